// Partition-centric layout of the PageRank side task's graph (internal to the library).
//
// The pull pass "acc[v] = sum over in-edges (u -> v) of contrib[u]" is a random 4-byte gather per edge when run
// straight off the CSR, and gathers, not bytes, are what a GPU runs out of.  The layout below turns the pass into
// two streaming sweeps whose random accesses all land in LDS (the two-phase partition-centric idea of Beamer et
// al., "propagation blocking", 2017, and Lakhotia et al., "PCPM", 2018, rebuilt around CDNA's 160 KB LDS):
//
//   * destination rows are cut into partitions of rows_per_part rows (8192, or 16384 from 2^22 vertices on);
//     sources into partitions of src_per_part (16384, or 32768 from 2^24 vertices on).  Larger partitions mean
//     fewer messages (more edges of a source fall into one partition) and longer bins of message traffic between
//     a source and a destination partition (M * rows_per_part * src_per_part / V^2 messages, which must not get
//     too short to stream), but only one workgroup per CU, and they must still leave every CU a tile: hence the
//     thresholds (256 gather tiles, 512 scatter tiles);
//   * all in-edges of one destination partition q are stored together, ordered by source u and then by row;
//     one MESSAGE is made per distinct (q, u) pair, however many rows of q the source u points to;
//   * scatter sweep, one workgroup per source partition p: the p-slice of contrib sits in LDS; for every q the
//     messages of bin (p, q) are written, msg[m] = contrib[src of m] -- sequential writes;
//   * gather sweep, one workgroup per destination partition q: 64-bit fixed-point accumulators for q's rows
//     sit in LDS; the id stream of q (one 16-bit local row id per edge, top bit set where a new message starts)
//     and q's messages are read sequentially and added into LDS with integer atomics.  Integer addition is
//     associative, so the sums do not depend on the order the hardware performs them in.
//
// Rows with more than hub_split in-edges ("hubs") would both unbalance their partition and serialise the LDS
// atomics, so each hub's in-edges are dealt out to virtual rows of at most hub_split edges, and the virtual rows
// are dealt round-robin over all partitions (each partition has kMaxVrowsPerPart spare accumulator slots behind
// its own rows); a small finishing step adds a hub's virtual rows up.  hub_split is kHubSplitMin unless the
// graph has so many hub edges that the spare slots would not hold them, in which case it is doubled until they do.
#pragma once

#include <cstdint>
#include <vector>

#include "common.h"

constexpr uint32_t kRowsSmall = 8192, kRowsLarge = 16384;   // destination rows per partition (8 B each in LDS)
constexpr uint32_t kSrcSmall = 16384, kSrcLarge = 32768;    // source vertices per scatter partition (4 B each in LDS)
constexpr int64_t kLargeRowsFrom = int64_t(1) << 22;        // vertex counts from which the large sizes are used
constexpr int64_t kLargeSrcFrom = int64_t(1) << 24;
constexpr uint32_t kHubSplitMin = 2048;      // rows with more in-edges than hub_split are split into virtual rows
constexpr uint32_t kMaxVrowsPerPart = 128;   // spare accumulator slots per partition for hubs' virtual rows
constexpr uint32_t kIdChunk = 512;           // ids per wavefront step (8 per lane, 64 apart)
constexpr uint32_t kHubsPerTile = 16;        // hubs finished per workgroup (16 lanes each)
constexpr int kKeyLocalBits = 15;            // sort key = partition << 46 | source << 15 | local row
constexpr uint32_t kLocalMask = (1u << kKeyLocalBits) - 1;
static_assert(kRowsLarge + kMaxVrowsPerPart <= (1u << kKeyLocalBits) && kSrcLarge <= 65536, "id fields");
constexpr int kKeySrcBits = 31;

struct PrLayout {
    int64_t V = 0, E = 0;
    uint64_t M = 0;                  // messages = distinct (destination partition, source) pairs
    uint32_t Q = 0;                  // destination partitions
    uint32_t P = 0;                  // source partitions
    uint32_t rows_per_part = kRowsSmall, src_per_part = kSrcSmall;
    uint32_t n_hubs = 0, n_vrows = 0;
    uint32_t hub_split = kHubSplitMin;
    uint32_t n_chunks = 0;           // ceil(E / kIdChunk)
    uint32_t n_hub_tiles = 1;

    // device arrays (allocated through the task's accounting allocator)
    uint16_t* ids16 = nullptr;       // [n_chunks * kIdChunk] local row id, bit 15 = first edge of a message;
                                     // each chunk stored transposed: stream position 64 j + lane at slot 8 lane + j
    uint16_t* src16 = nullptr;       // [M] source id relative to its source partition
    uint32_t* eoff = nullptr;        // [Q + 1] first edge (in sorted order) of every destination partition
    uint32_t* mbase = nullptr;       // [n_chunks + 1] messages that begin before each chunk
    uint2* bins = nullptr;           // [P * Q] message range [x, y) of bin (p, q), p-major
    int32_t* hub_row = nullptr;      // [n_hubs] row id of hub h
    uint32_t* hub_vbase = nullptr;   // [n_hubs + 1] first virtual row of hub h
    uint32_t* hub_of_p = nullptr;    // [P + 1] first hub (hubs are numbered in row order) of every source partition
    float* inv_tag = nullptr;        // [V] 1/outdeg (0 if dangling), sign bit set for hub rows

    // host copies used by the cost model
    std::vector<uint32_t> edges_of_q;    // [Q]
    std::vector<uint64_t> msgs_of_p;     // [P]

    // virtual rows dealt to partition q: those hv < n_vrows with hv % Q == q; hv sits in slot hv / Q
    uint32_t vrows_of_q(uint32_t q) const { return n_vrows > q ? (n_vrows - q + Q - 1) / Q : 0; }
};

// Builds the layout on `stream` from the caller's in-edge CSR (device pointers) and waits for it.
// rows_per_part / src_per_part: 0 = chosen from V, else one of the two sizes above (FR_ERR_ARG otherwise).
// Temporary memory is taken from and returned to `a`.  Returns FR_OK, FR_ERR_OOM, FR_ERR_HIP or FR_ERR_ARG
// (malformed CSR).  `hip_error` receives the failing HIP code, if any.
int pr_build_layout(PrLayout* L, int64_t V, int64_t E, const int32_t* row_ptr, const int32_t* col,
                    const int32_t* out_degree, uint32_t rows_per_part, uint32_t src_per_part, fr_alloc* a,
                    hipStream_t stream, int* hip_error);
