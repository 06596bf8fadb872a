// Partition-centric layout of the PageRank side task's graph (internal to the library).
//
// The pull pass "acc[v] = sum over in-edges (u -> v) of contrib[u]" is a random 4-byte gather per edge when run
// straight off the CSR, and gathers, not bytes, are what a GPU runs out of.  The layout below turns the pass into
// two streaming sweeps whose random accesses all land in LDS (the two-phase partition-centric idea of Beamer et
// al., "propagation blocking", 2017, and Lakhotia et al., "PCPM", 2018, rebuilt around CDNA's 160 KB LDS):
//
//   * vertices are renumbered by in-degree, largest first (ties by old id; without in-edges: by out-degree, largest
//     first); everything below is in new ids, and
//     perm[] leads back to the caller's ids when the final ranks are written.  With this order the rows that
//     receive most edges sit together, so that many edges of one source fall into one row range and share one
//     message: on an R-MAT graph of 2^22 vertices and 2^26 edges the messages drop from 0.50 to 0.20 per edge;
//   * destination rows are cut into RANGES of rows_per_part consecutive rows (8192, or 16384 from 2^22 vertices
//     on); sources into intervals of at most src_per_part (16384, or 32768 from 2^24 vertices on);
//   * all in-edges of one range j are stored together, ordered by source u and then by row; one MESSAGE is made
//     per distinct (j, u) pair, however many rows of j the source u points to;
//   * scatter sweep: contrib of a source interval p sits in LDS; for every range j the messages of bin (p, j)
//     are written, msg[m] = contrib[src of m] * 2^30 -- sequential writes;
//   * gather sweep: 64-bit fixed-point accumulators for the rows of one range sit in LDS; the id stream (one
//     16-bit local row id per edge, and one bit per edge that says where a new message starts) and the messages
//     are read sequentially and added into LDS with integer atomics.  Integer addition is associative, so the
//     sums do not depend on the order the hardware performs them in.
//
// Ordering by degree makes the ranges very unequal (the first range of that graph holds 42 % of the edges), so
// the unit of work is not the range but a TILE:
//   * a gather tile is a PIECE, a run of consecutive edges of one range (hence a source interval of it).  A range
//     heavier than a workgroup's share of the sweep is cut into several pieces and is a MERGED range: each of its
//     pieces stores its row sums as one row of fp32 partial sums (plain stores, no global atomics: 2.5 million
//     64-bit atomics from 150 workgroups were measured at 22 us on an otherwise idle chip), and the rows are
//     finished - partial sums added in a fixed tree order, then r and contrib - at the start of the next scatter
//     sweep.  This also spreads rows with very many in-edges over many workgroups; no other treatment of such rows
//     is needed.  A range with one piece is DIRECT: its piece finishes its rows itself;
//   * a scatter tile is a piece too: an interval of at most src_per_part consecutive sources, cut by weight
//     (messages + values read; narrow for the sources that point into many ranges); every source belongs to exactly
//     one piece, so the finishing of merged rows is done once per row.  The vertices without in-edges are ordered
//     by out-degree, so those of them without out-edges either, which send no message, form one run at the end; such
//     a run (any long run of sources without messages outside the merged ranges) is a VOID piece that belongs to no
//     tile;
//   * a launch has at most as many workgroups as run side by side; each starts on the tile of its own number and,
//     when done, takes the next tile nobody has taken yet (one atomic counter per task, reset by the last
//     workgroup to leave).  Tiles are in order of falling weight, so the light ones at the end fill the gaps the
//     heavy ones leave.  (With one fixed tile list per workgroup, cut by modelled weights, the sweeps of a graph of
//     2^26 vertices ran 14 % and 28 % over the mean time of their workgroups.)  What a tile computes does not depend
//     on which workgroup takes it;
//   * ranges behind the last row with an in-edge are EMPTY and have no gather piece: their rows' rank is the
//     iteration's base value, which the scatter sweep puts into its slice without reading a sum.
#pragma once

#include <cstdint>
#include <vector>

#include "common.h"

constexpr uint32_t kRowsSmall = 8192, kRowsLarge = 16384;   // destination rows per range (8 B each in LDS)
constexpr uint32_t kSrcSmall = 16384, kSrcLarge = 32768;    // source vertices per scatter partition (4 B each in LDS)
constexpr int64_t kLargeRowsFrom = int64_t(1) << 22;        // vertex counts from which the large sizes are used
constexpr int64_t kLargeSrcFrom = int64_t(1) << 24;
constexpr uint32_t kIdChunk = 512;           // ids per wavefront step (8 per lane, 64 apart)
constexpr uint32_t kStartWords = 12;         // 64-bit words of a chunk's message-start record
constexpr int kKeyLocalBits = 15;            // sort key = range << 46 | source << 15 | local row
constexpr uint32_t kLocalMask = (1u << kKeyLocalBits) - 1;
static_assert(kRowsLarge <= (1u << kKeyLocalBits) && kSrcLarge <= 65536, "id fields");
constexpr int kKeySrcBits = 31;
constexpr uint32_t kDefaultCus = 256;        // heavy ranges and source intervals are cut for this many workgroups side by side ...
constexpr uint64_t kMinTileEdges = 32768;    // ... but no smaller than this (in weight: times kGatherEdgeWeight)
constexpr uint64_t kMinTileMessages = 16384;
// weight of a gather tile = kGatherEdgeWeight * edges + kGatherMessageWeight * messages + kGatherRepeatWeight *
// repeated edges + kTileFixedWeight
constexpr uint64_t kGatherEdgeWeight = 2, kGatherMessageWeight = 0, kGatherRepeatWeight = 6, kTileFixedWeight = 147456;
// weight of a scatter tile = messages + values read for its sources (measured: a row of partial sums costs a tile
// about as much as a message, with one or with two workgroups per compute unit) + kScatterFixedWeight
constexpr uint64_t kScatterMessageWeight = 1, kScatterRowWeight = 1, kScatterFixedWeight = 8192;
// a slot's share of a sweep's weight from which on the sweep is cut fine: heavy parts for two pieces per slot, every
// piece a tile (measured: 2^24 vertices / 2^28 edges gains 15 % in the gather sweep and nothing in the scatter sweep,
// 2^26 / 2^30 gains 20 % and 24 %, 2^22 / 2^26 loses in both; three, four or six pieces per slot are no better than two)
constexpr uint64_t kGatherFineShare = 2000000, kScatterFineShare = 1000000;

// An id is stored as the byte offset of its row's 8-byte accumulator, or half of it where that needs 17 bits.
constexpr uint32_t id_scale_for(uint32_t rows_per_part) { return rows_per_part <= 8192 ? 8u : 4u; }

enum : uint32_t { kRangeDirect = 0, kRangeMerged = 1, kRangeEmpty = 2 };

constexpr uint32_t kNoPartial = 0xffffffffu;
constexpr uint32_t kNoVoid = 0xffffffffu;
constexpr uint64_t kVoidMin = 4096;           // sources in a run without messages from which on the run is a void piece
struct GatherPiece { uint32_t range, e0, e1, partial; };   // edges [e0, e1) of the sorted edge array; row of partial
                                                           // sums the piece writes (kNoPartial: direct range)
struct ScatterPiece { uint32_t u0, u1; };                  // sources [u0, u1)
struct RangeInfo { uint32_t cls_tiles, partial0; };        // class | gather tiles << 2; first row of partial sums
// a scatter tile: its piece p0 (p1 = p0 + 1), the piece's sources [u0, u1) and what range_info holds for the range of
// u0, so that the workgroup's first loads of vertex data depend on one load only
struct alignas(32) ScatterTile { uint32_t p0, p1, u0, u1; RangeInfo first; uint32_t pad[2]; };
static_assert(sizeof(ScatterTile) == 32, "read as two 16-byte words");
// a gather tile: its piece p0 (p1 = p0 + 1) and a copy of it, for the same reason
struct alignas(32) GatherTile { uint32_t p0, p1; GatherPiece first; uint32_t pad[2]; };
static_assert(sizeof(GatherTile) == 32, "read as two 16-byte words");

struct PrLayout {
    int64_t V = 0, E = 0;
    uint64_t M = 0;                  // messages = distinct (range, source) pairs
    uint32_t rows_per_part = kRowsSmall, src_per_part = kSrcSmall;
    uint32_t Q = 0;                  // ranges, ceil(V / rows_per_part)
    uint32_t Qe = 0;                 // ranges with at least one in-edge (they come first)
    uint32_t n_pieces = 0;           // gather pieces: runs of edges of one range
    uint32_t n_spieces = 0;          // scatter pieces: intervals of sources
    uint32_t n_gather = 0, n_scatter = 0;   // tiles (= pieces)
    uint32_t gather_slots = 0, scatter_slots = 0;   // workgroups of a sweep that run side by side
    uint32_t n_merged = 0;           // ranges cut into several gather pieces
    uint32_t n_partials = 0;         // gather pieces of merged ranges = rows of partial sums
    uint32_t n_finish = 0;           // merged + empty ranges (the tiles of the pass after the last iteration)
    bool scatter_packed = false;     // some scatter tile holds more than one piece
    uint32_t void_slot = kNoVoid;    // first void scatter piece (kNoVoid: none)
    uint64_t n_void_dangling = 0;    // rows of void pieces in ranges without in-edges
    uint32_t n_chunks = 0;           // ceil(E / kIdChunk)

    // device arrays (allocated through the task's accounting allocator)
    int32_t* perm = nullptr;         // [V] caller's id of new id v
    uint16_t* ids16 = nullptr;       // [n_chunks * kIdChunk] local row id times id_scale_for(rows_per_part);
                                     // each chunk stored transposed: stream position 64 j + lane at slot 8 lane + j
    uint64_t* starts = nullptr;      // [n_chunks * kStartWords] per chunk: eight words of message-start bits (one per 64
                                     // positions, shifted down by one) and, for the eight first positions, the byte offsets
                                     // of their messages from message mbase[chunk] - 1
    uint16_t* src16 = nullptr;       // [M] source id relative to the first source of its scatter piece
    uint32_t* mbase = nullptr;       // [n_chunks + 1] messages that begin before each chunk
    uint2* bins = nullptr;           // [n_spieces * Qe] message range [x, y) of (scatter piece, range), piece-major
    float* inv_out = nullptr;        // [V] 1/outdeg (0 if dangling)
    RangeInfo* range_info = nullptr; // [Q]
    GatherPiece* gather_pieces = nullptr;  // [n_pieces], heaviest ranges first
    GatherTile* gather_tiles = nullptr;    // [n_gather]
    ScatterPiece* scatter_pieces = nullptr;  // [n_spieces]
    ScatterTile* scatter_tiles = nullptr;  // [n_scatter]
    uint32_t* finish_ranges = nullptr;     // [n_finish] merged ranges, then empty ranges

    // host copies for the cost model
    std::vector<GatherPiece> gp;
    std::vector<GatherTile> gt;
    std::vector<uint64_t> gt_weight;     // weight of each gather tile (kTileFixedWeight included)
    std::vector<uint64_t> gt_edges;      // edges of each gather tile
    std::vector<ScatterPiece> sp;
    std::vector<ScatterTile> st;
    std::vector<uint64_t> st_msgs;       // messages of each scatter tile
    std::vector<uint64_t> st_rows;       // sources + partial sums added up, of each scatter tile
    std::vector<RangeInfo> ri;           // [Q]
    std::vector<uint32_t> fin;           // [n_finish]
};

// Builds the layout on `stream` from the caller's in-edge CSR (device pointers) and waits for it.
// rows_per_part / src_per_part: 0 = chosen from V, else one of the two sizes above (FR_ERR_ARG otherwise).
// Temporary memory is taken from and returned to `a`.  Returns FR_OK, FR_ERR_OOM, FR_ERR_HIP or FR_ERR_ARG
// (malformed CSR).  `hip_error` receives the failing HIP code, if any.
// cus: compute units the sweeps will have (heavy ranges and source intervals are cut for that many workgroups).
int pr_build_layout(PrLayout* L, int64_t V, int64_t E, const int32_t* row_ptr, const int32_t* col,
                    const int32_t* out_degree, uint32_t rows_per_part, uint32_t src_per_part, uint32_t cus, fr_alloc* a,
                    hipStream_t stream, int* hip_error);
