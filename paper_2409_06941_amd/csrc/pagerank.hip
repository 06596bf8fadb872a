// The PageRank side task: pull-based power iteration, fp32 ranks, for gfx950.
//
// The paper's graph-analytics side task (Section 6.1.4) with one iteration = one pass over the graph
// (Section 6.2), written as a step-wise task for the iterative interface (Section 4.2): work is cut into tiles
// that are fixed at init, a step is a run of consecutive tiles of one segment, and every tile computes the same
// bits whichever launch carries it, so pausing and resuming at any tile boundary cannot change the result.
//
// The pull pass runs on the partition-centric layout of pr_layout.h (vertices renumbered by in-degree).  One run =
//     V0, S_0 G_0, S_1 G_1, ..., S_{K-1} G_{K-1}, F
//   V0   vertex pass (tile = row range): dangling partials of r_0 = 1/V
//   S_k  scatter     (tile = source interval): contrib_k of the interval goes into LDS - r_0 / outdeg for k = 0,
//                    read back for rows of direct ranges, made on the spot for rows of merged ranges (partial
//                    sums of G_{k-1} added in tile order, then the vertex-pass arithmetic) and of empty ranges
//                    (r = base) - then one message per (range, source) is written
//   G_k  gather      (tile = run of edges of one range): id stream + messages -> 64-bit fixed-point sums in LDS;
//                    direct range: fused, the next vertex pass for its rows,
//                    r_{k+1} = base_k + d * sum, contrib_{k+1} = r_{k+1} / outdeg, dangling partials;
//                    merged range: the sums are stored as one row of fp32 partial sums
//   F    finish      (tile = merged or empty range): after the last iteration, r_K of their rows
// base_k = (1 - d)/V + d * D_k / V, D_k = fixed-order sum of the dangling partials of r_k.
// In the last iteration G writes r_K to ranks_out (through perm) instead of contrib; F does the same.
// No floating-point atomics anywhere: float sums have a fixed order, the LDS atomics add integers.

#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>

#include "freeride_device.h"
#include "pr_layout.h"

namespace {

constexpr int kBlock = 512;                     // threads per workgroup of the first vertex pass
constexpr int kGatherBlock = 1024;              // threads per workgroup of the gather sweep
constexpr int kGatherWaves = kGatherBlock / 64;
constexpr int kScatterBlock = 1024;             // threads per workgroup of the scatter sweep
constexpr int kScatterWaves = kScatterBlock / 64;
// row sums are kept as 64-bit fixed point with scale 2^62: contrib sums are <= 1, so they fit
constexpr float kFixInv = 1.0f / 4611686018427387904.0f;
// messages are contrib * 2^30: see to_fixed
constexpr float kMsgScale = 1073741824.0f;

// ---- fixed-order reductions ----
__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, 64);
    return x;
}

// Sum of a per-thread value over the workgroup, same association for a given blockDim.  All threads call.
__device__ __forceinline__ float block_sum(float x, float* lds /* one float per wavefront */)
{
    x = wave_sum(x);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    __syncthreads();
    if (lane == 0) lds[w] = x;
    __syncthreads();
    float s = 0.0f;
    const int nw = (int)(blockDim.x >> 6);
    for (int i = 0; i < nw; ++i) s += lds[i];
    return s;
}

// D = sum of dpart[0 .. n).  Every wavefront adds the whole array up by itself, in one fixed order (lane l takes
// the elements l, l + 64, l + 128, ... into four running sums in turn; the four are joined pairwise, the lanes by
// a butterfly), so all wavefronts of all kernels get the same bits, and no barrier stands between the loads of
// the array and the loads of the work that follows: the sum is only waited for where it is first used.
__device__ __forceinline__ float dangling_total(const float* __restrict__ dpart, uint32_t n)
{
    const uint32_t lane = threadIdx.x & 63;
    float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
    uint32_t i = lane;
    for (; i + 192 < n; i += 256) {
        const float a = dpart[i], b = dpart[i + 64], c = dpart[i + 128], d = dpart[i + 192];
        s0 += a; s1 += b; s2 += c; s3 += d;
    }
    if (i < n) s0 += dpart[i];
    if (i + 64 < n) s1 += dpart[i + 64];
    if (i + 128 < n) s2 += dpart[i + 128];
    return wave_sum((s0 + s1) + (s2 + s3));
}

struct DevArgs {
    int64_t V, E;
    uint32_t M, Q, Qe, n_gather, n_pieces, n_scatter, n_spieces, n_finish, n_dpart;
    uint32_t rows_per_part, rows_shift;           // rows per range and its log2
    uint32_t void_slot;                           // scatter piece whose slot of dangling partials takes the void pieces' mass (kNoVoid: none)
    float n_void_dangling;                        // rows of void pieces in ranges without in-edges: each holds the base value
    float damping;
    const uint16_t* ids16;
    const uint16_t* src16;
    const uint32_t* mbase;
    const uint64_t* starts;
    const uint2* bins;
    const float* inv_out;
    const int32_t* perm;
    const RangeInfo* range_info;
    const GatherPiece* gather_pieces;
    const GatherTile* gather_tiles;
    const ScatterPiece* scatter_pieces;
    const ScatterTile* scatter_tiles;
    const uint32_t* finish_ranges;
    float* msg;
    float* contrib;
    float* dpart;                 // [2][n_dpart]
    float* partials;              // [n_partials][rows_per_part]
    float* ranks_out;
    uint32_t* sched;              // [2] tiles handed out beyond a launch's first round; workgroups that have left
};

// What a step's kernels need to ask the device gate (Section 4.5's check, made by the GPU when the kernel starts).
struct GateArg {
    fr_gate* gate;                // NULL: no gate
    uint32_t slot, need_ticks;    // need_ticks: the whole step's modelled duration
    uint32_t tile_ticks;          // the modelled duration of the step's heaviest tile run alone
};

// Sum of a merged row's partial sums p_0 .. p_{nt-1}.  The order is fixed: sixteen leaves, leaf g = p_g + p_{g+16} +
// ... in rising order, joined by a balanced tree over g.  kLanes lanes (a power of two up to 16, consecutive in
// the wavefront, all active) share the row: lane `sub` owns the leaves sub * 16 / kLanes onwards, joins them, and
// the lanes' results are joined by butterfly exchanges, which is the same tree.  Every lane gets the sum.
template <int kLanes>
__device__ __forceinline__ float merged_sum(const DevArgs& A, RangeInfo info, uint32_t local, uint32_t sub)
{
    constexpr int kLeaves = 16 / kLanes;
    const uint32_t nt = info.cls_tiles >> 2;
    const float* p = A.partials + ((size_t)info.partial0 << A.rows_shift) + local;
    float s[kLeaves];
#pragma unroll
    for (int k = 0; k < kLeaves; ++k) s[k] = 0.0f;
    // (all loads of a round, up to sixteen, are issued before the first is used)
    for (uint32_t t0 = 0; t0 < nt; t0 += 16) {
        float x[kLeaves];
#pragma unroll
        for (int k = 0; k < kLeaves; ++k) {
            const uint32_t t = t0 + sub * kLeaves + k;
            x[k] = t < nt ? p[(size_t)t << A.rows_shift] : 0.0f;
        }
#pragma unroll
        for (int k = 0; k < kLeaves; ++k) s[k] += x[k];
    }
#pragma unroll
    for (int w = 1; w < kLeaves; w <<= 1)
#pragma unroll
        for (int k = 0; k + w < kLeaves; k += 2 * w) s[k] += s[k + w];
    float r = s[0];
#pragma unroll
    for (int off = 1; off < kLanes; off <<= 1) r += __shfl_xor(r, off, 64);
    return r;
}

// Rows [i0, i1) of a scatter tile's slice, all in one merged range: r = base + d * (sum of the row's partial sums),
// contrib = r / outdeg.  kLanes lanes work on a row.  Returns this thread's share of the dangling mass.
template <int kLanes, int kThreads>
__device__ __forceinline__ float fill_merged(const DevArgs& A, RangeInfo info, uint32_t u0, uint32_t i0, uint32_t i1, float base, float* slice)
{
    const uint32_t sub = threadIdx.x % kLanes;
    float dangling = 0.0f;
    for (uint32_t ib = i0; ib < i1; ib += kThreads / kLanes) {       // uniform trip count: the lanes exchange values
        const uint32_t i = ib + threadIdx.x / kLanes;
        if (i >= i1) continue;                                       // (all lanes of a row leave together)
        const uint32_t u = u0 + i;
        const float inv = A.inv_out[u];
        const float r = fmaf(A.damping, merged_sum<kLanes>(A, info, u & (A.rows_per_part - 1), sub), base);
        if (sub == 0) {
            slice[i] = r * inv * kMsgScale;
            dangling += (inv == 0.0f ? r : 0.0f);
        }
    }
    return dangling;
}

// contrib of the sources [u0, u0 + n) of a scatter tile for an iteration after the first, into `slice`; returns
// this thread's share of the dangling mass among the rows finished here.  The sources lie in a handful of ranges.
// kOneKind (the large slice): where these are all of one kind and not merged - nearly all pieces of the sources with
// few messages - every row needs one value from one array (its contrib, finished by the range's gather tile, or
// 1/outdeg if the rows have no in-edges), and the slice is read in rounds of kFillRound rows per thread whose loads
// are all issued before the first is used, whatever the ranges' boundaries: two memory latencies for 32768 sources
// (walked range by range, a round per range, it was three or four, and 24 us of a piece's 33 with four rows a round).
// Otherwise the tile is walked range by range, so that each loop has one kind of row.
// `first_info`: what range_info holds for the range of u0.
template <int kThreads, int kFillRound, bool kOneKind>
__device__ __forceinline__ float fill_slice(const DevArgs& A, uint32_t u0, uint32_t n, float base, float* slice, RangeInfo first_info)
{
    if constexpr (kOneKind) {
        const uint32_t q0 = u0 >> A.rows_shift, q_last = (u0 + n - 1) >> A.rows_shift;
        const uint32_t cls0 = first_info.cls_tiles & 3u;
        bool same = cls0 != kRangeMerged;
        for (uint32_t q = q0 + 1; q <= q_last; ++q) same = same && (A.range_info[q].cls_tiles & 3u) == cls0;
        if (same) {
            const float* __restrict__ from = (cls0 == kRangeDirect ? A.contrib : A.inv_out) + u0;
            float dangling = 0.0f;
            for (uint32_t ib = threadIdx.x; ib < n; ib += kFillRound * kThreads) {
                float v[kFillRound];
#pragma unroll
                for (int k = 0; k < kFillRound; ++k) {
                    const uint32_t i = ib + k * kThreads;
                    v[k] = i < n ? from[i] : 1.0f;
                }
                if (cls0 == kRangeDirect) {
#pragma unroll
                    for (int k = 0; k < kFillRound; ++k) {
                        const uint32_t i = ib + k * kThreads;
                        if (i < n) slice[i] = v[k] * kMsgScale;
                    }
                } else {
#pragma unroll
                    for (int k = 0; k < kFillRound; ++k) {
                        const uint32_t i = ib + k * kThreads;
                        if (i < n) slice[i] = base * v[k] * kMsgScale;
                        dangling += (v[k] == 0.0f ? base : 0.0f);
                    }
                }
            }
            return dangling;
        }
    }
    float dangling = 0.0f;
    for (uint32_t i0 = 0; i0 < n;) {
        const uint32_t q = (u0 + i0) >> A.rows_shift;
        const uint32_t range_end = ((q + 1) << A.rows_shift) - u0;
        const uint32_t i1 = range_end < n ? range_end : n;
        const RangeInfo info = i0 == 0 ? first_info : A.range_info[q];
        const uint32_t cls = info.cls_tiles & 3u;
        if (cls == kRangeDirect || cls == kRangeEmpty) {
            // one value per row: contrib, finished by the range's gather tile, or 1/outdeg of a row without in-edges.
            // All loads of a round are issued before the first is used: a round is kFillRound rows per thread, and a
            // range's share of the slice is no more than that at 1024 threads, so the slice costs one memory latency.
            const float* __restrict__ from = cls == kRangeDirect ? A.contrib : A.inv_out;
            for (uint32_t ib = i0 + threadIdx.x; ib < i1; ib += kFillRound * kThreads) {
                float v[kFillRound];
#pragma unroll
                for (int k = 0; k < kFillRound; ++k) {
                    const uint32_t i = ib + k * kThreads;
                    v[k] = i < i1 ? from[u0 + i] : 1.0f;
                }
                if (cls == kRangeDirect) {
#pragma unroll
                    for (int k = 0; k < kFillRound; ++k) {
                        const uint32_t i = ib + k * kThreads;
                        if (i < i1) slice[i] = v[k] * kMsgScale;
                    }
                } else {
#pragma unroll
                    for (int k = 0; k < kFillRound; ++k) {
                        const uint32_t i = ib + k * kThreads;
                        if (i < i1) slice[i] = base * v[k] * kMsgScale;
                        dangling += (v[k] == 0.0f ? base : 0.0f);
                    }
                }
            }
        } else {
            // few rows (sources with many messages; their rows are the ones with many partial sums): several lanes a row
            const uint32_t len = i1 - i0;
            if (len * 16 <= kThreads) dangling += fill_merged<16, kThreads>(A, info, u0, i0, i1, base, slice);
            else if (len * 4 <= kThreads) dangling += fill_merged<4, kThreads>(A, info, u0, i0, i1, base, slice);
            else if (len * 2 <= kThreads) dangling += fill_merged<2, kThreads>(A, info, u0, i0, i1, base, slice);
            else dangling += fill_merged<1, kThreads>(A, info, u0, i0, i1, base, slice);
        }
        i0 = i1;
    }
    return dangling;
}

// ---- V0 ----
__global__ __launch_bounds__(kBlock) void k_vertex0(DevArgs A, GateArg G, uint32_t tile0, int final_pass)
{
    __shared__ float red[8];
    if (!fr_gate_admit(G.gate, G.slot, G.need_ticks)) return;
    const uint32_t q = tile0 + blockIdx.x;
    const int64_t v0 = (int64_t)q << A.rows_shift;
    const float r0 = 1.0f / (float)A.V;
    float dangling = 0.0f;
    for (uint32_t i = threadIdx.x; i < A.rows_per_part; i += kBlock) {
        const int64_t v = v0 + i;
        if (v >= A.V) break;
        if (final_pass) A.ranks_out[v] = r0;              // every vertex gets the same value: no need for perm
        else dangling += (A.inv_out[v] == 0.0f ? r0 : 0.0f);
    }
    if (!final_pass) {
        const float total = block_sum(dangling, red);
        if (threadIdx.x == 0) A.dpart[q] = total;
        if (q == 0)
            for (uint32_t i = A.Q + threadIdx.x; i < A.n_dpart; i += kBlock) A.dpart[i] = 0.0f;
    }
    fr_gate_done(G.gate, G.slot);
}

// Workgroups are handed to the 8 XCDs round-robin (workgroup b runs on XCD b % 8), and every XCD has an L2 of its
// own.  This map gives every XCD runs of kTileRun consecutive tiles, the runs dealt round-robin: neighbouring tiles
// write neighbouring messages (and share the lines at the seams) through one L2, while the heaviest tiles, which
// come first and read the most partial sums, are spread over all XCDs (in one contiguous block per XCD they were
// measured to take twice as long to fill their slices).  It is a bijection on [0, n) for any n.
constexpr uint32_t kTileRun = 4;
__device__ __forceinline__ uint32_t xcd_runs(uint32_t b, uint32_t n)
{
    constexpr uint32_t kXcds = 8;
    const uint32_t full = n / (kXcds * kTileRun) * (kXcds * kTileRun);
    if (b >= full) return b;
    return ((b / kXcds / kTileRun) * kXcds + b % kXcds) * kTileRun + (b / kXcds) % kTileRun;
}

// ---- hand-out of a launch's tiles ----
// A launch covers the tiles tile0 .. tile0 + n - 1 of one segment with g <= n workgroups.  Workgroup b starts on
// the b-th of them (the first g dealt by first_round).  If n > g, it asks towards the end of every tile for the next
// tile nobody has taken: tile g + (value of a counter that every asker bumps); the answer is looked at once the
// tile in hand is done, so most of the atomic's round trip is covered (asked at the start of a tile, the answer
// stood in the way of the tile's first loads, which the hardware hands back in order: with all workgroups of
// a launch asking at once that was 10 to 20 us).  The last workgroup to leave puts the two words back to zero for
// the next launch (launches of one task run one after the other on one stream).  Which workgroup takes which tile has
// no bearing on what the tile computes.  Thread 0 only.
constexpr uint32_t kHandOutStopped = 1u << 30;      // set in the counter: every later asker is sent home
constexpr uint32_t kAskLater = 0xffffffffu;

__device__ __forceinline__ uint32_t ask_next_tile(uint32_t* sched)
{
    return gridDim.x + atomicAdd(&sched[0], 1u);        // (at or beyond the launch's tile count: nothing left)
}

// With the device gate: the time left in the bubble is no longer enough for another tile.  The hand-out stops - the
// tiles taken so far, which form the head of the launch's tile list, are finished by their workgroups - and the
// first workgroup to find this out records how many tiles that is.  Returns a tile number beyond the launch.
__device__ __forceinline__ uint32_t stop_hand_out(uint32_t* sched, const GateArg& G, uint32_t n_tiles)
{
    const uint32_t before = atomicOr(&sched[0], kHandOutStopped);
    if (!(before & kHandOutStopped)) {
        const uint32_t taken = gridDim.x + before < n_tiles ? gridDim.x + before : n_tiles;
        if (taken < n_tiles) fr_gate_stop_short(G.gate, G.slot, taken);
    }
    return n_tiles;
}

// The question for the next tile, put late in a tile (ahead_ticks: what of the tile is still to come): asked only
// if the gate leaves time for the rest of this tile and another one, else put off to the tile's end.
__device__ __forceinline__ uint32_t ask_if_time(uint32_t* sched, const GateArg& G)
{
    return fr_gate_may_take(G.gate, G.tile_ticks, G.tile_ticks) ? ask_next_tile(sched) : kAskLater;
}

// At a tile's end: the answer, asking now if that was put off and stopping the hand-out if time has run out.
__device__ __forceinline__ uint32_t settle_next_tile(uint32_t asked, uint32_t* sched, const GateArg& G, uint32_t n_tiles)
{
    if (asked != kAskLater) return asked;
    return fr_gate_may_take(G.gate, 0u, G.tile_ticks) ? ask_next_tile(sched) : stop_hand_out(sched, G, n_tiles);
}

__device__ __forceinline__ void leave_launch(uint32_t* sched)
{
    // (this thread's own asks have returned: their values were used)
    if (atomicAdd(&sched[1], 1u) == gridDim.x - 1) {
        __hip_atomic_store(&sched[0], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&sched[1], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// The two words start at zero (and every launch leaves them so).
__global__ void k_clear_sched(uint32_t* sched)
{
    if (threadIdx.x < 2) sched[threadIdx.x] = 0u;
}

// ---- S_k ----
// One workgroup per scatter tile at a time: contrib of its sources sits in LDS, and for every range j the messages of bin
// (tile, j) - a contiguous run [x, y) of message numbers - are written.  The unit of work is a GROUP of eight
// consecutive message numbers, aligned to eight: one 16-byte load brings the eight sources, eight LDS reads their
// contrib, two 16-byte stores write the messages (groups cut by the ends of a bin store element by element).
// The groups of all bins of a batch are numbered consecutively (prefix sums in LDS) and dealt to the threads
// round-robin, so bins of any length keep all lanes busy; a thread finds a group's bin by binary search.
// The load for a thread's next group is issued before the current one is worked on.
constexpr uint32_t kDescBatch = 1024;       // bins per batch
constexpr uint32_t kGroup = 8;

// Exclusive prefix sums of one value per thread over the workgroup (kScatterBlock threads); out[i] = sum of the
// values of threads < i for i <= kScatterBlock.  `wave_tot` holds kScatterWaves + 1 words.
__device__ __forceinline__ void block_exclusive_scan(uint32_t value, uint32_t* out, uint32_t* wave_tot)
{
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t incl = value;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t up = (uint32_t)__shfl_up((int)incl, off, 64);
        if (lane >= (uint32_t)off) incl += up;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t run = 0;
        for (int w = 0; w < kScatterWaves; ++w) { const uint32_t x = wave_tot[w]; wave_tot[w] = run; run += x; }
        wave_tot[kScatterWaves] = run;
    }
    __syncthreads();
    out[threadIdx.x] = wave_tot[wave] + incl - value;
    if (threadIdx.x == 0) out[kScatterBlock] = wave_tot[kScatterWaves];
    __syncthreads();
}

struct GroupRef {
    uint32_t m0;      // first message number of the group (multiple of kGroup)
    uint32_t bin;     // its bin in the batch
};

// Group number k of the batch: its bin is the last one whose first group number is <= k.
__device__ __forceinline__ GroupRef locate_group(uint32_t k, const uint32_t* gpre, const uint2* desc, uint32_t nb)
{
    uint32_t lo = 0, hi = nb;
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (gpre[mid] <= k) lo = mid;
        else hi = mid;
    }
    GroupRef g;
    g.bin = lo;
    g.m0 = (desc[lo].x / kGroup + (k - gpre[lo])) * kGroup;
    return g;
}

__device__ __forceinline__ void emit_group(const GroupRef& ref, const uint2* desc, const uint4& raw, const float* slice, uint32_t n,
                                           float* __restrict__ msg)
{
    struct { uint32_t m0, x, y; } g = {ref.m0, desc[ref.bin].x, desc[ref.bin].y};
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
    float val[kGroup];
#pragma unroll
    for (int e = 0; e < (int)kGroup; ++e) {
        const uint32_t src = (e & 1) ? (w[e >> 1] >> 16) : (w[e >> 1] & 0xffffu);
        val[e] = src < n ? slice[src] : 0.0f;
    }
    if (g.m0 >= g.x && g.m0 + kGroup <= g.y) {
        float4* out = reinterpret_cast<float4*>(msg + g.m0);
        out[0] = make_float4(val[0], val[1], val[2], val[3]);
        out[1] = make_float4(val[4], val[5], val[6], val[7]);
    } else {
#pragma unroll
        for (int e = 0; e < (int)kGroup; ++e)
            if (g.m0 + e >= g.x && g.m0 + e < g.y) msg[g.m0 + e] = val[e];
    }
}

// `parity` names the set of dangling partials that belongs to the iteration just finished (ignored when first).
// (two workgroups of the small size share a CU: 8 wavefronts per SIMD, hence at most 64 registers per lane)
// kPacked: some tile has more than one piece (kept apart: the loop over pieces costs the small size registers it
// does not have).
// kDynamic: the launch has more tiles than workgroups (else a workgroup's one tile is all it does, and the code of
// the hand-out, which costs registers too, is left out).
template <uint32_t kSrcPerPart, bool kPacked, bool kDynamic>
__global__ __launch_bounds__(kScatterBlock) __attribute__((amdgpu_waves_per_eu(kSrcPerPart == kSrcSmall ? 8 : 4, kSrcPerPart == kSrcSmall ? 8 : 4)))
void k_scatter(DevArgs A, GateArg G, uint32_t tile0, uint32_t n_tiles, int parity, int first)
{
    __shared__ __align__(16) float slice[kSrcPerPart];
    __shared__ uint2 desc[kDescBatch];
    __shared__ uint32_t gpre[kScatterBlock + 1];          // groups before each bin of the batch; [kScatterBlock] = all
    __shared__ uint32_t wave_tot[kScatterWaves + 1];
    __shared__ float red[kScatterWaves];
    __shared__ uint32_t next_local;
    static_assert(kDescBatch <= kScatterBlock, "one bin per thread");
    if (!fr_gate_admit(G.gate, G.slot, kDynamic ? G.tile_ticks : G.need_ticks)) return;
    const uint32_t Qe = A.Qe;
    float base = 0.0f;
    if (!first) {
        const float D = dangling_total(A.dpart + (size_t)parity * A.n_dpart, A.n_dpart);
        base = (1.0f - A.damping) / (float)A.V + A.damping * D / (float)A.V;
    }
    const uint4* src8 = reinterpret_cast<const uint4*>(A.src16);
    // rows a thread reads per round while the slice is filled (the small size has 64 registers per lane)
    constexpr int kFillRound = kSrcPerPart == kSrcSmall ? 4 : 16;
    uint32_t asked = kAskLater;          // thread 0: the answer to its question for the next tile
    bool last_piece = false;
    auto do_piece = [&](uint32_t t, ScatterPiece T, RangeInfo first_info) {
        // the first batch of bin descriptors is asked for now and used after the slice is filled
        uint2 d_first = make_uint2(0, 0);
        if (threadIdx.x < Qe) d_first = A.bins[(uint64_t)t * Qe + threadIdx.x];
        const uint32_t u0 = T.u0;
        const uint32_t n = T.u1 - T.u0 < kSrcPerPart ? T.u1 - T.u0 : kSrcPerPart;
        if (first) {
            const float r0 = 1.0f / (float)A.V;
            for (uint32_t ib = threadIdx.x; ib < n; ib += kFillRound * kScatterBlock) {
                float v[kFillRound];
#pragma unroll
                for (int k = 0; k < kFillRound; ++k) {
                    const uint32_t i = ib + k * kScatterBlock;
                    v[k] = i < n ? A.inv_out[u0 + i] : 0.0f;
                }
#pragma unroll
                for (int k = 0; k < kFillRound; ++k) {
                    const uint32_t i = ib + k * kScatterBlock;
                    if (i < n) slice[i] = r0 * v[k] * kMsgScale;
                }
            }
        } else {
            const float total = block_sum(fill_slice<kScatterBlock, kFillRound, kSrcPerPart == kSrcLarge>(A, u0, n, base, slice, first_info), red);
            if (threadIdx.x == 0) A.dpart[(size_t)(parity ^ 1) * A.n_dpart + A.n_pieces + t] = total;
        }
        for (uint32_t qb = 0; qb < Qe; qb += kDescBatch) {
            const uint32_t nb = Qe - qb < kDescBatch ? Qe - qb : kDescBatch;
            __syncthreads();                                     // slice filled / previous batch consumed
            uint32_t groups = 0;
            if (threadIdx.x < nb) {
                uint2 d = qb == 0 ? d_first : A.bins[(uint64_t)t * Qe + qb + threadIdx.x];
                if (d.y > A.M) d.y = A.M;
                if (d.x > d.y) d.x = d.y;
                desc[threadIdx.x] = d;
                if (d.y > d.x) groups = (d.y - 1) / kGroup - d.x / kGroup + 1;
            }
            block_exclusive_scan(groups, gpre, wave_tot);
            const uint32_t total = gpre[kScatterBlock];
            constexpr int kAhead = 4;                            // groups a thread has in flight
            for (uint32_t k0 = threadIdx.x; k0 < total; k0 += kAhead * kScatterBlock) {
                // the question for the next tile goes out with the tile's last groups: put earlier, a workgroup on a
                // heavy tile would book its next tile hundreds of microseconds before it is free to start it
                if constexpr (kDynamic)
                    if (threadIdx.x == 0 && last_piece && qb + kDescBatch >= Qe && k0 + kAhead * kScatterBlock >= total)
                        asked = ask_if_time(A.sched, G);
                GroupRef ref[kAhead];
                uint4 raw[kAhead];
#pragma unroll
                for (int a = 0; a < kAhead; ++a) {
                    const uint32_t k = k0 + a * kScatterBlock;
                    ref[a] = GroupRef{0, 0};
                    raw[a] = make_uint4(0, 0, 0, 0);
                    if (k < total) { ref[a] = locate_group(k, gpre, desc, nb); raw[a] = src8[ref[a].m0 / kGroup]; }
                }
#pragma unroll
                for (int a = 0; a < kAhead; ++a)
                    if (k0 + a * kScatterBlock < total) emit_group(ref[a], desc, raw[a], slice, n, A.msg);
            }
        }
    };
    uint32_t local = xcd_runs(blockIdx.x, gridDim.x);
    do {
        if (tile0 + local == 0 && !first && A.void_slot != kNoVoid && threadIdx.x == 0)       // (once per sweep)
            A.dpart[(size_t)(parity ^ 1) * A.n_dpart + A.n_pieces + A.void_slot] = base * A.n_void_dangling;
        asked = kAskLater;
        const uint4* rec = reinterpret_cast<const uint4*>(A.scatter_tiles + tile0 + local);
        const uint4 span = rec[0];                               // x, y: the tile's pieces, worked on one after the other;
        const uint4 span_info = rec[1];                          // z, w: the sources of the first; then their range
        if constexpr (!kPacked) {
            last_piece = true;
            do_piece(span.x, ScatterPiece{span.z, span.w}, RangeInfo{span_info.x, span_info.y});
            __syncthreads();                                     // the piece is done with slice and desc
        } else {
            for (uint32_t t = span.x; t < span.y; ++t) {
                last_piece = t + 1 == span.y;
                if (t == span.x) {
                    do_piece(t, ScatterPiece{span.z, span.w}, RangeInfo{span_info.x, span_info.y});
                } else {
                    const ScatterPiece T = A.scatter_pieces[t];
                    do_piece(t, T, first ? RangeInfo{kRangeEmpty, 0} : A.range_info[T.u0 >> A.rows_shift]);
                }
                __syncthreads();                                 // the piece is done with slice and desc
            }
        }
        if constexpr (kDynamic) {
            if (threadIdx.x == 0) next_local = settle_next_tile(asked, A.sched, G, n_tiles);
            __syncthreads();
            local = next_local;
        }
    } while (kDynamic && local < n_tiles);
    if constexpr (kDynamic)
        if (threadIdx.x == 0) leave_launch(A.sched);
    fr_gate_done(G.gate, G.slot);
}

// ---- G_k ----

// floor(x * 2^62) for 0 <= x <= 1, exactly, from t = x * 2^30 (the scatter sweep writes its messages scaled so: a
// power of two, hence exact, and one multiplication less per edge here): the integer part of t is the high word,
// its fraction times 2^32 (exact again, then truncated) the low word.
__device__ __forceinline__ unsigned long long to_fixed(float t)
{
    const uint32_t hi = (uint32_t)t;
    const uint32_t lo = (uint32_t)(__builtin_amdgcn_fractf(t) * 4294967296.0f);
    return ((unsigned long long)hi << 32) | lo;
}

__device__ __forceinline__ unsigned long long* acc_at(unsigned long long* acc, uint32_t byte_offset)
{
    return reinterpret_cast<unsigned long long*>(reinterpret_cast<char*>(acc) + byte_offset);
}

__device__ __forceinline__ uint32_t id_of(const uint4& raw, int j)
{
    const uint32_t w = (j >> 1) == 0 ? raw.x : (j >> 1) == 1 ? raw.y : (j >> 1) == 2 ? raw.z : raw.w;
    return (j & 1) ? (w >> 16) : (w & 0xffffu);
}

// One workgroup per gather tile; it takes the tile's pieces one after the other, the accumulators of the piece's
// range (one u64 per row) in LDS.  Per step a wavefront takes one chunk of 512 ids (8 per lane).  The loop is a
// three-stage software pipeline over the wavefront's chunks, so that no step waits on a load it has just issued:
//   A  ids, message-start record and message base of the chunk two steps on are requested;
//   B  this step's chunk (ids now here): the start bits tell every id which message it belongs to; the
//      messages are requested (64 consecutive ids per load, so the addresses are all but contiguous);
//   C  the chunk of the step before (messages now here): each id adds its message, as a 64-bit fixed-point
//      integer, to its row's accumulator with an LDS atomic.
// Chunks that lie wholly inside the tile's edge range and whose messages cannot pass the end of the message array -
// all but the first and last chunk of a tile - take a path without per-id checks (8 vector instructions per 64
// edges instead of 25).  On a graph of 2^26 edges the sweep then moves its bytes at about 4.7 TB/s, which is what
// the memory system gives this mix of streams: taking a sixth of the vector instructions out of the loop changed
// nothing, a third or fourth buffer of messages in flight made it 6 to 9 % slower, and so did start records that
// come through a vector load (one dword a lane, handed to the scalar side with readlane) instead of scalar loads.
// (two workgroups of the small size share a CU: 8 wavefronts per SIMD, hence at most 64 registers per lane)
template <uint32_t kRowsPerPart, bool kDynamic>
__global__ __launch_bounds__(kGatherBlock) __attribute__((amdgpu_waves_per_eu(kRowsPerPart == kRowsSmall ? 8 : 4, kRowsPerPart == kRowsSmall ? 8 : 4)))
void k_gather(DevArgs A, GateArg G, uint32_t tile0, uint32_t n_tiles, int parity, int final_pass, const uint64_t* __restrict__ starts,
              const uint32_t* __restrict__ mbase)
{
    constexpr uint32_t kAccSlots = kRowsPerPart;
    constexpr uint32_t kIdScale = id_scale_for(kRowsPerPart);
    static_assert(65535u * (8 / kIdScale) + 8 <= (kAccSlots + 1) * 8, "any id addresses a slot of acc");
    __shared__ unsigned long long acc[kAccSlots + 1];            // + the sink slot
    __shared__ float red[kGatherWaves];
    __shared__ uint32_t next_local;
    if (!fr_gate_admit(G.gate, G.slot, kDynamic ? G.tile_ticks : G.need_ticks)) return;
    const float D = dangling_total(A.dpart + (size_t)parity * A.n_dpart, A.n_dpart);
    const float base = (1.0f - A.damping) / (float)A.V + A.damping * D / (float)A.V;
    float* dnext = A.dpart + (size_t)(parity ^ 1) * A.n_dpart;
    if (tile0 == 0 && blockIdx.x == 0 && !final_pass)            // slots no gather piece writes: the scatter tiles of the next sweep
        for (uint32_t i = A.n_pieces + threadIdx.x; i < A.n_dpart; i += kGatherBlock) dnext[i] = 0.0f;     // fill theirs in, void pieces have none
    uint32_t local = blockIdx.x;
    do {
    const uint4* rec = reinterpret_cast<const uint4*>(A.gather_tiles + tile0 + local);
    const uint4 span = rec[0];                                   // x, y: the tile's pieces, worked on one after the other;
    const uint4 span_more = rec[1];                              // then a copy of the first (saves a dependent load)
    uint32_t asked = 0;
    for (uint32_t t = span.x; t < span.y; ++t) {
    const GatherPiece T = t == span.x ? GatherPiece{span.z, span.w, span_more.x, span_more.y} : A.gather_pieces[t];
    const uint32_t q = T.range;
    const int64_t left = A.V - (int64_t)q * kRowsPerPart;
    const uint32_t nrows = (uint32_t)(left < (int64_t)kRowsPerPart ? left : (int64_t)kRowsPerPart);
    for (uint32_t i = threadIdx.x; i < kAccSlots + 1; i += kGatherBlock) acc[i] = 0ull;
    __syncthreads();

    const uint32_t e0 = T.e0, e1 = T.e1 < (uint64_t)A.E ? T.e1 : (uint32_t)A.E;
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (e1 > e0) {
        const uint32_t c0 = e0 / kIdChunk, c1 = (e1 - 1) / kIdChunk;
        const uint4* ids4 = reinterpret_cast<const uint4*>(A.ids16);
        // Stage A's result: a chunk's ids, its message-start bits and the number of messages begun before it.  The
        // chunk number is the same in all lanes of a wavefront; saying so lets the bits and the count come through
        // the scalar unit, which leaves them where the arithmetic of stage B wants them.  There are kRing of these:
        // a buffer is asked for its next chunk as soon as stage B has used it, kRing - 1 steps before that chunk's
        // turn, so a wavefront has that many steps of work to cover the latency of the request.
        struct Ids {
            uint4 raw;
            uint32_t mb;
            uint64_t starts[8];      // row j: start bits of its positions 1 .. 63
            uint32_t first[8];       // row j: byte offset of the message of its position 0 from message mb - 1
        };
        constexpr int kRing = 2;     // (the records live in scalar registers: there is room for two)
        const uint32_t wave_u = (uint32_t)__builtin_amdgcn_readfirstlane((int)wave);
        auto load_ids = [&](Ids& I, uint32_t c) {
            if (c <= c1) {
                I.raw = ids4[(uint64_t)c * (kIdChunk / 8) + lane];
                I.mb = mbase[c];
                const uint64_t* rec = starts + (uint64_t)c * kStartWords;
#pragma unroll
                for (int j = 0; j < 8; ++j) I.starts[j] = rec[j];
#pragma unroll
                for (int j = 0; j < 8; ++j) I.first[j] = reinterpret_cast<const uint32_t*>(rec + 8)[j];
            }
        };
        // Stage B's result, waiting for stage C.  There are two of these, used in turn: copying one into the other
        // at the end of a step would make the step wait for the messages it has just asked for.  For the same reason
        // the loop below is written out once per combination of buffers.
        struct Pending {
            uint4 raw;
            float val[8];
            uint32_t ok;             // per-id validity bits of a checked chunk
            bool fast;               // the chunk took the unchecked path (wavefront-uniform)
        };
        Pending X, Y;
        X.ok = 0; X.fast = false; Y.ok = 0; Y.fast = false;
        X.raw = make_uint4(0, 0, 0, 0); Y.raw = make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int j = 0; j < 8; ++j) { X.val[j] = 0.0f; Y.val[j] = 0.0f; }

        // ---- stage B on chunk c: lane l holds the ids at stream positions 64 j + l of the chunk, so for a fixed j
        // the wavefront covers 64 consecutive ids (row j).  The message of the id in lane l is the message of the
        // row's first id plus the messages begun at positions 1 .. l, which is what mbcnt counts in the row's word.
        auto stage_b = [&](Pending& S, const Ids& I, uint32_t c) {
            S.raw = I.raw;
            S.ok = 0;
            const uint32_t mb = I.mb;
            const uint64_t first = (uint64_t)c * kIdChunk;
            // mb >= 1: the chunk's first id then has a message at or before it
            S.fast = first >= e0 && first + kIdChunk <= e1 && mb >= 1 && (uint64_t)mb + kIdChunk <= A.M;
            if (S.fast) {
                // messages mb - 1 .. mb + 511, inside [0, M): one base address for the chunk, 32-bit offsets from it
                const char* near = reinterpret_cast<const char*>(A.msg) + ((uint64_t)mb << 2) - 4;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const uint32_t before = __builtin_amdgcn_mbcnt_hi((uint32_t)(I.starts[j] >> 32),
                                                                      __builtin_amdgcn_mbcnt_lo((uint32_t)I.starts[j], 0u));
                    S.val[j] = *reinterpret_cast<const float*>(near + ((before << 2) + I.first[j]));
                }
            } else {
                const uint32_t ebase = c * kIdChunk + lane;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const uint32_t mi = mb - 1u + (I.first[j] >> 2) +
                                        __builtin_amdgcn_mbcnt_hi((uint32_t)(I.starts[j] >> 32),
                                                                  __builtin_amdgcn_mbcnt_lo((uint32_t)I.starts[j], 0u));
                    const uint32_t e = ebase + 64 * j;
                    const bool ok = e >= e0 && e < e1 && id_of(I.raw, j) < kAccSlots * kIdScale && mi < A.M;   // (mi wraps if no message precedes)
                    S.ok |= (ok ? 1u : 0u) << j;
                    S.val[j] = A.msg[ok ? mi : 0u];
                }
            }
        };
        // ---- stage C: the chunk's ids add their messages; leaves S empty.  An id is the byte offset of its row's
        // accumulator divided by 8 / kIdScale, so any 16-bit value stays inside `acc` (the sink slot is its end).
        auto stage_c = [&](Pending& S) {
            if (S.fast) {
#pragma unroll
                for (int j = 0; j < 8; ++j) atomicAdd(acc_at(acc, id_of(S.raw, j) * (8 / kIdScale)), to_fixed(S.val[j]));
            } else if (S.ok) {
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if ((S.ok >> j) & 1u) atomicAdd(acc_at(acc, id_of(S.raw, j) * (8 / kIdScale)), to_fixed(S.val[j]));
            }
            S.fast = false; S.ok = 0;
        };
        // one step: B on chunk c out of buffer I into `fresh`, I asked for the chunk kRing steps on, C on `due`
        uint32_t c = c0 + wave_u;
        auto step = [&](Ids& I, Pending& fresh, Pending& due) -> bool {
            if (c > c1) return false;
            stage_b(fresh, I, c);
            load_ids(I, c + kRing * kGatherWaves);
            stage_c(due);
            c += kGatherWaves;
            return true;
        };
        Ids I0, I1;
        I0.raw = I1.raw = make_uint4(0, 0, 0, 0);
        I0.mb = I1.mb = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) { I0.starts[j] = I1.starts[j] = 0; I0.first[j] = I1.first[j] = 0; }
        load_ids(I0, c);
        load_ids(I1, c + kGatherWaves);
        while (step(I0, X, Y) && step(I1, Y, X)) {}
        stage_c(X);          // drain: at most one of the two still holds a chunk
        stage_c(Y);
    }
    __syncthreads();
    if constexpr (kDynamic)
        if (t + 1 == span.y && threadIdx.x == 0) asked = ask_if_time(A.sched, G);   // covered by the row pass below

    if (T.partial != kNoPartial) {
        // merged range: the sums go out as one row of partial sums; the next scatter sweep (or F) finishes the rows
        float* out = A.partials + (size_t)T.partial * kRowsPerPart;
        for (uint32_t i = threadIdx.x; i < kRowsPerPart; i += kGatherBlock) out[i] = (float)acc[i] * kFixInv;
        if (threadIdx.x == 0 && !final_pass) dnext[t] = 0.0f;
    } else {
    // direct range: fused vertex pass for its rows
    const int64_t v0 = (int64_t)q * kRowsPerPart;
    float dangling = 0.0f;
    constexpr int kRowsPerThread = (kRowsPerPart + kGatherBlock - 1) / kGatherBlock;
    if (final_pass) {
#pragma unroll
        for (int k = 0; k < kRowsPerThread; ++k) {
            const uint32_t i = threadIdx.x + kGatherBlock * k;
            if (i < nrows) A.ranks_out[A.perm[v0 + i]] = fmaf(A.damping, (float)acc[i] * kFixInv, base);
        }
    } else {
        float inv[kRowsPerThread];
#pragma unroll
        for (int k = 0; k < kRowsPerThread; ++k) {
            const uint32_t i = threadIdx.x + kGatherBlock * k;
            inv[k] = i < nrows ? A.inv_out[v0 + i] : 1.0f;
        }
#pragma unroll
        for (int k = 0; k < kRowsPerThread; ++k) {
            const uint32_t i = threadIdx.x + kGatherBlock * k;
            if (i >= nrows) continue;
            const float r = fmaf(A.damping, (float)acc[i] * kFixInv, base);
            A.contrib[v0 + i] = r * inv[k];
            dangling += (inv[k] == 0.0f ? r : 0.0f);
        }
        const float total = block_sum(dangling, red);
        if (threadIdx.x == 0) dnext[t] = total;
    }
    }
    __syncthreads();                                             // the piece is done with acc
    }       // pieces
    if constexpr (kDynamic) {
        if (threadIdx.x == 0) next_local = settle_next_tile(asked, A.sched, G, n_tiles);
        __syncthreads();
        local = next_local;
    }
    } while (kDynamic && local < n_tiles);       // tiles
    if constexpr (kDynamic)
        if (threadIdx.x == 0) leave_launch(A.sched);
    fr_gate_done(G.gate, G.slot);
}

// ---- F ----
// After the last iteration: r_K of kFinishRows rows of one merged range (partial sums of G_{K-1}) or of one empty
// range (the base value) goes to ranks_out.
constexpr uint32_t kFinishRows = 2048;
__global__ __launch_bounds__(kBlock) void k_finish(DevArgs A, GateArg G, uint32_t tile0, int parity)
{
    if (!fr_gate_admit(G.gate, G.slot, G.need_ticks)) return;
    const uint32_t t = tile0 + blockIdx.x;
    const float D = dangling_total(A.dpart + (size_t)parity * A.n_dpart, A.n_dpart);
    const float base = (1.0f - A.damping) / (float)A.V + A.damping * D / (float)A.V;
    const uint32_t per_range = A.rows_per_part / kFinishRows;
    if (t / per_range < A.n_finish) {
        const uint32_t q = A.finish_ranges[t / per_range];
        const RangeInfo info = A.range_info[q];
        const bool merged = (info.cls_tiles & 3u) == kRangeMerged;
        const int64_t v0 = (int64_t)q << A.rows_shift;
        for (uint32_t k = threadIdx.x; k < kFinishRows; k += kBlock) {
            const uint32_t i = (t % per_range) * kFinishRows + k;
            const int64_t v = v0 + i;
            if (v >= A.V) break;
            A.ranks_out[A.perm[v]] = merged ? fmaf(A.damping, merged_sum<1>(A, info, i, 0), base) : base;
        }
    }
    fr_gate_done(G.gate, G.slot);
}

uint32_t ceil_div_u64(uint64_t a, uint64_t b) { return (uint32_t)((a + b - 1) / b); }

uint64_t ceil_fs_to_ns(unsigned __int128 fs)
{
    const uint64_t ns = (uint64_t)((fs + 999999) / 1000000);
    return ns ? ns : 1;
}

struct PrTask {
    fr_pagerank_desc d{};
    PrLayout L;
    std::vector<uint64_t> prefix[4];      // cumulative modelled tile costs per segment kind (after init)
    uint64_t footprint_after = 0, footprint_peak = 0;
    float *msg = nullptr, *contrib = nullptr, *dpart = nullptr, *partials = nullptr;
    uint32_t* sched = nullptr;
    uint32_t n_dpart = 0;
    DevArgs args{};
    bool inited = false;
    bool registered = false;
    fr_alloc own;                         // used by the standalone run only
    int hip_error = 0;
    uint32_t run = 0, seg = 0, tile = 0;  // cursor

    // V0, then S_k G_k for k < K, then F (no S, G, F at all when K = 0)
    uint32_t n_segments() const { return d.iterations == 0 ? 1u : 2u + 2u * (uint32_t)d.iterations; }
    int kind_of(uint32_t g) const
    {
        if (g == 0) return FR_PR_SEG_VERTEX;
        if (g + 1 == n_segments()) return FR_PR_SEG_FINISH;
        return ((g - 1) & 1u) ? FR_PR_SEG_GATHER : FR_PR_SEG_SCATTER;
    }
    uint32_t tiles_of(int kind) const
    {
        switch (kind) {
        case FR_PR_SEG_VERTEX: return L.Q;
        case FR_PR_SEG_SCATTER: return L.n_scatter;
        case FR_PR_SEG_GATHER: return L.n_gather;
        default: return std::max<uint32_t>(1, L.n_finish * (L.rows_per_part / kFinishRows));
        }
    }
    uint64_t rows_of_q(uint32_t q) const
    {
        return std::min<uint64_t>(L.rows_per_part, (uint64_t)L.V - (uint64_t)q * L.rows_per_part);
    }
};

void build_cost_tables(PrTask* p)
{
    const PrLayout& L = p->L;
    const uint64_t pe = p->d.fs_per_edge, pm = p->d.fs_per_message, pv = p->d.fs_per_vertex;
    auto& v = p->prefix[FR_PR_SEG_VERTEX];
    v.assign(L.Q + 1, 0);
    for (uint32_t q = 0; q < L.Q; ++q) v[q + 1] = v[q] + ceil_fs_to_ns((unsigned __int128)p->rows_of_q(q) * pv);
    auto& s = p->prefix[FR_PR_SEG_SCATTER];
    s.assign(L.n_scatter + 1, 0);
    for (uint32_t i = 0; i < L.n_scatter; ++i) {
        s[i + 1] = s[i] + ceil_fs_to_ns((unsigned __int128)(L.st_msgs[i] + L.st_rows[i]) * pm);   // a value read costs about a message
    }
    auto& g = p->prefix[FR_PR_SEG_GATHER];
    const uint32_t ng = p->tiles_of(FR_PR_SEG_GATHER);
    g.assign(ng + 1, 0);
    for (uint32_t t = 0; t < ng; ++t) {
        g[t + 1] = g[t] + ceil_fs_to_ns((unsigned __int128)L.gt_weight[t] * pe / 2);
    }
    auto& h = p->prefix[FR_PR_SEG_FINISH];
    const uint32_t nf = p->tiles_of(FR_PR_SEG_FINISH);
    h.assign(nf + 1, 0);
    for (uint32_t t = 0; t < nf; ++t) h[t + 1] = h[t] + std::max<uint64_t>(1, p->d.finish_tile_ns);
}

// `with`: the kernel arguments to use instead of the task's own (the run that works in the static scratch array).
int pr_launch(PrTask* p, uint32_t g, uint32_t tile0, uint32_t tile1, hipStream_t stream, GateArg G = GateArg{nullptr, 0, 0, 0},
              const DevArgs* with = nullptr)
{
    const DevArgs& args = with ? *with : p->args;
    const int kind = p->kind_of(g);
    if (tile1 <= tile0 || tile1 > p->tiles_of(kind)) return FR_ERR_ARG;
    const uint32_t n = tile1 - tile0;
    const uint32_t K = (uint32_t)p->d.iterations;
    if (kind == FR_PR_SEG_VERTEX) {
        hipLaunchKernelGGL(k_vertex0, dim3(n), dim3(kBlock), 0, stream, args, G, tile0, K == 0 ? 1 : 0);
    } else if (kind == FR_PR_SEG_FINISH) {
        // after G_{K-1}: the dangling partials of r_{K-1} sit in set (K-1) & 1
        hipLaunchKernelGGL(k_finish, dim3(n), dim3(kBlock), 0, stream, args, G, tile0, (int)((K - 1) & 1u));
    } else {
        const uint32_t k = (g - 1) / 2;
        if (kind == FR_PR_SEG_SCATTER) {    // S_k finishes rows of r_k with D_{k-1}: set (k-1) & 1
            const int parity = (int)((k + 1) & 1u), first = k == 0 ? 1 : 0;
            const uint32_t grid = std::min(n, p->L.scatter_slots);
            const bool packed = p->L.scatter_packed, dynamic = n > grid;
            auto go = [&](auto kernel) { hipLaunchKernelGGL(kernel, dim3(grid), dim3(kScatterBlock), 0, stream, args, G, tile0, n, parity, first); };
            if (p->L.src_per_part == kSrcLarge) {
                if (packed) { if (dynamic) go(k_scatter<kSrcLarge, true, true>); else go(k_scatter<kSrcLarge, true, false>); }
                else { if (dynamic) go(k_scatter<kSrcLarge, false, true>); else go(k_scatter<kSrcLarge, false, false>); }
            } else {
                if (packed) { if (dynamic) go(k_scatter<kSrcSmall, true, true>); else go(k_scatter<kSrcSmall, true, false>); }
                else { if (dynamic) go(k_scatter<kSrcSmall, false, true>); else go(k_scatter<kSrcSmall, false, false>); }
            }
        } else {
            const int parity = (int)(k & 1u), final_pass = (k + 1 == K) ? 1 : 0;
            const uint32_t grid = std::min(n, p->L.gather_slots);
            const bool dynamic = n > grid;
            auto go = [&](auto kernel) {
                hipLaunchKernelGGL(kernel, dim3(grid), dim3(kGatherBlock), 0, stream, args, G, tile0, n, parity, final_pass, args.starts, args.mbase);
            };
            if (p->L.rows_per_part == kRowsLarge) { if (dynamic) go(k_gather<kRowsLarge, true>); else go(k_gather<kRowsLarge, false>); }
            else { if (dynamic) go(k_gather<kRowsSmall, true>); else go(k_gather<kRowsSmall, false>); }
        }
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { p->hip_error = (int)e; return FR_ERR_HIP; }
    return FR_OK;
}

template <typename T>
bool take(fr_alloc* a, T** out, uint64_t count)
{
    *out = static_cast<T*>(fr_alloc_device(a, (size_t)(count ? count : 1) * sizeof(T)));
    return *out != nullptr;
}

// Compute units the stream may use (its CU mask, if it has one): the sweeps are cut into that many tiles.
uint32_t stream_cus(hipStream_t stream)
{
    int device = 0, cus = 0;
    if (hipGetDevice(&device) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || cus <= 0)
        cus = (int)kDefaultCus;
    uint32_t mask[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (hipExtStreamGetCUMask(stream, 8, mask) == hipSuccess) {
        int masked = 0;
        for (uint32_t w : mask) masked += __builtin_popcount(w);
        if (masked > 0 && masked < cus) cus = masked;
    } else {
        (void)hipGetLastError();          // a stream without a mask of its own
    }
    return (uint32_t)cus;
}

int pr_init(void* user, fr_alloc* a, void* stream_v)
{
    PrTask* p = static_cast<PrTask*>(user);
    hipStream_t stream = (hipStream_t)stream_v;
    if (a->host_only) return FR_ERR_ARG;      // this task needs a GPU
    const int64_t V = p->d.n_vertices, E = p->d.n_edges;
    // caller-provided buffers count against the task's limit: row_ptr, col, out_degree, ranks_out
    const uint64_t caller = 4ull * (uint64_t)(V + 1) + 4ull * (uint64_t)E + 4ull * (uint64_t)V + 4ull * (uint64_t)V;
    if (fr_alloc_charge(a, caller) != FR_OK) return FR_ERR_OOM;
    int rc = pr_build_layout(&p->L, V, E, p->d.row_ptr, p->d.col, p->d.out_degree, p->d.rows_per_partition,
                             p->d.sources_per_partition, stream_cus(stream), a, stream, &p->hip_error);
    if (rc != FR_OK) return rc;
    PrLayout& L = p->L;
    // dangling partials: one slot per range (V0), or one per gather piece followed by one per scatter piece
    p->n_dpart = std::max(L.Q, L.n_pieces + L.n_spieces);
    if (!take(a, &p->msg, L.M) || !take(a, &p->contrib, (uint64_t)V) || !take(a, &p->dpart, 2ull * p->n_dpart) ||
        !take(a, &p->partials, (uint64_t)L.n_partials * L.rows_per_part) || !take(a, &p->sched, 2))
        return a->hip_error ? FR_ERR_HIP : FR_ERR_OOM;
    hipLaunchKernelGGL(k_clear_sched, dim3(1), dim3(64), 0, stream, p->sched);
    if (hipStreamSynchronize(stream) != hipSuccess) return FR_ERR_HIP;
    DevArgs& A = p->args;
    A.V = V; A.E = E; A.M = (uint32_t)L.M; A.Q = L.Q; A.Qe = L.Qe;
    A.n_gather = L.n_gather; A.n_pieces = L.n_pieces; A.n_scatter = L.n_scatter; A.n_spieces = L.n_spieces;
    A.n_finish = L.n_finish;
    A.n_dpart = p->n_dpart; A.damping = p->d.damping;
    A.rows_per_part = L.rows_per_part;
    A.rows_shift = L.rows_per_part == kRowsLarge ? 14 : 13;
    A.void_slot = L.void_slot; A.n_void_dangling = (float)L.n_void_dangling;
    A.ids16 = L.ids16; A.src16 = L.src16; A.mbase = L.mbase; A.starts = L.starts; A.bins = L.bins;
    A.inv_out = L.inv_out; A.perm = L.perm; A.range_info = L.range_info;
    A.gather_pieces = L.gather_pieces; A.gather_tiles = L.gather_tiles;
    A.scatter_pieces = L.scatter_pieces; A.scatter_tiles = L.scatter_tiles; A.finish_ranges = L.finish_ranges;
    A.msg = p->msg; A.contrib = p->contrib; A.dpart = p->dpart; A.partials = p->partials; A.ranks_out = p->d.ranks_out;
    A.sched = p->sched;
    build_cost_tables(p);
    p->footprint_after = fr_alloc_used(a);
    p->footprint_peak = fr_alloc_peak(a);
    p->run = 0; p->seg = 0; p->tile = 0;
    p->inited = true;
    return FR_OK;
}

int pr_create(void* user)
{
    static_cast<PrTask*>(user)->registered = true;
    return FR_OK;
}

int pr_plan(void* user, uint64_t budget_ns, uint64_t launch_cost_ns, fr_step* out)
{
    PrTask* p = static_cast<PrTask*>(user);
    std::memset(out, 0, sizeof(*out));
    out->run = p->run; out->segment = p->seg; out->tile0 = p->tile; out->tile1 = p->tile;
    if (!p->inited) return FR_ERR_STATE;
    out->cost_class = (uint32_t)p->kind_of(p->seg);
    if (p->d.max_runs > 0 && p->run >= (uint32_t)p->d.max_runs) { out->finished = 1; return FR_OK; }
    const int kind = p->kind_of(p->seg);
    const std::vector<uint64_t>& pre = p->prefix[kind];
    const uint64_t floor_ns = p->d.min_step_ns[kind];
    if (floor_ns > budget_ns || launch_cost_ns > budget_ns - floor_ns) return FR_OK;     // even the shortest step is too long
    uint32_t n = 0;
    int rc = fr_chunk_fit(pre.data(), p->tiles_of(kind), p->tile, budget_ns, launch_cost_ns, &n);
    if (rc != FR_OK) return rc;
    if (n == 0) return FR_OK;
    // A launch of more tiles than workgroups runs in rounds, each workgroup taking a next tile when it is done with
    // one; the summed tile costs are what whole rounds take.  A step that does not reach the segment's end is
    // therefore cut to whole rounds (the tiles are in order of falling weight, so the light ones that close the
    // segment's last round smoothly are at its end): a round and a few tiles would take two rounds' time.
    const uint32_t slots = kind == FR_PR_SEG_SCATTER ? p->L.scatter_slots : kind == FR_PR_SEG_GATHER ? p->L.gather_slots : 0;
    if (slots && n > slots && p->tile + n < p->tiles_of(kind)) n = n / slots * slots;
    uint64_t cost = std::max(pre[p->tile + n] - pre[p->tile], floor_ns);
    if (slots && n <= slots) {
        // A step of up to a round: its tiles run side by side on part of the slots.  One tile alone takes the floor,
        // a full round the sum of its tiles' costs (each a share of a round), and in between the time was measured
        // to grow linearly with the number of tiles: the sum plus the floor's share of the slots left empty.
        // (a sweep of fewer tiles than slots is full with all of them)
        const uint32_t full = std::min(slots, p->tiles_of(kind));
        auto part = [&](uint32_t k) {
            return std::max(floor_ns, pre[p->tile + k] - pre[p->tile] + floor_ns * (full - k) / full);
        };
        const uint64_t room = budget_ns - launch_cost_ns;            // (launch_cost_ns <= budget_ns - floor_ns, above)
        while (n > 0 && part(n) > room) --n;
        if (n == 0) return FR_OK;
        cost = part(n);
    }
    out->tile1 = p->tile + n;
    out->modelled_ns = cost;
    if (slots && n > slots) {
        // the step's kernel hands its tiles out and can stop between them: what its heaviest tile - the first, they
        // are in order of falling weight - takes a workgroup, i.e. the slot's whole time for it (a tile's cost is its
        // share of a round of `slots` tiles side by side) and a quarter more.  (Not the floor of the segment, which is
        // the heaviest tile of the whole sweep run alone: the steps near a bubble's end are made of the light tiles.)
        const uint64_t heaviest = std::max<uint64_t>(10000, (pre[p->tile + 1] - pre[p->tile]) * slots * 5 / 4);
        out->gate_tile = (uint32_t)std::min<uint64_t>(heaviest, 4000000000ull);
    }
    if (kind == FR_PR_SEG_GATHER) {
        uint64_t edges = 0;
        for (uint32_t t = p->tile; t < p->tile + n && t < p->L.n_gather; ++t) edges += p->L.gt_edges[t];
        out->work_units = edges;
    }
    out->completes_run = (p->seg + 1 == p->n_segments() && out->tile1 == p->tiles_of(kind)) ? 1 : 0;
    return FR_OK;
}

int pr_run(void* user, void* stream, const fr_step* st)
{
    PrTask* p = static_cast<PrTask*>(user);
    if (!p->inited || st->run != p->run || st->segment != p->seg || st->tile0 != p->tile) return FR_ERR_STATE;
    int rc = pr_launch(p, p->seg, st->tile0, st->tile1, (hipStream_t)stream,
                       GateArg{static_cast<fr_gate*>(st->gate), st->gate_slot, st->gate_need_ticks, st->gate_tile});
    if (rc != FR_OK) return rc;
    p->tile = st->tile1;
    if (p->tile == p->tiles_of(p->kind_of(p->seg))) {
        p->tile = 0;
        if (++p->seg == p->n_segments()) { p->seg = 0; p->run++; }
    }
    return FR_OK;
}

// The device gate cut `first` off after `tiles_done` of its tiles, and every step after it did nothing: the cursor goes
// back to the first tile not done.  (A tile done twice computes the same values again: tiles only read what earlier
// segments wrote.)
int pr_rewind(void* user, const fr_step* first, uint32_t tiles_done, uint64_t* work_done)
{
    PrTask* p = static_cast<PrTask*>(user);
    if (!p->inited || !first || !work_done || first->segment >= p->n_segments()) return FR_ERR_ARG;
    const int kind = p->kind_of(first->segment);
    if (first->tile0 >= p->tiles_of(kind) || first->tile1 > p->tiles_of(kind) || tiles_done > first->tile1 - first->tile0) return FR_ERR_ARG;
    p->run = first->run; p->seg = first->segment; p->tile = first->tile0 + tiles_done;
    uint64_t edges = 0;
    if (kind == FR_PR_SEG_GATHER)
        for (uint32_t t = first->tile0; t < first->tile0 + tiles_done && t < p->L.n_gather; ++t) edges += p->L.gt_edges[t];
    *work_done = edges;
    if (p->tile == p->tiles_of(kind)) {            // (a step is only cut off before its last tile; kept for safety)
        p->tile = 0;
        if (++p->seg == p->n_segments()) { p->seg = 0; p->run++; }
    }
    return FR_OK;
}

int pr_stop(void* user)
{
    PrTask* p = static_cast<PrTask*>(user);
    p->inited = false;        // the runtime's allocator frees the device blocks
    p->registered = false;
    return FR_OK;
}

// ---- working memory of fr_pagerank_run_standalone_noalloc: messages, contributions, dangling partials and partial
// sums of one run live in this array instead of in memory taken from an allocator.  Every GPU the library is loaded
// on holds its own copy at its own address; host code never uses the array's name as an address, only the pointer
// hipGetSymbolAddress gave for the device at hand.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
unsigned char* g_scratch_ptr[kMaxDevices] = {};

size_t round256(size_t n) { return (n + 255) / 256 * 256; }

}  // namespace

extern "C" {

int fr_pagerank_make(const fr_pagerank_desc* d, fr_task_ops* ops_out, void** user_out, fr_task_profile* prof_out)
{
    if (!d || !ops_out || !user_out || !prof_out) return FR_ERR_ARG;
    if (d->n_vertices < 1 || d->n_vertices > 0x7fffffffLL || d->n_edges < 0 || d->n_edges > 0x7fffffffLL) return FR_ERR_ARG;
    if (!d->row_ptr || !d->out_degree || !d->ranks_out || (d->n_edges > 0 && !d->col)) return FR_ERR_ARG;
    if (d->iterations < 0 || d->iterations > 100000 || d->max_runs < 0) return FR_ERR_ARG;
    if (!(d->damping >= 0.0f && d->damping <= 1.0f)) return FR_ERR_ARG;
    PrTask* p = new (std::nothrow) PrTask();
    if (!p) return FR_ERR_ARG;
    p->d = *d;
    if (!p->d.fs_per_edge) p->d.fs_per_edge = 2000;
    if (!p->d.fs_per_message) p->d.fs_per_message = 2000;
    if (!p->d.fs_per_vertex) p->d.fs_per_vertex = 4000;
    if (!p->d.finish_tile_ns) p->d.finish_tile_ns = 2000;
    ops_out->create = pr_create;
    ops_out->init = pr_init;
    ops_out->plan_step = pr_plan;
    ops_out->run_step = pr_run;
    ops_out->stop = pr_stop;
    ops_out->rewind = pr_rewind;
    prof_out->mem_limit_bytes = d->mem_limit_bytes;
    prof_out->min_step_ns = 1;
    *user_out = p;
    return FR_OK;
}

int fr_pagerank_destroy(void* user)
{
    PrTask* p = static_cast<PrTask*>(user);
    if (!p) return FR_ERR_ARG;
    if (p->registered) return FR_ERR_STATE;
    if (p->inited) {
        (void)hipDeviceSynchronize();
        fr_alloc_release(&p->own);
    }
    delete p;
    return FR_OK;
}

int fr_pagerank_info(void* user, fr_pagerank_info_t* out)
{
    PrTask* p = static_cast<PrTask*>(user);
    if (!p || !out) return FR_ERR_ARG;
    if (p->prefix[0].empty()) return FR_ERR_STATE;       // known once InitSideTask has run
    std::memset(out, 0, sizeof(*out));
    out->messages = p->L.M;
    out->ranges = p->L.Q;
    out->nonempty_ranges = p->L.Qe;
    out->merged_ranges = p->L.n_merged;
    out->partial_rows = p->L.n_partials;
    out->gather_tiles = p->L.n_gather;
    out->scatter_tiles = p->L.n_scatter;
    out->rows_per_partition = p->L.rows_per_part;
    out->sources_per_partition = p->L.src_per_part;
    out->bytes_resident = p->footprint_after;
    out->bytes_peak = p->footprint_peak;
    out->scatter_slots = p->L.scatter_slots;
    out->gather_slots = p->L.gather_slots;
    return FR_OK;
}

int fr_pagerank_tiles(void* user, int32_t seg_kind, uint32_t* n_out)
{
    PrTask* p = static_cast<PrTask*>(user);
    if (!p || !n_out || seg_kind < 0 || seg_kind > 3) return FR_ERR_ARG;
    if (p->prefix[0].empty()) return FR_ERR_STATE;
    *n_out = p->tiles_of(seg_kind);
    return FR_OK;
}

int fr_pagerank_tile_costs(void* user, int32_t seg_kind, uint32_t* costs, size_t cap, size_t* n_out)
{
    PrTask* p = static_cast<PrTask*>(user);
    if (!p || !n_out || seg_kind < 0 || seg_kind > 3 || (!costs && cap)) return FR_ERR_ARG;
    if (p->prefix[0].empty()) return FR_ERR_STATE;
    const std::vector<uint64_t>& pre = p->prefix[seg_kind];
    const size_t n = pre.size() - 1;
    for (size_t t = 0; t < std::min(n, cap); ++t) costs[t] = (uint32_t)std::min<uint64_t>(pre[t + 1] - pre[t], 0xffffffffu);
    *n_out = n;
    return FR_OK;
}

int fr_pagerank_tile_work(void* user, int32_t seg_kind, uint64_t* work, size_t cap, size_t* n_out)
{
    PrTask* p = static_cast<PrTask*>(user);
    if (!p || !n_out || seg_kind < 0 || seg_kind > 3 || (!work && cap)) return FR_ERR_ARG;
    if (p->prefix[0].empty()) return FR_ERR_STATE;
    const size_t n = p->tiles_of(seg_kind);
    for (size_t t = 0; t < std::min(n, cap); ++t) {
        if (seg_kind == FR_PR_SEG_GATHER) work[t] = t < p->L.n_gather ? p->L.gt_edges[t] : 0;
        else if (seg_kind == FR_PR_SEG_SCATTER) work[t] = p->L.st_msgs[t];
        else if (seg_kind == FR_PR_SEG_VERTEX) work[t] = p->rows_of_q((uint32_t)t);
        else work[t] = 0;
    }
    *n_out = n;
    return FR_OK;
}

int fr_pagerank_tile_weights(void* user, int32_t seg_kind, uint64_t* weights, size_t cap, size_t* n_out)
{
    PrTask* p = static_cast<PrTask*>(user);
    if (!p || !n_out || seg_kind < 0 || seg_kind > 3 || (!weights && cap)) return FR_ERR_ARG;
    if (p->prefix[0].empty()) return FR_ERR_STATE;
    const size_t n = p->tiles_of(seg_kind);
    for (size_t t = 0; t < std::min(n, cap); ++t) {
        if (seg_kind == FR_PR_SEG_GATHER) weights[t] = p->L.gt_weight[t];
        else if (seg_kind == FR_PR_SEG_SCATTER) weights[t] = p->L.st_rows[t];
        else if (seg_kind == FR_PR_SEG_VERTEX) weights[t] = p->rows_of_q((uint32_t)t);
        else weights[t] = 0;
    }
    *n_out = n;
    return FR_OK;
}

int fr_pagerank_run_standalone(void* user, int32_t device_id, void* stream_v, uint32_t max_tiles, uint64_t* phase_ns)
{
    PrTask* p = static_cast<PrTask*>(user);
    if (!p || device_id < 0) return FR_ERR_ARG;
    if (p->registered) return FR_ERR_STATE;
    hipStream_t stream = (hipStream_t)stream_v;
    FR_HIP_TRY(hipSetDevice(device_id), p->hip_error);
    if (!p->inited) {
        fr_alloc_reset(&p->own, p->d.mem_limit_bytes, false, device_id);
        int rc = pr_init(p, &p->own, stream_v);
        if (rc != FR_OK) {
            const bool oom = p->own.oom;
            fr_alloc_release(&p->own);
            p->inited = false;
            return oom ? FR_ERR_OOM : rc;
        }
    }
    hipEvent_t ev[2] = {nullptr, nullptr};
    float ms_sum[4] = {0.f, 0.f, 0.f, 0.f};
    if (phase_ns) {
        FR_HIP_TRY(hipEventCreate(&ev[0]), p->hip_error);
        FR_HIP_TRY(hipEventCreate(&ev[1]), p->hip_error);
    }
    int rc = FR_OK;
    for (uint32_t g = 0; g < p->n_segments() && rc == FR_OK; ++g) {
        const int kind = p->kind_of(g);
        const uint32_t nt = p->tiles_of(kind);
        const uint32_t step = max_tiles ? max_tiles : nt;
        if (phase_ns) (void)hipEventRecord(ev[0], stream);
        for (uint32_t t0 = 0; t0 < nt && rc == FR_OK; t0 += step) rc = pr_launch(p, g, t0, std::min(nt, t0 + step), stream);
        if (phase_ns) {
            (void)hipEventRecord(ev[1], stream);
            (void)hipEventSynchronize(ev[1]);
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, ev[0], ev[1]) == hipSuccess) ms_sum[kind] += ms;
        }
    }
    hipError_t e = hipStreamSynchronize(stream);
    if (phase_ns) {
        for (int k = 0; k < 4; ++k) phase_ns[k] = (uint64_t)((double)ms_sum[k] * 1.0e6 + 0.5);
        (void)hipEventDestroy(ev[0]);
        (void)hipEventDestroy(ev[1]);
    }
    if (rc != FR_OK) return rc;
    if (e != hipSuccess) { p->hip_error = (int)e; return FR_ERR_HIP; }
    return FR_OK;
}

int fr_pagerank_run_standalone_noalloc(void* user, int32_t device_id, void* stream_v, uint32_t max_tiles)
{
    PrTask* p = static_cast<PrTask*>(user);
    if (!p || device_id < 0 || device_id >= kMaxDevices) return FR_ERR_ARG;
    if (p->registered || !p->inited) return FR_ERR_STATE;        // the layout must exist already: nothing is built here
    hipStream_t stream = (hipStream_t)stream_v;
    FR_HIP_TRY(hipSetDevice(device_id), p->hip_error);
    unsigned char* base = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mu);
        if (!g_scratch_ptr[device_id]) {
            void* sym = nullptr;
            FR_HIP_TRY(hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)), p->hip_error);
            g_scratch_ptr[device_id] = static_cast<unsigned char*>(sym);
        }
        base = g_scratch_ptr[device_id];
    }
    const PrLayout& L = p->L;
    const size_t b_msg = round256((size_t)std::max<uint64_t>(L.M, 1) * 4), b_contrib = round256((size_t)L.V * 4),
                 b_dpart = round256((size_t)2 * p->n_dpart * 4),
                 b_partials = round256((size_t)std::max<uint64_t>((uint64_t)L.n_partials * L.rows_per_part, 1) * 4);
    constexpr size_t b_sched = 256;
    if (b_msg + b_contrib + b_dpart + b_partials + b_sched > kStaticScratchBytes) return FR_ERR_ARG;   // too large for the array
    DevArgs A = p->args;
    A.msg = reinterpret_cast<float*>(base);
    A.contrib = reinterpret_cast<float*>(base + b_msg);
    A.dpart = reinterpret_cast<float*>(base + b_msg + b_contrib);
    A.partials = reinterpret_cast<float*>(base + b_msg + b_contrib + b_dpart);
    A.sched = reinterpret_cast<uint32_t*>(base + b_msg + b_contrib + b_dpart + b_partials);
    hipLaunchKernelGGL(k_clear_sched, dim3(1), dim3(64), 0, stream, A.sched);     // the hand-out words must start at zero
    int rc = FR_OK;
    for (uint32_t g = 0; g < p->n_segments() && rc == FR_OK; ++g) {
        const uint32_t nt = p->tiles_of(p->kind_of(g));
        const uint32_t step = max_tiles ? max_tiles : nt;
        for (uint32_t t0 = 0; t0 < nt && rc == FR_OK; t0 += step)
            rc = pr_launch(p, g, t0, std::min(nt, t0 + step), stream, GateArg{nullptr, 0, 0, 0}, &A);
    }
    hipError_t e = hipStreamSynchronize(stream);
    if (rc != FR_OK) return rc;
    if (e != hipSuccess) { p->hip_error = (int)e; return FR_ERR_HIP; }
    return FR_OK;
}

}  // extern "C"
