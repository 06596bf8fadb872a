// The PageRank side task: pull-based power iteration, fp32 ranks, for gfx950.
//
// The paper's graph-analytics side task (Section 6.1.4) with one iteration = one pass over the graph
// (Section 6.2), written as a step-wise task for the iterative interface (Section 4.2): work is cut into tiles
// that are fixed at init, a step is a run of consecutive tiles of one segment, and every tile computes the same
// bits whichever launch carries it, so pausing and resuming at any tile boundary cannot change the result.
//
// The pull pass runs on the partition-centric layout of pr_layout.h.  One run = segments
//     V0, S_0 G_0, S_1 G_1, ..., S_{K-1} G_{K-1}, H
//   V0   vertex pass (tile = destination partition): r_0 = 1/V, contrib_0 = r_0 / outdeg, dangling partials
//   S_k  scatter     (tile = source partition): contrib_k slice in LDS -> one message per (partition, source);
//                    for k > 0 the hubs that live in the slice are finished first (their virtual rows, summed by
//                    G_{k-1}, are added up and run through the vertex-pass arithmetic)
//   G_k  gather      (tile = destination partition): id stream + messages -> 64-bit fixed-point sums in LDS;
//                    then, fused, the next vertex pass for the partition's rows:
//                    r_{k+1} = base_k + d * sum, contrib_{k+1} = r_{k+1} / outdeg, dangling partials
//                    (sums of hubs' virtual rows are only stored)
//   H    hub finish  (tile = 16 hubs): after the last iteration, the hubs' r_K
// base_k = (1 - d)/V + d * D_k / V, D_k = fixed-order sum of the dangling partials of r_k.
// In the last iteration G writes r_K to ranks_out instead of contrib; H does the same for the hubs.
// No floating-point atomics anywhere: float sums have a fixed order, the LDS atomics add integers.

#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>

#include "freeride_device.h"
#include "pr_layout.h"

namespace {

#ifndef FR_GATHER_BLOCK
#define FR_GATHER_BLOCK 1024
#endif
#ifndef FR_SCATTER_BLOCK
#define FR_SCATTER_BLOCK 1024
#endif
constexpr int kBlock = 512;                     // threads per workgroup of the first vertex pass
constexpr int kGatherBlock = FR_GATHER_BLOCK;   // threads per workgroup of the gather sweep
constexpr int kGatherWaves = kGatherBlock / 64;
constexpr int kScatterBlock = FR_SCATTER_BLOCK; // threads per workgroup of the scatter sweep
constexpr int kScatterWaves = kScatterBlock / 64;
// row sums are kept as 64-bit fixed point with scale 2^62: contrib sums are <= 1, so they fit
constexpr float kFixInv = 1.0f / 4611686018427387904.0f;

// ---- fixed-order reductions ----
__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, 64);
    return x;
}

// Sum of a per-thread value over the workgroup, same association for a given blockDim.  All threads call.
__device__ __forceinline__ float block_sum(float x, float* lds /* >= 8 floats */)
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

// D = sum of dpart[0 .. n), in two halves so that the loads can be issued long before the sum is needed:
// dangling_partial (threads 0..255 each add up a strided share) and dangling_finish (fixed tree over those 256
// partial sums).  Every kernel that uses the pair gets the same bits whatever its workgroup size (>= 256).
__device__ __forceinline__ float dangling_partial(const float* __restrict__ dpart, uint32_t n)
{
    float s = 0.0f;
    if (threadIdx.x < 256) {
        uint32_t i = threadIdx.x;
        for (; i + 768 < n; i += 1024) {
            const float a = dpart[i], b = dpart[i + 256], c = dpart[i + 512], d = dpart[i + 768];
            s += a; s += b; s += c; s += d;
        }
        for (; i < n; i += 256) s += dpart[i];
    }
    return s;
}

// All threads call; all get the result.
__device__ __forceinline__ float dangling_finish(float s, float* lds /* >= 8 floats */)
{
    s = wave_sum(s);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    __syncthreads();
    if (lane == 0 && w < 4) lds[w] = s;
    __syncthreads();
    return (lds[0] + lds[1]) + (lds[2] + lds[3]);
}

__device__ __forceinline__ bool is_hub_tag(float tag) { return (__float_as_uint(tag) >> 31) != 0; }
__device__ __forceinline__ float inv_of_tag(float tag) { return __uint_as_float(__float_as_uint(tag) & 0x7fffffffu); }

enum : uint32_t { kShape_64x8 = 0, kShape_64x4, kShape_32x4, kShape_32x2 };

struct DevArgs {
    int64_t V, E;
    uint32_t M, Q, P, n_hubs, n_vrows, n_dpart;
    uint32_t scatter_shape;       // lanes per bin x messages per lane in the scatter sweep (kShape_*)
    uint32_t rows_per_part, src_per_part;
    float damping;
    const uint16_t* ids16;
    const uint16_t* src16;
    const uint32_t* eoff;
    const uint32_t* mbase;
    const uint2* bins;
    const int32_t* hub_row;
    const uint32_t* hub_vbase;
    const uint32_t* hub_of_p;
    const float* inv_tag;
    float* msg;
    float* contrib;
    float* dpart;                 // [2][n_dpart]
    unsigned long long* vacc;     // [n_vrows]
    float* ranks_out;
};

// What a step's kernels need to ask the device gate (Section 4.5's check, made by the GPU when the kernel starts).
struct GateArg {
    fr_gate* gate;                // NULL: no gate
    uint32_t slot, need_ticks;
};

// ---- V0 ----
__global__ __launch_bounds__(kBlock) void k_vertex0(DevArgs A, GateArg G, uint32_t tile0, int final_pass)
{
    __shared__ float red[8];
    if (!fr_gate_admit(G.gate, G.slot, G.need_ticks)) return;
    const uint32_t q = tile0 + blockIdx.x;
    const int64_t v0 = (int64_t)q * A.rows_per_part;
    const float r0 = 1.0f / (float)A.V;
    float dangling = 0.0f;
    for (uint32_t i = threadIdx.x; i < A.rows_per_part; i += kBlock) {
        const int64_t v = v0 + i;
        if (v >= A.V) break;
        if (final_pass) A.ranks_out[v] = r0;
        else {
            const float inv = inv_of_tag(A.inv_tag[v]);
            A.contrib[v] = r0 * inv;
            dangling += (inv == 0.0f ? r0 : 0.0f);
        }
    }
    if (!final_pass) {
        const float total = block_sum(dangling, red);
        if (threadIdx.x == 0) A.dpart[q] = total;
        if (q == 0)
            for (uint32_t i = A.Q + threadIdx.x; i < A.n_dpart; i += kBlock) A.dpart[i] = 0.0f;   // hub slots
    }
    fr_gate_done(G.gate);
}

// Workgroups are handed to the 8 XCDs round-robin (workgroup b runs on XCD b % 8), and every XCD has an L2 of its
// own.  This map gives XCD x the x-th contiguous eighth of a launch's n tiles, in order, so that tiles which touch
// neighbouring memory at about the same time do so through the same L2.  It is a bijection on [0, n) for any n.
__device__ __forceinline__ uint32_t xcd_contiguous(uint32_t b, uint32_t n)
{
    constexpr uint32_t kXcds = 8;
    const uint32_t x = b % kXcds, i = b / kXcds;
    const uint32_t rem = n % kXcds;
    return x * (n / kXcds) + (x < rem ? x : rem) + i;
}

// ---- S_k ----
// One workgroup per source partition: its slice of contrib sits in LDS, and for every destination partition q
// the messages of bin (p, q) are written in order.  Bin descriptors are staged in LDS a batch at a time; each
// wavefront works on two bins at once, eight messages per lane per step, so that sixteen independent loads are
// in flight before the first one is needed.
constexpr uint32_t kDescBatch = 1024;

// The messages of `nb` bins (ranges [x, y) of message numbers, staged in LDS) are produced from the slice.
// L lanes share a bin and move up to T messages each per step, for 16 / T bins at a time: a wavefront keeps
// sixteen loads per lane in flight over (16 / T) * (64 / L) bins.  Short bins (large graphs) want small L * T,
// so that lanes and issue slots are not spent on messages that are not there; long bins want L = 64, T = 8.
// The values written do not depend on L and T.
template <uint32_t L, uint32_t T>
__device__ __forceinline__ void scatter_bins(const uint16_t* __restrict__ src16, float* __restrict__ msg, const uint2* desc,
                                             uint32_t nb, const float* slice, uint32_t n)
{
    constexpr uint32_t H = 16 / T, kGroups = 64 / L;
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t grp = lane / L, sub = lane % L;
    for (uint32_t i = H * kGroups * wave; i < nb; i += H * kGroups * kScatterWaves) {
        uint32_t pos[H], end[H];
        bool more = false;
#pragma unroll
        for (uint32_t h = 0; h < H; ++h) {
            const uint32_t b = i + h * kGroups + grp;
            pos[h] = 0; end[h] = 0;
            if (b < nb) { pos[h] = desc[b].x; end[h] = desc[b].y; }
            more = more || pos[h] < end[h];
        }
        while (more) {
            uint32_t src[H][T];
#pragma unroll
            for (uint32_t h = 0; h < H; ++h)
#pragma unroll
                for (uint32_t t = 0; t < T; ++t) {
                    const uint32_t m = pos[h] + sub + L * t;
                    src[h][t] = m < end[h] ? src16[m] : 0u;
                }
            float val[H][T];
#pragma unroll
            for (uint32_t h = 0; h < H; ++h)
#pragma unroll
                for (uint32_t t = 0; t < T; ++t) val[h][t] = src[h][t] < n ? slice[src[h][t]] : 0.0f;
            more = false;
#pragma unroll
            for (uint32_t h = 0; h < H; ++h) {
#pragma unroll
                for (uint32_t t = 0; t < T; ++t) {
                    const uint32_t m = pos[h] + sub + L * t;
                    if (m < end[h]) msg[m] = val[h][t];
                }
                pos[h] = pos[h] + T * L < end[h] ? pos[h] + T * L : end[h];
                more = more || pos[h] < end[h];
            }
        }
    }
}

// `parity` names the set of dangling partials that belongs to the iteration just finished (ignored when first).
template <uint32_t kSrcPerPart>
__global__ __launch_bounds__(kScatterBlock) void k_scatter(DevArgs A, GateArg G, uint32_t tile0, int parity, int first)
{
    __shared__ __align__(16) float slice[kSrcPerPart];
    __shared__ uint2 desc[kDescBatch];
    __shared__ float red[32];
    if (!fr_gate_admit(G.gate, G.slot, G.need_ticks)) return;
    const uint32_t p = tile0 + xcd_contiguous(blockIdx.x, gridDim.x);
    const int64_t v0 = (int64_t)p * kSrcPerPart;
    const uint32_t n = (uint32_t)((A.V - v0) < (int64_t)kSrcPerPart ? (A.V - v0) : (int64_t)kSrcPerPart);
    const float d_part = first ? 0.0f : dangling_partial(A.dpart + (size_t)parity * A.n_dpart, A.n_dpart);
    for (uint32_t i = threadIdx.x * 4; i < n; i += kScatterBlock * 4) {
        if (i + 3 < n) *reinterpret_cast<float4*>(&slice[i]) = *reinterpret_cast<const float4*>(A.contrib + v0 + i);
        else
            for (uint32_t c = i; c < n; ++c) slice[c] = A.contrib[v0 + c];
    }
    if (!first) {
        // finish the hubs of this slice: 16 lanes add up a hub's virtual rows, the first of them applies
        // r = base + d * sum and puts contrib = r / outdeg into the slice
        const float D = dangling_finish(d_part, red);              // (its barriers also order the slice loads)
        const float base = (1.0f - A.damping) / (float)A.V + A.damping * D / (float)A.V;
        const uint32_t h0 = A.hub_of_p[p], h1 = A.hub_of_p[p + 1];
        const uint32_t sub = threadIdx.x & 15;
        float dangling = 0.0f;
        for (uint32_t hb = h0; hb < h1; hb += kScatterBlock / 16) {      // uniform trip count for the whole workgroup
            const uint32_t h = hb + (threadIdx.x >> 4);
            unsigned long long s = 0ull;
            if (h < h1 && h < A.n_hubs) {
                const uint32_t a = A.hub_vbase[h], b = A.hub_vbase[h + 1];
                for (uint32_t i = a + sub; i < b && i < A.n_vrows; i += 16) s += A.vacc[i];
            }
#pragma unroll
            for (int off = 8; off >= 1; off >>= 1) s += (unsigned long long)__shfl_xor((long long)s, off, 64);
            if (h < h1 && h < A.n_hubs && sub == 0) {
                const int64_t v = A.hub_row[h];
                const float inv = inv_of_tag(A.inv_tag[v]);
                const float r = fmaf(A.damping, (float)s * kFixInv, base);
                if (v >= v0 && v < v0 + (int64_t)n) slice[v - v0] = r * inv;
                dangling += (inv == 0.0f ? r : 0.0f);
            }
        }
        const float total = block_sum(dangling, red + 8);
        if (threadIdx.x == 0) A.dpart[(size_t)(parity ^ 1) * A.n_dpart + A.Q + p] = total;
    }
    const uint32_t Q = A.Q;
    for (uint32_t qb = 0; qb < Q; qb += kDescBatch) {
        const uint32_t nb = Q - qb < kDescBatch ? Q - qb : kDescBatch;
        __syncthreads();                                   // slice loaded / previous batch consumed
        for (uint32_t i = threadIdx.x; i < nb; i += kScatterBlock) {
            uint2 b = A.bins[(uint64_t)p * Q + qb + i];
            if (b.y > A.M) b.y = A.M;
            if (b.x > b.y) b.x = b.y;
            desc[i] = b;
        }
        __syncthreads();
        switch (A.scatter_shape) {
        case kShape_64x4: scatter_bins<64, 4>(A.src16, A.msg, desc, nb, slice, n); break;
        case kShape_32x4: scatter_bins<32, 4>(A.src16, A.msg, desc, nb, slice, n); break;
        case kShape_32x2: scatter_bins<32, 2>(A.src16, A.msg, desc, nb, slice, n); break;
        default: scatter_bins<64, 8>(A.src16, A.msg, desc, nb, slice, n); break;
        }
    }
    fr_gate_done(G.gate);
}

// ---- G_k ----

// floor(x * 2^62) for 0 <= x <= 1, exactly: x * 2^30 is exact, its integer part is the high word, its
// fraction times 2^32 (exact again, then truncated) the low word.
__device__ __forceinline__ unsigned long long to_fixed(float x)
{
    const float t = x * 1073741824.0f;
    const uint32_t hi = (uint32_t)t;
    const uint32_t lo = (uint32_t)(__builtin_amdgcn_fractf(t) * 4294967296.0f);
    return ((unsigned long long)hi << 32) | lo;
}

__device__ __forceinline__ uint32_t id_of(const uint4& raw, int j)
{
    const uint32_t w = (j >> 1) == 0 ? raw.x : (j >> 1) == 1 ? raw.y : (j >> 1) == 2 ? raw.z : raw.w;
    return (j & 1) ? (w >> 16) : (w & 0xffffu);
}

// One workgroup per destination partition; its accumulators (one u64 per row, plus the spare slots for hubs'
// virtual rows) sit in LDS.  Per step a wavefront takes one chunk of 512 ids (8 per lane).  The loop is a
// three-stage software pipeline over the wavefront's chunks, so that no step waits on a load it has just issued:
//   A  ids and message base of chunk i + 2 are requested;
//   B  chunk i + 1 (ids now here): ballots of the message-start flags tell every id which message it belongs
//      to; the messages are requested (64 consecutive ids per load, so the addresses are all but contiguous);
//   C  chunk i (messages now here): each id adds its message, as a 64-bit fixed-point integer, to its row's
//      accumulator with an LDS atomic.
// The sweep is bound by vector instruction issue, not by memory (about 30 instructions per 64 edges when every id
// is checked), so chunks that lie wholly inside the partition's edge range and whose messages cannot pass the end
// of the message array - all but the first and last chunk of a partition - take a path without per-id checks:
// ids out of range (which a sound layout never holds) are sent to a sink slot behind the accumulators.
// (two workgroups of the small size share a CU: 8 wavefronts per SIMD, hence at most 64 registers per lane)
template <uint32_t kRowsPerPart>
__global__ __launch_bounds__(kGatherBlock) __attribute__((amdgpu_waves_per_eu(kRowsPerPart == kRowsSmall ? 8 : 4, kRowsPerPart == kRowsSmall ? 8 : 4)))
void k_gather(DevArgs A, GateArg G, uint32_t tile0, int parity, int final_pass)
{
    constexpr uint32_t kAccSlots = kRowsPerPart + kMaxVrowsPerPart;
    __shared__ unsigned long long acc[kAccSlots + 1];            // + the sink slot
    __shared__ float red[32];
    if (!fr_gate_admit(G.gate, G.slot, G.need_ticks)) return;
    const uint32_t q = tile0 + blockIdx.x;
    const int64_t left = A.V - (int64_t)q * kRowsPerPart;
    const uint32_t nrows = (uint32_t)(left < (int64_t)kRowsPerPart ? left : (int64_t)kRowsPerPart);
    for (uint32_t i = threadIdx.x; i < kAccSlots + 1; i += kGatherBlock) acc[i] = 0ull;
    const float d_part = dangling_partial(A.dpart + (size_t)parity * A.n_dpart, A.n_dpart);
    __syncthreads();

    const uint32_t e0 = A.eoff[q], e1 = A.eoff[q + 1];
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (e1 > e0) {
        const uint32_t c0 = e0 / kIdChunk, c1 = (e1 - 1) / kIdChunk;
        const uint4* ids4 = reinterpret_cast<const uint4*>(A.ids16);
        // stage A's result: chunk cA, its ids and the number of messages begun before it
        uint32_t cA = c0 + wave;
        uint4 rawA = make_uint4(0, 0, 0, 0);
        uint32_t mbA = 0;
        if (cA <= c1) { rawA = ids4[(uint64_t)cA * (kIdChunk / 8) + lane]; mbA = A.mbase[cA]; }
        // stage B's result, waiting for stage C
        uint4 rawP = make_uint4(0, 0, 0, 0);
        float valP[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) valP[j] = 0.0f;
        uint32_t okP = 0;            // per-id validity bits of a checked chunk
        bool fastP = false;          // the chunk took the unchecked path (wavefront-uniform)
        while (cA <= c1) {
            // ---- stage B on chunk cA: lane l holds the ids at stream positions 64 j + l of the chunk, so for a
            // fixed j the wavefront covers 64 consecutive ids; a ballot of their flags plus a count of the set
            // bits below the lane tells every id how many messages have begun up to it.
            float valN[8];
            uint32_t okN = 0;
            const uint32_t mb = (uint32_t)__builtin_amdgcn_readfirstlane((int)mbA);
            const uint64_t first = (uint64_t)cA * kIdChunk;
            // mb >= 1: an id without a flag then still has a message before it (index >= 0 below)
            const bool fast = first >= e0 && first + kIdChunk <= e1 && mb >= 1 && (uint64_t)mb + kIdChunk <= A.M;
            if (fast) {
                uint32_t begun_m1 = mb - 1u;                               // messages begun before row j, minus one
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const uint32_t f = id_of(rawA, j) >> 15;
                    const unsigned long long ballot = __ballot(f != 0);
                    const uint32_t below = __builtin_amdgcn_mbcnt_hi((uint32_t)(ballot >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)ballot, 0u));
                    valN[j] = A.msg[begun_m1 + below + f];                 // in [mb - 1, mb + 511], inside [0, M)
                    begun_m1 += (uint32_t)__popcll(ballot);
                }
            } else {
                const uint32_t ebase = cA * kIdChunk + lane;
                uint32_t begun = mb;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const uint32_t id = id_of(rawA, j);
                    const uint32_t f = id >> 15;
                    const unsigned long long ballot = __ballot(f != 0);
                    const uint32_t below = __builtin_amdgcn_mbcnt_hi((uint32_t)(ballot >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)ballot, 0u));
                    const uint32_t mi = begun + below + f - 1;             // this id's message
                    begun += (uint32_t)__popcll(ballot);
                    const uint32_t e = ebase + 64 * j;
                    const bool ok = e >= e0 && e < e1 && (id & kLocalMask) < kAccSlots && mi < A.M;
                    okN |= (ok ? 1u : 0u) << j;
                    valN[j] = A.msg[ok ? mi : 0u];
                }
            }
            const uint4 rawN = rawA;
            // ---- stage A on this wavefront's next chunk
            cA += kGatherWaves;
            if (cA <= c1) { rawA = ids4[(uint64_t)cA * (kIdChunk / 8) + lane]; mbA = A.mbase[cA]; }
            else rawA = make_uint4(0, 0, 0, 0);
            // ---- stage C on the previous chunk
            if (fastP) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const uint32_t local = id_of(rawP, j) & kLocalMask;
                    atomicAdd(&acc[local < kAccSlots ? local : kAccSlots], to_fixed(valP[j]));
                }
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if ((okP >> j) & 1u) atomicAdd(&acc[id_of(rawP, j) & kLocalMask], to_fixed(valP[j]));
            }
            rawP = rawN;
            okP = okN;
            fastP = fast;
#pragma unroll
            for (int j = 0; j < 8; ++j) valP[j] = valN[j];
        }
        // drain: stage C on the last chunk
        if (fastP) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t local = id_of(rawP, j) & kLocalMask;
                atomicAdd(&acc[local < kAccSlots ? local : kAccSlots], to_fixed(valP[j]));
            }
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if ((okP >> j) & 1u) atomicAdd(&acc[id_of(rawP, j) & kLocalMask], to_fixed(valP[j]));
        }
    }
    __syncthreads();

    // virtual rows dealt to this partition: hv = q + slot * Q
    for (uint32_t slot = threadIdx.x; slot < kMaxVrowsPerPart; slot += kGatherBlock) {
        const uint64_t hv = (uint64_t)q + (uint64_t)slot * A.Q;
        if (hv < A.n_vrows) A.vacc[hv] = acc[kRowsPerPart + slot];
    }
    // fused vertex pass for the partition's own rows
    const float D = dangling_finish(d_part, red);
    const float base = (1.0f - A.damping) / (float)A.V + A.damping * D / (float)A.V;
    const int64_t v0 = (int64_t)q * kRowsPerPart;
    float dangling = 0.0f;
    constexpr int kRowsPerThread = (kRowsPerPart + kGatherBlock - 1) / kGatherBlock;
    float tag[kRowsPerThread];
#pragma unroll
    for (int t = 0; t < kRowsPerThread; ++t) {
        const uint32_t i = threadIdx.x + kGatherBlock * t;
        tag[t] = i < nrows ? A.inv_tag[v0 + i] : -0.0f;           // rows past the end behave like hubs: skipped
    }
#pragma unroll
    for (int t = 0; t < kRowsPerThread; ++t) {
        const uint32_t i = threadIdx.x + kGatherBlock * t;
        if (i >= nrows || is_hub_tag(tag[t])) continue;            // hubs are finished by H_k
        const float s = (float)acc[i] * kFixInv;
        const float r = fmaf(A.damping, s, base);
        if (final_pass) A.ranks_out[v0 + i] = r;
        else {
            A.contrib[v0 + i] = r * tag[t];
            dangling += (tag[t] == 0.0f ? r : 0.0f);
        }
    }
    if (!final_pass) {
        const float total = block_sum(dangling, red + 8);
        if (threadIdx.x == 0) A.dpart[(size_t)(parity ^ 1) * A.n_dpart + q] = total;
    }
    fr_gate_done(G.gate);
}

// ---- H_k ----
// 16 hubs per workgroup, 16 lanes per hub: the lanes add up the hub's virtual rows (integers, any order), the
// group's first lane applies the vertex-pass arithmetic.
__global__ __launch_bounds__(256) void k_hubfin(DevArgs A, GateArg G, uint32_t tile0, int parity, int final_pass)
{
    __shared__ float red[24];
    if (!fr_gate_admit(G.gate, G.slot, G.need_ticks)) return;
    const uint32_t t = tile0 + blockIdx.x;
    const float D = dangling_finish(dangling_partial(A.dpart + (size_t)parity * A.n_dpart, A.n_dpart), red);
    const float base = (1.0f - A.damping) / (float)A.V + A.damping * D / (float)A.V;
    const uint32_t h = t * kHubsPerTile + (threadIdx.x >> 4);
    const uint32_t sub = threadIdx.x & 15;
    float dangling = 0.0f;
    unsigned long long s = 0ull;
    if (h < A.n_hubs) {
        const uint32_t a = A.hub_vbase[h], b = A.hub_vbase[h + 1];
        for (uint32_t i = a + sub; i < b && i < A.n_vrows; i += 16) s += A.vacc[i];
    }
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1) s += (unsigned long long)__shfl_xor((long long)s, off, 64);
    if (h < A.n_hubs && sub == 0) {
        const int32_t v = A.hub_row[h];
        const float inv = inv_of_tag(A.inv_tag[v]);
        const float r = fmaf(A.damping, (float)s * kFixInv, base);
        if (final_pass) A.ranks_out[v] = r;
        else {
            A.contrib[v] = r * inv;
            dangling = (inv == 0.0f ? r : 0.0f);
        }
    }
    (void)dangling;          // H only runs after the last iteration: nothing reads its dangling sum
    fr_gate_done(G.gate);
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
    float *msg = nullptr, *contrib = nullptr, *dpart = nullptr;
    unsigned long long* vacc = nullptr;
    uint32_t n_dpart = 0;
    DevArgs args{};
    bool inited = false;
    bool registered = false;
    fr_alloc own;                         // used by the standalone run only
    int hip_error = 0;
    uint32_t run = 0, seg = 0, tile = 0;  // cursor

    // V0, then S_k G_k for k < K, then H (no S, G, H at all when K = 0)
    uint32_t n_segments() const { return d.iterations == 0 ? 1u : 2u + 2u * (uint32_t)d.iterations; }
    int kind_of(uint32_t g) const
    {
        if (g == 0) return FR_PR_SEG_VERTEX;
        if (g + 1 == n_segments()) return FR_PR_SEG_HUBFIN;
        return ((g - 1) & 1u) ? FR_PR_SEG_GATHER : FR_PR_SEG_SCATTER;
    }
    uint32_t tiles_of(int kind) const
    {
        switch (kind) {
        case FR_PR_SEG_VERTEX: return L.Q;
        case FR_PR_SEG_SCATTER: return L.P;
        case FR_PR_SEG_GATHER: return L.Q;
        default: return L.n_hub_tiles;
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
    s.assign(L.P + 1, 0);
    for (uint32_t i = 0; i < L.P; ++i) {
        const uint64_t srcs = std::min<uint64_t>(L.src_per_part, (uint64_t)L.V - (uint64_t)i * L.src_per_part);
        s[i + 1] = s[i] + ceil_fs_to_ns((unsigned __int128)L.msgs_of_p[i] * pm + (unsigned __int128)srcs * pv);
    }
    auto& g = p->prefix[FR_PR_SEG_GATHER];
    g.assign(L.Q + 1, 0);
    for (uint32_t q = 0; q < L.Q; ++q)
        g[q + 1] = g[q] + ceil_fs_to_ns((unsigned __int128)L.edges_of_q[q] * pe + (unsigned __int128)p->rows_of_q(q) * pv);
    auto& h = p->prefix[FR_PR_SEG_HUBFIN];
    h.assign(L.n_hub_tiles + 1, 0);
    for (uint32_t t = 0; t < L.n_hub_tiles; ++t) h[t + 1] = h[t] + std::max<uint64_t>(1, p->d.hubfin_tile_ns);
}

int pr_launch(PrTask* p, uint32_t g, uint32_t tile0, uint32_t tile1, hipStream_t stream, GateArg G = GateArg{nullptr, 0, 0})
{
    const int kind = p->kind_of(g);
    if (tile1 <= tile0 || tile1 > p->tiles_of(kind)) return FR_ERR_ARG;
    const uint32_t n = tile1 - tile0;
    const uint32_t K = (uint32_t)p->d.iterations;
    if (kind == FR_PR_SEG_VERTEX) {
        hipLaunchKernelGGL(k_vertex0, dim3(n), dim3(kBlock), 0, stream, p->args, G, tile0, K == 0 ? 1 : 0);
    } else if (kind == FR_PR_SEG_HUBFIN) {
        // after G_{K-1}: the dangling partials of r_{K-1} sit in set (K-1) & 1
        hipLaunchKernelGGL(k_hubfin, dim3(n), dim3(256), 0, stream, p->args, G, tile0, (int)((K - 1) & 1u), 1);
    } else {
        const uint32_t k = (g - 1) / 2;
        if (kind == FR_PR_SEG_SCATTER) {    // S_k finishes the hubs of r_k with D_{k-1}: set (k-1) & 1
            const int parity = (int)((k + 1) & 1u), first = k == 0 ? 1 : 0;
            if (p->L.src_per_part == kSrcLarge)
                hipLaunchKernelGGL(k_scatter<kSrcLarge>, dim3(n), dim3(kScatterBlock), 0, stream, p->args, G, tile0, parity, first);
            else
                hipLaunchKernelGGL(k_scatter<kSrcSmall>, dim3(n), dim3(kScatterBlock), 0, stream, p->args, G, tile0, parity, first);
        } else {
            const int parity = (int)(k & 1u), final_pass = (k + 1 == K) ? 1 : 0;
            if (p->L.rows_per_part == kRowsLarge)
                hipLaunchKernelGGL(k_gather<kRowsLarge>, dim3(n), dim3(kGatherBlock), 0, stream, p->args, G, tile0, parity, final_pass);
            else
                hipLaunchKernelGGL(k_gather<kRowsSmall>, dim3(n), dim3(kGatherBlock), 0, stream, p->args, G, tile0, parity, final_pass);
        }
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { p->hip_error = (int)e; return FR_ERR_HIP; }
    return FR_OK;
}

// Shape of the scatter sweep's inner loop (lanes per bin x messages per lane): the smallest step, L * T
// messages, that covers an average bin with a third to spare (measured: 27-message bins run fastest as 32 x 2,
// 94-message bins as 32 x 4, 305-message bins as 64 x 8).
uint32_t scatter_shape_for(uint64_t messages, uint64_t bins)
{
    const uint64_t want = bins ? 4 * (messages / bins) / 3 : 0;
    if (want <= 64) return kShape_32x2;
    if (want <= 128) return kShape_32x4;
    if (want <= 256) return kShape_64x4;
    return kShape_64x8;
}

template <typename T>
bool take(fr_alloc* a, T** out, uint64_t count)
{
    *out = static_cast<T*>(fr_alloc_device(a, (size_t)(count ? count : 1) * sizeof(T)));
    return *out != nullptr;
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
                             p->d.sources_per_partition, a, stream, &p->hip_error);
    if (rc != FR_OK) return rc;
    PrLayout& L = p->L;
    p->n_dpart = L.Q + L.P;                  // one slot per gather tile, one per scatter tile (its hubs)
    if (!take(a, &p->msg, L.M) || !take(a, &p->contrib, (uint64_t)V) || !take(a, &p->dpart, 2ull * p->n_dpart) ||
        !take(a, &p->vacc, (uint64_t)L.n_vrows))
        return a->hip_error ? FR_ERR_HIP : FR_ERR_OOM;
    DevArgs& A = p->args;
    A.V = V; A.E = E; A.M = (uint32_t)L.M; A.Q = L.Q; A.P = L.P; A.n_hubs = L.n_hubs; A.n_vrows = L.n_vrows;
    A.n_dpart = p->n_dpart; A.damping = p->d.damping;
    A.scatter_shape = scatter_shape_for(L.M, (uint64_t)L.P * L.Q);
    A.rows_per_part = L.rows_per_part; A.src_per_part = L.src_per_part;
    A.ids16 = L.ids16; A.src16 = L.src16; A.eoff = L.eoff; A.mbase = L.mbase; A.bins = L.bins;
    A.hub_row = L.hub_row; A.hub_vbase = L.hub_vbase; A.hub_of_p = L.hub_of_p; A.inv_tag = L.inv_tag;
    A.msg = p->msg; A.contrib = p->contrib; A.dpart = p->dpart; A.vacc = p->vacc; A.ranks_out = p->d.ranks_out;
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
    out->tile1 = p->tile + n;
    out->modelled_ns = std::max(pre[p->tile + n] - pre[p->tile], floor_ns);
    if (kind == FR_PR_SEG_GATHER) {
        uint64_t edges = 0;
        for (uint32_t q = p->tile; q < p->tile + n; ++q) edges += p->L.edges_of_q[q];
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
                       GateArg{static_cast<fr_gate*>(st->gate), st->gate_slot, st->gate_need_ticks});
    if (rc != FR_OK) return rc;
    p->tile = st->tile1;
    if (p->tile == p->tiles_of(p->kind_of(p->seg))) {
        p->tile = 0;
        if (++p->seg == p->n_segments()) { p->seg = 0; p->run++; }
    }
    return FR_OK;
}

// The device gate refused `first` and every step after it: they did nothing, so the cursor goes back to its start.
int pr_rewind(void* user, const fr_step* first)
{
    PrTask* p = static_cast<PrTask*>(user);
    if (!p->inited || !first || first->segment >= p->n_segments() || first->tile0 >= p->tiles_of(p->kind_of(first->segment)))
        return FR_ERR_ARG;
    p->run = first->run; p->seg = first->segment; p->tile = first->tile0;
    return FR_OK;
}

int pr_stop(void* user)
{
    PrTask* p = static_cast<PrTask*>(user);
    p->inited = false;        // the runtime's allocator frees the device blocks
    p->registered = false;
    return FR_OK;
}

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
    if (!p->d.hubfin_tile_ns) p->d.hubfin_tile_ns = 2000;
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
    out->partitions = p->L.Q;
    out->hub_split = p->L.hub_split;
    out->rows_per_partition = p->L.rows_per_part;
    out->sources_per_partition = p->L.src_per_part;
    out->source_partitions = p->L.P;
    out->hubs = p->L.n_hubs;
    out->virtual_rows = p->L.n_vrows;
    out->bytes_resident = p->footprint_after;
    out->bytes_peak = p->footprint_peak;
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
        if (seg_kind == FR_PR_SEG_GATHER) work[t] = p->L.edges_of_q[t];
        else if (seg_kind == FR_PR_SEG_SCATTER) work[t] = p->L.msgs_of_p[t];
        else if (seg_kind == FR_PR_SEG_VERTEX) work[t] = p->rows_of_q((uint32_t)t);
        else work[t] = 0;
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

}  // extern "C"
