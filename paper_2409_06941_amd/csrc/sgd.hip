// Graph SGD side task: stochastic gradient descent for matrix factorization over a rating graph, the second graph
// workload the paper harvests bubbles with (Section 6.1.4; Section 6.2: one iteration = one pass over the graph).
//
// The paper names the method only, so the arithmetic is the textbook one (Koren, Bell, Volinsky 2009): for every
// rating r_ui, one after the other,
//     e = r_ui - <p_u, q_i>,   p_u += gamma (e q_i - lambda p_u),   q_i += gamma (e p_u - lambda q_i)
// and the order of the updates is a stratified one (Gemulla et al. 2011), which a GPU can follow without races and
// without depending on timing: users and items are cut into B blocks of consecutive ids holding about E / B ratings
// each (block k begins at the first id with ceil(k E / B) or more ratings before it); the ratings of user block a
// and item block b are cell (a, b); an iteration is B strata, stratum s = the cells (a, (a + s) mod B), which share
// no user and no item and therefore run side by side; inside a cell the ratings are taken by user, then by item,
// one after the other.  Every rounding of an update is fixed (see k_sgd), so the factors do not depend on how the
// cells are grouped into launches, and an fp32 CPU implementation of the same steps gives the same bits.
//
// One run = K iterations = K * B segments (a segment is a stratum; a step is a run of consecutive cells of one
// stratum; tile = cell).  The factors carry over from run to run: the task keeps training.
//
// Layout, built once in InitSideTask: the ratings sorted by (stratum, user, item) as 64-bit keys
// (stratum << 54 | user << 27 | item) with the ratings alongside, and the start of every cell in that order.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <new>
#include <vector>

#include <rocprim/rocprim.hpp>

#include "common.h"
#include "freeride_device.h"

namespace {

constexpr int kSgdBlock = 256;
constexpr int kAhead = 2;                        // ratings whose rows are in flight ahead of the one being worked on (>= 2)
constexpr int kIdBits = 27;                      // users and items below 2^27, at most 1024 blocks
constexpr uint64_t kIdMask = (1ull << kIdBits) - 1;
constexpr int kStratumShift = 2 * kIdBits;
constexpr uint32_t kMaxBlocks = 1024;

struct SgdArgs {
    const uint64_t* keys;        // [E] sorted
    const float* rating;         // [E] in the order of keys
    const uint32_t* cell_ptr;    // [B * B + 1] first rating of cell s * B + a
    float* P;
    float* Q;
    float gamma, gl;             // gl = gamma * lambda, rounded once
};

struct GateArg {
    fr_gate* gate;
    uint32_t slot, need_ticks;
};

__device__ __forceinline__ uint32_t user_of(uint64_t key) { return (uint32_t)((key >> kIdBits) & kIdMask); }
__device__ __forceinline__ uint32_t item_of(uint64_t key) { return (uint32_t)(key & kIdMask); }

// One group of F lanes per cell, lane l holding dimension l of the factors; the cell's ratings one after the other.
// The update, with every rounding fixed:
//     t_l = p_l * q_l;  in rounds w = 1, 2, 4, .., F/2: t_l = t_l + t_(l xor w)   (all lanes end with the same sum)
//     e = r - t;  ge = gamma * e;  p_l' = fma(ge, q_l, fma(-gl, p_l, p_l));  q_l' = fma(ge, p_l, fma(-gl, q_l, q_l))
// A cell is one chain of dependent updates, so what it costs per rating is the latency of fetching the rating's
// rows.  The loop therefore looks two ratings ahead (and three for the keys): while rating x - 2 is being worked
// on, the rows of rating x are requested, unless they are held in registers by then (same user / same item as
// rating x - 1) or could still be written before they are used: q of rating x may be requested early only if its
// item differs from those of ratings x - 2 and x - 1; if it is the item of rating x - 2, the request waits until
// that rating's row has been stored (a wavefront's own store and later load of one address stay in order).  Users
// ascend inside a cell, so a row of P asked for early is never written in between.
// (The product p_l * q_l has to be kept from being folded into the first addition of the tree as a fused
// multiply-add: the rounded-operation intrinsics are plain operators to the compiler, so the product passes
// through an empty asm statement, which hides where it came from.)
__device__ __forceinline__ float rounded_product(float x, float y)
{
    float t = x * y;
    asm("" : "+v"(t));
    return t;
}

// The tree sum over a group of F lanes (F = 16, 32, 64; groups aligned in the wavefront): t_l + t_(l xor 1), then
// xor 2, 4, ... as defined above.  A butterfly with ds_bpermute costs an LDS round trip per round, which is most of
// what a rating costs a cell's chain, so the rounds inside a row of 16 lanes use DPP moves instead: quad
// permutations for xor 1 and 2; for xor 4 and 8 the half-row and row mirrors, which pair every lane with a lane of
// the other half - not lane l xor 4 itself, but by then all lanes of a quad (of a half-row) hold the same value, so
// the sums are the same numbers.  Rows are joined through readlane: row sums R_0 .. R_3, (R_0 + R_1) and
// (R_2 + R_3), then their sum - the same tree.  (readlane ignores the execution mask; a group only uses its own
// rows, whose lanes are all active together.)
template <int kCtrl>
__device__ __forceinline__ float add_dpp(float t)
{
    const int moved = __builtin_amdgcn_mov_dpp(__float_as_int(t), kCtrl, 0xf, 0xf, false);
    return __fadd_rn(t, __int_as_float(moved));
}

template <int F>
__device__ __forceinline__ float group_sum(float t)
{
    t = add_dpp<0xB1>(t);        // quad_perm [1, 0, 3, 2]
    t = add_dpp<0x4E>(t);        // quad_perm [2, 3, 0, 1]
    t = add_dpp<0x141>(t);       // row_half_mirror
    t = add_dpp<0x140>(t);       // row_mirror
    if constexpr (F == 16) return t;
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(t), 0));
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(t), 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(t), 32));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(t), 48));
    const float lo = __fadd_rn(r0, r1), hi = __fadd_rn(r2, r3);
    if constexpr (F == 32) return (threadIdx.x & 32) ? hi : lo;
    return __fadd_rn(lo, hi);
}

template <int F>
__global__ __launch_bounds__(kSgdBlock) void k_sgd(SgdArgs A, GateArg G, uint32_t cell0, uint32_t n_cells)
{
    if (!fr_gate_admit(G.gate, G.slot, G.need_ticks)) return;
    const uint32_t g = (blockIdx.x * kSgdBlock + threadIdx.x) / F, l = threadIdx.x % F;
    if (g < n_cells) {
        uint32_t e = A.cell_ptr[cell0 + g];
        const uint32_t e1 = A.cell_ptr[cell0 + g + 1];
        if (e < e1) {
            const float* __restrict__ rating = A.rating;
            const uint64_t* __restrict__ keys = A.keys;
            // Slot k holds rating e + k: slot 0 is being worked on, the rows of slots 1 .. kAhead have been asked
            // for, slot kAhead + 1 holds a key only.  Every iteration issues the same loads and stores whether
            // their values are needed or not (behind the cell's end: those of its last rating again), so that the
            // compiler can count what is in flight and waits only for the oldest request, not for all of them.
            uint32_t us[kAhead + 2], is[kAhead + 2];
            float rs[kAhead + 2], ps[kAhead + 1], qs[kAhead + 1];
            bool late[kAhead + 1] = {};
#pragma unroll
            for (int k = 0; k < kAhead + 2; ++k) {
                const uint32_t ek = e + k < e1 ? e + k : e1 - 1;
                const uint64_t key = keys[ek];
                us[k] = user_of(key); is[k] = item_of(key); rs[k] = rating[ek];
            }
#pragma unroll
            for (int k = 0; k < kAhead; ++k) {
                ps[k] = A.P[(size_t)us[k] * F + l];
                qs[k] = A.Q[(size_t)is[k] * F + l];
                bool clash = false;
#pragma unroll
                for (int j = 0; j + 1 < k; ++j) clash |= is[k] == is[j];
                late[k] = k >= 2 && is[k] != is[k - 1] && clash;
            }
            for (;;) {
                // the rows of slot kAhead.  q may be used as it arrives if no rating before it in flight writes it:
                // not the one just before it (then the registers are handed on) and none of the others (then the
                // row is asked for again once they have stored theirs: late)
                ps[kAhead] = A.P[(size_t)us[kAhead] * F + l];
                qs[kAhead] = A.Q[(size_t)is[kAhead] * F + l];
                {
                    bool clash = false;
#pragma unroll
                    for (int j = 0; j + 1 < kAhead; ++j) clash |= is[kAhead] == is[j];
                    late[kAhead] = is[kAhead] != is[kAhead - 1] && clash;
                }
                const uint32_t en = e + kAhead + 2 < e1 ? e + kAhead + 2 : e1 - 1;
                const uint64_t keyn = keys[en];
                const float rn = rating[en];
                const float p = ps[0], q = qs[0];
                const float t = group_sum<F>(rounded_product(p, q));
                const float ge = __fmul_rn(A.gamma, __fsub_rn(rs[0], t));
                const float p2 = __fmaf_rn(ge, q, __fmaf_rn(-A.gl, p, p));
                const float q2 = __fmaf_rn(ge, p, __fmaf_rn(-A.gl, q, q));
                A.P[(size_t)us[0] * F + l] = p2;
                A.Q[(size_t)is[0] * F + l] = q2;
                if (e + 1 >= e1) break;
                if (us[1] == us[0]) ps[1] = p2;          // the same user / item again: its row is in registers
                if (is[1] == is[0]) qs[1] = q2;
                // every rating before slot 1 has stored its row by now: a late row can be asked for
                const float again = A.Q[(size_t)is[2] * F + l];
                if (late[2]) qs[2] = again;
#pragma unroll
                for (int k = 0; k < kAhead; ++k) { ps[k] = ps[k + 1]; qs[k] = qs[k + 1]; }
#pragma unroll
                for (int k = 1; k < kAhead; ++k) late[k] = k == 1 ? false : late[k + 1];
#pragma unroll
                for (int k = 0; k < kAhead + 1; ++k) { us[k] = us[k + 1]; is[k] = is[k + 1]; rs[k] = rs[k + 1]; }
                us[kAhead + 1] = user_of(keyn); is[kAhead + 1] = item_of(keyn); rs[kAhead + 1] = rn;
                ++e;
            }
        }
    }
    fr_gate_done(G.gate, G.slot);
}

// ---- set-up kernels ----
__global__ void k_sgd_set(int32_t* p, int32_t v) { *p = v; }

__global__ __launch_bounds__(256) void k_sgd_validate(int64_t U, int64_t I, int64_t E, const int32_t* __restrict__ row_ptr,
                                                      const int32_t* __restrict__ item, int32_t* bad)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; u <= U; u += stride) {
        const int32_t a = row_ptr[u];
        if (a < 0 || a > E || (u == 0 && a != 0) || (u == U && a != E) || (u < U && row_ptr[u + 1] < a)) *bad = 1;
    }
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < E; e += stride)
        if (item[e] < 0 || item[e] >= I) *bad = 1;
}

// The block of id x: the last k below B with starts[k] <= x (empty blocks share their start with the next one).
__device__ __forceinline__ uint32_t block_of(const uint32_t* __restrict__ starts, uint32_t B, uint32_t x)
{
    uint32_t lo = 0, hi = B - 1;
    while (lo < hi) {
        const uint32_t mid = (lo + hi + 1) / 2;
        if (starts[mid] <= x) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}

__global__ __launch_bounds__(256) void k_sgd_zero(uint32_t* p, uint64_t n)
{
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

__global__ __launch_bounds__(256) void k_sgd_count_items(int64_t E, const int32_t* __restrict__ item, uint32_t* count)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e < E) atomicAdd(&count[item[e]], 1u);
}

// starts[k], k = 0 .. B: block k begins at the first id x with before[x] >= ceil(k E / B); before[x] = ratings of the
// ids below x (n + 1 entries, int32 or uint32: the values are below 2^31 either way).
__global__ __launch_bounds__(256) void k_sgd_starts(uint32_t n, const uint32_t* __restrict__ before, int64_t E, uint32_t B,
                                                    uint32_t* __restrict__ starts)
{
    const uint32_t k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k > B) return;
    if (k == 0 || k == B) { starts[k] = k == 0 ? 0u : n; return; }
    const uint64_t want = ((uint64_t)k * (uint64_t)E + B - 1) / B;
    uint32_t lo = 0, hi = n;                    // first x with before[x] >= want (before[n] = E >= want)
    while (lo < hi) {
        const uint32_t mid = lo + (hi - lo) / 2;
        if ((uint64_t)before[mid] < want) lo = mid + 1;
        else hi = mid;
    }
    starts[k] = lo;
}

// key of rating e; its user is found by bisection of row_ptr.  Also checks that items ascend inside a row.
__global__ __launch_bounds__(256) void k_sgd_keys(int64_t U, int64_t E, const int32_t* __restrict__ row_ptr,
                                                  const int32_t* __restrict__ item, uint32_t B,
                                                  const uint32_t* __restrict__ ustart, const uint32_t* __restrict__ istart,
                                                  uint64_t* __restrict__ keys, int32_t* bad)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= E) return;
    int64_t lo = 0, hi = U;                     // the last u with row_ptr[u] <= e
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) / 2;
        if (row_ptr[mid] <= e) lo = mid;
        else hi = mid;
    }
    const uint32_t u = (uint32_t)lo, i = (uint32_t)item[e];
    if (e > row_ptr[u] && item[e - 1] >= item[e]) *bad = 1;
    const uint32_t a = block_of(ustart, B, u), b = block_of(istart, B, i);
    const uint32_t s = (b + B - a) % B;
    keys[e] = ((uint64_t)s << kStratumShift) | ((uint64_t)u << kIdBits) | i;
}

__global__ __launch_bounds__(256) void k_sgd_cells(int64_t E, uint32_t B, const uint32_t* __restrict__ ustart,
                                                   const uint64_t* __restrict__ keys, uint32_t* __restrict__ cell_ptr)
{
    const uint32_t c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c > B * B) return;
    const uint64_t s = c / B, a = c % B;
    const uint64_t want = c == B * B ? ~0ull : (s << kStratumShift) | ((uint64_t)ustart[a] << kIdBits);
    int64_t lo = 0, hi = E;                     // first rating with key >= want
    while (lo < hi) {
        const int64_t mid = (lo + hi) / 2;
        if (keys[mid] < want) lo = mid + 1;
        else hi = mid;
    }
    cell_ptr[c] = (uint32_t)lo;
}

uint64_t ceil_fs_to_ns(unsigned __int128 fs)
{
    const uint64_t ns = (uint64_t)((fs + 999999) / 1000000);
    return ns ? ns : 1;
}

struct SgdTask {
    fr_sgd_desc d{};
    uint32_t B = 0;
    uint32_t *ustart = nullptr, *istart = nullptr;      // device, B + 1 entries each
    std::vector<uint32_t> ustart_host, istart_host;
    uint64_t* keys = nullptr;
    float* rating = nullptr;
    uint32_t* cell_ptr = nullptr;
    std::vector<uint32_t> cells;          // host copy of cell_ptr
    std::vector<uint64_t> prefix;         // cumulative modelled cost of the cells, in the order of cell_ptr
    uint32_t max_cell = 0;
    uint64_t chain_ratings = 0;           // sum over the strata of their largest cell
    uint64_t footprint_after = 0, footprint_peak = 0;
    SgdArgs args{};
    bool inited = false, registered = false;
    fr_alloc own;                         // used by the standalone run only
    int hip_error = 0;
    uint32_t run = 0, seg = 0, tile = 0;  // cursor

    uint32_t n_segments() const { return (uint32_t)d.iterations * B; }
};

int sgd_launch(SgdTask* p, uint32_t seg, uint32_t tile0, uint32_t tile1, hipStream_t stream, GateArg G = GateArg{nullptr, 0, 0})
{
    if (tile1 <= tile0 || tile1 > p->B || seg >= p->n_segments()) return FR_ERR_ARG;
    const uint32_t s = seg % p->B, n = tile1 - tile0, cell0 = s * p->B + tile0;
    const int F = p->d.factors;
    const unsigned grid = (unsigned)(((uint64_t)n * F + kSgdBlock - 1) / kSgdBlock);
    if (F == 64) hipLaunchKernelGGL(k_sgd<64>, dim3(grid), dim3(kSgdBlock), 0, stream, p->args, G, cell0, n);
    else if (F == 32) hipLaunchKernelGGL(k_sgd<32>, dim3(grid), dim3(kSgdBlock), 0, stream, p->args, G, cell0, n);
    else hipLaunchKernelGGL(k_sgd<16>, dim3(grid), dim3(kSgdBlock), 0, stream, p->args, G, cell0, n);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { p->hip_error = (int)e; return FR_ERR_HIP; }
    return FR_OK;
}

#define SGD_HIP(expr) do { hipError_t e__ = (expr); if (e__ != hipSuccess) { p->hip_error = (int)e__; return FR_ERR_HIP; } } while (0)
#define SGD_NEED(ptr) do { if (!(ptr)) return a->hip_error ? FR_ERR_HIP : FR_ERR_OOM; } while (0)

int sgd_init(void* user, fr_alloc* a, void* stream_v)
{
    SgdTask* p = static_cast<SgdTask*>(user);
    hipStream_t stream = (hipStream_t)stream_v;
    if (a->host_only) return FR_ERR_ARG;      // this task needs a GPU
    const int64_t U = p->d.n_users, I = p->d.n_items, E = p->d.n_ratings;
    const int F = p->d.factors;
    // caller-provided buffers count against the task's limit
    const uint64_t caller = 4ull * (uint64_t)(U + 1) + 8ull * (uint64_t)E + 4ull * (uint64_t)F * (uint64_t)(U + I);
    if (fr_alloc_charge(a, caller) != FR_OK) return FR_ERR_OOM;
    const uint32_t B = p->B;

    int32_t* bad = static_cast<int32_t*>(fr_alloc_device(a, sizeof(int32_t)));
    SGD_NEED(bad);
    hipLaunchKernelGGL(k_sgd_set, dim3(1), dim3(1), 0, stream, bad, 0);
    const unsigned vgrid = (unsigned)std::min<int64_t>((std::max<int64_t>(U + 1, E) + 255) / 256, 65536);
    hipLaunchKernelGGL(k_sgd_validate, dim3(vgrid), dim3(256), 0, stream, U, I, E, p->d.row_ptr, p->d.item, bad);
    int32_t bad_host = 0;
    SGD_HIP(hipMemcpyAsync(&bad_host, bad, sizeof(int32_t), hipMemcpyDeviceToHost, stream));
    SGD_HIP(hipStreamSynchronize(stream));
    if (bad_host) return FR_ERR_ARG;          // (indices are only trusted from here on)

    // ---- blocks of about E / B ratings
    p->ustart = static_cast<uint32_t*>(fr_alloc_device(a, ((uint64_t)B + 1) * 4));
    p->istart = static_cast<uint32_t*>(fr_alloc_device(a, ((uint64_t)B + 1) * 4));
    SGD_NEED(p->ustart); SGD_NEED(p->istart);
    {
        uint32_t* count = static_cast<uint32_t*>(fr_alloc_device(a, ((uint64_t)I + 1) * 4));
        uint32_t* before = static_cast<uint32_t*>(fr_alloc_device(a, ((uint64_t)I + 1) * 4));
        SGD_NEED(count); SGD_NEED(before);
        hipLaunchKernelGGL(k_sgd_zero, dim3((unsigned)((I + 1 + 255) / 256)), dim3(256), 0, stream, count, (uint64_t)I + 1);
        if (E > 0) hipLaunchKernelGGL(k_sgd_count_items, dim3((unsigned)((E + 255) / 256)), dim3(256), 0, stream, E, p->d.item, count);
        size_t bytes = 0;
        SGD_HIP(rocprim::exclusive_scan(nullptr, bytes, count, before, 0u, (size_t)I + 1, rocprim::plus<uint32_t>(), stream));
        void* tmp = fr_alloc_device(a, bytes ? bytes : 1);
        SGD_NEED(tmp);
        SGD_HIP(rocprim::exclusive_scan(tmp, bytes, count, before, 0u, (size_t)I + 1, rocprim::plus<uint32_t>(), stream));
        hipLaunchKernelGGL(k_sgd_starts, dim3((B + 1 + 255) / 256), dim3(256), 0, stream, (uint32_t)I, before, E, B, p->istart);
        hipLaunchKernelGGL(k_sgd_starts, dim3((B + 1 + 255) / 256), dim3(256), 0, stream, (uint32_t)U,
                           reinterpret_cast<const uint32_t*>(p->d.row_ptr), E, B, p->ustart);
        p->ustart_host.assign((size_t)B + 1, 0); p->istart_host.assign((size_t)B + 1, 0);
        SGD_HIP(hipMemcpyAsync(p->ustart_host.data(), p->ustart, ((size_t)B + 1) * 4, hipMemcpyDeviceToHost, stream));
        SGD_HIP(hipMemcpyAsync(p->istart_host.data(), p->istart, ((size_t)B + 1) * 4, hipMemcpyDeviceToHost, stream));
        SGD_HIP(hipStreamSynchronize(stream));
        (void)fr_alloc_free(a, tmp); (void)fr_alloc_free(a, before); (void)fr_alloc_free(a, count);
    }

    const uint64_t n = (uint64_t)(E ? E : 1);
    uint64_t* keys_a = static_cast<uint64_t*>(fr_alloc_device(a, n * 8));
    uint64_t* keys_b = static_cast<uint64_t*>(fr_alloc_device(a, n * 8));
    float* val_b = static_cast<float*>(fr_alloc_device(a, n * 4));
    SGD_NEED(keys_a); SGD_NEED(keys_b); SGD_NEED(val_b);
    p->cell_ptr = static_cast<uint32_t*>(fr_alloc_device(a, ((uint64_t)B * B + 1) * 4));
    SGD_NEED(p->cell_ptr);
    if (E > 0) {
        hipLaunchKernelGGL(k_sgd_keys, dim3((unsigned)((E + 255) / 256)), dim3(256), 0, stream, U, E, p->d.row_ptr, p->d.item, B,
                           p->ustart, p->istart, keys_a, bad);
        SGD_HIP(hipMemcpyAsync(&bad_host, bad, sizeof(int32_t), hipMemcpyDeviceToHost, stream));
        SGD_HIP(hipStreamSynchronize(stream));
        if (bad_host) return FR_ERR_ARG;      // items of a row not ascending / not distinct
        size_t bytes = 0;
        unsigned end_bit = kStratumShift;
        while (end_bit < 64 && (1ull << (end_bit - kStratumShift)) < (uint64_t)B) ++end_bit;
        // (the overload with separate input and output arrays: the caller's ratings are only read)
        SGD_HIP(rocprim::radix_sort_pairs(nullptr, bytes, keys_a, keys_b, p->d.rating, val_b, (size_t)E, 0u, end_bit, stream));
        void* tmp = fr_alloc_device(a, bytes ? bytes : 1);
        SGD_NEED(tmp);
        SGD_HIP(rocprim::radix_sort_pairs(tmp, bytes, keys_a, keys_b, p->d.rating, val_b, (size_t)E, 0u, end_bit, stream));
        SGD_HIP(hipStreamSynchronize(stream));
        (void)fr_alloc_free(a, tmp);
    }
    (void)fr_alloc_free(a, keys_a);
    (void)fr_alloc_free(a, bad);
    p->keys = keys_b;
    p->rating = val_b;
    hipLaunchKernelGGL(k_sgd_cells, dim3((B * B + 1 + 255) / 256), dim3(256), 0, stream, E, B, p->ustart, p->keys, p->cell_ptr);
    p->cells.assign((size_t)B * B + 1, 0);
    SGD_HIP(hipMemcpyAsync(p->cells.data(), p->cell_ptr, p->cells.size() * 4, hipMemcpyDeviceToHost, stream));
    SGD_HIP(hipStreamSynchronize(stream));
    if (p->cells[0] != 0 || p->cells[(size_t)B * B] != (uint32_t)E) return FR_ERR_ARG;
    p->prefix.assign((size_t)B * B + 1, 0);
    p->max_cell = 0;
    p->chain_ratings = 0;
    uint32_t stratum_max = 0;
    for (size_t c = 0; c < (size_t)B * B; ++c) {
        if (p->cells[c + 1] < p->cells[c]) return FR_ERR_ARG;
        const uint32_t len = p->cells[c + 1] - p->cells[c];
        p->max_cell = std::max(p->max_cell, len);
        stratum_max = std::max(stratum_max, len);
        if ((c + 1) % B == 0) { p->chain_ratings += stratum_max; stratum_max = 0; }
        p->prefix[c + 1] = p->prefix[c] + ceil_fs_to_ns((unsigned __int128)len * p->d.fs_per_rating);
    }
    SgdArgs& A = p->args;
    A.keys = p->keys; A.rating = p->rating; A.cell_ptr = p->cell_ptr; A.P = p->d.P; A.Q = p->d.Q;
    A.gamma = p->d.gamma; A.gl = p->d.gamma * p->d.lambda;
    p->footprint_after = fr_alloc_used(a);
    p->footprint_peak = fr_alloc_peak(a);
    p->run = 0; p->seg = 0; p->tile = 0;
    p->inited = true;
    return FR_OK;
}

int sgd_create(void* user)
{
    static_cast<SgdTask*>(user)->registered = true;
    return FR_OK;
}

int sgd_plan(void* user, uint64_t budget_ns, uint64_t launch_cost_ns, fr_step* out)
{
    SgdTask* p = static_cast<SgdTask*>(user);
    std::memset(out, 0, sizeof(*out));
    out->run = p->run; out->segment = p->seg; out->tile0 = p->tile; out->tile1 = p->tile;
    if (!p->inited) return FR_ERR_STATE;
    if (p->d.max_runs > 0 && p->run >= (uint32_t)p->d.max_runs) { out->finished = 1; return FR_OK; }
    const uint64_t floor_ns = p->d.min_step_ns;
    if (floor_ns > budget_ns || launch_cost_ns > budget_ns - floor_ns) return FR_OK;     // even the shortest step is too long
    const uint64_t* pre = p->prefix.data() + (size_t)(p->seg % p->B) * p->B;             // this stratum's cells
    uint32_t n = 0;
    int rc = fr_chunk_fit(pre, p->B, p->tile, budget_ns, launch_cost_ns, &n);
    if (rc != FR_OK) return rc;
    if (n == 0) return FR_OK;
    const uint32_t c0 = (p->seg % p->B) * p->B;
    uint64_t cost = std::max(pre[p->tile + n] - pre[p->tile], floor_ns);
    if (p->d.fs_per_chain_rating) {
        uint32_t longest = 0;
        for (uint32_t t = p->tile; t < p->tile + n; ++t) longest = std::max(longest, p->cells[c0 + t + 1] - p->cells[c0 + t]);
        cost = std::max(cost, ceil_fs_to_ns((unsigned __int128)longest * p->d.fs_per_chain_rating));
        if (cost > budget_ns || launch_cost_ns > budget_ns - cost) return FR_OK;     // the chain does not fit
    }
    out->tile1 = p->tile + n;
    out->modelled_ns = cost;
    out->work_units = p->cells[c0 + out->tile1] - p->cells[c0 + p->tile];
    out->completes_run = (p->seg + 1 == p->n_segments() && out->tile1 == p->B) ? 1 : 0;
    return FR_OK;
}

int sgd_run(void* user, void* stream, const fr_step* st)
{
    SgdTask* p = static_cast<SgdTask*>(user);
    if (!p->inited || st->run != p->run || st->segment != p->seg || st->tile0 != p->tile) return FR_ERR_STATE;
    int rc = sgd_launch(p, p->seg, st->tile0, st->tile1, (hipStream_t)stream,
                        GateArg{static_cast<fr_gate*>(st->gate), st->gate_slot, st->gate_need_ticks});
    if (rc != FR_OK) return rc;
    p->tile = st->tile1;
    if (p->tile == p->B) {
        p->tile = 0;
        if (++p->seg == p->n_segments()) { p->seg = 0; p->run++; }
    }
    return FR_OK;
}

// (this task's steps are all or nothing - plan_step leaves gate_tile at 0 and the kernel never stops between cells,
// whose updates are made in place and must not be made twice - so tiles_done is always 0)
int sgd_rewind(void* user, const fr_step* first, uint32_t tiles_done, uint64_t* work_done)
{
    SgdTask* p = static_cast<SgdTask*>(user);
    if (!p->inited || !first || !work_done || tiles_done != 0 || first->segment >= p->n_segments() || first->tile0 >= p->B) return FR_ERR_ARG;
    p->run = first->run; p->seg = first->segment; p->tile = first->tile0;
    *work_done = 0;
    return FR_OK;
}

int sgd_stop(void* user)
{
    SgdTask* p = static_cast<SgdTask*>(user);
    p->inited = false;        // the runtime's allocator frees the device blocks
    p->registered = false;
    return FR_OK;
}

}  // namespace

extern "C" {

int fr_sgd_make(const fr_sgd_desc* d, fr_task_ops* ops_out, void** user_out, fr_task_profile* prof_out)
{
    if (!d || !ops_out || !user_out || !prof_out) return FR_ERR_ARG;
    const int64_t most = (int64_t)kIdMask - kMaxBlocks;      // (a block's first id, rounded up, still fits the key field)
    if (d->n_users < 1 || d->n_users > most || d->n_items < 1 || d->n_items > most) return FR_ERR_ARG;
    if (d->n_ratings < 0 || d->n_ratings > 0x7fffffffLL) return FR_ERR_ARG;
    if (!d->row_ptr || !d->P || !d->Q || (d->n_ratings > 0 && (!d->item || !d->rating))) return FR_ERR_ARG;
    if (d->factors != 16 && d->factors != 32 && d->factors != 64) return FR_ERR_ARG;
    if (d->blocks < 0 || d->blocks > (int32_t)kMaxBlocks) return FR_ERR_ARG;
    if (d->iterations < 1 || d->iterations > 100000 || d->max_runs < 0) return FR_ERR_ARG;
    if (!(d->gamma >= 0.0f) || !(d->lambda >= 0.0f)) return FR_ERR_ARG;
    SgdTask* p = new (std::nothrow) SgdTask();
    if (!p) return FR_ERR_ARG;
    p->d = *d;
    // blocks: as many as there are cells to run side by side, but cells of a few dozen ratings at least
    uint32_t B = (uint32_t)d->blocks;
    if (B == 0) {
        B = kMaxBlocks;
        while (B > 1 && (uint64_t)d->n_ratings / ((uint64_t)B * B) < 32) B /= 2;
    }
    B = (uint32_t)std::min<int64_t>(B, std::min(d->n_users, d->n_items));
    if ((uint64_t)p->d.iterations * B > 0xffffffffull) { delete p; return FR_ERR_ARG; }
    p->B = B;
    if (!p->d.fs_per_rating) p->d.fs_per_rating = 1000000;
    ops_out->create = sgd_create;
    ops_out->init = sgd_init;
    ops_out->plan_step = sgd_plan;
    ops_out->run_step = sgd_run;
    ops_out->stop = sgd_stop;
    ops_out->rewind = sgd_rewind;
    prof_out->mem_limit_bytes = d->mem_limit_bytes;
    prof_out->min_step_ns = d->min_step_ns ? d->min_step_ns : 1;
    *user_out = p;
    return FR_OK;
}

int fr_sgd_destroy(void* user)
{
    SgdTask* p = static_cast<SgdTask*>(user);
    if (!p) return FR_ERR_ARG;
    if (p->registered) return FR_ERR_STATE;
    if (p->inited) {
        (void)hipDeviceSynchronize();
        fr_alloc_release(&p->own);
    }
    delete p;
    return FR_OK;
}

int fr_sgd_info(void* user, fr_sgd_info_t* out)
{
    SgdTask* p = static_cast<SgdTask*>(user);
    if (!p || !out) return FR_ERR_ARG;
    if (p->prefix.empty()) return FR_ERR_STATE;          // known once InitSideTask has run
    std::memset(out, 0, sizeof(*out));
    out->blocks = p->B;
    out->largest_cell = p->max_cell;
    out->chain_ratings = p->chain_ratings;
    out->bytes_resident = p->footprint_after;
    out->bytes_peak = p->footprint_peak;
    return FR_OK;
}

int fr_sgd_block_starts(void* user, int32_t items, uint32_t* starts_host, size_t cap, size_t* n_out)
{
    SgdTask* p = static_cast<SgdTask*>(user);
    if (!p || !n_out || (!starts_host && cap)) return FR_ERR_ARG;
    if (p->prefix.empty()) return FR_ERR_STATE;
    const std::vector<uint32_t>& v = items ? p->istart_host : p->ustart_host;
    for (size_t k = 0; k < std::min(v.size(), cap); ++k) starts_host[k] = v[k];
    *n_out = v.size();
    return FR_OK;
}

int fr_sgd_cell_sizes(void* user, uint32_t stratum, uint32_t* sizes_host, size_t cap, size_t* n_out)
{
    SgdTask* p = static_cast<SgdTask*>(user);
    if (!p || !n_out || (!sizes_host && cap)) return FR_ERR_ARG;
    if (p->prefix.empty()) return FR_ERR_STATE;
    if (stratum >= p->B) return FR_ERR_ARG;
    for (size_t a = 0; a < std::min<size_t>(p->B, cap); ++a)
        sizes_host[a] = p->cells[(size_t)stratum * p->B + a + 1] - p->cells[(size_t)stratum * p->B + a];
    *n_out = p->B;
    return FR_OK;
}

int fr_sgd_run_standalone(void* user, int32_t device_id, void* stream_v, uint32_t max_cells, uint64_t* ns_out)
{
    SgdTask* p = static_cast<SgdTask*>(user);
    if (!p || device_id < 0) return FR_ERR_ARG;
    if (p->registered) return FR_ERR_STATE;
    hipStream_t stream = (hipStream_t)stream_v;
    FR_HIP_TRY(hipSetDevice(device_id), p->hip_error);
    if (!p->inited) {
        fr_alloc_reset(&p->own, p->d.mem_limit_bytes, false, device_id);
        int rc = sgd_init(p, &p->own, stream_v);
        if (rc != FR_OK) {
            const bool oom = p->own.oom;
            fr_alloc_release(&p->own);
            p->inited = false;
            return oom ? FR_ERR_OOM : rc;
        }
    }
    hipEvent_t ev[2] = {nullptr, nullptr};
    if (ns_out) {
        FR_HIP_TRY(hipEventCreate(&ev[0]), p->hip_error);
        FR_HIP_TRY(hipEventCreate(&ev[1]), p->hip_error);
        (void)hipEventRecord(ev[0], stream);
    }
    int rc = FR_OK;
    const uint32_t step = max_cells ? max_cells : p->B;
    for (uint32_t g = 0; g < p->n_segments() && rc == FR_OK; ++g)
        for (uint32_t t0 = 0; t0 < p->B && rc == FR_OK; t0 += step) rc = sgd_launch(p, g, t0, std::min(p->B, t0 + step), stream);
    if (ns_out) (void)hipEventRecord(ev[1], stream);
    hipError_t e = hipStreamSynchronize(stream);
    if (ns_out) {
        float ms = 0.f;
        *ns_out = hipEventElapsedTime(&ms, ev[0], ev[1]) == hipSuccess ? (uint64_t)((double)ms * 1.0e6 + 0.5) : 0;
        (void)hipEventDestroy(ev[0]);
        (void)hipEventDestroy(ev[1]);
    }
    if (rc != FR_OK) return rc;
    if (e != hipSuccess) { p->hip_error = (int)e; return FR_ERR_HIP; }
    return FR_OK;
}

}  // extern "C"
