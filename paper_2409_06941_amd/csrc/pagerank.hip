// The PageRank side task: pull-based power iteration, fp32 ranks, for gfx950.
//
// The paper's graph-analytics side task (Section 6.1.4) with one iteration = one pass over the graph
// (Section 6.2), written as a step-wise task for the iterative interface (Section 4.2): work is cut into tiles
// that are fixed at init, a step is a run of consecutive tiles of one segment, and every tile computes the same
// bits whichever launch carries it, so pausing and resuming at any tile boundary cannot change the result.
//
// The pull pass runs on the partition-centric layout of pr_layout.h.  One run = segments
//     V0, S_0 G_0 H_0, S_1 G_1 H_1, ..., S_{K-1} G_{K-1} H_{K-1}
//   V0   vertex pass (tile = destination partition): r_0 = 1/V, contrib_0 = r_0 / outdeg, dangling partials
//   S_k  scatter     (tile = source partition): contrib_k slice in LDS -> one message per (partition, source)
//   G_k  gather      (tile = destination partition): id stream + messages -> 64-bit fixed-point sums in LDS;
//                    then, fused, the next vertex pass for the partition's rows:
//                    r_{k+1} = base_k + d * sum, contrib_{k+1} = r_{k+1} / outdeg, dangling partials
//                    (hub partitions only store their virtual rows' sums)
//   H_k  hub finish  (tile = 256 hubs): add a hub's virtual rows, same vertex-pass arithmetic
// base_k = (1 - d)/V + d * D_k / V, D_k = fixed-order sum of the dangling partials of r_k.
// In the last iteration G and H write r_K to ranks_out instead of contrib.
// No floating-point atomics anywhere: float sums have a fixed order, the LDS atomics add integers.

#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>

#include "pr_layout.h"

namespace {

constexpr int kBlock = 512;                     // threads per workgroup of the sweeps (8 wavefronts)
constexpr int kWaves = kBlock / 64;
constexpr float kFixScale = 4611686018427387904.0f;        // 2^62: contrib sums are <= 1, so they fit u64
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

// D = sum of dpart[0 .. n): strided over the first 256 threads, then a fixed tree, so every kernel that calls
// this gets the same bits whatever its workgroup size (>= 256).  All threads call; all get the result.
__device__ __forceinline__ float dangling_total(const float* __restrict__ dpart, uint32_t n, float* lds /* >= 8 */)
{
    float s = 0.0f;
    if (threadIdx.x < 256)
        for (uint32_t i = threadIdx.x; i < n; i += 256) s += dpart[i];
    s = wave_sum(s);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    __syncthreads();
    if (lane == 0 && w < 4) lds[w] = s;
    __syncthreads();
    return (lds[0] + lds[1]) + (lds[2] + lds[3]);
}

__device__ __forceinline__ bool is_hub_tag(float tag) { return (__float_as_uint(tag) >> 31) != 0; }
__device__ __forceinline__ float inv_of_tag(float tag) { return __uint_as_float(__float_as_uint(tag) & 0x7fffffffu); }

struct DevArgs {
    int64_t V, E;
    uint32_t M, q_reg, q_hub, P, n_hubs, n_dpart;
    float damping;
    const uint16_t* ids16;
    const uint16_t* src16;
    const uint32_t* eoff;
    const uint32_t* mbase;
    const uint2* bins;
    const int32_t* hub_row;
    const uint32_t* hub_vbase;
    const float* inv_tag;
    float* msg;
    float* contrib;
    float* dpart;                 // [2][n_dpart]
    unsigned long long* vacc;     // [q_hub * kVrowsPerHubPart]
    float* ranks_out;
};

// ---- V0 ----
__global__ __launch_bounds__(kBlock) void k_vertex0(DevArgs A, uint32_t tile0, int final_pass)
{
    __shared__ float red[8];
    const uint32_t q = tile0 + blockIdx.x;
    const int64_t v0 = (int64_t)q * kRowsPerPart;
    const float r0 = 1.0f / (float)A.V;
    float dangling = 0.0f;
    for (uint32_t i = threadIdx.x; i < kRowsPerPart; i += kBlock) {
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
            for (uint32_t i = A.q_reg + threadIdx.x; i < A.n_dpart; i += kBlock) A.dpart[i] = 0.0f;   // hub slots
    }
}

// ---- S_k ----
__global__ __launch_bounds__(kBlock) void k_scatter(DevArgs A, uint32_t tile0)
{
    __shared__ __align__(16) float slice[kSrcPerPart];
    __shared__ uint32_t next_bin;
    const uint32_t p = tile0 + blockIdx.x;
    const int64_t v0 = (int64_t)p * kSrcPerPart;
    const uint32_t n = (uint32_t)((A.V - v0) < (int64_t)kSrcPerPart ? (A.V - v0) : (int64_t)kSrcPerPart);
    for (uint32_t i = threadIdx.x * 4; i < n; i += kBlock * 4) {
        if (i + 3 < n) *reinterpret_cast<float4*>(&slice[i]) = *reinterpret_cast<const float4*>(A.contrib + v0 + i);
        else
            for (uint32_t c = i; c < n; ++c) slice[c] = A.contrib[v0 + c];
    }
    if (threadIdx.x == 0) next_bin = kWaves;
    __syncthreads();
    const uint32_t Q = A.q_reg + A.q_hub;
    const int lane = threadIdx.x & 63;
    uint32_t q = threadIdx.x >> 6;                  // every wavefront starts on its own bin, then takes the next free one
    while (q < Q) {
        const uint2 b = A.bins[(uint64_t)p * Q + q];
        const uint32_t end = b.y < A.M ? b.y : A.M;
        for (uint32_t m = b.x + lane; m < end; m += 64) {
            const uint32_t s = A.src16[m];
            A.msg[m] = s < n ? slice[s] : 0.0f;
        }
        uint32_t nq = 0;
        if (lane == 0) nq = atomicAdd(&next_bin, 1u);
        q = __shfl(nq, 0, 64);
    }
}

// ---- G_k ----
__device__ __forceinline__ uint32_t wave_exclusive_scan(uint32_t x, int lane)
{
    uint32_t incl = x;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t y = __shfl_up(incl, off, 64);
        if (lane >= off) incl += y;
    }
    return incl - x;
}

__global__ __launch_bounds__(kBlock) void k_gather(DevArgs A, uint32_t tile0, int parity, int final_pass)
{
    __shared__ unsigned long long acc[kRowsPerPart];
    __shared__ float red[8];
    const uint32_t q = tile0 + blockIdx.x;
    const bool hub_part = q >= A.q_reg;
    uint32_t nrows;
    if (!hub_part) {
        const int64_t left = A.V - (int64_t)q * kRowsPerPart;
        nrows = (uint32_t)(left < (int64_t)kRowsPerPart ? left : (int64_t)kRowsPerPart);
    } else nrows = kVrowsPerHubPart;
    for (uint32_t i = threadIdx.x; i < nrows; i += kBlock) acc[i] = 0ull;
    __syncthreads();

    const uint32_t e0 = A.eoff[q], e1 = A.eoff[q + 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (e1 > e0) {
        const uint32_t c0 = e0 / kIdChunk, c1 = (e1 - 1) / kIdChunk;
        for (uint32_t c = c0 + wave; c <= c1; c += kWaves) {
            const uint4 raw = reinterpret_cast<const uint4*>(A.ids16)[(uint64_t)c * (kIdChunk / 8) + lane];
            const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
            uint32_t id[8];
#pragma unroll
            for (int j = 0; j < 4; ++j) { id[2 * j] = w[j] & 0xffffu; id[2 * j + 1] = w[j] >> 16; }
            uint32_t nf = 0;
#pragma unroll
            for (int j = 0; j < 8; ++j) nf += id[j] >> 15;
            uint32_t ord = A.mbase[c] + wave_exclusive_scan(nf, lane);     // messages begun before this lane's ids
            const uint32_t ebase = c * kIdChunk + lane * 8;
            float val = 0.0f;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t f = id[j] >> 15;
                ord += f;
                if (f | (j == 0)) {
                    const uint32_t mi = ord - 1;
                    val = mi < A.M ? A.msg[mi] : 0.0f;
                }
                const uint32_t e = ebase + j;
                const uint32_t loc = id[j] & 0x3fffu;
                if (e >= e0 && e < e1 && loc < nrows)
                    atomicAdd(&acc[loc], (unsigned long long)(val * kFixScale));
            }
        }
    }
    __syncthreads();

    if (hub_part) {
        const uint32_t vb = (q - A.q_reg) * kVrowsPerHubPart;
        for (uint32_t i = threadIdx.x; i < nrows; i += kBlock) A.vacc[vb + i] = acc[i];
        return;
    }
    const float D = dangling_total(A.dpart + (size_t)parity * A.n_dpart, A.n_dpart, red);
    const float base = (1.0f - A.damping) / (float)A.V + A.damping * D / (float)A.V;
    const int64_t v0 = (int64_t)q * kRowsPerPart;
    float dangling = 0.0f;
    for (uint32_t i = threadIdx.x; i < nrows; i += kBlock) {
        const float tag = A.inv_tag[v0 + i];
        if (is_hub_tag(tag)) continue;                 // finished by H_k
        const float s = (float)acc[i] * kFixInv;
        const float r = fmaf(A.damping, s, base);
        if (final_pass) A.ranks_out[v0 + i] = r;
        else {
            A.contrib[v0 + i] = r * tag;
            dangling += (tag == 0.0f ? r : 0.0f);
        }
    }
    if (!final_pass) {
        const float total = block_sum(dangling, red);
        if (threadIdx.x == 0) A.dpart[(size_t)(parity ^ 1) * A.n_dpart + q] = total;
    }
}

// ---- H_k ----
__global__ __launch_bounds__(kHubsPerTile) void k_hubfin(DevArgs A, uint32_t tile0, int parity, int final_pass)
{
    __shared__ float red[8];
    const uint32_t t = tile0 + blockIdx.x;
    const float D = dangling_total(A.dpart + (size_t)parity * A.n_dpart, A.n_dpart, red);
    const float base = (1.0f - A.damping) / (float)A.V + A.damping * D / (float)A.V;
    const uint32_t h = t * kHubsPerTile + threadIdx.x;
    float dangling = 0.0f;
    if (h < A.n_hubs) {
        unsigned long long s = 0ull;
        const uint32_t a = A.hub_vbase[h], b = A.hub_vbase[h + 1];
        for (uint32_t i = a; i < b && i < A.q_hub * kVrowsPerHubPart; ++i) s += A.vacc[i];
        const int32_t v = A.hub_row[h];
        const float inv = inv_of_tag(A.inv_tag[v]);
        const float r = fmaf(A.damping, (float)s * kFixInv, base);
        if (final_pass) A.ranks_out[v] = r;
        else {
            A.contrib[v] = r * inv;
            dangling = (inv == 0.0f ? r : 0.0f);
        }
    }
    if (!final_pass) {
        const float total = block_sum(dangling, red);
        if (threadIdx.x == 0) A.dpart[(size_t)(parity ^ 1) * A.n_dpart + A.q_reg + t] = total;
    }
}

uint32_t ceil_div_u64(uint64_t a, uint64_t b) { return (uint32_t)((a + b - 1) / b); }

uint64_t ceil_ps_to_ns(unsigned __int128 ps)
{
    const uint64_t ns = (uint64_t)((ps + 999) / 1000);
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

    uint32_t n_segments() const { return 1u + 3u * (uint32_t)d.iterations; }
    int kind_of(uint32_t g) const { return g == 0 ? FR_PR_SEG_VERTEX : 1 + (int)((g - 1) % 3u); }
    uint32_t tiles_of(int kind) const
    {
        switch (kind) {
        case FR_PR_SEG_VERTEX: return L.q_reg;
        case FR_PR_SEG_SCATTER: return L.P;
        case FR_PR_SEG_GATHER: return L.Q();
        default: return L.n_hub_tiles;
        }
    }
    uint64_t rows_of_q(uint32_t q) const
    {
        if (q >= L.q_reg) return kVrowsPerHubPart;
        return std::min<uint64_t>(kRowsPerPart, (uint64_t)L.V - (uint64_t)q * kRowsPerPart);
    }
};

void build_cost_tables(PrTask* p)
{
    const PrLayout& L = p->L;
    const uint64_t pe = p->d.ps_per_edge, pm = p->d.ps_per_message, pv = p->d.ps_per_vertex;
    auto& v = p->prefix[FR_PR_SEG_VERTEX];
    v.assign(L.q_reg + 1, 0);
    for (uint32_t q = 0; q < L.q_reg; ++q) v[q + 1] = v[q] + ceil_ps_to_ns((unsigned __int128)p->rows_of_q(q) * pv);
    auto& s = p->prefix[FR_PR_SEG_SCATTER];
    s.assign(L.P + 1, 0);
    for (uint32_t i = 0; i < L.P; ++i) {
        const uint64_t srcs = std::min<uint64_t>(kSrcPerPart, (uint64_t)L.V - (uint64_t)i * kSrcPerPart);
        s[i + 1] = s[i] + ceil_ps_to_ns((unsigned __int128)L.msgs_of_p[i] * pm + (unsigned __int128)srcs * pv);
    }
    auto& g = p->prefix[FR_PR_SEG_GATHER];
    g.assign(L.Q() + 1, 0);
    for (uint32_t q = 0; q < L.Q(); ++q)
        g[q + 1] = g[q] + ceil_ps_to_ns((unsigned __int128)L.edges_of_q[q] * pe + (unsigned __int128)p->rows_of_q(q) * pv);
    auto& h = p->prefix[FR_PR_SEG_HUBFIN];
    h.assign(L.n_hub_tiles + 1, 0);
    for (uint32_t t = 0; t < L.n_hub_tiles; ++t) h[t + 1] = h[t] + std::max<uint64_t>(1, p->d.hubfin_tile_ns);
}

int pr_launch(PrTask* p, uint32_t g, uint32_t tile0, uint32_t tile1, hipStream_t stream)
{
    const int kind = p->kind_of(g);
    if (tile1 <= tile0 || tile1 > p->tiles_of(kind)) return FR_ERR_ARG;
    const uint32_t n = tile1 - tile0;
    const uint32_t K = (uint32_t)p->d.iterations;
    if (kind == FR_PR_SEG_VERTEX) {
        hipLaunchKernelGGL(k_vertex0, dim3(n), dim3(kBlock), 0, stream, p->args, tile0, K == 0 ? 1 : 0);
    } else {
        const uint32_t k = (g - 1) / 3;
        const int parity = (int)(k & 1u), final_pass = (k + 1 == K) ? 1 : 0;
        if (kind == FR_PR_SEG_SCATTER) hipLaunchKernelGGL(k_scatter, dim3(n), dim3(kBlock), 0, stream, p->args, tile0);
        else if (kind == FR_PR_SEG_GATHER) hipLaunchKernelGGL(k_gather, dim3(n), dim3(kBlock), 0, stream, p->args, tile0, parity, final_pass);
        else hipLaunchKernelGGL(k_hubfin, dim3(n), dim3(kHubsPerTile), 0, stream, p->args, tile0, parity, final_pass);
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

int pr_init(void* user, fr_alloc* a, void* stream_v)
{
    PrTask* p = static_cast<PrTask*>(user);
    hipStream_t stream = (hipStream_t)stream_v;
    if (a->host_only) return FR_ERR_ARG;      // this task needs a GPU
    const int64_t V = p->d.n_vertices, E = p->d.n_edges;
    // caller-provided buffers count against the task's limit: row_ptr, col, out_degree, ranks_out
    const uint64_t caller = 4ull * (uint64_t)(V + 1) + 4ull * (uint64_t)E + 4ull * (uint64_t)V + 4ull * (uint64_t)V;
    if (fr_alloc_charge(a, caller) != FR_OK) return FR_ERR_OOM;
    int rc = pr_build_layout(&p->L, V, E, p->d.row_ptr, p->d.col, p->d.out_degree, a, stream, &p->hip_error);
    if (rc != FR_OK) return rc;
    PrLayout& L = p->L;
    p->n_dpart = L.q_reg + L.n_hub_tiles;
    if (!take(a, &p->msg, L.M) || !take(a, &p->contrib, (uint64_t)V) || !take(a, &p->dpart, 2ull * p->n_dpart) ||
        !take(a, &p->vacc, (uint64_t)std::max<uint32_t>(L.q_hub, 1) * kVrowsPerHubPart))
        return a->hip_error ? FR_ERR_HIP : FR_ERR_OOM;
    DevArgs& A = p->args;
    A.V = V; A.E = E; A.M = (uint32_t)L.M; A.q_reg = L.q_reg; A.q_hub = L.q_hub; A.P = L.P; A.n_hubs = L.n_hubs;
    A.n_dpart = p->n_dpart; A.damping = p->d.damping;
    A.ids16 = L.ids16; A.src16 = L.src16; A.eoff = L.eoff; A.mbase = L.mbase; A.bins = L.bins;
    A.hub_row = L.hub_row; A.hub_vbase = L.hub_vbase; A.inv_tag = L.inv_tag;
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
    if (p->d.max_runs > 0 && p->run >= (uint32_t)p->d.max_runs) { out->finished = 1; return FR_OK; }
    const int kind = p->kind_of(p->seg);
    const std::vector<uint64_t>& pre = p->prefix[kind];
    uint32_t n = 0;
    int rc = fr_chunk_fit(pre.data(), p->tiles_of(kind), p->tile, budget_ns, launch_cost_ns, &n);
    if (rc != FR_OK) return rc;
    if (n == 0) return FR_OK;
    out->tile1 = p->tile + n;
    out->modelled_ns = pre[p->tile + n] - pre[p->tile];
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
    int rc = pr_launch(p, p->seg, st->tile0, st->tile1, (hipStream_t)stream);
    if (rc != FR_OK) return rc;
    p->tile = st->tile1;
    if (p->tile == p->tiles_of(p->kind_of(p->seg))) {
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
    if (!p->d.ps_per_edge) p->d.ps_per_edge = 2;
    if (!p->d.ps_per_message) p->d.ps_per_message = 2;
    if (!p->d.ps_per_vertex) p->d.ps_per_vertex = 4;
    if (!p->d.hubfin_tile_ns) p->d.hubfin_tile_ns = 2000;
    ops_out->create = pr_create;
    ops_out->init = pr_init;
    ops_out->plan_step = pr_plan;
    ops_out->run_step = pr_run;
    ops_out->stop = pr_stop;
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
    out->regular_partitions = p->L.q_reg;
    out->hub_partitions = p->L.q_hub;
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
