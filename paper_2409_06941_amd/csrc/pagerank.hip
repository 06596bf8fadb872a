// The PageRank side task: pull-based power iteration over an in-edge CSR, fp32, for gfx950.
//
// The paper's graph-analytics side task (Section 6.1.4) with one iteration = one pass over the graph
// (Section 6.2), written as a step-wise task for the iterative interface (Section 4.2): work is cut into tiles
// that are fixed at init, a step is a run of consecutive tiles of one segment, and every tile computes the same
// bits whichever launch carries it, so pausing and resuming at any tile boundary cannot change the result.
//
// One run = segments V_0 P_0 E_0 V_1 P_1 E_1 ... V_K :
//   V_k  vertex pass   r_k = 1/V (k = 0) or base_{k-1} + d * acc_{k-1};  contrib_k = r_k * (1/outdeg) (0 if
//                      dangling);  dpart[tile] = sum of dangling r_k in the tile;  V_K writes r_K to ranks_out
//   P_k  pull pass     acc_k[v] = sum over row v of contrib_k[col[j]]  -- the SpMV, almost all of the bytes
//   E_k  epilogue      rows cut by pull-tile borders are summed from per-tile head/tail partials;
//                      base_k = (1 - d)/V + d * (sum of dpart) / V
// No floating-point atomics anywhere: every sum has a fixed order.

#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>

#include "common.h"

namespace {

constexpr int kPullTile = 4096;      // edges per pull tile (one workgroup)
constexpr int kVertexTile = 4096;    // vertices per vertex tile (one workgroup)
constexpr int kBlock = 256;          // threads per workgroup (4 wavefronts)
constexpr int kFixPerTile = kBlock;  // pull tiles whose cut rows one epilogue tile repairs
constexpr int kLongRow = 32;         // in-tile row pieces longer than this are summed by a whole wavefront
constexpr int kMaxLong = kPullTile / (kLongRow + 1) + 2;

// ---- fixed-order reductions ----
__device__ __forceinline__ float wave_sum(float x)
{
    // xor butterfly over the 64 lanes; the same pairing every time
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, 64);
    return x;
}

__device__ __forceinline__ float block_sum(float x, float* lds4)
{
    x = wave_sum(x);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    if (lane == 0) lds4[w] = x;
    __syncthreads();
    return (lds4[0] + lds4[1]) + (lds4[2] + lds4[3]);
}

// ---- init kernels ----
__global__ __launch_bounds__(kBlock) void k_init_vertices(int64_t V, const int32_t* __restrict__ outdeg,
                                                          float* __restrict__ inv_outdeg, float* __restrict__ acc)
{
    const int64_t v = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= V) return;
    const int32_t d = outdeg[v];
    inv_outdeg[v] = d > 0 ? 1.0f / (float)d : 0.0f;
    acc[v] = 0.0f;     // rows without in-edges are never written by the pull pass
}

// Row that holds edge e: the v with row_ptr[v] <= e < row_ptr[v + 1].
__device__ __forceinline__ int32_t row_of_edge(const int32_t* __restrict__ row_ptr, int64_t V, int64_t e)
{
    int64_t lo = 0, hi = V;            // first index in [0, V] whose row_ptr exceeds e
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if ((int64_t)row_ptr[mid] > e) hi = mid;
        else lo = mid + 1;
    }
    return (int32_t)(lo - 1);
}

__global__ __launch_bounds__(kBlock) void k_tile_rows(uint32_t n_pull, int64_t E, int64_t V,
                                                      const int32_t* __restrict__ row_ptr,
                                                      int32_t* __restrict__ first_row, int32_t* __restrict__ last_row)
{
    const uint32_t t = blockIdx.x * kBlock + threadIdx.x;
    if (t >= n_pull) return;
    const int64_t e0 = (int64_t)t * kPullTile;
    if (e0 >= E) { first_row[t] = 0; last_row[t] = -1; return; }
    const int64_t e1 = e0 + kPullTile < E ? e0 + kPullTile : E;
    first_row[t] = row_of_edge(row_ptr, V, e0);
    last_row[t] = row_of_edge(row_ptr, V, e1 - 1);
}

__global__ void k_set_i32(int32_t* p, int32_t value) { *p = value; }

// Structure check of the caller's CSR so that no later kernel can index out of bounds.
__global__ __launch_bounds__(kBlock) void k_validate(int64_t V, int64_t E, const int32_t* __restrict__ row_ptr,
                                                     const int32_t* __restrict__ col, int32_t* __restrict__ bad)
{
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    int err = 0;
    if (i == 0 && (row_ptr[0] != 0 || (int64_t)row_ptr[V] != E)) err = 1;
    for (int64_t v = i; v < V; v += stride) {
        const int32_t a = row_ptr[v], b = row_ptr[v + 1];
        if (a > b || a < 0 || (int64_t)b > E) err = 1;
    }
    for (int64_t e = i; e < E; e += stride) {
        const int32_t c = col[e];
        if (c < 0 || (int64_t)c >= V) err = 1;
    }
    if (err) *bad = 1;
}

// ---- V_k: vertex pass ----
// mode 0: first iteration (r = 1/V); mode 1: r = base + d * acc; mode 2: like 1 but writes ranks_out (final pass;
// with K = 0 the host passes mode 3 = first and final at once).
__global__ __launch_bounds__(kBlock) void k_vertex(int mode, uint32_t tile0, int64_t V, float damping,
                                                   const float* __restrict__ base, const float* __restrict__ acc,
                                                   const float* __restrict__ inv_outdeg, float* __restrict__ contrib,
                                                   float* __restrict__ dpart, float* __restrict__ ranks_out)
{
    __shared__ float red[4];
    const uint32_t t = tile0 + blockIdx.x;
    const int64_t v0 = (int64_t)t * kVertexTile;
    const bool first = (mode == 0 || mode == 3), final_pass = (mode >= 2);
    const float b = first ? 0.0f : base[0];
    const float r0 = 1.0f / (float)V;
    float dangling = 0.0f;
#pragma unroll
    for (int j = 0; j < kVertexTile / (4 * kBlock); ++j) {
        const int64_t v = v0 + 4 * ((int64_t)threadIdx.x + (int64_t)kBlock * j);
        if (v + 3 < V) {
            const float4 inv = *reinterpret_cast<const float4*>(inv_outdeg + v);
            float4 r;
            if (first) r = make_float4(r0, r0, r0, r0);
            else {
                const float4 a = *reinterpret_cast<const float4*>(acc + v);
                r = make_float4(fmaf(damping, a.x, b), fmaf(damping, a.y, b), fmaf(damping, a.z, b), fmaf(damping, a.w, b));
            }
            if (final_pass) *reinterpret_cast<float4*>(ranks_out + v) = r;
            else {
                *reinterpret_cast<float4*>(contrib + v) = make_float4(r.x * inv.x, r.y * inv.y, r.z * inv.z, r.w * inv.w);
                dangling += (inv.x == 0.0f ? r.x : 0.0f);
                dangling += (inv.y == 0.0f ? r.y : 0.0f);
                dangling += (inv.z == 0.0f ? r.z : 0.0f);
                dangling += (inv.w == 0.0f ? r.w : 0.0f);
            }
        } else {
            for (int c = 0; c < 4; ++c) {
                if (v + c >= V) break;
                const float inv = inv_outdeg[v + c];
                const float r = first ? r0 : fmaf(damping, acc[v + c], b);
                if (final_pass) ranks_out[v + c] = r;
                else {
                    contrib[v + c] = r * inv;
                    dangling += (inv == 0.0f ? r : 0.0f);
                }
            }
        }
    }
    if (!final_pass) {
        const float total = block_sum(dangling, red);
        if (threadIdx.x == 0) dpart[t] = total;
    }
}

// ---- P_k: pull pass (SpMV) ----
// One workgroup per tile of kPullTile consecutive CSR entries.  The tile's col slab is streamed with 16-byte
// loads, contrib is gathered, and the products are staged in LDS; then every row piece inside the slab is summed
// in CSR order: short pieces by one lane, long pieces by a wavefront (lane-strided, then a fixed butterfly).
// A row lying wholly inside the slab gets its acc written here; a row that began in an earlier slab leaves its
// piece in head[t], one that runs past the slab's end leaves it in tail[t]; E_k adds those up.
__device__ __forceinline__ void store_piece(int64_t lo, int64_t hi, int64_t e0, int64_t e1, int32_t v, uint32_t t,
                                            float s, float* __restrict__ acc, float* __restrict__ head,
                                            float* __restrict__ tail)
{
    if (lo >= e0 && hi <= e1) acc[v] = s;
    else if (lo < e0) head[t] = s;
    else tail[t] = s;
}

__global__ __launch_bounds__(kBlock) void k_pull(uint32_t tile0, int64_t E, const int32_t* __restrict__ row_ptr,
                                                 const int32_t* __restrict__ col, const float* __restrict__ contrib,
                                                 const int32_t* __restrict__ first_row,
                                                 const int32_t* __restrict__ last_row, float* __restrict__ acc,
                                                 float* __restrict__ head, float* __restrict__ tail)
{
    __shared__ __align__(16) float vals[kPullTile];
    __shared__ int32_t long_rows[kMaxLong];
    __shared__ int32_t long_count;

    const uint32_t t = tile0 + blockIdx.x;
    const int64_t e0 = (int64_t)t * kPullTile;
    if (e0 >= E) return;
    const int64_t e1 = e0 + kPullTile < E ? e0 + kPullTile : E;
    const int ne = (int)(e1 - e0);

    if (threadIdx.x == 0) long_count = 0;
    if (ne == kPullTile) {
        const int4* c4 = reinterpret_cast<const int4*>(col + e0);
        int4 c[kPullTile / (4 * kBlock)];
#pragma unroll
        for (int j = 0; j < kPullTile / (4 * kBlock); ++j) c[j] = c4[threadIdx.x + kBlock * j];
#pragma unroll
        for (int j = 0; j < kPullTile / (4 * kBlock); ++j) {
            float4 g;
            g.x = contrib[c[j].x]; g.y = contrib[c[j].y]; g.z = contrib[c[j].z]; g.w = contrib[c[j].w];
            reinterpret_cast<float4*>(vals)[threadIdx.x + kBlock * j] = g;
        }
    } else {
        for (int i = threadIdx.x; i < ne; i += kBlock) vals[i] = contrib[col[e0 + i]];
    }
    __syncthreads();

    const int32_t rf = first_row[t], rl = last_row[t];
    for (int32_t v = rf + (int32_t)threadIdx.x; v <= rl; v += kBlock) {
        const int64_t lo = row_ptr[v], hi = row_ptr[v + 1];
        const int a = (int)((lo > e0 ? lo : e0) - e0), b = (int)((hi < e1 ? hi : e1) - e0);
        if (b <= a) continue;
        if (b - a > kLongRow) {
            const int k = atomicAdd(&long_count, 1);      // list order does not matter: rows are independent
            long_rows[k] = v;
            continue;
        }
        float s = 0.0f;
        for (int i = a; i < b; ++i) s += vals[i];
        store_piece(lo, hi, e0, e1, v, t, s, acc, head, tail);
    }
    __syncthreads();

    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int nlong = long_count;
    for (int k = w; k < nlong; k += kBlock / 64) {
        const int32_t v = long_rows[k];
        const int64_t lo = row_ptr[v], hi = row_ptr[v + 1];
        const int a = (int)((lo > e0 ? lo : e0) - e0), b = (int)((hi < e1 ? hi : e1) - e0);
        float s = 0.0f;
        for (int i = a + lane; i < b; i += 64) s += vals[i];
        s = wave_sum(s);
        if (lane == 0) store_piece(lo, hi, e0, e1, v, t, s, acc, head, tail);
    }
}

// ---- E_k: epilogue ----
// Tiles 0 .. n_fix-1: lane p repairs the row that starts in pull tile p and runs past its end:
//   acc[v] = tail[p] + head[p + 1] + head[p + 2] + ...  (every later tile the row reaches, in order).
// Tile n_fix: base = (1 - d)/V + d * D / V with D the fixed-order sum of the vertex tiles' dangling partials.
__global__ __launch_bounds__(kBlock) void k_epilogue(uint32_t tile0, uint32_t n_fix, uint32_t n_pull, int64_t E,
                                                     int64_t V, float damping, const int32_t* __restrict__ row_ptr,
                                                     const int32_t* __restrict__ last_row,
                                                     const float* __restrict__ head, const float* __restrict__ tail,
                                                     float* __restrict__ acc, const float* __restrict__ dpart,
                                                     uint32_t n_vertex_tiles, float* __restrict__ base)
{
    __shared__ float red[4];
    const uint32_t t = tile0 + blockIdx.x;
    if (t < n_fix) {
        const uint32_t p = t * kFixPerTile + threadIdx.x;
        if (p >= n_pull) return;
        const int64_t e0 = (int64_t)p * kPullTile;
        if (e0 >= E) return;
        const int64_t e1 = e0 + kPullTile < E ? e0 + kPullTile : E;
        const int32_t v = last_row[p];
        const int64_t lo = row_ptr[v], hi = row_ptr[v + 1];
        if (hi > e1 && lo >= e0) {
            float s = tail[p];
            for (uint32_t q = p + 1; q < n_pull && (int64_t)q * kPullTile < hi; ++q) s += head[q];
            acc[v] = s;
        }
        return;
    }
    float s = 0.0f;
    for (uint32_t i = threadIdx.x; i < n_vertex_tiles; i += kBlock) s += dpart[i];
    const float D = block_sum(s, red);
    if (threadIdx.x == 0) base[0] = (1.0f - damping) / (float)V + damping * D / (float)V;
}

uint32_t ceil_div_u64(uint64_t a, uint64_t b) { return (uint32_t)((a + b - 1) / b); }

struct PrTask {
    fr_pagerank_desc d{};
    uint32_t n_vertex = 0, n_pull = 0, n_fix = 0, n_epi = 0;
    std::vector<uint64_t> prefix[3];      // cumulative modelled tile costs per segment kind
    uint64_t footprint = 0, internal_bytes = 0;
    // device
    float *inv_outdeg = nullptr, *contrib = nullptr, *acc = nullptr, *dpart = nullptr, *head = nullptr,
          *tail = nullptr, *base = nullptr;
    int32_t *first_row = nullptr, *last_row = nullptr, *bad = nullptr;
    bool inited = false;
    bool registered = false;
    fr_alloc own;                         // used by the standalone run only
    int hip_error = 0;
    // cursor
    uint32_t run = 0, seg = 0, tile = 0;

    uint32_t n_segments() const { return 3u * (uint32_t)d.iterations + 1u; }
    int kind_of(uint32_t seg_index) const { return seg_index == 3u * (uint32_t)d.iterations ? FR_PR_SEG_VERTEX : (int)(seg_index % 3u); }
    uint32_t tiles_of(int kind) const { return kind == FR_PR_SEG_VERTEX ? n_vertex : kind == FR_PR_SEG_PULL ? n_pull : n_epi; }
};

uint64_t ceil_ps_to_ns(uint64_t units, uint64_t ps)
{
    const unsigned __int128 x = (unsigned __int128)units * ps + 999;
    const uint64_t ns = (uint64_t)(x / 1000);
    return ns ? ns : 1;
}

int pr_launch(PrTask* p, uint32_t seg_index, uint32_t tile0, uint32_t tile1, hipStream_t stream)
{
    const int kind = p->kind_of(seg_index);
    const uint32_t n = tile1 - tile0;
    if (tile1 <= tile0 || tile1 > p->tiles_of(kind)) return FR_ERR_ARG;
    const int64_t V = p->d.n_vertices, E = p->d.n_edges;
    const uint32_t K = (uint32_t)p->d.iterations;
    if (kind == FR_PR_SEG_VERTEX) {
        const uint32_t k = seg_index / 3;
        int mode = (k == 0) ? 0 : 1;
        if (k == K) mode = (K == 0) ? 3 : 2;
        hipLaunchKernelGGL(k_vertex, dim3(n), dim3(kBlock), 0, stream, mode, tile0, V, p->d.damping, p->base, p->acc,
                           p->inv_outdeg, p->contrib, p->dpart, p->d.ranks_out);
    } else if (kind == FR_PR_SEG_PULL) {
        hipLaunchKernelGGL(k_pull, dim3(n), dim3(kBlock), 0, stream, tile0, E, p->d.row_ptr, p->d.col, p->contrib,
                           p->first_row, p->last_row, p->acc, p->head, p->tail);
    } else {
        hipLaunchKernelGGL(k_epilogue, dim3(n), dim3(kBlock), 0, stream, tile0, p->n_fix, p->n_pull, E, V, p->d.damping,
                           p->d.row_ptr, p->last_row, p->head, p->tail, p->acc, p->dpart, p->n_vertex, p->base);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { p->hip_error = (int)e; return FR_ERR_HIP; }
    return FR_OK;
}

template <typename T>
bool take(fr_alloc* a, T** out, size_t count)
{
    *out = static_cast<T*>(fr_alloc_device(a, count * sizeof(T)));
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
    if (!take(a, &p->inv_outdeg, (size_t)V) || !take(a, &p->contrib, (size_t)V) || !take(a, &p->acc, (size_t)V) ||
        !take(a, &p->dpart, p->n_vertex) || !take(a, &p->head, p->n_pull) || !take(a, &p->tail, p->n_pull) ||
        !take(a, &p->base, 1) || !take(a, &p->first_row, p->n_pull) || !take(a, &p->last_row, p->n_pull) ||
        !take(a, &p->bad, 1))
        return a->hip_error ? FR_ERR_HIP : FR_ERR_OOM;

    hipLaunchKernelGGL(k_set_i32, dim3(1), dim3(1), 0, stream, p->bad, 0);
    const uint32_t vgrid = (uint32_t)std::min<int64_t>((std::max<int64_t>(V, E) + kBlock - 1) / kBlock, 65536);
    hipLaunchKernelGGL(k_validate, dim3(vgrid), dim3(kBlock), 0, stream, V, E, p->d.row_ptr, p->d.col, p->bad);
    int32_t bad = 0;
    FR_HIP_TRY(hipMemcpyAsync(&bad, p->bad, sizeof(int32_t), hipMemcpyDeviceToHost, stream), p->hip_error);
    FR_HIP_TRY(hipStreamSynchronize(stream), p->hip_error);
    if (bad) return FR_ERR_ARG;               // malformed CSR: refuse before any kernel indexes with it

    hipLaunchKernelGGL(k_init_vertices, dim3(ceil_div_u64((uint64_t)V, kBlock)), dim3(kBlock), 0, stream, V,
                       p->d.out_degree, p->inv_outdeg, p->acc);
    hipLaunchKernelGGL(k_tile_rows, dim3(ceil_div_u64(p->n_pull, kBlock)), dim3(kBlock), 0, stream, p->n_pull, E, V,
                       p->d.row_ptr, p->first_row, p->last_row);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { p->hip_error = (int)e; return FR_ERR_HIP; }
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
    if (p->d.max_runs > 0 && p->run >= (uint32_t)p->d.max_runs) { out->finished = 1; return FR_OK; }
    const int kind = p->kind_of(p->seg);
    const std::vector<uint64_t>& pre = p->prefix[kind];
    uint32_t n = 0;
    int rc = fr_chunk_fit(pre.data(), p->tiles_of(kind), p->tile, budget_ns, launch_cost_ns, &n);
    if (rc != FR_OK) return rc;
    if (n == 0) return FR_OK;
    out->tile1 = p->tile + n;
    out->modelled_ns = pre[p->tile + n] - pre[p->tile];
    if (kind == FR_PR_SEG_PULL) {
        const uint64_t a = std::min<uint64_t>((uint64_t)p->tile * kPullTile, (uint64_t)p->d.n_edges);
        const uint64_t b = std::min<uint64_t>((uint64_t)(p->tile + n) * kPullTile, (uint64_t)p->d.n_edges);
        out->work_units = b - a;
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
    if (((uintptr_t)d->col & 15) || ((uintptr_t)d->ranks_out & 15)) return FR_ERR_ARG;
    if (d->iterations < 0 || d->iterations > 100000 || d->max_runs < 0) return FR_ERR_ARG;
    if (!(d->damping >= 0.0f && d->damping <= 1.0f)) return FR_ERR_ARG;
    PrTask* p = new (std::nothrow) PrTask();
    if (!p) return FR_ERR_ARG;
    p->d = *d;
    if (!p->d.ps_per_edge) p->d.ps_per_edge = 4;          // about 1.4 TB/s of CSR entries
    if (!p->d.ps_per_vertex) p->d.ps_per_vertex = 8;
    if (!p->d.epilogue_tile_ns) p->d.epilogue_tile_ns = 2000;
    const uint64_t V = (uint64_t)d->n_vertices, E = (uint64_t)d->n_edges;
    p->n_vertex = ceil_div_u64(V, kVertexTile);
    p->n_pull = E ? ceil_div_u64(E, kPullTile) : 1;
    p->n_fix = ceil_div_u64(p->n_pull, kFixPerTile);
    p->n_epi = p->n_fix + 1;
    p->prefix[FR_PR_SEG_VERTEX].assign(p->n_vertex + 1, 0);
    for (uint32_t t = 0; t < p->n_vertex; ++t) {
        const uint64_t nv = std::min<uint64_t>(kVertexTile, V - (uint64_t)t * kVertexTile);
        p->prefix[FR_PR_SEG_VERTEX][t + 1] = p->prefix[FR_PR_SEG_VERTEX][t] + ceil_ps_to_ns(nv, p->d.ps_per_vertex);
    }
    p->prefix[FR_PR_SEG_PULL].assign(p->n_pull + 1, 0);
    for (uint32_t t = 0; t < p->n_pull; ++t) {
        const uint64_t done = (uint64_t)t * kPullTile;
        const uint64_t ne = done < E ? std::min<uint64_t>(kPullTile, E - done) : 0;
        p->prefix[FR_PR_SEG_PULL][t + 1] = p->prefix[FR_PR_SEG_PULL][t] + ceil_ps_to_ns(ne, p->d.ps_per_edge);
    }
    p->prefix[FR_PR_SEG_EPILOGUE].assign(p->n_epi + 1, 0);
    for (uint32_t t = 0; t < p->n_epi; ++t)
        p->prefix[FR_PR_SEG_EPILOGUE][t + 1] = p->prefix[FR_PR_SEG_EPILOGUE][t] + p->d.epilogue_tile_ns;
    auto r256 = [](uint64_t b) { return (b + 255) & ~255ull; };
    p->internal_bytes = 3 * r256(4 * V) + r256(4ull * p->n_vertex) + 4 * r256(4ull * p->n_pull) + 2 * r256(4);
    p->footprint = 4 * (V + 1) + 4 * E + 8 * V + p->internal_bytes;

    ops_out->create = pr_create;
    ops_out->init = pr_init;
    ops_out->plan_step = pr_plan;
    ops_out->run_step = pr_run;
    ops_out->stop = pr_stop;
    prof_out->mem_limit_bytes = d->mem_limit_bytes;
    uint64_t min_step = ~0ull;
    for (int k = 0; k < 3; ++k)
        for (size_t t = 0; t + 1 < p->prefix[k].size(); ++t) min_step = std::min(min_step, p->prefix[k][t + 1] - p->prefix[k][t]);
    prof_out->min_step_ns = min_step;
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

int fr_pagerank_footprint(void* user, uint64_t* bytes_out)
{
    if (!user || !bytes_out) return FR_ERR_ARG;
    *bytes_out = static_cast<PrTask*>(user)->footprint;
    return FR_OK;
}

int fr_pagerank_tiles(void* user, int32_t seg_kind, uint32_t* n_out)
{
    if (!user || !n_out || seg_kind < 0 || seg_kind > 2) return FR_ERR_ARG;
    *n_out = static_cast<PrTask*>(user)->tiles_of(seg_kind);
    return FR_OK;
}

int fr_pagerank_tile_costs(void* user, int32_t seg_kind, uint32_t* costs, size_t cap, size_t* n_out)
{
    if (!user || !n_out || seg_kind < 0 || seg_kind > 2 || (!costs && cap)) return FR_ERR_ARG;
    PrTask* p = static_cast<PrTask*>(user);
    const std::vector<uint64_t>& pre = p->prefix[seg_kind];
    const size_t n = pre.size() - 1;
    for (size_t t = 0; t < std::min(n, cap); ++t) costs[t] = (uint32_t)(pre[t + 1] - pre[t]);
    *n_out = n;
    return FR_OK;
}

int fr_pagerank_tile_shape(uint32_t* pull_edges, uint32_t* vertex_vertices)
{
    if (!pull_edges || !vertex_vertices) return FR_ERR_ARG;
    *pull_edges = kPullTile;
    *vertex_vertices = kVertexTile;
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
        if (rc != FR_OK) { fr_alloc_release(&p->own); p->inited = false; return p->own.oom ? FR_ERR_OOM : rc; }
    }
    hipEvent_t ev[2] = {nullptr, nullptr};
    float ms_sum[3] = {0.f, 0.f, 0.f};
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
        for (int k = 0; k < 3; ++k) phase_ns[k] = (uint64_t)((double)ms_sum[k] * 1.0e6 + 0.5);
        (void)hipEventDestroy(ev[0]);
        (void)hipEventDestroy(ev[1]);
    }
    if (rc != FR_OK) return rc;
    if (e != hipSuccess) { p->hip_error = (int)e; return FR_ERR_HIP; }
    return FR_OK;
}

}  // extern "C"
