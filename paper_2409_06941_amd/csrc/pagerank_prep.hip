// Builds the partition-centric layout (pr_layout.h) of the PageRank side task on the GPU, once, in InitSideTask
// (Section 4.1 of the paper: the transition that loads the task's context into GPU memory).
//
// Pipeline: check the CSR -> mark hubs and number their virtual rows (scan) -> one 64-bit key per edge
// (partition, source, local row) -> radix sort -> message starts (flags, scan) -> id stream, message sources,
// per-partition offsets, per-bin message ranges.  rocPRIM supplies the device-wide sort and scans; they run
// once per task and are not part of any iteration.

#include <cstring>

#include <rocprim/rocprim.hpp>

#include <algorithm>

#include "pr_layout.h"

namespace {

constexpr int kBlk = 256;

inline unsigned blocks_for(uint64_t n) { return (unsigned)((n + kBlk - 1) / kBlk); }

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

__global__ void k_set_i32(int32_t* p, int32_t value) { *p = value; }

// Structure check of the caller's CSR so that no later kernel can index out of bounds.
__global__ __launch_bounds__(kBlk) void k_validate(int64_t V, int64_t E, const int32_t* __restrict__ row_ptr,
                                                   const int32_t* __restrict__ col, int32_t* __restrict__ bad)
{
    const int64_t i = (int64_t)blockIdx.x * kBlk + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * kBlk;
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

// packed[v] = (virtual rows of v) << 32 | (1 if v is a hub)
__global__ __launch_bounds__(kBlk) void k_hub_mark(int64_t V, uint32_t split, const int32_t* __restrict__ row_ptr, uint64_t* __restrict__ packed)
{
    const int64_t v = (int64_t)blockIdx.x * kBlk + threadIdx.x;
    if (v >= V) return;
    const uint32_t indeg = (uint32_t)(row_ptr[v + 1] - row_ptr[v]);
    const bool hub = indeg > split;
    const uint64_t nsplit = hub ? ((uint64_t)indeg + split - 1) / split : 0;
    packed[v] = (nsplit << 32) | (hub ? 1u : 0u);
}

__global__ __launch_bounds__(kBlk) void k_hub_tables(int64_t V, uint32_t split, const int32_t* __restrict__ row_ptr,
                                                     const uint64_t* __restrict__ scanned, uint32_t n_hubs,
                                                     uint32_t n_vrows, int32_t* __restrict__ hub_row,
                                                     uint32_t* __restrict__ hub_vbase)
{
    const int64_t v = (int64_t)blockIdx.x * kBlk + threadIdx.x;
    if (v == 0) hub_vbase[n_hubs] = n_vrows;
    if (v >= V) return;
    const uint32_t indeg = (uint32_t)(row_ptr[v + 1] - row_ptr[v]);
    if (indeg <= split) return;
    const uint32_t h = (uint32_t)(scanned[v] & 0xffffffffu);
    if (h < n_hubs) {
        hub_row[h] = (int32_t)v;
        hub_vbase[h] = (uint32_t)(scanned[v] >> 32);
    }
}

// 1/outdeg (0 for dangling vertices) with the sign bit marking hub rows.
__global__ __launch_bounds__(kBlk) void k_inv_tag(int64_t V, uint32_t split, const int32_t* __restrict__ row_ptr,
                                                  const int32_t* __restrict__ outdeg, float* __restrict__ inv_tag)
{
    const int64_t v = (int64_t)blockIdx.x * kBlk + threadIdx.x;
    if (v >= V) return;
    const int32_t d = outdeg[v];
    float inv = d > 0 ? 1.0f / (float)d : 0.0f;
    if ((uint32_t)(row_ptr[v + 1] - row_ptr[v]) > split) inv = __uint_as_float(__float_as_uint(inv) | 0x80000000u);
    inv_tag[v] = inv;
}

// Virtual row hv of a hub goes to partition hv % Q, accumulator slot rows_per_part + hv / Q.
__global__ __launch_bounds__(kBlk) void k_keys(int64_t V, int64_t E, uint32_t split, const int32_t* __restrict__ row_ptr,
                                               const int32_t* __restrict__ col, const uint64_t* __restrict__ scanned,
                                               uint32_t Q, uint32_t rows_per_part, uint64_t* __restrict__ keys)
{
    const int64_t e = (int64_t)blockIdx.x * kBlk + threadIdx.x;
    if (e >= E) return;
    const int32_t v = row_of_edge(row_ptr, V, e);
    const int64_t begin = row_ptr[v];
    const uint32_t indeg = (uint32_t)(row_ptr[v + 1] - begin);
    uint64_t q, local;
    if (indeg > split) {
        const uint64_t hv = (scanned[v] >> 32) + (uint64_t)(e - begin) / split;
        q = hv % Q;
        local = rows_per_part + hv / Q;
    } else {
        q = (uint64_t)v / rows_per_part;
        local = (uint64_t)v % rows_per_part;
    }
    keys[e] = (q << (kKeyLocalBits + kKeySrcBits)) | ((uint64_t)(uint32_t)col[e] << kKeyLocalBits) | local;
}

// 1 where edge e (in sorted order) is the first of its (partition, source) group, i.e. starts a message.
__host__ __device__ __forceinline__ uint32_t flag_of(const uint64_t* __restrict__ keys, int64_t e)
{
    return (e == 0 || (keys[e] >> kKeyLocalBits) != (keys[e - 1] >> kKeyLocalBits)) ? 1u : 0u;
}

struct FlagOf {
    const uint64_t* keys;
    __host__ __device__ uint32_t operator()(size_t e) const { return flag_of(keys, (int64_t)e); }
};

// Id stream and message sources.  Inside every chunk of kIdChunk ids the stream is stored transposed: stream
// position r = 64 * j + lane of the chunk sits at slot 8 * lane + j, so that one 16-byte load hands a lane the
// ids 64 apart and, for a fixed j, the 64 lanes of a wavefront hold 64 consecutive ids of the stream.
__device__ __forceinline__ int64_t id_slot(int64_t e)
{
    const int64_t r = e % kIdChunk;
    return e - r + (r % 64) * (kIdChunk / 64) + r / 64;
}

__global__ __launch_bounds__(kBlk) void k_emit(int64_t E, int64_t padded, uint64_t M, const uint64_t* __restrict__ keys,
                                               const uint32_t* __restrict__ incl, uint32_t src_per_part,
                                               uint16_t* __restrict__ ids16, uint16_t* __restrict__ src16)
{
    const int64_t e = (int64_t)blockIdx.x * kBlk + threadIdx.x;
    if (e >= padded) return;
    if (e >= E) { ids16[id_slot(e)] = 0; return; }
    const uint64_t k = keys[e];
    const uint32_t f = flag_of(keys, e);
    ids16[id_slot(e)] = (uint16_t)((k & ((1u << kKeyLocalBits) - 1)) | (f << 15));
    if (f) {
        const uint64_t m = (uint64_t)incl[e] - 1;
        const uint32_t u = (uint32_t)((k >> kKeyLocalBits) & 0x7fffffffu);
        if (m < M) src16[m] = (uint16_t)(u % src_per_part);
    }
}

__global__ __launch_bounds__(kBlk) void k_mbase(int64_t E, uint32_t n_chunks, uint32_t M, const uint64_t* __restrict__ keys,
                                                const uint32_t* __restrict__ incl, uint32_t* __restrict__ mbase)
{
    const uint32_t c = blockIdx.x * kBlk + threadIdx.x;
    if (c > n_chunks) return;
    const int64_t e = (int64_t)c * kIdChunk;
    mbase[c] = e < E ? incl[e] - flag_of(keys, e) : M;
}

__device__ __forceinline__ int64_t lower_bound_key(const uint64_t* __restrict__ keys, int64_t E, uint64_t target)
{
    int64_t lo = 0, hi = E;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (keys[mid] < target) lo = mid + 1;
        else hi = mid;
    }
    return lo;
}

__global__ __launch_bounds__(kBlk) void k_eoff(uint32_t Q, int64_t E, const uint64_t* __restrict__ keys, uint32_t* __restrict__ eoff)
{
    const uint32_t q = blockIdx.x * kBlk + threadIdx.x;
    if (q > Q) return;
    eoff[q] = (uint32_t)lower_bound_key(keys, E, (uint64_t)q << (kKeyLocalBits + kKeySrcBits));
}

// bins[p * Q + q] = message range of the edges of partition q whose source lies in source partition p.
// The first edge of a bin always starts a message, so "messages before it" = incl - 1 there.
__global__ __launch_bounds__(kBlk) void k_bins(uint32_t P, uint32_t Q, int64_t E, uint32_t M, uint64_t src_per_part,
                                               const uint64_t* __restrict__ keys, const uint32_t* __restrict__ incl,
                                               uint2* __restrict__ bins)
{
    const uint64_t idx = (uint64_t)blockIdx.x * kBlk + threadIdx.x;
    if (idx >= (uint64_t)P * Q) return;
    const uint64_t p = idx / Q, q = idx % Q;
    const uint64_t base = q << (kKeyLocalBits + kKeySrcBits);
    const int64_t lo = lower_bound_key(keys, E, base + ((p * src_per_part) << kKeyLocalBits));
    const int64_t hi = lower_bound_key(keys, E, base + (((p + 1) * src_per_part) << kKeyLocalBits));
    uint2 r;
    r.x = lo < E ? incl[lo] - 1 : M;
    r.y = hi < E ? incl[hi] - 1 : M;
    if (r.y < r.x) r.y = r.x;
    bins[idx] = r;
}

// hub_of_p[p] = first hub whose row id is >= p * src_per_part (hub_row is ascending).
__global__ __launch_bounds__(kBlk) void k_hub_of_p(uint32_t P, uint32_t n_hubs, uint32_t src_per_part, const int32_t* __restrict__ hub_row,
                                                   uint32_t* __restrict__ hub_of_p)
{
    const uint32_t p = blockIdx.x * kBlk + threadIdx.x;
    if (p > P) return;
    const int64_t target = (int64_t)p * src_per_part;
    uint32_t lo = 0, hi = n_hubs;
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if ((int64_t)hub_row[mid] < target) lo = mid + 1;
        else hi = mid;
    }
    hub_of_p[p] = lo;
}

__global__ __launch_bounds__(kBlk) void k_msgs_of_p(uint32_t P, uint32_t Q, const uint2* __restrict__ bins, uint64_t* __restrict__ out)
{
    const uint32_t p = blockIdx.x * kBlk + threadIdx.x;
    if (p >= P) return;
    uint64_t s = 0;
    for (uint32_t q = 0; q < Q; ++q) s += bins[(uint64_t)p * Q + q].y - bins[(uint64_t)p * Q + q].x;
    out[p] = s;
}

struct Scratch {
    fr_alloc* a;
    std::vector<void*> held;
    template <typename T>
    T* take(uint64_t count)
    {
        void* p = fr_alloc_device(a, (size_t)(count ? count : 1) * sizeof(T));
        if (p) held.push_back(p);
        return static_cast<T*>(p);
    }
    void drop(void* p)
    {
        for (size_t i = 0; i < held.size(); ++i)
            if (held[i] == p) { (void)fr_alloc_free(a, p); held.erase(held.begin() + (long)i); return; }
    }
    ~Scratch()
    {
        for (void* p : held) (void)fr_alloc_free(a, p);
    }
};

template <typename T>
bool keep(fr_alloc* a, T** out, uint64_t count)
{
    *out = static_cast<T*>(fr_alloc_device(a, (size_t)(count ? count : 1) * sizeof(T)));
    return *out != nullptr;
}

}  // namespace

#define PREP_HIP(expr)                                             \
    do {                                                           \
        hipError_t e__ = (expr);                                   \
        if (e__ != hipSuccess) { *hip_error = (int)e__; return FR_ERR_HIP; } \
    } while (0)
#define PREP_NEED(ptr)                                             \
    do {                                                           \
        if (!(ptr)) { if (a->hip_error) *hip_error = a->hip_error; return a->hip_error ? FR_ERR_HIP : FR_ERR_OOM; } \
    } while (0)

int pr_build_layout(PrLayout* L, int64_t V, int64_t E, const int32_t* row_ptr, const int32_t* col,
                    const int32_t* out_degree, uint32_t rows_per_part, uint32_t src_per_part, fr_alloc* a,
                    hipStream_t stream, int* hip_error)
{
    if (!rows_per_part) rows_per_part = V >= kLargeRowsFrom ? kRowsLarge : kRowsSmall;
    if (!src_per_part) src_per_part = V >= kLargeSrcFrom ? kSrcLarge : kSrcSmall;
    if ((rows_per_part != kRowsSmall && rows_per_part != kRowsLarge) || (src_per_part != kSrcSmall && src_per_part != kSrcLarge))
        return FR_ERR_ARG;
    L->V = V; L->E = E;
    L->rows_per_part = rows_per_part; L->src_per_part = src_per_part;
    L->Q = (uint32_t)((V + rows_per_part - 1) / rows_per_part);
    L->P = (uint32_t)((V + src_per_part - 1) / src_per_part);
    L->n_chunks = (uint32_t)((E + kIdChunk - 1) / kIdChunk);
    const int64_t padded = (int64_t)std::max<uint32_t>(L->n_chunks, 1) * kIdChunk;
    const uint32_t Q = L->Q;
    if ((uint64_t)Q >= (1ull << (63 - kKeyLocalBits - kKeySrcBits))) return FR_ERR_ARG;

    Scratch tmp{a, {}};

    // ---- refuse a malformed CSR before anything indexes with it
    int32_t* bad = tmp.take<int32_t>(1);
    PREP_NEED(bad);
    hipLaunchKernelGGL(k_set_i32, dim3(1), dim3(1), 0, stream, bad, 0);
    const unsigned vgrid = std::min<unsigned>(blocks_for((uint64_t)std::max<int64_t>(V, E)), 65536u);
    hipLaunchKernelGGL(k_validate, dim3(vgrid), dim3(kBlk), 0, stream, V, E, row_ptr, col, bad);
    int32_t bad_host = 0;
    PREP_HIP(hipMemcpyAsync(&bad_host, bad, sizeof(int32_t), hipMemcpyDeviceToHost, stream));
    PREP_HIP(hipStreamSynchronize(stream));
    if (bad_host) return FR_ERR_ARG;

    // ---- hubs and their virtual rows; the split length doubles until the spare slots hold all virtual rows
    uint64_t* packed = tmp.take<uint64_t>((uint64_t)V);
    uint64_t* scanned = tmp.take<uint64_t>((uint64_t)V);
    PREP_NEED(packed); PREP_NEED(scanned);
    void* scan_tmp = nullptr;
    size_t scan_bytes = 0;
    PREP_HIP(rocprim::exclusive_scan(nullptr, scan_bytes, packed, scanned, uint64_t(0), (size_t)V, rocprim::plus<uint64_t>(), stream));
    scan_tmp = tmp.take<uint8_t>(scan_bytes);
    PREP_NEED(scan_tmp);
    uint32_t split = kHubSplitMin;
    for (;;) {
        hipLaunchKernelGGL(k_hub_mark, dim3(blocks_for((uint64_t)V)), dim3(kBlk), 0, stream, V, split, row_ptr, packed);
        PREP_HIP(rocprim::exclusive_scan(scan_tmp, scan_bytes, packed, scanned, uint64_t(0), (size_t)V, rocprim::plus<uint64_t>(), stream));
        uint64_t last_packed = 0, last_scanned = 0;
        PREP_HIP(hipMemcpyAsync(&last_packed, packed + (V - 1), 8, hipMemcpyDeviceToHost, stream));
        PREP_HIP(hipMemcpyAsync(&last_scanned, scanned + (V - 1), 8, hipMemcpyDeviceToHost, stream));
        PREP_HIP(hipStreamSynchronize(stream));
        const uint64_t totals = last_packed + last_scanned;
        L->n_hubs = (uint32_t)(totals & 0xffffffffu);
        L->n_vrows = (uint32_t)(totals >> 32);
        if ((uint64_t)L->n_vrows <= (uint64_t)kMaxVrowsPerPart * Q) break;
        if (split >= 0x40000000u) return FR_ERR_ARG;       // cannot happen for E < 2^31
        split *= 2;
    }
    L->hub_split = split;
    L->n_hub_tiles = std::max<uint32_t>(1, (L->n_hubs + kHubsPerTile - 1) / kHubsPerTile);

    if (!keep(a, &L->hub_row, L->n_hubs) || !keep(a, &L->hub_vbase, (uint64_t)L->n_hubs + 1) || !keep(a, &L->inv_tag, (uint64_t)V))
        PREP_NEED((void*)nullptr);
    hipLaunchKernelGGL(k_hub_tables, dim3(blocks_for((uint64_t)V)), dim3(kBlk), 0, stream, V, split, row_ptr, scanned, L->n_hubs,
                       L->n_vrows, L->hub_row, L->hub_vbase);
    hipLaunchKernelGGL(k_inv_tag, dim3(blocks_for((uint64_t)V)), dim3(kBlk), 0, stream, V, split, row_ptr, out_degree, L->inv_tag);
    if (!keep(a, &L->hub_of_p, (uint64_t)L->P + 1)) PREP_NEED((void*)nullptr);
    hipLaunchKernelGGL(k_hub_of_p, dim3(blocks_for((uint64_t)L->P + 1)), dim3(kBlk), 0, stream, L->P, L->n_hubs, src_per_part, L->hub_row, L->hub_of_p);

    tmp.drop(packed);
    tmp.drop(scan_tmp);

    // ---- sort the edges by (partition, source, local row); set-up scratch is returned as soon as it is done with
    uint64_t* keys = nullptr;
    uint32_t* incl = nullptr;
    uint32_t M = 0;
    if (E > 0) {
        uint64_t* keys_a = tmp.take<uint64_t>((uint64_t)E);
        uint64_t* keys_b = tmp.take<uint64_t>((uint64_t)E);
        PREP_NEED(keys_a); PREP_NEED(keys_b);
        hipLaunchKernelGGL(k_keys, dim3(blocks_for((uint64_t)E)), dim3(kBlk), 0, stream, V, E, split, row_ptr, col, scanned, Q, rows_per_part, keys_a);
        unsigned end_bit = kKeyLocalBits + kKeySrcBits;
        while (end_bit < 63 && (1ull << (end_bit - kKeyLocalBits - kKeySrcBits)) < (uint64_t)Q) ++end_bit;
        {
            rocprim::double_buffer<uint64_t> db(keys_a, keys_b);
            size_t bytes = 0;
            PREP_HIP(rocprim::radix_sort_keys(nullptr, bytes, db, (size_t)E, 0u, end_bit, stream));
            void* t = tmp.take<uint8_t>(bytes);
            PREP_NEED(t);
            PREP_HIP(rocprim::radix_sort_keys(t, bytes, db, (size_t)E, 0u, end_bit, stream));
            PREP_HIP(hipStreamSynchronize(stream));
            keys = db.current();
            tmp.drop(t);
            tmp.drop(keys == keys_a ? keys_b : keys_a);
        }
        tmp.drop(scanned);
        incl = tmp.take<uint32_t>((uint64_t)E);
        PREP_NEED(incl);
        {
            auto flags = rocprim::make_transform_iterator(rocprim::make_counting_iterator<size_t>(0), FlagOf{keys});
            size_t bytes = 0;
            PREP_HIP(rocprim::inclusive_scan(nullptr, bytes, flags, incl, (size_t)E, rocprim::plus<uint32_t>(), stream));
            void* t = tmp.take<uint8_t>(bytes);
            PREP_NEED(t);
            PREP_HIP(rocprim::inclusive_scan(t, bytes, flags, incl, (size_t)E, rocprim::plus<uint32_t>(), stream));
        }
        PREP_HIP(hipMemcpyAsync(&M, incl + (E - 1), 4, hipMemcpyDeviceToHost, stream));
        PREP_HIP(hipStreamSynchronize(stream));
    } else {
        tmp.drop(scanned);
    }

    // ---- the arrays that stay
    if (!keep(a, &L->ids16, (uint64_t)padded) || !keep(a, &L->eoff, (uint64_t)Q + 1) ||
        !keep(a, &L->mbase, (uint64_t)L->n_chunks + 1) || !keep(a, &L->bins, (uint64_t)L->P * Q))
        PREP_NEED((void*)nullptr);
    L->M = M;
    if (!keep(a, &L->src16, (uint64_t)M)) PREP_NEED((void*)nullptr);

    hipLaunchKernelGGL(k_emit, dim3(blocks_for((uint64_t)padded)), dim3(kBlk), 0, stream, E, padded, (uint64_t)M, keys, incl,
                       src_per_part, L->ids16, L->src16);
    hipLaunchKernelGGL(k_mbase, dim3(blocks_for((uint64_t)L->n_chunks + 1)), dim3(kBlk), 0, stream, E, L->n_chunks, M, keys, incl, L->mbase);
    hipLaunchKernelGGL(k_eoff, dim3(blocks_for((uint64_t)Q + 1)), dim3(kBlk), 0, stream, Q, E, keys, L->eoff);
    hipLaunchKernelGGL(k_bins, dim3(blocks_for((uint64_t)L->P * Q)), dim3(kBlk), 0, stream, L->P, Q, E, M, (uint64_t)src_per_part, keys, incl, L->bins);
    uint64_t* mp = tmp.take<uint64_t>(L->P);
    PREP_NEED(mp);
    hipLaunchKernelGGL(k_msgs_of_p, dim3(blocks_for(L->P)), dim3(kBlk), 0, stream, L->P, Q, L->bins, mp);
    PREP_HIP(hipGetLastError());

    // ---- host copies for the cost model
    std::vector<uint32_t> eoff_host((size_t)Q + 1);
    L->msgs_of_p.assign(L->P, 0);
    PREP_HIP(hipMemcpyAsync(eoff_host.data(), L->eoff, ((size_t)Q + 1) * 4, hipMemcpyDeviceToHost, stream));
    PREP_HIP(hipMemcpyAsync(L->msgs_of_p.data(), mp, (size_t)L->P * 8, hipMemcpyDeviceToHost, stream));
    PREP_HIP(hipStreamSynchronize(stream));
    L->edges_of_q.resize(Q);
    for (uint32_t q = 0; q < Q; ++q) L->edges_of_q[q] = eoff_host[q + 1] - eoff_host[q];
    if (eoff_host[Q] != (uint32_t)E) return FR_ERR_ARG;
    return FR_OK;     // `tmp` returns the scratch blocks to the allocator
}
