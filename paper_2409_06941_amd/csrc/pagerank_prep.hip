// Builds the partition-centric layout (pr_layout.h) of the PageRank side task on the GPU, once, in InitSideTask
// (Section 4.1 of the paper: the transition that loads the task's context into GPU memory).
//
// Pipeline: check the CSR -> order the vertices by in-degree (radix sort; perm and its inverse) -> one 64-bit key
// per edge (range, source, local row) in new ids -> radix sort -> message starts (flags, scan) -> messages per
// source (histogram, scan) -> scatter tiles (host) -> id stream, message sources, edge offsets of the ranges ->
// gather tiles and range classes (host) -> message range of every (scatter tile, range).  rocPRIM supplies the
// device-wide sorts and scans; they run once per task and are not part of any iteration.

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

// Vertex order: larger in-degree first, ties by the caller's id - except among the vertices without in-edges, which
// are ordered by falling out-degree first.  Those vertices have no row sums to gather, so their order is free as far
// as the gather sweep goes, and for the scatter sweep it lines up the ones without out-edges, which send no message,
// in one run at the very end that no scatter piece has to load.  (Breaking all ties by out-degree gives a few more
// such runs and made the gather sweep 2 to 6 % slower on R-MAT graphs: rows of like out-degree are like in whom
// they are pointed to by, and the ids of a wavefront's 64 edges then fall on fewer accumulators.)
// Two sorts of 64-bit keys: by (out-degree falling, id), then by (in-degree falling, id or, without in-edges, the
// rank in the first order).
__global__ __launch_bounds__(kBlk) void k_vertex_keys_out(int64_t V, const int32_t* __restrict__ outdeg, uint64_t* __restrict__ keys)
{
    const int64_t v = (int64_t)blockIdx.x * kBlk + threadIdx.x;
    if (v >= V) return;
    const uint32_t d = (uint32_t)(outdeg[v] < 0 ? 0 : outdeg[v]);
    keys[v] = ((uint64_t)(0x7fffffffu - d) << 32) | (uint64_t)(uint32_t)v;
}

__global__ __launch_bounds__(kBlk) void k_vertex_keys_in(int64_t V, const int32_t* __restrict__ row_ptr, const uint64_t* __restrict__ by_out,
                                                         uint64_t* __restrict__ keys)
{
    const int64_t i = (int64_t)blockIdx.x * kBlk + threadIdx.x;
    if (i >= V) return;
    uint32_t v = (uint32_t)(by_out[i] & 0xffffffffu);
    if ((int64_t)v >= V) v = 0;                        // cannot happen: the keys hold 0 .. V-1
    const uint32_t indeg = (uint32_t)(row_ptr[v + 1] - row_ptr[v]);
    keys[i] = ((uint64_t)(0x7fffffffu - indeg) << 32) | (uint64_t)(indeg ? v : (uint32_t)i);
}

// perm[new] = old, inv[old] = new, inv_out[new] = 1/outdeg (0 for dangling vertices)
__global__ __launch_bounds__(kBlk) void k_perm(int64_t V, const uint64_t* __restrict__ sorted, const uint64_t* __restrict__ by_out,
                                               const int32_t* __restrict__ outdeg, int32_t* __restrict__ perm, int32_t* __restrict__ inv,
                                               float* __restrict__ inv_out)
{
    const int64_t n = (int64_t)blockIdx.x * kBlk + threadIdx.x;
    if (n >= V) return;
    uint32_t old = (uint32_t)(sorted[n] & 0xffffffffu);          // the id, or for a vertex without in-edges its rank by out-degree
    if ((int64_t)old >= V) old = 0;                    // cannot happen
    if ((sorted[n] >> 32) == 0x7fffffffull) {
        old = (uint32_t)(by_out[old] & 0xffffffffu);
        if ((int64_t)old >= V) old = 0;                // cannot happen
    }
    perm[n] = (int32_t)old;
    inv[old] = (int32_t)n;
    const int32_t d = outdeg[old];
    inv_out[n] = d > 0 ? 1.0f / (float)d : 0.0f;
}

__global__ __launch_bounds__(kBlk) void k_keys(int64_t V, int64_t E, const int32_t* __restrict__ row_ptr,
                                               const int32_t* __restrict__ col, const int32_t* __restrict__ inv,
                                               uint32_t rows_per_part, uint64_t* __restrict__ keys)
{
    const int64_t e = (int64_t)blockIdx.x * kBlk + threadIdx.x;
    if (e >= E) return;
    const uint64_t v = (uint64_t)(uint32_t)inv[row_of_edge(row_ptr, V, e)];
    const uint64_t u = (uint64_t)(uint32_t)inv[col[e]];
    keys[e] = ((v / rows_per_part) << (kKeyLocalBits + kKeySrcBits)) | (u << kKeyLocalBits) | (v % rows_per_part);
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

// Scatter tile that holds source u: the t with ubound[t] <= u < ubound[t + 1].
__device__ __forceinline__ uint32_t tile_of_source(const uint32_t* __restrict__ ubound, uint32_t n_tiles, uint32_t u)
{
    uint32_t lo = 0, hi = n_tiles;             // first index in [0, n_tiles] whose bound exceeds u
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if (ubound[mid] > u) hi = mid;
        else lo = mid + 1;
    }
    return lo ? lo - 1 : 0;
}

// cnt[u] += 1 for every message of source u (set-up only; integer atomics)
__global__ __launch_bounds__(kBlk) void k_count_messages(int64_t E, int64_t V, const uint64_t* __restrict__ keys, uint32_t* __restrict__ cnt)
{
    const int64_t e = (int64_t)blockIdx.x * kBlk + threadIdx.x;
    if (e >= E || !flag_of(keys, e)) return;
    const uint32_t u = (uint32_t)((keys[e] >> kKeyLocalBits) & 0x7fffffffu);
    if ((int64_t)u < V) atomicAdd(&cnt[u], 1u);
}

__global__ __launch_bounds__(kBlk) void k_zero_u32(uint64_t n, uint32_t* p)
{
    const uint64_t i = (uint64_t)blockIdx.x * kBlk + threadIdx.x;
    if (i < n) p[i] = 0u;
}

__global__ __launch_bounds__(kBlk) void k_emit(int64_t E, int64_t padded, uint64_t M, const uint64_t* __restrict__ keys,
                                               const uint32_t* __restrict__ incl, const uint32_t* __restrict__ ubound,
                                               uint32_t n_tiles, uint32_t id_scale, uint16_t* __restrict__ ids16,
                                               uint16_t* __restrict__ src16)
{
    const int64_t e = (int64_t)blockIdx.x * kBlk + threadIdx.x;
    if (e >= padded) return;
    if (e >= E) { ids16[id_slot(e)] = 0; return; }
    const uint64_t k = keys[e];
    const uint32_t f = flag_of(keys, e);
    ids16[id_slot(e)] = (uint16_t)((k & ((1u << kKeyLocalBits) - 1)) * id_scale);
    if (f) {
        const uint64_t m = (uint64_t)incl[e] - 1;
        const uint32_t u = (uint32_t)((k >> kKeyLocalBits) & 0x7fffffffu);
        if (m < M) src16[m] = (uint16_t)(u - ubound[tile_of_source(ubound, n_tiles, u)]);
    }
}

// Message-start record of chunk c, kStartWords 64-bit words: words 0 .. 7 = for row j (stream positions 64 j .. 64 j + 63
// of the chunk) the start bits of positions 1 .. 63 in bits 0 .. 62 (bit l set: position l + 1 begins a message);
// words 8 .. 11 = eight 32-bit words, for the first position of each row four times the distance of its message from
// message mbase[c] - 1 (0 .. 2048: a byte offset into the messages).  The message of position l of row j is then:
// mbase[c] - 1 + first[j] / 4 + (set bits below l in word j).
__global__ __launch_bounds__(kBlk) void k_starts(int64_t E, uint64_t n_rows, const uint64_t* __restrict__ keys,
                                                 const uint32_t* __restrict__ incl, uint64_t* __restrict__ starts)
{
    const uint64_t w = (uint64_t)blockIdx.x * kBlk + threadIdx.x;
    if (w >= n_rows) return;
    uint64_t bits = 0;
    for (int l = 1; l < 64; ++l) {
        const int64_t e = (int64_t)(w * 64) + l;
        if (e < E && flag_of(keys, e)) bits |= 1ull << (l - 1);
    }
    const int64_t e0 = (int64_t)(w * 64);
    uint64_t* rec = starts + (w / 8) * kStartWords;
    rec[w % 8] = bits;
    const int64_t ec = (int64_t)(w / 8) * kIdChunk;          // the chunk's first position
    reinterpret_cast<uint32_t*>(rec + 8)[w % 8] = e0 < E ? 4u * (incl[e0] - (incl[ec] - flag_of(keys, ec))) : 0u;
}

__global__ __launch_bounds__(kBlk) void k_mbase(int64_t E, uint32_t n_chunks, uint32_t M, const uint64_t* __restrict__ keys,
                                                const uint32_t* __restrict__ incl, uint32_t* __restrict__ mbase)
{
    const uint32_t c = blockIdx.x * kBlk + threadIdx.x;
    if (c > n_chunks) return;
    const int64_t e = (int64_t)c * kIdChunk;
    mbase[c] = e < E ? incl[e] - flag_of(keys, e) : M;
}

// rep[c] = edges of chunk c that repeat their predecessor (same range, source and row: a multi-edge).  Adjacent in
// the stream, they hit one accumulator from neighbouring lanes, which the LDS serialises; the tile cutter counts them.
__global__ __launch_bounds__(kBlk) void k_chunk_repeats(int64_t E, uint32_t n_chunks, const uint64_t* __restrict__ keys,
                                                        uint32_t* __restrict__ rep)
{
    const uint32_t c = blockIdx.x;
    if (c >= n_chunks) return;
    __shared__ uint32_t total;
    if (threadIdx.x == 0) total = 0;
    __syncthreads();
    uint32_t mine = 0;
    for (uint32_t r = threadIdx.x; r < kIdChunk; r += kBlk) {
        const int64_t e = (int64_t)c * kIdChunk + r;
        if (e >= 1 && e < E && keys[e] == keys[e - 1]) ++mine;
    }
    if (mine) atomicAdd(&total, mine);
    __syncthreads();
    if (threadIdx.x == 0) rep[c] = total;
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

// bins[t * Qe + j] = message range of the edges of range j whose source lies in scatter tile t.
// The first edge of a bin always starts a message, so "messages before it" = incl - 1 there.
__global__ __launch_bounds__(kBlk) void k_bins(uint32_t n_tiles, uint32_t Qe, int64_t E, uint32_t M, const uint32_t* __restrict__ ubound,
                                               const uint64_t* __restrict__ keys, const uint32_t* __restrict__ incl,
                                               uint2* __restrict__ bins)
{
    const uint64_t idx = (uint64_t)blockIdx.x * kBlk + threadIdx.x;
    if (idx >= (uint64_t)n_tiles * Qe) return;
    const uint64_t t = idx / Qe, j = idx % Qe;
    const uint64_t base = j << (kKeyLocalBits + kKeySrcBits);
    const int64_t lo = lower_bound_key(keys, E, base + ((uint64_t)ubound[t] << kKeyLocalBits));
    const int64_t hi = lower_bound_key(keys, E, base + ((uint64_t)ubound[t + 1] << kKeyLocalBits));
    uint2 r;
    r.x = lo < E ? incl[lo] - 1 : M;
    r.y = hi < E ? incl[hi] - 1 : M;
    if (r.y < r.x) r.y = r.x;
    bins[idx] = r;
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
                    const int32_t* out_degree, uint32_t rows_per_part, uint32_t src_per_part, uint32_t cus, fr_alloc* a,
                    hipStream_t stream, int* hip_error)
{
    if (!cus) cus = kDefaultCus;
    if (!rows_per_part) rows_per_part = V >= kLargeRowsFrom ? kRowsLarge : kRowsSmall;
    if (!src_per_part) src_per_part = V >= kLargeSrcFrom ? kSrcLarge : kSrcSmall;
    if ((rows_per_part != kRowsSmall && rows_per_part != kRowsLarge) || (src_per_part != kSrcSmall && src_per_part != kSrcLarge))
        return FR_ERR_ARG;
    L->V = V; L->E = E;
    L->rows_per_part = rows_per_part; L->src_per_part = src_per_part;
    L->Q = (uint32_t)((V + rows_per_part - 1) / rows_per_part);
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

    // ---- vertices in order of falling in-degree; those without in-edges by falling out-degree
    if (!keep(a, &L->perm, (uint64_t)V) || !keep(a, &L->inv_out, (uint64_t)V)) PREP_NEED((void*)nullptr);
    int32_t* inv = tmp.take<int32_t>((uint64_t)V);
    PREP_NEED(inv);
    {
        uint64_t* by_out = tmp.take<uint64_t>((uint64_t)V);
        uint64_t* vk_a = tmp.take<uint64_t>((uint64_t)V);
        uint64_t* vk_b = tmp.take<uint64_t>((uint64_t)V);
        PREP_NEED(by_out); PREP_NEED(vk_a); PREP_NEED(vk_b);
        size_t bytes = 0;
        {
            rocprim::double_buffer<uint64_t> probe(vk_a, vk_b);
            PREP_HIP(rocprim::radix_sort_keys(nullptr, bytes, probe, (size_t)V, 0u, 64u, stream));
        }
        void* t = tmp.take<uint8_t>(bytes);
        PREP_NEED(t);
        hipLaunchKernelGGL(k_vertex_keys_out, dim3(blocks_for((uint64_t)V)), dim3(kBlk), 0, stream, V, out_degree, vk_a);
        rocprim::double_buffer<uint64_t> first(vk_a, vk_b);
        PREP_HIP(rocprim::radix_sort_keys(t, bytes, first, (size_t)V, 0u, 64u, stream));
        PREP_HIP(hipMemcpyAsync(by_out, first.current(), (size_t)V * 8, hipMemcpyDeviceToDevice, stream));
        hipLaunchKernelGGL(k_vertex_keys_in, dim3(blocks_for((uint64_t)V)), dim3(kBlk), 0, stream, V, row_ptr, by_out, vk_a);
        rocprim::double_buffer<uint64_t> second(vk_a, vk_b);
        PREP_HIP(rocprim::radix_sort_keys(t, bytes, second, (size_t)V, 0u, 64u, stream));
        hipLaunchKernelGGL(k_perm, dim3(blocks_for((uint64_t)V)), dim3(kBlk), 0, stream, V, second.current(), by_out, out_degree, L->perm, inv, L->inv_out);
        PREP_HIP(hipStreamSynchronize(stream));
        tmp.drop(t); tmp.drop(vk_a); tmp.drop(vk_b); tmp.drop(by_out);
    }

    // ---- sort the edges by (range, source, local row); set-up scratch is returned as soon as it is done with
    uint64_t* keys = nullptr;
    uint32_t* incl = nullptr;
    uint32_t M = 0;
    if (E > 0) {
        uint64_t* keys_a = tmp.take<uint64_t>((uint64_t)E);
        uint64_t* keys_b = tmp.take<uint64_t>((uint64_t)E);
        PREP_NEED(keys_a); PREP_NEED(keys_b);
        hipLaunchKernelGGL(k_keys, dim3(blocks_for((uint64_t)E)), dim3(kBlk), 0, stream, V, E, row_ptr, col, inv, rows_per_part, keys_a);
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
        incl = tmp.take<uint32_t>((uint64_t)E);
        PREP_NEED(incl);
        {
            auto flags = rocprim::make_transform_iterator(rocprim::make_counting_iterator<size_t>(0), FlagOf{keys});
            size_t bytes = 0;
            PREP_HIP(rocprim::inclusive_scan(nullptr, bytes, flags, incl, (size_t)E, rocprim::plus<uint32_t>(), stream));
            void* t = tmp.take<uint8_t>(bytes);
            PREP_NEED(t);
            PREP_HIP(rocprim::inclusive_scan(t, bytes, flags, incl, (size_t)E, rocprim::plus<uint32_t>(), stream));
            PREP_HIP(hipMemcpyAsync(&M, incl + (E - 1), 4, hipMemcpyDeviceToHost, stream));
            PREP_HIP(hipStreamSynchronize(stream));
            tmp.drop(t);
        }
    }
    tmp.drop(inv);
    L->M = M;

    // ---- scatter pieces: source intervals of about equal numbers of messages
    std::vector<uint32_t> cum((size_t)V + 1, 0u);            // messages of the sources before u
    if (E > 0) {
        uint32_t* cnt = tmp.take<uint32_t>((uint64_t)V + 1);
        uint32_t* cum_dev = tmp.take<uint32_t>((uint64_t)V + 1);
        PREP_NEED(cnt); PREP_NEED(cum_dev);
        hipLaunchKernelGGL(k_zero_u32, dim3(blocks_for((uint64_t)V + 1)), dim3(kBlk), 0, stream, (uint64_t)V + 1, cnt);
        hipLaunchKernelGGL(k_count_messages, dim3(blocks_for((uint64_t)E)), dim3(kBlk), 0, stream, E, V, keys, cnt);
        size_t bytes = 0;
        PREP_HIP(rocprim::exclusive_scan(nullptr, bytes, cnt, cum_dev, 0u, (size_t)V + 1, rocprim::plus<uint32_t>(), stream));
        void* t = tmp.take<uint8_t>(bytes);
        PREP_NEED(t);
        PREP_HIP(rocprim::exclusive_scan(t, bytes, cnt, cum_dev, 0u, (size_t)V + 1, rocprim::plus<uint32_t>(), stream));
        PREP_HIP(hipMemcpyAsync(cum.data(), cum_dev, ((size_t)V + 1) * 4, hipMemcpyDeviceToHost, stream));
        PREP_HIP(hipStreamSynchronize(stream));
        tmp.drop(t); tmp.drop(cnt); tmp.drop(cum_dev);
        if (cum[(size_t)V] != M) return FR_ERR_ARG;
    }
    // ---- the arrays that stay
    if (!keep(a, &L->ids16, (uint64_t)padded) || !keep(a, &L->starts, (uint64_t)padded / kIdChunk * kStartWords) || !keep(a, &L->mbase, (uint64_t)L->n_chunks + 1) || !keep(a, &L->src16, ((uint64_t)M + 15) / 8 * 8))     // read eight at a time
        PREP_NEED((void*)nullptr);
    uint32_t* eoff = tmp.take<uint32_t>((uint64_t)Q + 1);
    PREP_NEED(eoff);
    hipLaunchKernelGGL(k_starts, dim3(blocks_for((uint64_t)padded / 64)), dim3(kBlk), 0, stream, E, (uint64_t)padded / 64, keys, incl, L->starts);
    hipLaunchKernelGGL(k_mbase, dim3(blocks_for((uint64_t)L->n_chunks + 1)), dim3(kBlk), 0, stream, E, L->n_chunks, M, keys, incl, L->mbase);
    hipLaunchKernelGGL(k_eoff, dim3(blocks_for((uint64_t)Q + 1)), dim3(kBlk), 0, stream, Q, E, keys, eoff);
    std::vector<uint32_t> eoff_host((size_t)Q + 1);
    PREP_HIP(hipMemcpyAsync(eoff_host.data(), eoff, ((size_t)Q + 1) * 4, hipMemcpyDeviceToHost, stream));
    PREP_HIP(hipStreamSynchronize(stream));
    if (eoff_host[0] != 0 || eoff_host[Q] != (uint32_t)E) return FR_ERR_ARG;

    // ---- gather tiles and range classes.  Rows are in order of falling in-degree, so the ranges with edges come first.
    uint32_t Qe = 0;
    for (uint32_t j = 0; j < Q; ++j)
        if (eoff_host[j + 1] > eoff_host[j]) Qe = j + 1;
    if (Qe == 0) Qe = 1;          // a graph without edges: range 0 still gets a (direct) gather tile
    L->Qe = Qe;
    // weight of the stream up to every chunk boundary: an edge counts 1, a message kGatherMessageWeight more, a
    // repeated edge kGatherRepeatWeight more (measured on single tiles: 0.09 ns, 0.18 ns and 0.28 ns a piece)
    std::vector<uint64_t> wcum((size_t)L->n_chunks + 1, 0);
    if (E > 0) {
        uint32_t* rep = tmp.take<uint32_t>((uint64_t)L->n_chunks);
        PREP_NEED(rep);
        hipLaunchKernelGGL(k_chunk_repeats, dim3(L->n_chunks), dim3(kBlk), 0, stream, E, L->n_chunks, keys, rep);
        std::vector<uint32_t> rep_host(L->n_chunks), mbase_host((size_t)L->n_chunks + 1);
        PREP_HIP(hipMemcpyAsync(rep_host.data(), rep, (size_t)L->n_chunks * 4, hipMemcpyDeviceToHost, stream));
        PREP_HIP(hipMemcpyAsync(mbase_host.data(), L->mbase, ((size_t)L->n_chunks + 1) * 4, hipMemcpyDeviceToHost, stream));
        PREP_HIP(hipStreamSynchronize(stream));
        tmp.drop(rep);
        for (uint32_t c = 0; c < L->n_chunks; ++c) {
            const uint64_t edges = std::min<uint64_t>(kIdChunk, (uint64_t)E - (uint64_t)c * kIdChunk);
            wcum[c + 1] = wcum[c] + kGatherEdgeWeight * edges + kGatherMessageWeight * (uint64_t)(mbase_host[c + 1] - mbase_host[c]) +
                          kGatherRepeatWeight * (uint64_t)rep_host[c];
        }
    }
    auto weight_at = [&](uint64_t e) -> uint64_t {          // weight of the edges before e (linear inside a chunk)
        const uint64_t c = e / kIdChunk;
        if (c >= L->n_chunks) return wcum[L->n_chunks];
        const uint64_t held = std::min<uint64_t>(kIdChunk, (uint64_t)E - c * kIdChunk);      // the last chunk may be short
        return wcum[c] + (wcum[c + 1] - wcum[c]) * std::min(e - c * kIdChunk, held) / held;
    };
    L->gp.clear(); L->gt.clear(); L->gt_weight.clear(); L->gt_edges.clear();
    L->ri.assign(Q, RangeInfo{kRangeEmpty, 0}); L->fin.clear();
    {
        // A piece costs its weight plus a fixed part (kTileFixedWeight: the chain of dependent loads at its start and
        // the row pass at its end).  Ranges are cut into pieces of at most `body` weight; pieces are then grouped, in
        // order, into tiles of at most body + kTileFixedWeight.  A launch has no more workgroups than run side by
        // side (`slots`), each of which takes the next tile when it is done with one.  Where a slot's share of the
        // sweep is long against what a tile costs to start and to end (kGatherFineShare), heavy ranges are cut for
        // two pieces per slot and every piece is a tile of its own, so that the many light tiles at the end fill
        // the gaps the heavy ones leave; below that there are no more tiles than slots, light pieces share tiles, and
        // `body` is the smallest (to 2 %) that achieves it.
        const uint64_t slots = (uint64_t)cus * (rows_per_part == kRowsSmall ? 2 : 1);
        std::vector<uint64_t> w(Qe);
        uint64_t total = 0;
        for (uint32_t j = 0; j < Qe; ++j) { w[j] = weight_at(eoff_host[j + 1]) - weight_at(eoff_host[j]); total += w[j]; }
        const uint64_t share = (total + slots - 1) / slots;
        const uint64_t fine = share >= kGatherFineShare ? 2 : 1;
        std::vector<GatherPiece> pieces;
        std::vector<uint64_t> piece_w;
        std::vector<uint2> tiles;
        uint64_t body = std::max<uint64_t>(kMinTileEdges * kGatherEdgeWeight, (total + slots * fine - 1) / (slots * fine));
        for (int round = 0; round < 400; ++round, body += body / 50 + 1) {
            pieces.clear(); piece_w.clear(); tiles.clear();
            L->ri.assign(Q, RangeInfo{kRangeEmpty, 0});
            L->fin.clear();
            L->n_merged = 0; L->n_partials = 0;
            for (uint32_t j = 0; j < Qe; ++j) {
                const uint64_t e0 = eoff_host[j], e1 = eoff_host[j + 1];
                const uint64_t nt = std::max<uint64_t>(1, (w[j] + body - 1) / body);
                std::vector<uint64_t> cuts;                      // chunk boundaries strictly inside (e0, e1)
                const uint64_t w0 = weight_at(e0);
                for (uint64_t i = 1; i < nt; ++i) {
                    const uint64_t want = w0 + w[j] * i / nt;
                    const uint64_t c = (uint64_t)(std::lower_bound(wcum.begin(), wcum.end(), want) - wcum.begin());
                    const uint64_t cut = c * kIdChunk;
                    if (cut > (cuts.empty() ? e0 : cuts.back()) && cut < e1) cuts.push_back(cut);
                }
                if (cuts.empty()) {
                    pieces.push_back(GatherPiece{j, (uint32_t)e0, (uint32_t)e1, kNoPartial});
                    piece_w.push_back(w[j] + kTileFixedWeight);
                    L->ri[j] = RangeInfo{kRangeDirect | (1u << 2), 0};
                    continue;
                }
                L->ri[j] = RangeInfo{kRangeMerged | ((uint32_t)(cuts.size() + 1) << 2), L->n_partials};
                L->fin.push_back(j);
                L->n_merged++;
                cuts.push_back(e1);
                uint64_t lo = e0;
                for (uint64_t hi : cuts) {
                    pieces.push_back(GatherPiece{j, (uint32_t)lo, (uint32_t)hi, L->n_partials++});
                    piece_w.push_back(weight_at(hi) - weight_at(lo) + kTileFixedWeight);
                    lo = hi;
                }
            }
            uint64_t in_tile = 0;
            uint32_t first = 0;
            for (uint32_t i = 0; i < pieces.size(); ++i) {
                if (i > first && (fine > 1 || in_tile + piece_w[i] > body + kTileFixedWeight)) {
                    tiles.push_back(make_uint2(first, i));
                    first = i; in_tile = 0;
                }
                in_tile += piece_w[i];
            }
            tiles.push_back(make_uint2(first, (uint32_t)pieces.size()));
            if (fine > 1 || tiles.size() <= slots) break;
        }
        for (uint32_t j = Qe; j < Q; ++j) L->fin.push_back(j);
        L->gp = pieces;
        L->gt.clear();
        for (const uint2& t : tiles) L->gt.push_back(GatherTile{t.x, t.y, pieces[t.x], {0, 0}});
        for (const uint2& t : tiles) {
            uint64_t wsum = 0, esum = 0;
            for (uint32_t i = t.x; i < t.y; ++i) { wsum += piece_w[i]; esum += (uint64_t)pieces[i].e1 - pieces[i].e0; }
            L->gt_weight.push_back(wsum);
            L->gt_edges.push_back(esum);
        }
    }
    L->gather_slots = cus * (rows_per_part == kRowsSmall ? 2u : 1u);
    L->scatter_slots = cus * (src_per_part == kSrcSmall ? 2u : 1u);
    L->n_pieces = (uint32_t)L->gp.size();
    L->n_gather = (uint32_t)L->gt.size();
    L->n_finish = (uint32_t)L->fin.size();

    // ---- scatter pieces and tiles.  A piece is an interval of at most src_per_part sources and at most `target`
    // weight, where a message weighs kScatterMessageWeight and a source kScatterRowWeight times the values read to
    // finish it (its contrib or 1/outdeg, and the partial sums of a row of a merged range); the pieces of the sources
    // with few messages are as wide as allowed and light whatever the target.  A tile is a run of consecutive pieces
    // whose costs (weight + kScatterFixedWeight a piece, for the chain of dependent loads at its start) add up to at
    // most target + kScatterFixedWeight.  A launch has no more workgroups than run side by side (`slots`), each of
    // which takes the next tile when it is done with one; with `fine` tiles per slot the light tiles at the end fill
    // the gaps the heavy ones leave, which pays where a slot's share of the sweep is long: from kScatterFineShare on
    // the pieces are cut for two per slot and each is a tile of its own.  Below that the target is the smallest one
    // (to 2 %) that leaves no more tiles than slots.
    std::vector<uint32_t> ubound;
    std::vector<uint8_t> piece_void;
    std::vector<uint2> stiles;
    {
        std::vector<uint64_t> per_row(Q), rows_before((size_t)Q + 1, 0);
        for (uint32_t j = 0; j < Q; ++j) {
            per_row[j] = 1 + ((L->ri[j].cls_tiles & 3u) == kRangeMerged ? (L->ri[j].cls_tiles >> 2) : 0u);
            const uint64_t lo = (uint64_t)j * rows_per_part, hi = std::min<uint64_t>((uint64_t)V, lo + rows_per_part);
            rows_before[j + 1] = rows_before[j] + (hi - lo) * per_row[j];
        }
        // Runs of kVoidMin or more consecutive sources that send no message (vertices without out-edges: the order by
        // in-degree, then out-degree, lines them up at the end of every class of equal in-degree) become VOID pieces,
        // which no tile holds: nothing of them is loaded.  Not in merged ranges, whose rows the scatter sweep
        // finishes.  Their dangling mass is not lost: in a range with in-edges the gather tile counts it, and in a
        // range without, every such row holds the base value, so the sweep adds base x their number in one go.
        std::vector<std::pair<uint64_t, uint64_t>> voids;
        std::vector<uint64_t> void_rows_before_void;        // rows in the void runs before each of them
        {
            uint64_t first_voidable = std::min<uint64_t>((uint64_t)V, src_per_part);      // (the first piece always exists)
            for (uint32_t j = 0; j < Q; ++j)
                if ((L->ri[j].cls_tiles & 3u) == kRangeMerged) first_voidable = std::max(first_voidable, std::min<uint64_t>((uint64_t)V, ((uint64_t)j + 1) * rows_per_part));
            uint64_t run_start = first_voidable, rows = 0;
            for (uint64_t u = first_voidable; u <= (uint64_t)V; ++u) {
                if (u < (uint64_t)V && cum[u + 1] == cum[u]) continue;
                if (u - run_start >= kVoidMin) { voids.push_back({run_start, u}); void_rows_before_void.push_back(rows); rows += u - run_start; }
                run_start = u + 1;
            }
            void_rows_before_void.push_back(rows);
        }
        auto void_rows_before = [&](uint64_t u) -> uint64_t {        // rows of void runs among the sources before u
            const size_t k = (size_t)(std::upper_bound(voids.begin(), voids.end(), std::pair<uint64_t, uint64_t>(u, ~(uint64_t)0)) - voids.begin());   // runs starting at or before u
            if (k == 0) return 0;
            return void_rows_before_void[k - 1] + std::min(u, voids[k - 1].second) - voids[k - 1].first;
        };
        auto weight_before = [&](uint64_t u) -> uint64_t {
            const uint64_t j = std::min<uint64_t>(u / rows_per_part, Q);
            const uint64_t rows = rows_before[j] + (j < Q ? (u - j * rows_per_part) * per_row[j] : 0);
            return kScatterMessageWeight * (uint64_t)cum[u] + kScatterRowWeight * (rows - void_rows_before(u));
        };
        auto cut = [&](uint64_t target) {
            ubound.clear(); piece_void.clear();
            uint64_t u = 0;
            size_t vi = 0;
            while (u < (uint64_t)V) {
                if (vi < voids.size() && u == voids[vi].first) {
                    ubound.push_back((uint32_t)u); piece_void.push_back(1);
                    u = voids[vi++].second;
                    continue;
                }
                uint64_t limit = std::min<uint64_t>((uint64_t)V, u + src_per_part);
                if (vi < voids.size()) limit = std::min(limit, voids[vi].first);
                const uint64_t want = weight_before(u) + target;
                uint64_t lo = u + 1, hi = limit;             // the first end in (u, limit] that reaches `want`, else limit
                while (lo < hi) {
                    const uint64_t mid = (lo + hi) / 2;
                    if (weight_before(mid) >= want) hi = mid;
                    else lo = mid + 1;
                }
                ubound.push_back((uint32_t)u); piece_void.push_back(0);
                u = lo;
            }
            ubound.push_back((uint32_t)V);
        };
        auto live_pieces = [&]() { size_t n = 0; for (uint8_t v : piece_void) n += v ? 0 : 1; return n; };
        auto pack = [&](uint64_t limit) {                    // (limit 0: a tile per piece); void pieces are in no tile
            stiles.clear();
            const uint32_t n = (uint32_t)ubound.size() - 1;
            uint64_t in_tile = 0;
            uint32_t first = 0;
            bool open = false;
            for (uint32_t i = 0; i < n; ++i) {
                if (piece_void[i]) {
                    if (open) stiles.push_back(make_uint2(first, i));
                    open = false;
                    continue;
                }
                const uint64_t c = weight_before(ubound[i + 1]) - weight_before(ubound[i]) + kScatterFixedWeight;
                if (open && in_tile + c > limit) {
                    stiles.push_back(make_uint2(first, i));
                    open = false;
                }
                if (!open) { first = i; in_tile = 0; open = true; }
                in_tile += c;
            }
            if (open) stiles.push_back(make_uint2(first, n));
        };
        const uint64_t slots = (uint64_t)cus * (src_per_part == kSrcSmall ? 2 : 1);
        const uint64_t all = weight_before((uint64_t)V), least = kMinTileMessages * kScatterMessageWeight;
        const uint64_t share = (all + slots - 1) / slots;
        const uint64_t fine = share >= kScatterFineShare ? 2 : 1;
        const uint64_t start = std::max<uint64_t>(least, (all + slots * fine - 1) / (slots * fine));
        bool done = false;
        if (fine > 1) {
            cut(start);
            pack(0);
            done = true;
        } else if (src_per_part == kSrcSmall) {
            // the small kernel is faster without the loop over pieces: a tile per piece, if a target up to one
            // compute unit's share of the weight leaves few enough pieces
            const uint64_t most = std::max<uint64_t>(least, (all + cus - 1) / cus);
            for (uint64_t target = start;; target = std::min(most, target + target / 50 + 1)) {
                cut(target);
                if (live_pieces() <= slots) { pack(0); done = true; break; }
                if (target >= most) break;
            }
        }
        if (!done)
            for (uint64_t target = start;; target += target / 50 + 1) {
                cut(target);
                pack(target + kScatterFixedWeight);
                if (stiles.size() <= slots) break;
            }
    }
    L->n_spieces = (uint32_t)ubound.size() - 1;
    // the void pieces' rows in ranges without in-edges (all dangling: no message means no out-edge), and the slot of
    // the dangling partials that takes base x their number
    L->void_slot = kNoVoid; L->n_void_dangling = 0;
    {
        const uint64_t first_empty_row = std::min<uint64_t>((uint64_t)V, (uint64_t)Qe * rows_per_part);
        for (uint32_t i = 0; i < L->n_spieces; ++i) {
            if (!piece_void[i]) continue;
            if (L->void_slot == kNoVoid) L->void_slot = i;
            const uint64_t u0 = std::max<uint64_t>(ubound[i], first_empty_row), u1 = ubound[i + 1];
            if (u1 > u0) L->n_void_dangling += u1 - u0;
        }
    }
    uint32_t* ubound_dev = tmp.take<uint32_t>(ubound.size());
    PREP_NEED(ubound_dev);
    PREP_HIP(hipMemcpyAsync(ubound_dev, ubound.data(), ubound.size() * 4, hipMemcpyHostToDevice, stream));
    hipLaunchKernelGGL(k_emit, dim3(blocks_for((uint64_t)padded)), dim3(kBlk), 0, stream, E, padded, (uint64_t)M, keys, incl,
                       ubound_dev, L->n_spieces, id_scale_for(rows_per_part), L->ids16, L->src16);

    // ---- what the cost model needs of every scatter tile
    L->sp.clear(); L->st.clear(); L->st_msgs.clear(); L->st_rows.clear();
    {
        std::vector<uint64_t> msgs(L->n_spieces), rows(L->n_spieces);
        for (uint32_t t = 0; t < L->n_spieces; ++t) {
            const uint64_t u0 = ubound[t], u1 = ubound[t + 1];
            uint64_t partials = 0;
            for (uint64_t j = u0 / rows_per_part; j < Q && j * rows_per_part < u1; ++j) {
                if ((L->ri[j].cls_tiles & 3u) != kRangeMerged) continue;
                const uint64_t lo = std::max<uint64_t>(u0, j * rows_per_part), hi = std::min<uint64_t>(u1, (j + 1) * (uint64_t)rows_per_part);
                partials += (hi - lo) * (L->ri[j].cls_tiles >> 2);
            }
            L->sp.push_back(ScatterPiece{(uint32_t)u0, (uint32_t)u1});
            msgs[t] = (uint64_t)cum[u1] - cum[u0];
            rows[t] = (u1 - u0) + partials;
        }
        for (const uint2& t : stiles) {
            L->st.push_back(ScatterTile{t.x, t.y, L->sp[t.x].u0, L->sp[t.x].u1, L->ri[L->sp[t.x].u0 / rows_per_part], {0, 0}});
            uint64_t m = 0, r = 0;
            for (uint32_t i = t.x; i < t.y; ++i) { m += msgs[i]; r += rows[i]; }
            L->st_msgs.push_back(m);
            L->st_rows.push_back(r);
        }
    }
    L->n_scatter = (uint32_t)L->st.size();
    L->scatter_packed = false;
    for (const ScatterTile& t : L->st) L->scatter_packed = L->scatter_packed || t.p1 - t.p0 > 1;

    if (!keep(a, &L->bins, (uint64_t)L->n_spieces * Qe) || !keep(a, &L->range_info, (uint64_t)Q) ||
        !keep(a, &L->gather_pieces, (uint64_t)L->n_pieces) || !keep(a, &L->gather_tiles, (uint64_t)L->n_gather) || !keep(a, &L->scatter_pieces, (uint64_t)L->n_spieces) || !keep(a, &L->scatter_tiles, (uint64_t)L->n_scatter) ||
        !keep(a, &L->finish_ranges, (uint64_t)L->n_finish))
        PREP_NEED((void*)nullptr);
    if (Qe)
        hipLaunchKernelGGL(k_bins, dim3(blocks_for((uint64_t)L->n_spieces * Qe)), dim3(kBlk), 0, stream, L->n_spieces, Qe, E, M, ubound_dev,
                           keys, incl, L->bins);
    PREP_HIP(hipGetLastError());
    PREP_HIP(hipMemcpyAsync(L->range_info, L->ri.data(), (size_t)Q * sizeof(RangeInfo), hipMemcpyHostToDevice, stream));
    PREP_HIP(hipMemcpyAsync(L->gather_pieces, L->gp.data(), (size_t)L->n_pieces * sizeof(GatherPiece), hipMemcpyHostToDevice, stream));
    PREP_HIP(hipMemcpyAsync(L->gather_tiles, L->gt.data(), (size_t)L->n_gather * sizeof(GatherTile), hipMemcpyHostToDevice, stream));
    PREP_HIP(hipMemcpyAsync(L->scatter_pieces, L->sp.data(), (size_t)L->n_spieces * sizeof(ScatterPiece), hipMemcpyHostToDevice, stream));
    PREP_HIP(hipMemcpyAsync(L->scatter_tiles, L->st.data(), (size_t)L->n_scatter * sizeof(ScatterTile), hipMemcpyHostToDevice, stream));
    if (L->n_finish)
        PREP_HIP(hipMemcpyAsync(L->finish_ranges, L->fin.data(), (size_t)L->n_finish * 4, hipMemcpyHostToDevice, stream));
    PREP_HIP(hipStreamSynchronize(stream));       // the host vectors and `tmp` go away after this
    return FR_OK;     // `tmp` returns the scratch blocks to the allocator
}
