// Stage load generator: what the emulated pipeline stage runs between bubbles.
//
// The paper harvests the bubbles of a transformer language model trained with pipeline parallelism
// (Section 6.1.3); its forward and backward passes per micro-batch are the stage's busy periods (Section 2.1).
// Here one busy period is a burst of bf16 GEMMs with the shapes of `layers` transformer blocks, run on the
// MFMA units with fp32 accumulation, or (for the small timed configuration) a kernel that spins on the GPU
// clock for a fixed time.

#include <algorithm>
#include <new>

#include "common.h"

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int BM = 256, BN = 128, BK = 64;     // workgroup tile
constexpr int kThreads = 512;                  // 8 wavefronts as 4 x 2, each 64 x 64 of C
constexpr int kLdsRow = BK + 8;                // bf16 elements per LDS row: 128 B of data + 16 B pad, which spreads
                                               // the rows one 16-byte-per-lane LDS access touches over the banks
constexpr int kXcds = 8;

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float x)
{
    uint32_t u = __float_as_uint(x);
    u += 0x7fffu + ((u >> 16) & 1u);           // round to nearest even (inputs here are finite)
    return (uint16_t)(u >> 16);
}

// C[M, N] = A[M, K] * B[N, K]^T, bf16 in / bf16 out, fp32 accumulate.  M multiple of 256, N of 128, K of 64.
// Per k-tile: the registers holding the tile go to LDS, the next tile's global loads are issued into the same
// registers, and the tile is multiplied out of LDS (4 k-steps of v_mfma_f32_32x32x16_bf16, 2 x 2 MFMA tiles per
// wavefront).  Two workgroups share a CU (54 KB of LDS and 128 registers per lane each), so one multiplies while
// the other sits at its barrier.  The staging registers are named scalars on purpose: as small private arrays
// they are moved to LDS or scratch by the compiler and the kernel runs three times slower.
// Workgroups are dealt round-robin over the 8 XCDs by the hardware; the tile map undoes that so that each XCD
// walks a contiguous run of tiles (same A rows, consecutive B columns) and reuses its own L2.
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(4, 4)))
void k_gemm_bf16_nt(const uint16_t* __restrict__ A, const uint16_t* __restrict__ B, uint16_t* __restrict__ C, int M, int N, int K)
{
    constexpr int kPiecesPerRow = BK / 8, kRowsPerPass = kThreads / kPiecesPerRow;     // 8 pieces of 16 B, 64 rows
    __shared__ __align__(16) uint16_t sA[BM * kLdsRow];
    __shared__ __align__(16) uint16_t sB[BN * kLdsRow];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int tiles_n = N / BN, n_tiles = (int)gridDim.x;
    int tile = (int)blockIdx.x;
    if (n_tiles % kXcds == 0) tile = (tile % kXcds) * (n_tiles / kXcds) + tile / kXcds;
    const int bm = (tile / tiles_n) * BM, bn = (tile % tiles_n) * BN;

    const int ld_row = tid / kPiecesPerRow, ld_k = (tid % kPiecesPerRow) * 8;
    const uint16_t* gA = A + (size_t)(bm + ld_row) * K + ld_k;
    const uint16_t* gB = B + (size_t)(bn + ld_row) * K + ld_k;
    const size_t step = (size_t)kRowsPerPass * K;

    f32x16 acc00, acc01, acc10, acc11;
#pragma unroll
    for (int r = 0; r < 16; ++r) { acc00[r] = 0.0f; acc01[r] = 0.0f; acc10[r] = 0.0f; acc11[r] = 0.0f; }

    uint4 a0 = *reinterpret_cast<const uint4*>(gA), a1 = *reinterpret_cast<const uint4*>(gA + step);
    uint4 a2 = *reinterpret_cast<const uint4*>(gA + 2 * step), a3 = *reinterpret_cast<const uint4*>(gA + 3 * step);
    uint4 b0 = *reinterpret_cast<const uint4*>(gB), b1 = *reinterpret_cast<const uint4*>(gB + step);

    const int frag_row = lane & 31, frag_k = (lane >> 5) * 8;
    uint16_t* wA = &sA[ld_row * kLdsRow + ld_k];
    uint16_t* wB = &sB[ld_row * kLdsRow + ld_k];
    const uint16_t* rA = &sA[(wm * 64 + frag_row) * kLdsRow + frag_k];
    const uint16_t* rB = &sB[(wn * 64 + frag_row) * kLdsRow + frag_k];
    constexpr int kPass = kRowsPerPass * kLdsRow;
    for (int k0 = 0; k0 < K; k0 += BK) {
        __syncthreads();                       // previous tile fully consumed
        *reinterpret_cast<uint4*>(wA) = a0;
        *reinterpret_cast<uint4*>(wA + kPass) = a1;
        *reinterpret_cast<uint4*>(wA + 2 * kPass) = a2;
        *reinterpret_cast<uint4*>(wA + 3 * kPass) = a3;
        *reinterpret_cast<uint4*>(wB) = b0;
        *reinterpret_cast<uint4*>(wB + kPass) = b1;
        __syncthreads();
        if (k0 + BK < K) {                     // fetch the next tile while this one is multiplied
            const uint16_t* pA = gA + k0 + BK;
            const uint16_t* pB = gB + k0 + BK;
            a0 = *reinterpret_cast<const uint4*>(pA);
            a1 = *reinterpret_cast<const uint4*>(pA + step);
            a2 = *reinterpret_cast<const uint4*>(pA + 2 * step);
            a3 = *reinterpret_cast<const uint4*>(pA + 3 * step);
            b0 = *reinterpret_cast<const uint4*>(pB);
            b1 = *reinterpret_cast<const uint4*>(pB + step);
        }
#pragma unroll
        for (int kk = 0; kk < BK; kk += 16) {
            const bf16x8 fa0 = *reinterpret_cast<const bf16x8*>(rA + kk);
            const bf16x8 fa1 = *reinterpret_cast<const bf16x8*>(rA + 32 * kLdsRow + kk);
            const bf16x8 fb0 = *reinterpret_cast<const bf16x8*>(rB + kk);
            const bf16x8 fb1 = *reinterpret_cast<const bf16x8*>(rB + 32 * kLdsRow + kk);
            acc00 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa0, fb0, acc00, 0, 0, 0);
            acc01 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa0, fb1, acc01, 0, 0, 0);
            acc10 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa1, fb0, acc10, 0, 0, 0);
            acc11 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa1, fb1, acc11, 0, 0, 0);
        }
    }

    // accumulator layout of the 32 x 32 MFMA: lane l holds column l % 32, rows 8 * (r / 4) + 4 * (l / 32) + r % 4
    const int col = bn + wn * 64 + (lane & 31), row_in = (lane >> 5) * 4;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int row = bm + wm * 64 + 8 * (r >> 2) + row_in + (r & 3);
        C[(size_t)row * N + col] = f32_to_bf16_rne(acc00[r]);
        C[(size_t)row * N + col + 32] = f32_to_bf16_rne(acc01[r]);
        C[(size_t)(row + 32) * N + col] = f32_to_bf16_rne(acc10[r]);
        C[(size_t)(row + 32) * N + col + 32] = f32_to_bf16_rne(acc11[r]);
    }
}

// Seeded fill: bf16 values uniform in [-1/8, 1/8) from a counter-based 64-bit mixer.
__global__ __launch_bounds__(256) void k_fill_bf16(uint16_t* __restrict__ p, uint64_t n, uint64_t seed)
{
    const uint64_t stride = (uint64_t)gridDim.x * 256;
    for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
        uint64_t z = seed + i * 0x9E3779B97F4A7C15ull;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        z ^= z >> 31;
        const float u = (float)(z >> 40) * (1.0f / 16777216.0f);      // [0, 1)
        p[i] = f32_to_bf16_rne((u - 0.5f) * 0.25f);
    }
}

// Spins until the GPU's constant-rate clock has advanced by `ticks`, with a hard cap on loop trips so that the
// kernel ends even if the clock did not advance.
__global__ void k_busywait(uint64_t ticks, uint64_t max_trips)
{
    const uint64_t t0 = wall_clock64();
    for (uint64_t i = 0; i < max_trips; ++i) {
        if (wall_clock64() - t0 >= ticks) break;
        __builtin_amdgcn_s_sleep(16);
    }
}

// Keeps compute units busy with register-only arithmetic (no memory traffic) until the GPU's constant-rate clock has
// advanced by `ticks`: what fills the bubbles of the baseline that differs from a harvested epoch only by the side
// task's memory traffic.  The trip cap ends the kernel even if the clock did not advance; the result is stored only
// if it is NaN (it never is), so the loop cannot be optimised away.
__global__ __launch_bounds__(256) void k_alu_fill(uint64_t ticks, uint64_t max_trips, float* sink)
{
    const uint64_t t0 = wall_clock64();
    float a = (float)threadIdx.x * 1.0e-3f, b = 0.999f, c = 1.0e-4f;
    for (uint64_t i = 0; i < max_trips; ++i) {
        if (wall_clock64() - t0 >= ticks) break;
#pragma unroll
        for (int k = 0; k < 64; ++k) a = fmaf(a, b, c);
    }
    if (a != a && sink) *sink = a;
}

struct GemmShape { int M, N, K; size_t a_off, b_off, c_off; };   // offsets in bf16 elements into the workspace

}  // namespace

struct fr_load {
    fr_load_desc d{};
    int wall_clock_khz = 100000;
    std::vector<GemmShape> fp, bp;
    uint64_t fp_flops = 0, bp_flops = 0;
    int hip_error = 0;
};

namespace {

uint64_t r128(uint64_t elems) { return (elems + 127) & ~127ull; }

// Lays out operands in the workspace and lists the GEMMs of one forward and one backward burst.
// Per layer, with T tokens, hidden h, feed-forward width f:
//   forward : QKV [T,h]x[h,3h], projection [T,h]x[h,h], up [T,h]x[h,f], down [T,f]x[f,h]
//   backward: for each forward GEMM  Y[T,n] = X[T,k] W[n,k]^T  the data gradient  dX[T,k] = dY[T,n] W
//             (M = T, N = k, K = n) and the weight gradient  dW[n,k] = dY^T X  (M = n, N = k, K = T).
// Weights are distinct per layer; activations, gradients and the weight-gradient scratch are shared by layers.
uint64_t plan_gpt(fr_load* l, bool fill_lists)
{
    const fr_load_desc& d = l->d;
    const uint64_t T = d.tokens, h = d.hidden, f = d.ffn;
    uint64_t off = 0;
    auto take = [&](uint64_t elems) { uint64_t o = off; off += r128(elems); return o; };
    const uint64_t n_out[4] = {3 * h, h, f, h}, k_in[4] = {h, h, h, f};
    uint64_t maxn = 0, maxk = 0, maxw = 0;
    for (int g = 0; g < 4; ++g) { maxn = std::max(maxn, n_out[g]); maxk = std::max(maxk, k_in[g]); maxw = std::max(maxw, n_out[g] * k_in[g]); }
    const uint64_t x = take(T * maxk), y = take(T * maxn), dy = take(T * maxn), dx = take(T * maxk);
    const uint64_t xt = take(T * maxk), dyt = take(T * maxn), dw = take(maxw), wt = take(maxw);
    for (int layer = 0; layer < d.layers; ++layer) {
        for (int g = 0; g < 4; ++g) {
            const uint64_t w = take(n_out[g] * k_in[g]);
            if (!fill_lists) continue;
            l->fp.push_back({(int)T, (int)n_out[g], (int)k_in[g], x, w, y});
            // dX = dY[T, n] x (W^T)[k, n]^T : the B operand is K-contiguous when read from the transposed copy
            l->bp.push_back({(int)T, (int)k_in[g], (int)n_out[g], dy, wt, dx});
            // dW = (dY^T)[n, T] x (X^T)[k, T]^T
            l->bp.push_back({(int)n_out[g], (int)k_in[g], (int)T, dyt, xt, dw});
        }
    }
    return off;
}

int gemm_launch(const void* A, const void* B, void* C, int M, int N, int K, hipStream_t stream)
{
    const unsigned grid = (unsigned)((M / BM) * (N / BN));
    hipLaunchKernelGGL(k_gemm_bf16_nt, dim3(grid), dim3(kThreads), 0, stream, (const uint16_t*)A, (const uint16_t*)B,
                       (uint16_t*)C, M, N, K);
    return hipGetLastError() == hipSuccess ? FR_OK : FR_ERR_HIP;
}

// Part `part` of `parts` of a burst: the GEMMs of the layers [part * layers / parts, (part + 1) * layers / parts)
// (the list holds the layers one after the other, the same number of GEMMs each), or that share of a busy-wait.
int burst(fr_load* l, const std::vector<GemmShape>& list, uint64_t ns, hipStream_t stream, int part = 0, int parts = 1)
{
    if (parts < 1 || part < 0 || part >= parts) return FR_ERR_ARG;
    if (l->d.kind == FR_LOAD_BUSYWAIT) return fr_busywait_launch(ns / (uint64_t)parts, l->wall_clock_khz, stream);
    if (l->d.layers % parts != 0) return FR_ERR_ARG;
    const size_t per_layer = list.size() / (size_t)l->d.layers, layers = (size_t)l->d.layers / (size_t)parts;
    uint16_t* ws = static_cast<uint16_t*>(l->d.workspace);
    for (size_t i = (size_t)part * layers * per_layer; i < ((size_t)part + 1) * layers * per_layer; ++i) {
        const GemmShape& g = list[i];
        int rc = gemm_launch(ws + g.a_off, ws + g.b_off, ws + g.c_off, g.M, g.N, g.K, stream);
        if (rc != FR_OK) return rc;
    }
    return FR_OK;
}

}  // namespace

int fr_busywait_launch(uint64_t ns, int wall_clock_khz, hipStream_t stream)
{
    const uint64_t ticks = (uint64_t)((unsigned __int128)ns * (uint64_t)wall_clock_khz / 1000000ull);
    const uint64_t max_trips = ns / 20 + 4096;        // one trip takes well over 20 ns
    hipLaunchKernelGGL(k_busywait, dim3(1), dim3(64), 0, stream, ticks, max_trips);
    return hipGetLastError() == hipSuccess ? FR_OK : FR_ERR_HIP;
}

int fr_alufill_launch(uint64_t ns, int wall_clock_khz, uint32_t workgroups, hipStream_t stream)
{
    const uint64_t ticks = (uint64_t)((unsigned __int128)ns * (uint64_t)wall_clock_khz / 1000000ull);
    const uint64_t max_trips = ns / 50 + 4096;        // one trip (64 dependent fused multiply-adds) takes well over 50 ns
    hipLaunchKernelGGL(k_alu_fill, dim3(workgroups ? workgroups : 1), dim3(256), 0, stream, ticks, max_trips, (float*)nullptr);
    return hipGetLastError() == hipSuccess ? FR_OK : FR_ERR_HIP;
}

extern "C" {

int fr_gemm_bf16(const void* A, const void* B, void* C, int32_t M, int32_t N, int32_t K, void* stream)
{
    if (!A || !B || !C || M <= 0 || N <= 0 || K <= 0) return FR_ERR_ARG;
    if (M % 256 || N % 256 || K % 64) return FR_ERR_ARG;
    if (((uintptr_t)A | (uintptr_t)B | (uintptr_t)C) & 15) return FR_ERR_ARG;
    if ((uint64_t)(M / BM) * (uint64_t)(N / BN) > 0x7fffffffull) return FR_ERR_ARG;
    return gemm_launch(A, B, C, M, N, K, (hipStream_t)stream);
}

int fr_load_workspace_bytes(const fr_load_desc* d, uint64_t* bytes_out)
{
    if (!d || !bytes_out) return FR_ERR_ARG;
    if (d->kind == FR_LOAD_BUSYWAIT) { *bytes_out = 0; return FR_OK; }
    if (d->kind != FR_LOAD_GPT) return FR_ERR_ARG;
    if (d->layers < 1 || d->layers > 1024 || d->hidden < 256 || d->ffn < 256 || d->tokens < 256) return FR_ERR_ARG;
    if (d->hidden % 256 || d->ffn % 256 || d->tokens % 256) return FR_ERR_ARG;
    if (d->hidden > 65536 || d->ffn > 262144 || d->tokens > 1048576) return FR_ERR_ARG;
    fr_load tmp;
    tmp.d = *d;
    *bytes_out = plan_gpt(&tmp, false) * 2;
    return FR_OK;
}

int fr_load_make(const fr_load_desc* d, void* stream, fr_load** out)
{
    if (!d || !out) return FR_ERR_ARG;
    uint64_t need = 0;
    int rc = fr_load_workspace_bytes(d, &need);
    if (rc != FR_OK) return rc;
    fr_load* l = new (std::nothrow) fr_load();
    if (!l) return FR_ERR_ARG;
    l->d = *d;
    if (d->kind == FR_LOAD_BUSYWAIT) {
        if (d->fp_ns == 0 || d->bp_ns == 0 || d->fp_ns > 10000000000ull || d->bp_ns > 10000000000ull) { delete l; return FR_ERR_ARG; }
        int dev = 0, khz = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess || khz <= 0) {
            delete l;
            return FR_ERR_HIP;
        }
        l->wall_clock_khz = khz;
        *out = l;
        return FR_OK;
    }
    if (!d->workspace || d->workspace_bytes < need || ((uintptr_t)d->workspace & 255)) { delete l; return FR_ERR_ARG; }
    plan_gpt(l, true);
    for (const GemmShape& g : l->fp) l->fp_flops += 2ull * g.M * g.N * g.K;
    for (const GemmShape& g : l->bp) l->bp_flops += 2ull * g.M * g.N * g.K;
    hipLaunchKernelGGL(k_fill_bf16, dim3(4096), dim3(256), 0, (hipStream_t)stream, (uint16_t*)d->workspace, need / 2, d->seed);
    if (hipGetLastError() != hipSuccess || hipStreamSynchronize((hipStream_t)stream) != hipSuccess) { delete l; return FR_ERR_HIP; }
    *out = l;
    return FR_OK;
}

int fr_load_destroy(fr_load* l)
{
    if (!l) return FR_ERR_ARG;
    delete l;
    return FR_OK;
}

int fr_load_fp(fr_load* l, void* stream)
{
    if (!l) return FR_ERR_ARG;
    return burst(l, l->fp, l->d.fp_ns, (hipStream_t)stream);
}

int fr_load_bp(fr_load* l, void* stream)
{
    if (!l) return FR_ERR_ARG;
    return burst(l, l->bp, l->d.bp_ns, (hipStream_t)stream);
}

int fr_load_part(fr_load* l, void* stream, int32_t kind, int32_t part, int32_t parts)
{
    if (!l || (kind != 0 && kind != 1)) return FR_ERR_ARG;
    return kind == 0 ? burst(l, l->fp, l->d.fp_ns, (hipStream_t)stream, part, parts)
                     : burst(l, l->bp, l->d.bp_ns, (hipStream_t)stream, part, parts);
}

int fr_load_flops(fr_load* l, uint64_t* fp, uint64_t* bp)
{
    if (!l || !fp || !bp) return FR_ERR_ARG;
    *fp = l->fp_flops;
    *bp = l->bp_flops;
    return FR_OK;
}

}  // extern "C"
