/*
 * Seeded synthetic graph inputs: edge generators and the in-edge CSR builder.
 *
 * This file holds input construction only (random structure, sorting, counting).
 * None of PageRank's arithmetic and none of the schedule logic lives here; both the
 * CPU oracle's tests and the GPU path's tests draw their inputs from this module.
 *
 * Randomness is counter based: every draw is a pure function of (seed, edge index,
 * level), so any edge can be produced independently and in parallel, and two builds
 * from one seed give byte-identical arrays.  The 64-bit mixer is the SplitMix64
 * output function (Steele, Lea, Flood 2014; public domain reference by S. Vigna).
 *
 * Graphs stand in for the social graph the paper feeds its PageRank side task
 * (Section 6.1.4), which is not available here.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

static inline uint64_t mix64(uint64_t z)
{
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

/* Per-edge key: one mix of the seed stream, one of the edge index. */
static inline uint64_t edge_key(uint64_t seed, uint64_t stream, uint64_t i)
{
    return mix64(mix64(seed * 0xD1342543DE82EF95ull + stream) ^ (i * 0x9E3779B97F4A7C15ull));
}

/* 24-bit uniform integer for (key, level). */
static inline uint32_t draw24(uint64_t key, uint64_t level)
{
    return (uint32_t)(mix64(key + level * 0xA0761D6478BD642Full) >> 40);
}

/* Seeded bijection on [0, 2^scale): affine map with odd multiplier, an invertible
 * xor-shift, and a second affine map.  Scatters the R-MAT hubs over the id space. */
static inline uint32_t relabel(uint32_t x, int scale, uint64_t m1, uint64_t c1, uint64_t m2, uint64_t c2)
{
    if (scale == 0) return 0;
    const uint64_t mask = (scale >= 64) ? ~0ull : ((1ull << scale) - 1);
    uint64_t y = ((uint64_t)x * m1 + c1) & mask;
    int sh = (scale + 1) / 2;
    y ^= (y >> sh);
    y = (y * m2 + c2) & mask;
    return (uint32_t)y;
}

/*
 * R-MAT edges (Chakrabarti, Zhan, Faloutsos 2004): for each of `scale` bit levels one
 * uniform draw picks quadrant a / b / c / d; quadrants c and d set the source (row) bit,
 * b and d set the destination (column) bit.  No per-level noise.  When permute != 0 both
 * endpoints go through the seeded bijection.
 * Returns 0, or -1 on bad arguments.
 */
int wl_rmat_edges(int scale, int64_t n_edges, double a, double b, double c,
                  uint64_t seed, int permute, int32_t *src, int32_t *dst)
{
    if (scale < 0 || scale > 30 || n_edges < 0 || a < 0 || b < 0 || c < 0 || a + b + c > 1.0) return -1;
    const uint32_t ta = (uint32_t)ceil(a * 16777216.0);
    const uint32_t tb = (uint32_t)ceil((a + b) * 16777216.0);
    const uint32_t tc = (uint32_t)ceil((a + b + c) * 16777216.0);
    const uint64_t m1 = mix64(seed ^ 0x1111) | 1ull, c1 = mix64(seed ^ 0x2222);
    const uint64_t m2 = mix64(seed ^ 0x3333) | 1ull, c2 = mix64(seed ^ 0x4444);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_edges; ++i) {
        const uint64_t key = edge_key(seed, 1, (uint64_t)i);
        uint32_t u = 0, v = 0;
        for (int l = 0; l < scale; ++l) {
            const uint32_t x = draw24(key, (uint64_t)l);
            const uint32_t rbit = (x >= tb);                /* quadrants c, d */
            const uint32_t cbit = (x >= ta && x < tb) || (x >= tc); /* quadrants b, d */
            u = (u << 1) | rbit;
            v = (v << 1) | cbit;
        }
        if (permute) {
            u = relabel(u, scale, m1, c1, m2, c2);
            v = relabel(v, scale, m1, c1, m2, c2);
        }
        src[i] = (int32_t)u;
        dst[i] = (int32_t)v;
    }
    return 0;
}

/*
 * Fixed out-degree random graph: every vertex u emits exactly `degree` edges whose
 * destinations are independent and uniform on [0, n_vertices).  Edge index is
 * u * degree + slot.  Returns 0, or -1 on bad arguments.
 */
int wl_fixed_outdeg_edges(int64_t n_vertices, int degree, uint64_t seed, int32_t *src, int32_t *dst)
{
    if (n_vertices <= 0 || n_vertices > 0x7fffffffLL || degree < 0) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t u = 0; u < n_vertices; ++u) {
        const uint64_t key = edge_key(seed, 2, (uint64_t)u);
        for (int s = 0; s < degree; ++s) {
            const uint64_t h = mix64(key + (uint64_t)s * 0xA0761D6478BD642Full);
            const uint64_t t = (uint64_t)(((__uint128_t)h * (uint64_t)n_vertices) >> 64);
            src[u * degree + s] = (int32_t)u;
            dst[u * degree + s] = (int32_t)t;
        }
    }
    return 0;
}

/*
 * In-edge CSR of a directed edge list (u -> v): row v lists the sources of v's in-edges
 * in ascending source id, duplicates adjacent; multi-edges and self-loops are kept.
 * out_degree[u] counts edges leaving u with multiplicity.
 * Built as a two-pass stable counting sort: edges by source, then by destination.
 * row_ptr has n_vertices + 1 entries; col has n_edges entries.
 * Returns 0, -1 on bad arguments (including an endpoint out of range), -2 on allocation failure.
 */
int wl_build_in_csr(int64_t n_vertices, int64_t n_edges, const int32_t *src, const int32_t *dst,
                    int32_t *row_ptr, int32_t *col, int32_t *out_degree)
{
    if (n_vertices < 0 || n_edges < 0 || n_edges > 0x7fffffffLL || n_vertices > 0x7fffffffLL) return -1;
    for (int64_t i = 0; i < n_edges; ++i)
        if (src[i] < 0 || src[i] >= n_vertices || dst[i] < 0 || dst[i] >= n_vertices) return -1;

    int64_t *cursor = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n_vertices + 1));
    int32_t *by_src = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_edges > 0 ? n_edges : 1));
    if (!cursor || !by_src) { free(cursor); free(by_src); return -2; }

    memset(out_degree, 0, sizeof(int32_t) * (size_t)n_vertices);
    memset(row_ptr, 0, sizeof(int32_t) * (size_t)(n_vertices + 1));
    for (int64_t i = 0; i < n_edges; ++i) { out_degree[src[i]]++; row_ptr[dst[i] + 1]++; }
    for (int64_t v = 0; v < n_vertices; ++v) row_ptr[v + 1] += row_ptr[v];

    /* pass 1: destinations grouped by source, edge order kept inside a group */
    int64_t run = 0;
    for (int64_t u = 0; u < n_vertices; ++u) { cursor[u] = run; run += out_degree[u]; }
    for (int64_t i = 0; i < n_edges; ++i) by_src[cursor[src[i]]++] = dst[i];

    /* pass 2: walk sources in ascending order and append each to its destination's row */
    for (int64_t v = 0; v < n_vertices; ++v) cursor[v] = row_ptr[v];
    int64_t pos = 0;
    for (int64_t u = 0; u < n_vertices; ++u) {
        const int64_t end = pos + out_degree[u];
        for (; pos < end; ++pos) col[cursor[by_src[pos]]++] = (int32_t)u;
    }
    free(cursor);
    free(by_src);
    return 0;
}

/* 64-bit FNV-1a over a byte buffer: used by tests to fingerprint generated arrays. */
uint64_t wl_fnv1a(const void *data, int64_t n_bytes)
{
    const uint8_t *p = (const uint8_t *)data;
    uint64_t h = 0xcbf29ce484222325ull;
    for (int64_t i = 0; i < n_bytes; ++i) { h ^= p[i]; h *= 0x100000001b3ull; }
    return h;
}
