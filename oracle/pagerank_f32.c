/*
 * The timed CPU baseline of the PageRank side task: the same power iteration as pagerank.c (textbook pull form,
 * exactly K Jacobi iterations, dangling mass spread uniformly; the paper's Section 6.1.4 names the task, Section
 * 6.2 its unit of work, one iteration = one pass over the graph, and Table 1 reports such a CPU column), with the
 * ranks and the row sums in fp32 and the rows dealt to threads.  TEST INFRASTRUCTURE ONLY, like everything under
 * oracle/: it is what bench.py times on the host's cores (one thread and all of them); the parity authority is the
 * fp64 file, and this one is pinned against it and against the ring and star closed forms.
 *
 *     r_0[v]     = 1 / V
 *     D_k        = sum of r_k[u] over vertices u with no out-edges           (added up in fp64: one scalar)
 *     base_k     = (1 - d) / V + d * D_k / V
 *     r_{k+1}[v] = base_k + d * sum over in-edges (u -> v) of r_k[u] / outdeg[u]      (fp32, sequential per row)
 *
 * Each row is summed sequentially in CSR order, so the result does not depend on the number of threads.
 */
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/*
 * row_ptr[V + 1], col[E]: in-edge CSR (col holds sources).  outdeg[V]: out-degrees.  ranks_out[V]: r_K (fp32).
 * n_threads <= 0 means "all available".  Returns the number of threads used (>= 1), -1 on bad arguments, -2 on
 * allocation failure.
 */
int oracle_pagerank_fp32(int64_t V, const int32_t *row_ptr, const int32_t *col, const int32_t *outdeg,
                         float damping, int iterations, int n_threads, float *ranks_out)
{
    if (V <= 0 || iterations < 0 || !row_ptr || !outdeg || !ranks_out) return -1;
    float *r = (float *)malloc(sizeof(float) * (size_t)V);
    float *q = (float *)malloc(sizeof(float) * (size_t)V);     /* r[u] / outdeg[u], 0 if dangling */
    float *rn = (float *)malloc(sizeof(float) * (size_t)V);
    if (!r || !q || !rn) { free(r); free(q); free(rn); return -2; }
    int used = 1;
#ifdef _OPENMP
    if (n_threads <= 0) n_threads = omp_get_max_threads();
    used = n_threads;
#else
    (void)n_threads;
#endif
    for (int64_t v = 0; v < V; ++v) r[v] = 1.0f / (float)V;

    for (int k = 0; k < iterations; ++k) {
        double dangling = 0.0;
#pragma omp parallel for schedule(static) num_threads(used) reduction(+ : dangling)
        for (int64_t u = 0; u < V; ++u) {
            if (outdeg[u] == 0) { dangling += (double)r[u]; q[u] = 0.0f; }
            else q[u] = r[u] / (float)outdeg[u];
        }
        const float base = (float)((1.0 - (double)damping) / (double)V + (double)damping * dangling / (double)V);
#pragma omp parallel for schedule(dynamic, 4096) num_threads(used)
        for (int64_t v = 0; v < V; ++v) {
            float s = 0.0f;
            for (int64_t j = row_ptr[v]; j < row_ptr[v + 1]; ++j) s += q[col[j]];
            rn[v] = base + damping * s;
        }
        float *t = r; r = rn; rn = t;
    }
    for (int64_t v = 0; v < V; ++v) ranks_out[v] = r[v];
    free(r); free(q); free(rn);
    return used;
}
