/*
 * CPU oracle for the PageRank side task.  TEST INFRASTRUCTURE ONLY: nothing on the
 * product path may call this; it exists so that tests, the smoke check and the
 * benchmark's CPU-baseline leg have an independent answer to compare with.
 *
 * What it computes.  The paper names the side task (Section 6.1.4: graph analytics,
 * PageRank; Section 6.2: one iteration = one pass of the algorithm over the input
 * graph) but not its arithmetic, so this is the textbook power iteration
 * (Page, Brin, Motwani, Winograd 1999) in pull form, in fp64, written out plainly:
 *
 *     r_0[v]     = 1 / V
 *     D_k        = sum of r_k[u] over vertices u with no out-edges
 *     base_k     = (1 - d) / V + d * D_k / V
 *     r_{k+1}[v] = base_k + d * sum over in-edges (u -> v) of r_k[u] / outdeg[u]
 *
 * for exactly K iterations (no convergence test), Jacobi style: iteration k + 1 reads
 * only iteration k.  Dangling mass is spread uniformly, which keeps sum(r) = 1.
 * Multi-edges and self-loops count with multiplicity.  Row sums run sequentially in
 * CSR order.  The quotient r_k[u] / outdeg[u] is formed once per vertex and reused for
 * every edge leaving u; that is the same fp64 value the per-edge division would give.
 *
 * The loop over rows may run on several threads (rows are independent, each row is
 * still summed sequentially, so the result does not depend on the thread count).
 *
 * Pinned by tests against closed forms (ring, three kinds of star), sum(r) = 1,
 * dense Google-matrix powers on 8-vertex graphs and a dense eigen-solver.
 */
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/*
 * row_ptr[V + 1], col[E]: in-edge CSR (col holds sources).  outdeg[V]: out-degrees.
 * ranks_out[V]: r_K.  n_threads <= 0 means "all available".
 * Returns the number of threads used (>= 1), or -1 on bad arguments, -2 on allocation failure.
 */
int oracle_pagerank_fp64(int64_t V, const int32_t *row_ptr, const int32_t *col, const int32_t *outdeg,
                         double damping, int iterations, int n_threads, double *ranks_out)
{
    if (V <= 0 || iterations < 0 || !row_ptr || !outdeg || !ranks_out) return -1;
    double *r = (double *)malloc(sizeof(double) * (size_t)V);
    double *q = (double *)malloc(sizeof(double) * (size_t)V);   /* r[u] / outdeg[u], 0 if dangling */
    double *rn = (double *)malloc(sizeof(double) * (size_t)V);
    if (!r || !q || !rn) { free(r); free(q); free(rn); return -2; }
    int used = 1;
#ifdef _OPENMP
    if (n_threads <= 0) n_threads = omp_get_max_threads();
    used = n_threads;
#else
    (void)n_threads;
#endif
    for (int64_t v = 0; v < V; ++v) r[v] = 1.0 / (double)V;

    for (int k = 0; k < iterations; ++k) {
        double dangling = 0.0;
        for (int64_t u = 0; u < V; ++u) {
            if (outdeg[u] == 0) { dangling += r[u]; q[u] = 0.0; }
            else q[u] = r[u] / (double)outdeg[u];
        }
        const double base = (1.0 - damping) / (double)V + damping * dangling / (double)V;
#pragma omp parallel for schedule(dynamic, 4096) num_threads(used)
        for (int64_t v = 0; v < V; ++v) {
            double s = 0.0;
            for (int64_t j = row_ptr[v]; j < row_ptr[v + 1]; ++j) s += q[col[j]];
            rn[v] = base + damping * s;
        }
        double *t = r; r = rn; rn = t;
    }
    for (int64_t v = 0; v < V; ++v) ranks_out[v] = r[v];
    free(r); free(q); free(rn);
    return used;
}
