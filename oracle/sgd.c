/*
 * CPU oracle for the Graph SGD side task.  TEST INFRASTRUCTURE ONLY: nothing on the
 * product path may call this.
 *
 * What it computes.  The paper names the side task (Section 6.1.4: graph analytics,
 * "Graph SGD", stochastic gradient descent for matrix factorization after Koren, Bell
 * and Volinsky 2009; Section 6.2: one iteration = one pass over the input graph) but
 * neither its arithmetic nor the order of its updates, so this is the textbook method:
 * ratings r_ui on the edges (u, i) of a bipartite graph, factors p_u, q_i of F numbers
 * each, and for every rating, one after the other,
 *
 *     e    = r_ui - <p_u, q_i>
 *     p_u' = p_u + gamma * (e * q_i - lambda * p_u)
 *     q_i' = q_i + gamma * (e * p_u - lambda * q_i)        (both from the old p_u, q_i)
 *
 * i.e. a step of length gamma down the gradient of
 *     1/2 (r_ui - <p_u, q_i>)^2 + lambda/2 (|p_u|^2 + |q_i|^2).
 *
 * Order of the updates (the paper is silent; a parallel machine needs one that does not
 * depend on timing).  Stratified SGD (Gemulla, Nijkamp, Haas, Sismanis 2011): users and
 * items are cut into B blocks of consecutive ids holding about E / B ratings each - user
 * block k begins at the first user with ceil(k E / B) or more ratings before it, item
 * block k at the first item with that many ratings of smaller items, block 0 at id 0 (a
 * block may be empty) - and the ratings of user block a and item block b form cell (a, b).
 * One iteration
 * is B strata; stratum s holds the cells (a, (a + s) mod B), a = 0 .. B - 1, no two of
 * which share a user or an item.  Here the cells of a stratum are taken in order of a,
 * and inside a cell the ratings by user and then by item; since the cells of a stratum
 * touch disjoint factors, any interleaving of them gives the same result, which is what
 * lets a GPU run them side by side.
 *
 * Two entry points:
 *   oracle_sgd_fp64          the formulas above as written, in double.
 *   oracle_sgd_fp32_ordered  the same steps in float with every rounding pinned down, so
 *                            that an fp32 implementation can be compared bit for bit:
 *                              t_l  = p_l * q_l                      (rounded products)
 *                              dot  = tree sum of t over l: F a power of two; in round
 *                                     w = 1, 2, 4, .. every t_l becomes t_l + t_(l xor w)
 *                              e    = r - dot,  ge = gamma * e,  gl = gamma * lambda
 *                              p_l' = fma(ge, q_l, fma(-gl, p_l, p_l))
 *                              q_l' = fma(ge, p_l, fma(-gl, q_l, q_l))
 *                            (compile without floating-point contraction).
 *
 * Pinned by tests: a hand-worked update, the gradient of the objective by finite
 * differences, exact low-rank ratings as a fixed point, the visiting order against a
 * brute-force enumeration with block starts computed independently, and fp32 against
 * fp64.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* Calls visit(ctx, u, e) for every rating e of user u in the order defined above.  Items inside a row of the
   CSR must ascend. */
typedef void (*visit_fn)(void* ctx, int64_t u, int64_t e);

/* starts[k], k = 0 .. B: first id of block k; before[x] = ratings of the ids below x, x = 0 .. n. */
static void block_starts(int64_t n, const int64_t* before, int64_t E, int32_t B, int64_t* starts)
{
    int64_t x = 0;
    starts[0] = 0;
    for (int32_t k = 1; k < B; ++k) {
        const int64_t want = ((int64_t)k * E + B - 1) / B;
        while (x < n && before[x] < want) ++x;
        starts[k] = x;
    }
    starts[B] = n;
}

static int make_blocks(int64_t U, int64_t I, const int32_t* row_ptr, const int32_t* item, int32_t B, int64_t* ustart,
                       int64_t* istart)
{
    const int64_t E = row_ptr[U];
    int64_t* before = (int64_t*)calloc((size_t)((U > I ? U : I) + 2), sizeof(int64_t));
    if (!before) return -3;
    for (int64_t u = 0; u <= U; ++u) before[u] = row_ptr[u];
    block_starts(U, before, E, B, ustart);
    for (int64_t i = 0; i <= I; ++i) before[i] = 0;
    for (int64_t e = 0; e < E; ++e) before[item[e] + 1]++;
    for (int64_t i = 0; i < I; ++i) before[i + 1] += before[i];
    block_starts(I, before, E, B, istart);
    free(before);
    return 0;
}

static int for_each_rating(int64_t U, int64_t I, const int32_t* row_ptr, const int32_t* item, int32_t B, visit_fn visit,
                           void* ctx)
{
    if (U < 1 || I < 1 || B < 1) return -1;
    int64_t* ustart = (int64_t*)malloc(sizeof(int64_t) * 2 * ((size_t)B + 1));
    if (!ustart) return -3;
    int64_t* istart = ustart + B + 1;
    if (make_blocks(U, I, row_ptr, item, B, ustart, istart) != 0) { free(ustart); return -3; }
    for (int32_t s = 0; s < B; ++s) {
        for (int32_t a = 0; a < B; ++a) {
            const int32_t b = (int32_t)(((int64_t)a + s) % B);
            const int64_t i0 = istart[b], i1 = istart[b + 1];
            for (int64_t u = ustart[a]; u < ustart[a + 1]; ++u) {
                int64_t lo = row_ptr[u], hi = row_ptr[u + 1];       /* first rating of the row with item >= i0 */
                while (lo < hi) {
                    const int64_t mid = (lo + hi) / 2;
                    if (item[mid] < i0) lo = mid + 1;
                    else hi = mid;
                }
                for (int64_t e = lo; e < row_ptr[u + 1] && item[e] < i1; ++e) visit(ctx, u, e);
            }
        }
    }
    free(ustart);
    return 0;
}

/* ---- the blocks alone (for the tests) ---- */
int oracle_sgd_blocks(int64_t U, int64_t I, const int32_t* row_ptr, const int32_t* item, int32_t B, int64_t* ustart,
                      int64_t* istart)
{
    if (U < 1 || I < 1 || B < 1) return -1;
    return make_blocks(U, I, row_ptr, item, B, ustart, istart);
}

/* ---- the order alone (for the tests of the order) ---- */
struct order_ctx { int64_t* out; int64_t n; };
static void visit_order(void* c, int64_t u, int64_t e)
{
    struct order_ctx* o = (struct order_ctx*)c;
    (void)u;
    o->out[o->n++] = e;
}
int oracle_sgd_order(int64_t U, int64_t I, const int32_t* row_ptr, const int32_t* item, int32_t B, int64_t* order_out)
{
    struct order_ctx o = {order_out, 0};
    if (for_each_rating(U, I, row_ptr, item, B, visit_order, &o) != 0) return -1;
    return o.n == row_ptr[U] ? 0 : -2;
}

/* ---- fp64 ---- */
struct sgd64 { const int32_t* item; const float* rating; int32_t F; double gamma, lambda; double *P, *Q; };
static void visit64(void* c, int64_t u, int64_t e)
{
    struct sgd64* g = (struct sgd64*)c;
    double* p = g->P + u * g->F;
    double* q = g->Q + (int64_t)g->item[e] * g->F;
    double dot = 0.0;
    for (int32_t l = 0; l < g->F; ++l) dot += p[l] * q[l];
    const double err = (double)g->rating[e] - dot;
    for (int32_t l = 0; l < g->F; ++l) {
        const double pl = p[l], ql = q[l];
        p[l] = pl + g->gamma * (err * ql - g->lambda * pl);
        q[l] = ql + g->gamma * (err * pl - g->lambda * ql);
    }
}
int oracle_sgd_fp64(int64_t U, int64_t I, const int32_t* row_ptr, const int32_t* item, const float* rating, int32_t F,
                    double gamma, double lambda, int32_t K, int32_t B, double* P, double* Q)
{
    struct sgd64 g = {item, rating, F, gamma, lambda, P, Q};
    if (F < 1 || K < 0) return -1;
    for (int32_t k = 0; k < K; ++k)
        if (for_each_rating(U, I, row_ptr, item, B, visit64, &g) != 0) return -1;
    return 0;
}

/* ---- fp32, every rounding as stated in the header ---- */
struct sgd32 { const int32_t* item; const float* rating; int32_t F; float gamma, gl; float *P, *Q; float* t; };
static void visit32(void* c, int64_t u, int64_t e)
{
    struct sgd32* g = (struct sgd32*)c;
    float* p = g->P + u * g->F;
    float* q = g->Q + (int64_t)g->item[e] * g->F;
    float* t = g->t;
    float* t2 = g->t + g->F;
    for (int32_t l = 0; l < g->F; ++l) t[l] = p[l] * q[l];
    for (int32_t w = 1; w < g->F; w <<= 1) {
        for (int32_t l = 0; l < g->F; ++l) t2[l] = t[l] + t[l ^ w];
        memcpy(t, t2, sizeof(float) * (size_t)g->F);
    }
    const float err = g->rating[e] - t[0];
    const float ge = g->gamma * err;
    for (int32_t l = 0; l < g->F; ++l) {
        const float pl = p[l], ql = q[l];
        p[l] = fmaf(ge, ql, fmaf(-g->gl, pl, pl));
        q[l] = fmaf(ge, pl, fmaf(-g->gl, ql, ql));
    }
}
int oracle_sgd_fp32_ordered(int64_t U, int64_t I, const int32_t* row_ptr, const int32_t* item, const float* rating,
                            int32_t F, float gamma, float lambda, int32_t K, int32_t B, float* P, float* Q)
{
    if (F < 1 || (F & (F - 1)) != 0 || K < 0) return -1;
    struct sgd32 g = {item, rating, F, gamma, gamma * lambda, P, Q, NULL};
    g.t = (float*)malloc(sizeof(float) * 2 * (size_t)F);
    if (!g.t) return -3;
    int rc = 0;
    for (int32_t k = 0; k < K && rc == 0; ++k) rc = for_each_rating(U, I, row_ptr, item, B, visit32, &g);
    free(g.t);
    return rc;
}
