/*
 * TEST INFRASTRUCTURE ONLY -- plain float64 reference ("oracle") for probabilistic-circuit
 * forward pass, PC flows and the EM update.  Nothing in the product path may call this file;
 * it shares no code, headers or tables with the GPU library.
 *
 * The circuit is handed over as a DAG of node blocks (K node slots per block), but every
 * function below works node by node, edge by edge, straight from the definitions:
 *   forward   Def. 1 / Eq. (1): input = f_n(x), product = product of children, sum = weighted
 *             sum of children; evaluated in log space (Sec. 3), marginalised variables give
 *             probability 1 (Sec. 2).
 *   backward  Def. 2: root flow 1; sum/input nodes add their parents' flows; a product node c
 *             receives theta_{n,c} p_c / p_n F_n from every sum parent n; the edge flow
 *             F_{n,c} = theta_{n,c} p_c / p_n F_n is accumulated over the batch per parameter
 *             (tied edges share one accumulator, App. A.3).
 *   EM        theta_new = normalised accumulated flows; theta <- (1-a) theta + a theta_new
 *             (Sec. 2, App. C.3).  The paper does not print theta_new; the normalised-flow
 *             form with an optional pseudocount is the reading used here.
 *
 * Node (u, k) = node k of block u has index u*K + k.  Sum edge e = (u -> c) with parameter
 * block p: weight of (u,i) -> (c,j) is theta[(p+1)*K*K + i*K + j] (block 0 of theta is unused
 * padding).  Product block u: node (u,k) has children (c,k) for every child block c.
 * Input block u on variable v with table t: f(x) = tables[(t*n_cats + x_v)*K + k]; a value x_v
 * outside 0..n_cats-1 has f(x) = 0, so the sample's likelihood is 0 and (every node on a path
 * from the root has that variable in its scope, hence probability 0, and a sum node of
 * probability 0 passes no flow on) the sample adds nothing to any accumulated flow.
 *
 * Parallelism: OpenMP over samples (forward, node flows) or over the row index inside a
 * block (parameter flows), so no two threads ever add into the same accumulator.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { T_INPUT = 0, T_PRODUCT = 1, T_SUM = 2 };

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Children-before-parents order of the blocks (iterative depth-first post-order).
 * Returns 0, or -1 if the DAG has a cycle. */
int orc_topo_order(int32_t n_blocks, const int64_t *child_ptr, const int32_t *child, int32_t *order)
{
    uint8_t *state = (uint8_t *)calloc((size_t)n_blocks, 1);      /* 0 new, 1 open, 2 done */
    int32_t *stack = (int32_t *)malloc(sizeof(int32_t) * (size_t)n_blocks);
    int64_t *next = (int64_t *)malloc(sizeof(int64_t) * (size_t)n_blocks);
    int32_t n_out = 0, rc = 0;
    for (int32_t s = 0; s < n_blocks && rc == 0; ++s) {
        if (state[s]) continue;
        int32_t top = 0;
        stack[0] = s; state[s] = 1; next[s] = child_ptr[s];
        while (top >= 0) {
            int32_t u = stack[top];
            if (next[u] < child_ptr[u + 1]) {
                int32_t c = child[next[u]++];
                if (state[c] == 1) { rc = -1; break; }
                if (state[c] == 0) { state[c] = 1; next[c] = child_ptr[c]; stack[++top] = c; }
            } else {
                state[u] = 2; order[n_out++] = u; --top;
            }
        }
    }
    free(state); free(stack); free(next);
    return rc;
}

static double log_add_terms(const double *t, int64_t n)
{
    /* log sum_i exp(t_i), -inf when every term is -inf */
    double m = -INFINITY;
    for (int64_t i = 0; i < n; ++i) if (t[i] > m) m = t[i];
    if (m == -INFINITY) return -INFINITY;
    double s = 0.0;
    for (int64_t i = 0; i < n; ++i) s += exp(t[i] - m);
    return m + log(s);
}

/* Forward pass.  lp: [B][n_blocks*K] log-probability of every node; ll: [B] root (node 0 of
 * root_block).  mask (may be NULL): mask[b*n_vars+v] != 0 marginalises variable v in sample b. */
int orc_forward(int32_t K, int32_t n_blocks, int32_t root_block, const uint8_t *type,
                const int64_t *child_ptr, const int32_t *child, const int32_t *param_blk,
                const int32_t *in_var, const int32_t *in_table, int32_t n_vars, int32_t n_cats,
                const float *theta, const float *tables, const int32_t *x, const uint8_t *mask,
                int32_t B, double *lp, double *ll)
{
    int32_t *order = (int32_t *)malloc(sizeof(int32_t) * (size_t)n_blocks);
    if (orc_topo_order(n_blocks, child_ptr, child, order) != 0) { free(order); return -1; }
    const int64_t n_nodes = (int64_t)n_blocks * K;
    int64_t max_deg = 1;
    for (int32_t u = 0; u < n_blocks; ++u)
        if (child_ptr[u + 1] - child_ptr[u] > max_deg) max_deg = child_ptr[u + 1] - child_ptr[u];

#pragma omp parallel
    {
        double *terms = (double *)malloc(sizeof(double) * (size_t)(max_deg * K));
#pragma omp for schedule(dynamic, 1)
        for (int32_t b = 0; b < B; ++b) {
            double *L = lp + (int64_t)b * n_nodes;
            for (int32_t o = 0; o < n_blocks; ++o) {
                const int32_t u = order[o];
                const int64_t e0 = child_ptr[u], e1 = child_ptr[u + 1];
                for (int32_t k = 0; k < K; ++k) {
                    double v;
                    if (type[u] == T_INPUT) {
                        const int32_t var = in_var[u];
                        if (mask && mask[(int64_t)b * n_vars + var]) {
                            v = 0.0;                                   /* marginalised: p = 1 */
                        } else {
                            const int32_t xv = x[(int64_t)b * n_vars + var];
                            /* a value outside 0..n_cats-1 is outside the support of the categorical
                             * distribution: f(x) = 0 (Def. 1 with f_n a probability mass function) */
                            v = (xv < 0 || xv >= n_cats) ? -INFINITY
                                : log((double)tables[((int64_t)in_table[u] * n_cats + xv) * K + k]);
                        }
                    } else if (type[u] == T_PRODUCT) {
                        v = 0.0;
                        for (int64_t e = e0; e < e1; ++e) v += L[(int64_t)child[e] * K + k];
                    } else {
                        int64_t n = 0;
                        for (int64_t e = e0; e < e1; ++e) {
                            const float *th = theta + ((int64_t)param_blk[e] + 1) * K * K + (int64_t)k * K;
                            const double *Lc = L + (int64_t)child[e] * K;
                            for (int32_t j = 0; j < K; ++j)
                                if (th[j] > 0.0f && Lc[j] > -INFINITY)
                                    terms[n++] = log((double)th[j]) + Lc[j];
                        }
                        v = log_add_terms(terms, n);
                    }
                    L[(int64_t)u * K + k] = v;
                }
            }
            ll[b] = L[(int64_t)root_block * K];
        }
        free(terms);
    }
    free(order);
    return 0;
}

/* Node flows.  flow: [B][n_blocks*K] (overwritten).  Needs lp from orc_forward on the same inputs. */
int orc_node_flows(int32_t K, int32_t n_blocks, int32_t root_block, const uint8_t *type,
                   const int64_t *child_ptr, const int32_t *child, const int32_t *param_blk,
                   const float *theta, int32_t B, const double *lp, double *flow)
{
    int32_t *order = (int32_t *)malloc(sizeof(int32_t) * (size_t)n_blocks);
    if (orc_topo_order(n_blocks, child_ptr, child, order) != 0) { free(order); return -1; }
    const int64_t n_nodes = (int64_t)n_blocks * K;

#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t b = 0; b < B; ++b) {
        const double *L = lp + (int64_t)b * n_nodes;
        double *F = flow + (int64_t)b * n_nodes;
        for (int64_t i = 0; i < n_nodes; ++i) F[i] = 0.0;
        if (L[(int64_t)root_block * K] > -INFINITY) F[(int64_t)root_block * K] = 1.0;
        for (int32_t o = n_blocks - 1; o >= 0; --o) {               /* parents before children */
            const int32_t u = order[o];
            if (type[u] == T_INPUT) continue;
            for (int32_t k = 0; k < K; ++k) {
                const double Fn = F[(int64_t)u * K + k];
                if (Fn == 0.0) continue;
                const double Ln = L[(int64_t)u * K + k];
                for (int64_t e = child_ptr[u]; e < child_ptr[u + 1]; ++e) {
                    if (type[u] == T_PRODUCT) {
                        F[(int64_t)child[e] * K + k] += Fn;
                    } else {
                        if (Ln == -INFINITY) continue;
                        const float *th = theta + ((int64_t)param_blk[e] + 1) * K * K + (int64_t)k * K;
                        for (int32_t j = 0; j < K; ++j) {
                            const double Lc = L[(int64_t)child[e] * K + j];
                            if (th[j] > 0.0f && Lc > -INFINITY)
                                F[(int64_t)child[e] * K + j] += exp(log((double)th[j]) + Lc - Ln) * Fn;
                        }
                    }
                }
            }
        }
    }
    free(order);
    return 0;
}

/* Parameter flows, summed over the batch and ADDED into theta_flow [(n_param_blocks+1)*K*K]
 * and table_flow [n_tables*n_cats*K]. */
int orc_param_flows(int32_t K, int32_t n_blocks, const uint8_t *type,
                    const int64_t *child_ptr, const int32_t *child, const int32_t *param_blk,
                    const int32_t *in_var, const int32_t *in_table, int32_t n_vars, int32_t n_cats,
                    const float *theta, const int32_t *x, const uint8_t *mask, int32_t B,
                    const double *lp, const double *flow, double *theta_flow, double *table_flow)
{
    const int64_t n_nodes = (int64_t)n_blocks * K;
#pragma omp parallel for schedule(static)
    for (int32_t k = 0; k < K; ++k) {                               /* row k of every block */
        for (int32_t u = 0; u < n_blocks; ++u) {
            for (int32_t b = 0; b < B; ++b) {
                const double *L = lp + (int64_t)b * n_nodes;
                const double Fn = flow[(int64_t)b * n_nodes + (int64_t)u * K + k];
                if (Fn == 0.0) continue;
                if (type[u] == T_INPUT) {
                    const int32_t var = in_var[u];
                    if (mask && mask[(int64_t)b * n_vars + var]) continue;
                    const int32_t xv = x[(int64_t)b * n_vars + var];
                    if (xv < 0 || xv >= n_cats) continue;               /* p(x) = 0: no table entry to credit */
                    table_flow[((int64_t)in_table[u] * n_cats + xv) * K + k] += Fn;
                } else if (type[u] == T_SUM) {
                    const double Ln = L[(int64_t)u * K + k];
                    if (Ln == -INFINITY) continue;
                    for (int64_t e = child_ptr[u]; e < child_ptr[u + 1]; ++e) {
                        const int64_t off = ((int64_t)param_blk[e] + 1) * K * K + (int64_t)k * K;
                        for (int32_t j = 0; j < K; ++j) {
                            const double Lc = L[(int64_t)child[e] * K + j];
                            if (theta[off + j] > 0.0f && Lc > -INFINITY)
                                theta_flow[off + j] += exp(log((double)theta[off + j]) + Lc - Ln) * Fn;
                        }
                    }
                }
            }
        }
    }
    return 0;
}

/* EM update in place (theta, tables are fp32 like the GPU's; arithmetic in double).
 * Sum node (u,i): Z = sum of its accumulated edge flows, n_ch = number of real children;
 *   new = (G + pc/n_ch) / (Z + pc);  theta <- (1-a) theta + a new;   unchanged if Z + pc == 0.
 * Entries in placeholder rows / columns (i >= n_real[u] or j >= n_real[child]) stay untouched.
 * Sum blocks that share parameter blocks (tying) are updated once.
 * Table column (t,k): same over categories with n_ch = n_cats.  Flows are zeroed afterwards. */
int orc_em_step(int32_t K, int32_t n_blocks, const uint8_t *type, const int32_t *n_real,
                const int64_t *child_ptr, const int32_t *child, const int32_t *param_blk,
                int32_t n_param_blocks, int32_t n_cats, int32_t n_tables,
                float *theta, float *tables, double *theta_flow, double *table_flow,
                double step, double pseudocount)
{
    uint8_t *done = (uint8_t *)calloc((size_t)n_param_blocks + 1, 1);
    for (int32_t u = 0; u < n_blocks; ++u) {
        if (type[u] != T_SUM || child_ptr[u] == child_ptr[u + 1]) continue;
        if (done[param_blk[child_ptr[u]] + 1]) continue;
        for (int32_t i = 0; i < n_real[u]; ++i) {
            double Z = 0.0; int64_t n_ch = 0;
            for (int64_t e = child_ptr[u]; e < child_ptr[u + 1]; ++e) {
                const int64_t off = ((int64_t)param_blk[e] + 1) * K * K + (int64_t)i * K;
                for (int32_t j = 0; j < n_real[child[e]]; ++j) { Z += theta_flow[off + j]; ++n_ch; }
            }
            if (Z + pseudocount <= 0.0) continue;
            for (int64_t e = child_ptr[u]; e < child_ptr[u + 1]; ++e) {
                const int64_t off = ((int64_t)param_blk[e] + 1) * K * K + (int64_t)i * K;
                for (int32_t j = 0; j < n_real[child[e]]; ++j) {
                    const double nw = (theta_flow[off + j] + pseudocount / (double)n_ch) / (Z + pseudocount);
                    theta[off + j] = (float)((1.0 - step) * (double)theta[off + j] + step * nw);
                }
            }
        }
        for (int64_t e = child_ptr[u]; e < child_ptr[u + 1]; ++e) done[param_blk[e] + 1] = 1;
    }
    free(done);
    for (int32_t t = 0; t < n_tables; ++t)
        for (int32_t k = 0; k < K; ++k) {
            double Z = 0.0;
            for (int32_t c = 0; c < n_cats; ++c) Z += table_flow[((int64_t)t * n_cats + c) * K + k];
            if (Z + pseudocount <= 0.0) continue;
            for (int32_t c = 0; c < n_cats; ++c) {
                const int64_t off = ((int64_t)t * n_cats + c) * K + k;
                const double nw = (table_flow[off] + pseudocount / (double)n_cats) / (Z + pseudocount);
                tables[off] = (float)((1.0 - step) * (double)tables[off] + step * nw);
            }
        }
    memset(theta_flow, 0, sizeof(double) * (size_t)(n_param_blocks + 1) * K * K);
    memset(table_flow, 0, sizeof(double) * (size_t)n_tables * n_cats * K);
    return 0;
}
