/*
 * CPU checker for graph-random-feature (GRF) masked linear attention.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * method computes, written from the paper (arXiv 2410.03462).  Only the tests, the
 * smoke check and the benchmark's "cpu_baseline" leg may call it.  It shares no code
 * with the HIP library and is never a fallback for it.
 *
 * Everything is single-threaded, fp64 accumulation, host pointers.
 *
 * Parity pins (see tests): Philox against the published known-answer vectors;
 * walks against the closed-form halting and transition laws; features against
 * dense matrix powers (exactly on degree-1 graphs, in expectation elsewhere);
 * factorised attention against the O(N^2) definition.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ Philox4x32-10
 * Counter-based generator of Salmon, Moraes, Dror, Shaw, "Parallel random numbers:
 * as easy as 1, 2, 3" (SC'11).  The paper does not name a generator; the walks
 * only need reproducible uniform 32-bit words keyed by (seed, node, walk).
 */
void grf_ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* ------------------------------------------------------------------ one halting walk
 * Sec. 3.3 (GRF definition) and Thm 3.1: a simple random walk out of `start` that,
 * before every hop, halts with probability p_halt and otherwise moves to a
 * uniformly chosen neighbour.  At most max_nodes nodes are visited (f vanishes
 * beyond index max_nodes-1, so later deposits would be multiplied by zero).
 *
 * For the prefix of t hops the importance weight is
 *     (product of traversed edge weights) / (probability of that prefix)
 *   = prod_s  W[u_s, u_{s+1}] * deg(u_s) / (1 - p_halt),
 * and 1 for the 0-hop prefix.
 *
 * Random stream: Philox counter (node, walk, block, 0), key (seed_lo, seed_hi).
 * Block b serves hops 2b+1 and 2b+2: words 0,1 are the (halt, neighbour) draws of
 * hop 2b+1, words 2,3 those of hop 2b+2.  halt iff draw < floor(p_halt * 2^32);
 * neighbour index = floor(draw * deg / 2^32).
 *
 * nodes[t], loads[t] for t < returned length.
 */
static int one_walk(const int32_t* row_ptr, const int32_t* col, const float* w,
                    int64_t start, int64_t walk, int max_nodes, double p_halt, uint64_t seed,
                    int32_t* nodes, double* loads)
{
    const uint64_t threshold = (uint64_t)floor(p_halt * 4294967296.0);
    const uint32_t key[2] = { (uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32) };
    uint32_t x[4] = {0, 0, 0, 0};
    int64_t u = start;
    double load = 1.0;
    int len = 0;
    nodes[len] = (int32_t)u; loads[len] = load; ++len;
    for (int t = 1; t < max_nodes; ++t) {
        const int64_t deg = (int64_t)row_ptr[u + 1] - (int64_t)row_ptr[u];
        if (deg == 0) break;
        const int within = (t - 1) & 1;
        if (within == 0) {
            const uint32_t ctr[4] = { (uint32_t)start, (uint32_t)walk, (uint32_t)((t - 1) >> 1), 0u };
            grf_ref_philox4x32_10(ctr, key, x);
        }
        const uint32_t draw_halt = x[2 * within];
        const uint32_t draw_nbr = x[2 * within + 1];
        if ((uint64_t)draw_halt < threshold) break;
        const int64_t pick = (int64_t)(((uint64_t)draw_nbr * (uint64_t)deg) >> 32);
        const int64_t e = (int64_t)row_ptr[u] + pick;
        load = load * (double)w[e] * (double)deg / (1.0 - p_halt);
        u = col[e];
        nodes[len] = (int32_t)u; loads[len] = load; ++len;
    }
    return len;
}

/* Trajectories only: traj[n][n_walks][max_nodes], -1 padded; loads_opt same shape or NULL. */
void grf_ref_sample_walks(int64_t n, const int32_t* row_ptr, const int32_t* col, const float* w,
                          double p_halt, int32_t n_walks, int32_t max_nodes, uint64_t seed,
                          int32_t* traj, double* loads_opt)
{
    int32_t* nodes = (int32_t*)malloc(sizeof(int32_t) * (size_t)max_nodes);
    double* loads = (double*)malloc(sizeof(double) * (size_t)max_nodes);
    for (int64_t i = 0; i < n; ++i)
        for (int32_t k = 0; k < n_walks; ++k) {
            const int len = one_walk(row_ptr, col, w, i, k, max_nodes, p_halt, seed, nodes, loads);
            int32_t* out = traj + ((size_t)i * n_walks + k) * max_nodes;
            for (int t = 0; t < max_nodes; ++t) out[t] = t < len ? nodes[t] : -1;
            if (loads_opt) {
                double* lo = loads_opt + ((size_t)i * n_walks + k) * max_nodes;
                for (int t = 0; t < max_nodes; ++t) lo[t] = t < len ? loads[t] : 0.0;
            }
        }
    free(nodes); free(loads);
}

/* ------------------------------------------------------------------ GRF rows, Eq. (GRF definition)
 *   phi_hat(v_i)_q = (1/n) * sum over walks k, over prefix subwalks ending at q, of
 *                    weight(prefix) * f[len(prefix)]
 * Every visited node is an entry of the row (kept even if its sum is 0).  Columns
 * ascending.  Sums are taken in (walk, hop) order in fp64 and rounded once to fp32.
 *
 * Two-call protocol: with col_out == NULL only row_ptr_out[n+1] is written and nnz
 * returned; otherwise col_out[nnz] and val_out[n_f][nnz] are filled as well.
 * f is [n_f][f_len]; all n_f value planes share one set of walks (the features are
 * linear in f).
 */
int64_t grf_ref_sample(int64_t n, const int32_t* row_ptr, const int32_t* col, const float* w,
                       const float* f, int32_t f_len, int32_t n_f,
                       double p_halt, int32_t n_walks, uint64_t seed,
                       int32_t* row_ptr_out, int32_t* col_out, float* val_out)
{
    const size_t cap = (size_t)n_walks * (size_t)f_len;
    int32_t* nodes = (int32_t*)malloc(sizeof(int32_t) * (size_t)f_len);
    double* loads = (double*)malloc(sizeof(double) * (size_t)f_len);
    int32_t* cols = (int32_t*)malloc(sizeof(int32_t) * cap);
    double* sums = (double*)malloc(sizeof(double) * cap * (size_t)n_f);
    int64_t nnz_total = (col_out == NULL) ? 0 : (int64_t)row_ptr_out[n];
    int64_t running = 0;
    for (int64_t i = 0; i < n; ++i) {
        size_t cnt = 0;
        for (int32_t k = 0; k < n_walks; ++k) {
            const int len = one_walk(row_ptr, col, w, i, k, f_len, p_halt, seed, nodes, loads);
            for (int t = 0; t < len; ++t) {
                size_t s = 0;
                while (s < cnt && cols[s] != nodes[t]) ++s;
                if (s == cnt) {
                    cols[cnt] = nodes[t];
                    for (int32_t h = 0; h < n_f; ++h) sums[cnt * n_f + h] = 0.0;
                    ++cnt;
                }
                for (int32_t h = 0; h < n_f; ++h)
                    sums[s * n_f + h] += loads[t] * (double)f[(size_t)h * f_len + t];
            }
        }
        if (col_out == NULL) {
            row_ptr_out[i] = (int32_t)running;
        } else {
            /* insertion sort of the row by column */
            for (size_t a = 1; a < cnt; ++a) {
                size_t b = a;
                while (b > 0 && cols[b - 1] > cols[b]) {
                    int32_t tc = cols[b]; cols[b] = cols[b - 1]; cols[b - 1] = tc;
                    for (int32_t h = 0; h < n_f; ++h) {
                        double tv = sums[b * n_f + h];
                        sums[b * n_f + h] = sums[(b - 1) * n_f + h];
                        sums[(b - 1) * n_f + h] = tv;
                    }
                    --b;
                }
            }
            for (size_t s = 0; s < cnt; ++s) {
                col_out[running + (int64_t)s] = cols[s];
                for (int32_t h = 0; h < n_f; ++h)
                    val_out[(size_t)h * (size_t)nnz_total + (size_t)running + s] =
                        (float)(sums[s * n_f + h] / (double)n_walks);
            }
        }
        running += (int64_t)cnt;
    }
    if (col_out == NULL) row_ptr_out[n] = (int32_t)running;
    free(nodes); free(loads); free(cols); free(sums);
    return running;
}

/* ------------------------------------------------------------------ feature map */
static inline double feature(float x, int32_t feature_map)
{
    /* 0: ReLU (the map used in the paper's experiments); 1: identity (tests only);
     * 2: elu(x) + 1, the deterministic map of the linear transformer that Sec. 2 and Alg. 1
     *    step 3 name as an alternative (the paper prints it as "elu(x)+x"; the cited work's
     *    map is elu(x)+1 = x+1 for x > 0 and exp(x) otherwise, which is what keeps it positive). */
    if (feature_map == 0) return x > 0.0f ? (double)x : 0.0;
    if (feature_map == 2) return x > 0.0f ? (double)x + 1.0 : exp((double)x);
    return (double)x;
}

/* d phi(x) / dx for the same maps (ReLU: 0 at x = 0). */
static inline double feature_grad(float x, int32_t feature_map)
{
    if (feature_map == 0) return x > 0.0f ? 1.0 : 0.0;
    if (feature_map == 2) return x > 0.0f ? 1.0 : exp((double)x);
    return 1.0;
}

/* ------------------------------------------------------------------ Alg. 1, step 5, first product
 * Block l of  Phi_{K,G}^T V  and of  Phi_{K,G}^T 1 :
 *     S_l = sum_j phi_hat(v_j)_l * phi(k_j) v_j^T   (m x d),     z_l = sum_j phi_hat(v_j)_l * phi(k_j)   (m)
 * with m = d for the elementwise feature maps used here.  One (batch, head) slice:
 * K, V are [n][d]; phi is CSR (row_ptr, col, val); S is [n][d][d] (feature index
 * first), z is [n][d]; both fp64, overwritten.  Contributors are met in ascending j.
 */
void grf_ref_buckets(int64_t n, int32_t d, const float* K, const float* V,
                     const int32_t* phi_row_ptr, const int32_t* phi_col, const float* phi_val,
                     int32_t feature_map, double* S, double* z)
{
    memset(S, 0, sizeof(double) * (size_t)n * d * d);
    memset(z, 0, sizeof(double) * (size_t)n * d);
    for (int64_t j = 0; j < n; ++j)
        for (int64_t e = phi_row_ptr[j]; e < phi_row_ptr[j + 1]; ++e) {
            const int64_t l = phi_col[e];
            const double g = (double)phi_val[e];
            double* Sl = S + (size_t)l * d * d;
            double* zl = z + (size_t)l * d;
            for (int32_t a = 0; a < d; ++a) {
                const double ka = g * feature(K[j * d + a], feature_map);
                zl[a] += ka;
                for (int32_t b = 0; b < d; ++b) Sl[a * d + b] += ka * (double)V[j * d + b];
            }
        }
}

/* ------------------------------------------------------------------ Alg. 1, step 5, second product and D
 *     num_i = sum_l phi_hat(v_i)_l * phi(q_i)^T S_l   (d),     den_i = sum_l phi_hat(v_i)_l * phi(q_i)^T z_l
 * fp64, l ascending.  The attention output is num_i / den_i (no epsilon: Eq. 12 has none).
 */
void grf_ref_gather(int64_t n, int32_t d, const float* Q,
                    const int32_t* phi_row_ptr, const int32_t* phi_col, const float* phi_val,
                    int32_t feature_map, const double* S, const double* z,
                    double* num, double* den)
{
    for (int64_t i = 0; i < n; ++i) {
        double* ni = num + (size_t)i * d;
        for (int32_t b = 0; b < d; ++b) ni[b] = 0.0;
        double di = 0.0;
        for (int64_t e = phi_row_ptr[i]; e < phi_row_ptr[i + 1]; ++e) {
            const int64_t l = phi_col[e];
            const double g = (double)phi_val[e];
            const double* Sl = S + (size_t)l * d * d;
            const double* zl = z + (size_t)l * d;
            for (int32_t a = 0; a < d; ++a) {
                const double qa = g * feature(Q[i * d + a], feature_map);
                di += qa * zl[a];
                for (int32_t b = 0; b < d; ++b) ni[b] += qa * Sl[a * d + b];
            }
        }
        den[i] = di;
    }
}

/* ------------------------------------------------------------------ one output row from the definition
 * Eq. (2) with M_hat = Phi_hat Phi_hat^T written out for a single query row i:
 *     num_i = sum_j M_hat_ij (phi(q_i) . phi(k_j)) v_j,    den_i = sum_j M_hat_ij (phi(q_i) . phi(k_j)),
 *     M_hat_ij = sum_l phi_hat(v_i)_l phi_hat(v_j)_l.
 * Used to spot-check single rows at sizes where the full S array is too large.
 * mask_row is caller scratch of n doubles.
 */
void grf_ref_row_direct(int64_t n, int32_t d, int64_t i, const float* Q, const float* K, const float* V,
                        const int32_t* phi_row_ptr, const int32_t* phi_col, const float* phi_val,
                        int32_t feature_map, double* mask_row, double* num_i, double* den_i)
{
    double* dense_i = (double*)calloc((size_t)n, sizeof(double));
    for (int64_t e = phi_row_ptr[i]; e < phi_row_ptr[i + 1]; ++e) dense_i[phi_col[e]] = (double)phi_val[e];
    for (int32_t b = 0; b < d; ++b) num_i[b] = 0.0;
    double di = 0.0;
    for (int64_t j = 0; j < n; ++j) {
        double mij = 0.0;
        for (int64_t e = phi_row_ptr[j]; e < phi_row_ptr[j + 1]; ++e)
            mij += dense_i[phi_col[e]] * (double)phi_val[e];
        mask_row[j] = mij;
        if (mij == 0.0) continue;
        double a = 0.0;
        for (int32_t c = 0; c < d; ++c)
            a += feature(Q[i * d + c], feature_map) * feature(K[j * d + c], feature_map);
        di += mij * a;
        for (int32_t b = 0; b < d; ++b) num_i[b] += mij * a * (double)V[j * d + b];
    }
    *den_i = di;
    free(dense_i);
}

/* ------------------------------------------------------------------ App. D, Alg. 2: asymmetric GRFs
 * Keys use the one-hot feature (f^(2) = delta_0, Phi^(2) = I), queries the walks with modulation
 * f^(1) = f (so f plays the role of alpha).  Following the algorithm's own loop structure, for every
 * node i, every walk out of i and every visited (t, v_j):
 *     w = phi(q_i)^T phi(k_j) * f_t * weight(prefix of t hops)
 *     F_i += w * v_j,     S_i += w
 * One (batch, head) slice.  num_i = F_i / n_walks and den_i = S_i / n_walks are returned (the 1/n of
 * the GRF definition on both; it cancels in the output F_i / S_i -- the extra factor n that the
 * printed normalisation line carries has no counterpart in the accumulations and is not applied).
 */
void grf_ref_asymmetric_walks(int64_t n, const int32_t* row_ptr, const int32_t* col, const float* w,
                              const float* f, int32_t f_len, double p_halt, int32_t n_walks, uint64_t seed,
                              int32_t d, const float* Q, const float* K, const float* V, int32_t feature_map,
                              double* num, double* den)
{
    int32_t* nodes = (int32_t*)malloc(sizeof(int32_t) * (size_t)f_len);
    double* loads = (double*)malloc(sizeof(double) * (size_t)f_len);
    for (int64_t i = 0; i < n; ++i) {
        double* Fi = num + (size_t)i * d;
        for (int32_t b = 0; b < d; ++b) Fi[b] = 0.0;
        double Si = 0.0;
        for (int32_t k = 0; k < n_walks; ++k) {
            const int len = one_walk(row_ptr, col, w, i, k, f_len, p_halt, seed, nodes, loads);
            for (int t = 0; t < len; ++t) {
                const int64_t j = nodes[t];
                double a = 0.0;
                for (int32_t c = 0; c < d; ++c)
                    a += feature(Q[i * d + c], feature_map) * feature(K[j * d + c], feature_map);
                const double wgt = a * (double)f[t] * loads[t];
                Si += wgt;
                for (int32_t b = 0; b < d; ++b) Fi[b] += wgt * (double)V[j * d + b];
            }
        }
        for (int32_t b = 0; b < d; ++b) Fi[b] /= (double)n_walks;
        den[i] = Si / (double)n_walks;
    }
    free(nodes); free(loads);
}

/* ------------------------------------------------------------------ gradients of Eq. 7 (training; Alg. 1 has learnable f)
 * One (batch, head) slice.  The forward pass is
 *     num_i = sum_l Phi_il phi(q_i)^T S_l,   den_i = sum_l Phi_il phi(q_i)^T z_l,   out_i = num_i / den_i,
 *     S_l = sum_j Phi_jl phi(k_j) v_j^T,     z_l = sum_j Phi_jl phi(k_j).
 * With v'_j = [v_j, 1] (length d+1) both products are one: num'_i = [num_i, den_i] = sum_l Phi_il phi(q_i)^T S'_l,
 * S'_l = sum_j Phi_jl phi(k_j) v'_j^T.  Given dout = dL/dout, the chain rule through the division gives
 *     g'_i = dL/dnum'_i = [ dout_i / den_i ,  -(dout_i . out_i) / den_i ],
 * and L depends on the inputs through  sum_{i,l,j} Phi_il Phi_jl (phi(q_i) . phi(k_j)) (v'_j . g'_i).  Hence, with
 *     T'_l = sum_i Phi_il phi(q_i) g'_i^T   (d x (d+1), the query-side counterpart of S'_l),
 *     dL/dphi(q_i) = sum_l Phi_il S'_l g'_i
 *     dL/dphi(k_j) = sum_l Phi_jl T'_l v'_j
 *     dL/dv_j      = sum_l Phi_jl T_l^T phi(k_j)            (T_l = first d columns of T'_l)
 *     dL/dPhi_il   = phi(q_i)^T S'_l g'_i + phi(k_i)^T T'_l v'_i     (entry (i,l) acts once as a query-side
 *                                                                      and once as a key-side factor)
 * and dL/dq = dL/dphi(q) * phi'(q) elementwise, likewise for k.
 *
 * out [n][d] and den [n] are the forward results the caller saved (fp64 here).  dphi has one value per stored
 * entry of Phi_hat, in CSR order.  Everything fp64.
 */
void grf_ref_attention_backward(int64_t n, int32_t d, const float* Q, const float* K, const float* V,
                                const int32_t* phi_row_ptr, const int32_t* phi_col, const float* phi_val,
                                int32_t feature_map, const double* out, const double* den, const double* dout,
                                double* dQ, double* dK, double* dV, double* dphi)
{
    const int32_t e1 = d + 1;
    double* Sp = (double*)calloc((size_t)n * d * e1, sizeof(double));
    double* Tp = (double*)calloc((size_t)n * d * e1, sizeof(double));
    double* gp = (double*)malloc(sizeof(double) * (size_t)n * e1);
    double* fq = (double*)malloc(sizeof(double) * (size_t)n * d);
    double* fk = (double*)malloc(sizeof(double) * (size_t)n * d);
    for (int64_t i = 0; i < n; ++i) {
        double dot = 0.0;
        for (int32_t c = 0; c < d; ++c) {
            gp[i * e1 + c] = dout[i * d + c] / den[i];
            dot += dout[i * d + c] * out[i * d + c];
            fq[i * d + c] = feature(Q[i * d + c], feature_map);
            fk[i * d + c] = feature(K[i * d + c], feature_map);
        }
        gp[i * e1 + d] = -dot / den[i];
    }
    /* key-side buckets S'_l and query-side buckets T'_l */
    for (int64_t j = 0; j < n; ++j)
        for (int64_t e = phi_row_ptr[j]; e < phi_row_ptr[j + 1]; ++e) {
            const int64_t l = phi_col[e];
            const double g = (double)phi_val[e];
            double* Sl = Sp + (size_t)l * d * e1;
            double* Tl = Tp + (size_t)l * d * e1;
            for (int32_t a = 0; a < d; ++a) {
                const double ka = g * fk[j * d + a], qa = g * fq[j * d + a];
                for (int32_t c = 0; c < d; ++c) Sl[a * e1 + c] += ka * (double)V[j * d + c];
                Sl[a * e1 + d] += ka;
                for (int32_t c = 0; c < e1; ++c) Tl[a * e1 + c] += qa * gp[j * e1 + c];
            }
        }
    memset(dV, 0, sizeof(double) * (size_t)n * d);
    for (int64_t i = 0; i < n; ++i) {
        double* dfq = dQ + (size_t)i * d;
        double* dfk = dK + (size_t)i * d;
        for (int32_t a = 0; a < d; ++a) { dfq[a] = 0.0; dfk[a] = 0.0; }
        for (int64_t e = phi_row_ptr[i]; e < phi_row_ptr[i + 1]; ++e) {
            const int64_t l = phi_col[e];
            const double g = (double)phi_val[e];
            const double* Sl = Sp + (size_t)l * d * e1;
            const double* Tl = Tp + (size_t)l * d * e1;
            double de = 0.0;
            for (int32_t a = 0; a < d; ++a) {
                double u = 0.0, r = 0.0;
                for (int32_t c = 0; c < e1; ++c) u += Sl[a * e1 + c] * gp[i * e1 + c];
                for (int32_t c = 0; c < d; ++c) r += Tl[a * e1 + c] * (double)V[i * d + c];
                r += Tl[a * e1 + d];
                dfq[a] += g * u;
                dfk[a] += g * r;
                de += fq[i * d + a] * u + fk[i * d + a] * r;
                for (int32_t c = 0; c < d; ++c) dV[i * d + c] += g * Tl[a * e1 + c] * fk[i * d + a];
            }
            dphi[e] = de;
        }
        for (int32_t a = 0; a < d; ++a) {
            dfq[a] *= feature_grad(Q[i * d + a], feature_map);
            dfk[a] *= feature_grad(K[i * d + a], feature_map);
        }
    }
    free(Sp); free(Tp); free(gp); free(fq); free(fk);
}

/* ------------------------------------------------------------------ gradient with respect to the modulation f
 * Eq. (GRF definition): Phi_iq = (1/n) sum_k sum_t [omega_k(t) = q] load_{k,t} f_t  is linear in f, so
 *     dL/df_t = (1/n) sum_i sum_k load_{k,t} * (dL/dPhi)[i, omega_k(t)]
 * over the same walks (same seed).  dphi is [n_f][nnz] in the CSR order of the pattern (phi_row_ptr, phi_col),
 * df is [n_f][f_len]; fp64.
 */
void grf_ref_sample_backward(int64_t n, const int32_t* row_ptr, const int32_t* col, const float* w,
                             int32_t f_len, int32_t n_f, double p_halt, int32_t n_walks, uint64_t seed,
                             const int32_t* phi_row_ptr, const int32_t* phi_col, int64_t nnz,
                             const double* dphi, double* df)
{
    int32_t* nodes = (int32_t*)malloc(sizeof(int32_t) * (size_t)f_len);
    double* loads = (double*)malloc(sizeof(double) * (size_t)f_len);
    for (int64_t x = 0; x < (int64_t)n_f * f_len; ++x) df[x] = 0.0;
    for (int64_t i = 0; i < n; ++i)
        for (int32_t k = 0; k < n_walks; ++k) {
            const int len = one_walk(row_ptr, col, w, i, k, f_len, p_halt, seed, nodes, loads);
            for (int t = 0; t < len; ++t) {
                int64_t e = phi_row_ptr[i];
                while (e < phi_row_ptr[i + 1] && phi_col[e] != nodes[t]) ++e;
                if (e == phi_row_ptr[i + 1]) continue;      /* cannot happen for a pattern sampled with the same arguments */
                for (int32_t h = 0; h < n_f; ++h)
                    df[(size_t)h * f_len + t] += loads[t] * dphi[(size_t)h * (size_t)nnz + (size_t)e] / (double)n_walks;
            }
        }
    free(nodes); free(loads);
}

/* ------------------------------------------------------------------ gradients of single rows from Eq. (2) directly
 * For node i, with M_hat_ij = sum_l Phi_il Phi_jl (symmetric) and g' as above (gp is [n][d+1], precomputed):
 *     dL/dphi(q_i) = sum_j M_hat_ij (v'_j . g'_i) phi(k_j)
 *     dL/dphi(k_i) = sum_j M_hat_ij (v'_i . g'_j) phi(q_j)
 *     dL/dv_i      = sum_j M_hat_ij (phi(q_j) . phi(k_i)) g_j
 * O(N r) per row; used to spot-check rows at sizes where the bucket arrays are too large.
 */
void grf_ref_row_direct_backward(int64_t n, int32_t d, int64_t i, const float* Q, const float* K, const float* V,
                                 const int32_t* phi_row_ptr, const int32_t* phi_col, const float* phi_val,
                                 int32_t feature_map, const double* gp, double* dq_i, double* dk_i, double* dv_i)
{
    const int32_t e1 = d + 1;
    double* dense_i = (double*)calloc((size_t)n, sizeof(double));
    for (int64_t e = phi_row_ptr[i]; e < phi_row_ptr[i + 1]; ++e) dense_i[phi_col[e]] = (double)phi_val[e];
    for (int32_t a = 0; a < d; ++a) { dq_i[a] = 0.0; dk_i[a] = 0.0; dv_i[a] = 0.0; }
    for (int64_t j = 0; j < n; ++j) {
        double mij = 0.0;
        for (int64_t e = phi_row_ptr[j]; e < phi_row_ptr[j + 1]; ++e)
            mij += dense_i[phi_col[e]] * (double)phi_val[e];
        if (mij == 0.0) continue;
        double vj_gi = gp[i * e1 + d], vi_gj = gp[j * e1 + d], qj_ki = 0.0;
        for (int32_t c = 0; c < d; ++c) {
            vj_gi += (double)V[j * d + c] * gp[i * e1 + c];
            vi_gj += (double)V[i * d + c] * gp[j * e1 + c];
            qj_ki += feature(Q[j * d + c], feature_map) * feature(K[i * d + c], feature_map);
        }
        for (int32_t a = 0; a < d; ++a) {
            dq_i[a] += mij * vj_gi * feature(K[j * d + a], feature_map);
            dk_i[a] += mij * vi_gj * feature(Q[j * d + a], feature_map);
            dv_i[a] += mij * qj_ki * gp[j * e1 + a];
        }
    }
    for (int32_t a = 0; a < d; ++a) {
        dq_i[a] *= feature_grad(Q[i * d + a], feature_map);
        dk_i[a] *= feature_grad(K[i * d + a], feature_map);
    }
    free(dense_i);
}

/* dL/dPhi for the single stored entry e = (i, l) from the formula above, with S'_l and T'_l formed by a scan
 * over all entries of column l. */
double grf_ref_dphi_entry_direct(int64_t n, int32_t d, int64_t i, int64_t l, const float* Q, const float* K, const float* V,
                                 const int32_t* phi_row_ptr, const int32_t* phi_col, const float* phi_val,
                                 int32_t feature_map, const double* gp)
{
    const int32_t e1 = d + 1;
    double* Sl = (double*)calloc((size_t)d * e1, sizeof(double));
    double* Tl = (double*)calloc((size_t)d * e1, sizeof(double));
    for (int64_t j = 0; j < n; ++j)
        for (int64_t e = phi_row_ptr[j]; e < phi_row_ptr[j + 1]; ++e) {
            if (phi_col[e] != l) continue;
            const double g = (double)phi_val[e];
            for (int32_t a = 0; a < d; ++a) {
                const double ka = g * feature(K[j * d + a], feature_map), qa = g * feature(Q[j * d + a], feature_map);
                for (int32_t c = 0; c < d; ++c) Sl[a * e1 + c] += ka * (double)V[j * d + c];
                Sl[a * e1 + d] += ka;
                for (int32_t c = 0; c < e1; ++c) Tl[a * e1 + c] += qa * gp[j * e1 + c];
            }
        }
    double de = 0.0;
    for (int32_t a = 0; a < d; ++a) {
        double u = 0.0, r = Tl[a * e1 + d];
        for (int32_t c = 0; c < e1; ++c) u += Sl[a * e1 + c] * gp[i * e1 + c];
        for (int32_t c = 0; c < d; ++c) r += Tl[a * e1 + c] * (double)V[i * d + c];
        de += feature(Q[i * d + a], feature_map) * u + feature(K[i * d + a], feature_map) * r;
    }
    free(Sl); free(Tl);
    return de;
}

/* ------------------------------------------------------------------ gradients of asymmetric-GRF attention (App. D)
 * Forward (the per-end-node form of Alg. 2):  num'_i = [num_i, den_i] = sum_j Phi_ij (phi(q_i) . phi(k_j)) v'_j,
 * out_i = num_i / den_i, the sum running over the stored entries of row i.  With g'_i as for the symmetric case,
 * L depends on the inputs through  sum_(i,j) Phi_ij a_ij c_ij,  a_ij = phi(q_i) . phi(k_j),  c_ij = v'_j . g'_i:
 *     dL/dPhi_ij   = a_ij c_ij                     dL/dphi(q_i) = sum_j Phi_ij c_ij phi(k_j)
 *     dL/dphi(k_j) = sum_i Phi_ij c_ij phi(q_i)    dL/dv_j      = sum_i Phi_ij a_ij g_i
 * One slice, fp64; dphi in CSR order.
 */
void grf_ref_asymmetric_backward(int64_t n, int32_t d, const float* Q, const float* K, const float* V,
                                 const int32_t* phi_row_ptr, const int32_t* phi_col, const float* phi_val,
                                 int32_t feature_map, const double* out, const double* den, const double* dout,
                                 double* dQ, double* dK, double* dV, double* dphi)
{
    double* g = (double*)malloc(sizeof(double) * (size_t)(d + 1));
    for (int64_t x = 0; x < n * (int64_t)d; ++x) { dQ[x] = 0.0; dK[x] = 0.0; dV[x] = 0.0; }
    for (int64_t i = 0; i < n; ++i) {
        double dot = 0.0;
        for (int32_t c = 0; c < d; ++c) { g[c] = dout[i * d + c] / den[i]; dot += dout[i * d + c] * out[i * d + c]; }
        g[d] = -dot / den[i];
        for (int64_t e = phi_row_ptr[i]; e < phi_row_ptr[i + 1]; ++e) {
            const int64_t j = phi_col[e];
            const double w = (double)phi_val[e];
            double a = 0.0, c = g[d];
            for (int32_t x = 0; x < d; ++x) {
                a += feature(Q[i * d + x], feature_map) * feature(K[j * d + x], feature_map);
                c += (double)V[j * d + x] * g[x];
            }
            dphi[e] = a * c;
            for (int32_t x = 0; x < d; ++x) {
                dQ[i * d + x] += w * c * feature(K[j * d + x], feature_map);
                dK[j * d + x] += w * c * feature(Q[i * d + x], feature_map);
                dV[j * d + x] += w * a * g[x];
            }
        }
    }
    for (int64_t x = 0; x < n * (int64_t)d; ++x) {
        dQ[x] *= feature_grad(Q[x], feature_map);
        dK[x] *= feature_grad(K[x], feature_map);
    }
    free(g);
}

/* ------------------------------------------------------------------ k-nearest-neighbour graph of a point cloud
 * For dynamic point clouds the paper builds the graph on the fly from each node's k nearest neighbours
 * (Sec. 4, point-cloud experiment; App. C).  Brute force: every pair is examined.
 *
 * The squared distance is taken in fp32, each operation rounded on its own (build with -ffp-contract=off):
 *     fl(fl(fl(dx*dx) + fl(dy*dy)) + fl(dz*dz)),  dx = fl(x_i - x_j);
 * neighbours are ordered by (squared distance, index).  The fp32 arithmetic is part of the definition because it
 * decides an integer (which points are neighbours); both the checker and the library take it in this precision.
 *
 * knn_idx [n][k] (-1 where fewer than k other points exist), knn_d2 [n][k].
 */
static float squared_distance_f32(const float* a, const float* b)
{
    const float dx = a[0] - b[0], dy = a[1] - b[1], dz = a[2] - b[2];
    const float xx = dx * dx, yy = dy * dy, zz = dz * dz;
    const float xy = xx + yy;
    return xy + zz;
}

/* The same for the n_rows query points listed in rows[] only: knn_idx, knn_d2 are [n_rows][k]. */
void grf_ref_knn_lists_rows(int64_t n, const float* pts, int32_t k, int64_t n_rows, const int64_t* rows,
                            int32_t* knn_idx, float* knn_d2);

void grf_ref_knn_lists(int64_t n, const float* pts, int32_t k, int32_t* knn_idx, float* knn_d2)
{
    int64_t* rows = (int64_t*)malloc(sizeof(int64_t) * (size_t)(n > 0 ? n : 1));
    for (int64_t i = 0; i < n; ++i) rows[i] = i;
    grf_ref_knn_lists_rows(n, pts, k, n, rows, knn_idx, knn_d2);
    free(rows);
}

void grf_ref_knn_lists_rows(int64_t n, const float* pts, int32_t k, int64_t n_rows, const int64_t* rows,
                            int32_t* knn_idx, float* knn_d2)
{
    for (int64_t r = 0; r < n_rows; ++r) {
        const int64_t i = rows[r];
        int32_t* bi = knn_idx + (size_t)r * k;
        float* bd = knn_d2 + (size_t)r * k;
        int32_t cnt = 0;
        for (int64_t j = 0; j < n; ++j) {
            if (j == i) continue;
            const float d = squared_distance_f32(pts + 3 * i, pts + 3 * j);
            if (cnt == k && !(d < bd[k - 1])) continue;        /* j ascending: an equal distance never displaces */
            int32_t s = cnt < k ? cnt : k - 1;
            while (s > 0 && bd[s - 1] > d) { bd[s] = bd[s - 1]; bi[s] = bi[s - 1]; --s; }
            bd[s] = d; bi[s] = (int32_t)j;
            if (cnt < k) ++cnt;
        }
        for (int32_t s = cnt; s < k; ++s) { bi[s] = -1; bd[s] = INFINITY; }
    }
}

/* CSR graph from the lists: directed (row i = its k neighbours) or symmetric closure (i ~ j if either lists the
 * other); columns ascending; weights 1/deg(i) (kind 0), exp(-dist/sigma) (1) or exp(-dist^2/(2 sigma^2)) (2), the
 * last two divided by their row sum; fp64.  Two calls: with col_out == NULL only row_ptr_out is written and nnz
 * returned. */
int64_t grf_ref_knn_graph(int64_t n, int32_t k, const int32_t* knn_idx, const float* knn_d2,
                          int32_t symmetrise, int32_t weight_kind, double sigma,
                          int32_t* row_ptr_out, int32_t* col_out, double* w_out)
{
    int64_t running = 0;
    int32_t* cols = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    double* d2s = (double*)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
    for (int64_t i = 0; i < n; ++i) {
        int64_t cnt = 0;
        for (int32_t s = 0; s < k; ++s)
            if (knn_idx[i * k + s] >= 0) { cols[cnt] = knn_idx[i * k + s]; d2s[cnt] = (double)knn_d2[i * k + s]; ++cnt; }
        if (symmetrise)
            for (int64_t j = 0; j < n; ++j) {
                if (j == i) continue;
                int lists_i = 0, listed = 0;
                double d2 = 0.0;
                for (int32_t s = 0; s < k; ++s) if (knn_idx[j * k + s] == (int32_t)i) { lists_i = 1; d2 = (double)knn_d2[j * k + s]; }
                for (int32_t s = 0; s < k; ++s) if (knn_idx[i * k + s] == (int32_t)j) listed = 1;
                if (lists_i && !listed) { cols[cnt] = (int32_t)j; d2s[cnt] = d2; ++cnt; }
            }
        row_ptr_out[i] = (int32_t)running;
        if (col_out != NULL) {
            for (int64_t a = 1; a < cnt; ++a) {
                int64_t b = a;
                while (b > 0 && cols[b - 1] > cols[b]) {
                    int32_t tc = cols[b]; cols[b] = cols[b - 1]; cols[b - 1] = tc;
                    double td = d2s[b]; d2s[b] = d2s[b - 1]; d2s[b - 1] = td;
                    --b;
                }
            }
            /* exp(-d/sigma) / sum exp(-d/sigma), with numerator and denominator both divided by the largest term
             * (that of the nearest neighbour) so that a far-away row does not become 0 / 0 */
            double total = 0.0, nearest = INFINITY;
            for (int64_t a = 0; a < cnt; ++a) if (d2s[a] < nearest) nearest = d2s[a];
            for (int64_t a = 0; a < cnt; ++a) {
                double raw = 1.0;
                if (weight_kind == 1) raw = exp(-(sqrt(d2s[a]) - sqrt(nearest)) / sigma);
                if (weight_kind == 2) raw = exp(-(d2s[a] - nearest) / (2.0 * sigma * sigma));
                d2s[a] = raw;
                total += raw;
            }
            for (int64_t a = 0; a < cnt; ++a) {
                col_out[running + a] = cols[a];
                w_out[running + a] = d2s[a] / total;
            }
        }
        running += cnt;
    }
    row_ptr_out[n] = (int32_t)running;
    free(cols); free(d2s);
    return running;
}
