/*
 * memo_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain, slow, fp64 CPU statement of what the Memo hot path computes, written
 * from the paper (arXiv 2407.12117).  Only tests, the smoke check and the
 * cpu_baseline leg of the benchmark may call it.  It shares no code, header,
 * table or helper with the HIP library and includes nothing from it.
 *
 * What is stated here
 *   - Causal softmax self-attention, O = softmax(Q K^T / sqrt(d)) V with the
 *     decoder-only causal mask (Section 2.1.1 "Architecture"; Section 2.1.3,
 *     the formula for O).  FlashAttention is exact (Section 2.1.3), so the
 *     oracle is the plain definition: every score of a row is formed, the row
 *     maximum is taken, the exponentials are summed (two-pass softmax) and the
 *     weighted sum of value rows is taken.  No tiling, no running maximum.
 *   - The per-row logsumexp LSE_i = ln sum_j exp(s_ij) of the scaled scores,
 *     the "compact state" FlashAttention keeps (Section 2.1.3).
 *   - The gradients dQ, dK, dV of the scalar L = sum(O * dO) by the chain rule
 *     through the three steps above (Section 2.1.3 says the backward pass
 *     re-forms the intermediates; the formulas are the ordinary derivative of
 *     the definition and are pinned by finite differences in the tests).
 *   - Token-wise swap bookkeeping (Section 4.1 "Token-wise Recomputation and
 *     Swapping"): a fraction alpha of the tokens of a saved activation is
 *     offloaded, the rest is dropped and recomputed later.  k = floor(alpha*S)
 *     in IEEE double, the first k token rows are the swapped ones, rows [k,S)
 *     are the recompute set.
 *   - The choice of alpha (Section 4.1, the two constraints under "max alpha").
 *
 * Layout: attention tensors are [B, S, H, d] row-major doubles (token-major as
 * the paper's (b, s, h) with h = H*d); LSE is [B, H, S].
 *
 * Readings taken where the paper is silent: mask is inclusive (j <= i); scale
 * is an explicit argument; heads are independent (no grouped K/V).
 *
 * OpenMP pragmas only spread independent rows / columns over cores so that the
 * baseline timing uses the host's cores; they do not change any arithmetic.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------------ */
/* One head: rows are rs doubles apart (rs = H*d in the [B,S,H,d] layout).   */
/* ------------------------------------------------------------------------ */

/* Scores, softmax and output of query row i.
 * p[0..i] receives P_ij = exp(s_ij - LSE_i); returns LSE_i; o_i[0..d) = O_i.  */
static double row_forward(int64_t i, int d, double scale,
                          const double *q, const double *k, const double *v,
                          int64_t rs, double *p, double *o_i)
{
    const double *qi = q + i * rs;
    double m = -INFINITY;
    for (int64_t j = 0; j <= i; ++j) {          /* causal: keys 0..i */
        const double *kj = k + j * rs;
        double dot = 0.0;
        for (int c = 0; c < d; ++c) dot += qi[c] * kj[c];
        p[j] = scale * dot;
        if (p[j] > m) m = p[j];
    }
    double l = 0.0;
    for (int64_t j = 0; j <= i; ++j) l += exp(p[j] - m);
    const double lse = m + log(l);
    for (int64_t j = 0; j <= i; ++j) p[j] = exp(p[j] - lse);
    for (int c = 0; c < d; ++c) o_i[c] = 0.0;
    for (int64_t j = 0; j <= i; ++j) {
        const double *vj = v + j * rs;
        for (int c = 0; c < d; ++c) o_i[c] += p[j] * vj[c];
    }
    return lse;
}

/* D_i = sum_c dO_ic O_ic */
static double row_delta(int d, const double *do_i, const double *o_i)
{
    double D = 0.0;
    for (int c = 0; c < d; ++c) D += do_i[c] * o_i[c];
    return D;
}

/* dQ_i = scale * sum_{j<=i} dS_ij k_j, dS_ij = P_ij (dP_ij - D_i),
 * dP_ij = sum_c dO_ic v_jc.  p[0..i] holds P_ij. */
static void row_dq(int64_t i, int d, double scale, const double *p, double D,
                   const double *k, const double *v, const double *do_i,
                   int64_t rs, double *dq_i)
{
    for (int c = 0; c < d; ++c) dq_i[c] = 0.0;
    for (int64_t j = 0; j <= i; ++j) {
        const double *vj = v + j * rs, *kj = k + j * rs;
        double dP = 0.0;
        for (int c = 0; c < d; ++c) dP += do_i[c] * vj[c];
        const double dS = p[j] * (dP - D);
        for (int c = 0; c < d; ++c) dq_i[c] += scale * dS * kj[c];
    }
}

/* Column j of the backward: dV_j = sum_{i>=j} P_ij dO_i,
 * dK_j = scale * sum_{i>=j} dS_ij q_i.  lse[], delta[] are indexed by the
 * absolute row i and must be valid for i >= j. */
static void col_dkdv(int64_t j, int64_t S, int d, double scale,
                     const double *q, const double *k, const double *v,
                     const double *d_o, int64_t rs,
                     const double *lse, const double *delta,
                     double *dk_j, double *dv_j)
{
    const double *kj = k + j * rs, *vj = v + j * rs;
    for (int c = 0; c < d; ++c) { dk_j[c] = 0.0; dv_j[c] = 0.0; }
    for (int64_t i = j; i < S; ++i) {
        const double *qi = q + i * rs, *doi = d_o + i * rs;
        double dot = 0.0, dP = 0.0;
        for (int c = 0; c < d; ++c) { dot += qi[c] * kj[c]; dP += doi[c] * vj[c]; }
        const double P = exp(scale * dot - lse[i]);
        const double dS = P * (dP - delta[i]);
        for (int c = 0; c < d; ++c) {
            dv_j[c] += P * doi[c];
            dk_j[c] += scale * dS * qi[c];
        }
    }
}

/* ------------------------------------------------------------------------ */
/* Dense entry points, [B,S,H,d]                                             */
/* ------------------------------------------------------------------------ */

void memo_oracle_attn_fwd(int B, int64_t S, int H, int d, double scale,
                          const double *q, const double *k, const double *v,
                          double *o, double *lse /* [B,H,S] */)
{
    const int64_t rs = (int64_t)H * d;
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < H; ++h) {
            const int64_t base = (int64_t)b * S * rs + (int64_t)h * d;
            double *lse_bh = lse + ((int64_t)b * H + h) * S;
#pragma omp parallel
            {
                double *p = (double *)malloc(sizeof(double) * (size_t)S);
#pragma omp for schedule(dynamic, 8)
                for (int64_t i = 0; i < S; ++i)
                    lse_bh[i] = row_forward(i, d, scale, q + base, k + base, v + base,
                                            rs, p, o + base + i * rs);
                free(p);
            }
        }
}

void memo_oracle_attn_bwd(int B, int64_t S, int H, int d, double scale,
                          const double *q, const double *k, const double *v,
                          const double *d_o,
                          double *dq, double *dk, double *dv)
{
    const int64_t rs = (int64_t)H * d;
    double *lse = (double *)malloc(sizeof(double) * (size_t)S);
    double *delta = (double *)malloc(sizeof(double) * (size_t)S);
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < H; ++h) {
            const int64_t base = (int64_t)b * S * rs + (int64_t)h * d;
            /* rows: LSE_i, D_i, dQ_i */
#pragma omp parallel
            {
                double *p = (double *)malloc(sizeof(double) * (size_t)S);
                double *o_i = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(dynamic, 8)
                for (int64_t i = 0; i < S; ++i) {
                    lse[i] = row_forward(i, d, scale, q + base, k + base, v + base, rs, p, o_i);
                    delta[i] = row_delta(d, d_o + base + i * rs, o_i);
                    row_dq(i, d, scale, p, delta[i], k + base, v + base,
                           d_o + base + i * rs, rs, dq + base + i * rs);
                }
                free(p);
                free(o_i);
            }
            /* columns: dK_j, dV_j */
#pragma omp parallel for schedule(dynamic, 8)
            for (int64_t j = 0; j < S; ++j)
                col_dkdv(j, S, d, scale, q + base, k + base, v + base, d_o + base, rs,
                         lse, delta, dk + base + j * rs, dv + base + j * rs);
        }
    free(lse);
    free(delta);
}

/* ------------------------------------------------------------------------ */
/* Sampled entry points on one head, tensors [S,d] contiguous.  Same row and */
/* column routines as above; used where the dense pass would take hours.     */
/* ------------------------------------------------------------------------ */

/* Forward and dQ for the listed query rows.  o_out, dq_out: [nrows,d];
 * lse_out, delta_out: [nrows].  d_o may be NULL (then dq_out/delta_out are
 * not written). */
void memo_oracle_head_rows(int64_t S, int d, double scale,
                           const double *q, const double *k, const double *v,
                           const double *d_o,
                           int64_t nrows, const int64_t *rows,
                           double *o_out, double *lse_out,
                           double *delta_out, double *dq_out)
{
    (void)S;
#pragma omp parallel
    {
        double *p = (double *)malloc(sizeof(double) * (size_t)S);
#pragma omp for schedule(dynamic, 1)
        for (int64_t r = 0; r < nrows; ++r) {
            const int64_t i = rows[r];
            lse_out[r] = row_forward(i, d, scale, q, k, v, d, p, o_out + r * d);
            if (d_o) {
                delta_out[r] = row_delta(d, d_o + i * d, o_out + r * d);
                row_dq(i, d, scale, p, delta_out[r], k, v, d_o + i * d, d, dq_out + r * d);
            }
        }
        free(p);
    }
}

/* dK, dV for key columns [j0, S): needs LSE_i, D_i of rows i >= j0 only.
 * dk_out, dv_out: [S-j0, d]. */
void memo_oracle_head_dkdv_tail(int64_t S, int d, double scale,
                                const double *q, const double *k, const double *v,
                                const double *d_o, int64_t j0,
                                double *dk_out, double *dv_out)
{
    const int64_t n = S - j0;
    double *lse = (double *)malloc(sizeof(double) * (size_t)S);
    double *delta = (double *)malloc(sizeof(double) * (size_t)S);
#pragma omp parallel
    {
        double *p = (double *)malloc(sizeof(double) * (size_t)S);
        double *o_i = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(dynamic, 1)
        for (int64_t i = j0; i < S; ++i) {
            lse[i] = row_forward(i, d, scale, q, k, v, d, p, o_i);
            delta[i] = row_delta(d, d_o + i * d, o_i);
        }
        free(p);
        free(o_i);
    }
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t t = 0; t < n; ++t)
        col_dkdv(j0 + t, S, d, scale, q, k, v, d_o, d, lse, delta,
                 dk_out + t * d, dv_out + t * d);
    free(lse);
    free(delta);
}

/* ------------------------------------------------------------------------ */
/* Token-wise swap bookkeeping (Section 4.1)                                 */
/* ------------------------------------------------------------------------ */

/* Number of swapped tokens: floor(alpha * S) in double; -1 if the arguments
 * are not a valid split (alpha outside [0,1] or not finite, S < 0). */
int64_t memo_oracle_split_tokens(int64_t S, double alpha)
{
    if (S < 0 || !(alpha >= 0.0) || !(alpha <= 1.0)) return -1;
    double kf = floor(alpha * (double)S);
    int64_t k = (int64_t)kf;
    if (k < 0) k = 0;
    if (k > S) k = S;
    return k;
}

/* out[0]=k swapped tokens, out[1]=S-k tokens to recompute, out[2]=bytes
 * swapped, out[3]=bytes dropped, out[4]=byte offset of the first recompute
 * row.  Returns 0, or -1 on invalid arguments. */
int memo_oracle_swap_plan(int64_t S, int64_t row_bytes, double alpha, int64_t out[5])
{
    const int64_t k = memo_oracle_split_tokens(S, alpha);
    if (k < 0 || row_bytes <= 0) return -1;
    out[0] = k;
    out[1] = S - k;
    out[2] = k * row_bytes;
    out[3] = (S - k) * row_bytes;
    out[4] = k * row_bytes;
    return 0;
}

/* Offload: the first k rows go to the host store; nothing else is read.
 * Returns bytes copied, -1 on invalid arguments, -2 if the host store is too
 * small (the paper's host out-of-memory case). */
int64_t memo_oracle_swap_out(const unsigned char *act, int64_t S, int64_t row_bytes,
                             double alpha, unsigned char *host, int64_t host_capacity)
{
    int64_t plan[5];
    if (memo_oracle_swap_plan(S, row_bytes, alpha, plan) != 0) return -1;
    if (plan[2] > host_capacity) return -2;
    if (plan[2] > 0) memcpy(host, act, (size_t)plan[2]);   /* alpha = 0: nothing to copy, host may be NULL */
    return plan[2];
}

/* Prefetch: the swapped rows come back to rows [0,k); rows [k,S) are left as
 * they are (they are rebuilt by recomputation, not by this call). */
int64_t memo_oracle_swap_in(unsigned char *act, int64_t S, int64_t row_bytes,
                            double alpha, const unsigned char *host, int64_t host_capacity)
{
    int64_t plan[5];
    if (memo_oracle_swap_plan(S, row_bytes, alpha, plan) != 0) return -1;
    if (plan[2] > host_capacity) return -2;
    if (plan[2] > 0) memcpy(act, host, (size_t)plan[2]);
    return plan[2];
}

/* ------------------------------------------------------------------------ */
/* Choice of alpha (Section 4.1, the problem "max alpha s.t. ...")           */
/*   (S_in + S_attn + alpha S_oth) / B      <= T_layer                        */
/*   (n-2) (S_in + S_attn + alpha S_oth)    <= M_cpu                          */
/* The oracle does not use the closed form: it scans alpha downwards on a     */
/* grid of `steps` equal parts of [0,1] and returns the largest grid point    */
/* that satisfies both constraints, or -1 if even alpha = 0 violates one.     */
/* ------------------------------------------------------------------------ */
double memo_oracle_alpha_grid(double s_in, double s_attn, double s_oth,
                              double bandwidth, double t_layer,
                              int n_layers, double m_cpu, int steps)
{
    for (int t = steps; t >= 0; --t) {
        const double a = (double)t / (double)steps;
        const double bytes = s_in + s_attn + a * s_oth;
        if (bytes / bandwidth <= t_layer && (double)(n_layers - 2) * bytes <= m_cpu)
            return a;
    }
    return -1.0;
}

int memo_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
