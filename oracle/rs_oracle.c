/*
 * TEST INFRASTRUCTURE ONLY: slow fp64 CPU checker for the representation-shift hot path.
 *
 * Nothing in the product path may include, link or call this file; it shares no
 * code with the HIP kernels.  Every function is the plain definition from the
 * paper written out with double arithmetic and no intermediate rounding:
 *
 *   - self-attention, Eq. (1) of Sec. 3.1, multi-head form, attention map
 *     materialised row by row;
 *   - the pre-LayerNorm block, Eqs. (5) and (6) of Sec. 3.3;
 *   - the representation shift s = D(F(x), x), Eq. (4) of Sec. 3.2, with the
 *     L2 / L1 / cosine distances listed under "Distance metrics" in Sec. 3.3;
 *   - pruning of the lowest-score tokens (Sec. 3.1, reduced token set
 *     x~ in R^{(N-r) x C}; Sec. 3.2, "dropped the tokens having the lowest k").
 *
 * Readings where the paper is silent (scale per head, exact-erf GELU, biased
 * variance, tie rule, ascending kept order) are stated at each function.
 *
 * OpenMP is used only to spread independent (image, row) iterations over cores.
 * All matrices are row-major; linear weights are [in, out] as in [Q,K,V] = xW.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int rs_oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void rs_oracle_set_num_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* LayerNorm over the last axis: mean and biased (population) variance of each
 * row, (x-mean)/sqrt(var+eps)*gamma+beta.  (LN of Eqs. (5),(6); the paper does
 * not state eps or the variance convention: eps is an argument, variance is the
 * population one, as in every ViT implementation.) */
void rs_oracle_layernorm(const double *x, const double *gamma, const double *beta,
                         double eps, int64_t M, int64_t D, double *out) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        const double *r = x + i * D;
        double mean = 0.0;
        for (int64_t j = 0; j < D; ++j) mean += r[j];
        mean /= (double)D;
        double var = 0.0;
        for (int64_t j = 0; j < D; ++j) var += (r[j] - mean) * (r[j] - mean);
        var /= (double)D;
        double inv = 1.0 / sqrt(var + eps);
        for (int64_t j = 0; j < D; ++j)
            out[i * D + j] = (r[j] - mean) * inv * (gamma ? gamma[j] : 1.0) + (beta ? beta[j] : 0.0);
    }
}

/* GELU with the exact Gaussian CDF: x * Phi(x) = 0.5 x (1 + erf(x / sqrt 2)).
 * (The paper only says "MLP"; the erf form is the ViT/DeiT one.) */
double rs_oracle_gelu(double x) { return 0.5 * x * (1.0 + erf(x / sqrt(2.0))); }

/* out[M,N] = a[M,K] @ w[K,N] + bias[N]; the sum over k runs in ascending k for
 * every output element. */
void rs_oracle_linear(const double *a, const double *w, const double *bias,
                      int64_t M, int64_t K, int64_t N, double *out) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        double *o = out + i * N;
        for (int64_t j = 0; j < N; ++j) o[j] = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double aik = a[i * K + k];
            const double *wr = w + k * N;
            for (int64_t j = 0; j < N; ++j) o[j] += aik * wr[j];
        }
        if (bias)
            for (int64_t j = 0; j < N; ++j) o[j] += bias[j];
    }
}

/* Multi-head softmax attention, Eq. (1): for every (image, head, query row)
 * S_j = scale * <q, k_j>;  P = softmax_j(S) with the row maximum subtracted;
 * o = sum_j P_j v_j.  The full row of the attention map is materialised.
 * Element (b, n, h, d) of q/k/v sits at b*sb + n*sn + h*sh + d (strides in
 * elements, shared by q, k and v); o uses its own strides.  The paper writes the
 * scale as 1/sqrt(C); the caller passes the scale (1/sqrt(dh) per head in ViTs). */
void rs_oracle_attention(const double *q, const double *k, const double *v, double *o,
                         int64_t B, int64_t H, int64_t N, int64_t dh,
                         int64_t sb, int64_t sn, int64_t sh,
                         int64_t osb, int64_t osn, int64_t osh, double scale) {
#pragma omp parallel
    {
        double *row = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
#pragma omp for collapse(3) schedule(static)
        for (int64_t b = 0; b < B; ++b)
            for (int64_t h = 0; h < H; ++h)
                for (int64_t i = 0; i < N; ++i) {
                    const double *qi = q + b * sb + i * sn + h * sh;
                    double mx = -INFINITY;
                    for (int64_t j = 0; j < N; ++j) {
                        const double *kj = k + b * sb + j * sn + h * sh;
                        double s = 0.0;
                        for (int64_t d = 0; d < dh; ++d) s += qi[d] * kj[d];
                        s *= scale;
                        row[j] = s;
                        if (s > mx) mx = s;
                    }
                    double den = 0.0;
                    for (int64_t j = 0; j < N; ++j) {
                        row[j] = exp(row[j] - mx);
                        den += row[j];
                    }
                    double *oi = o + b * osb + i * osn + h * osh;
                    for (int64_t d = 0; d < dh; ++d) oi[d] = 0.0;
                    for (int64_t j = 0; j < N; ++j) {
                        const double *vj = v + b * sb + j * sn + h * sh;
                        double p = row[j] / den;
                        for (int64_t d = 0; d < dh; ++d) oi[d] += p * vj[d];
                    }
                }
        free(row);
    }
}

/* Representation shift per token, Eq. (4): s_i = D(F(x)_i, x_i).
 * dist 0: L2  ||f_out - f_in||_2      (default of the paper)
 * dist 1: L1  ||f_out - f_in||_1
 * dist 2: cosine distance 1 - <a,b>/(||a|| ||b||)   ("Distance metrics", Sec. 3.3) */
void rs_oracle_shift_scores(const double *f_out, const double *f_in, int64_t M, int64_t D,
                            int dist, double *scores) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        const double *a = f_out + i * D, *b = f_in + i * D;
        if (dist == 0) {
            double s = 0.0;
            for (int64_t j = 0; j < D; ++j) s += (a[j] - b[j]) * (a[j] - b[j]);
            scores[i] = sqrt(s);
        } else if (dist == 1) {
            double s = 0.0;
            for (int64_t j = 0; j < D; ++j) s += fabs(a[j] - b[j]);
            scores[i] = s;
        } else {
            double ab = 0.0, aa = 0.0, bb = 0.0;
            for (int64_t j = 0; j < D; ++j) {
                ab += a[j] * b[j];
                aa += a[j] * a[j];
                bb += b[j] * b[j];
            }
            scores[i] = 1.0 - ab / (sqrt(aa) * sqrt(bb));
        }
    }
}

/* Token selection (Sec. 3.1 / 3.2: drop the lowest-score tokens).  Per image:
 * tokens [0, n_prefix) are always kept (the class token); the other tokens are
 * ordered by (score descending, index ascending) with a full insertion sort and
 * the first n_keep of them survive; kept_idx lists prefix + survivors in
 * ascending index order, K = n_prefix + n_keep entries per image.
 * Tie rule and output order are this build's reading; the paper is silent. */
void rs_oracle_topk(const double *scores, int64_t B, int64_t N, int64_t n_prefix,
                    int64_t n_keep, int32_t *kept_idx) {
    int64_t K = n_prefix + n_keep;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b) {
        const double *s = scores + b * N;
        int64_t n = N - n_prefix;
        int32_t *order = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
        /* insertion sort by (score desc, index asc): stable on ascending input */
        for (int64_t t = 0; t < n; ++t) {
            int32_t idx = (int32_t)(n_prefix + t);
            int64_t p = t;
            while (p > 0 && s[order[p - 1]] < s[idx]) {
                order[p] = order[p - 1];
                --p;
            }
            order[p] = idx;
        }
        char *keep = (char *)calloc((size_t)(N > 0 ? N : 1), 1);
        for (int64_t i = 0; i < n_prefix; ++i) keep[i] = 1;
        for (int64_t t = 0; t < n_keep; ++t) keep[order[t]] = 1;
        int64_t w = 0;
        for (int64_t i = 0; i < N; ++i)
            if (keep[i]) kept_idx[b * K + w++] = (int32_t)i;
        free(keep);
        free(order);
    }
}

/* Reduced token set: out[b, j, :] = src[b, kept_idx[b, j], :]. */
void rs_oracle_gather(const double *src, const int32_t *kept_idx, int64_t B, int64_t N,
                      int64_t K, int64_t D, double *out) {
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t b = 0; b < B; ++b)
        for (int64_t j = 0; j < K; ++j)
            memcpy(out + (b * K + j) * D, src + (b * N + kept_idx[b * K + j]) * D,
                   sizeof(double) * (size_t)D);
}

/* One pre-LN encoder block, Eqs. (5),(6):
 *   sa   = SA(LN(x))              SA = multi-head attention followed by the output projection
 *   x1   = sa + x
 *   mlp  = W2 GELU(W1 LN(x1) + b1) + b2
 *   xhat = mlp + x1
 * and the representation shift s_i = D(f_out_i, f_in_i) for the operation `op`
 * ("Operation choice", Sec. 3.3):
 *   op 0  case (ii), the MLP:       D(MLP(LN(x1)), x1)   -- branch output versus the
 *                                                           residual-stream input (the default)
 *   op 1  case (i), attention:      D(SA(LN(x)), x)
 *   op 2  case (iii), whole block:  D(xhat, x)
 * plus the two other readings of "the shift around the MLP" that the text leaves open:
 *   op 3  residual stream before and after the MLP:  D(xhat, x1)
 *   op 4  the MLP's own input and output:            D(MLP(v), v),  v = LN(x1)
 * W_qkv columns are ordered [Q | K | V], each H heads of dh = D/H.
 * Any bias may be NULL (= zero).  Outputs (each may be NULL): sa, x1, mlp, xhat [B*N, D];
 * scores [B*N].  Returns 0, -1 if an allocation fails, -2 for an unknown op. */
int rs_oracle_block(int64_t B, int64_t N, int64_t D, int64_t H, int64_t Dm,
                    double ln_eps, double attn_scale, int dist, int op,
                    const double *x,
                    const double *ln1_g, const double *ln1_b,
                    const double *w_qkv, const double *b_qkv,
                    const double *w_proj, const double *b_proj,
                    const double *ln2_g, const double *ln2_b,
                    const double *w_fc1, const double *b_fc1,
                    const double *w_fc2, const double *b_fc2,
                    double *sa_out, double *x1_out, double *mlp_out, double *xhat_out,
                    double *scores) {
    int64_t M = B * N, dh = D / H;
    size_t md = (size_t)M * (size_t)D;
    double *u = (double *)malloc(sizeof(double) * md);
    double *qkv = (double *)malloc(sizeof(double) * md * 3);
    double *att = (double *)malloc(sizeof(double) * md);
    double *x1 = (double *)malloc(sizeof(double) * md);
    double *hid = (double *)malloc(sizeof(double) * (size_t)M * (size_t)Dm);
    double *mlp = (double *)malloc(sizeof(double) * md);
    double *sa = (double *)malloc(sizeof(double) * md);
    double *xhat = (double *)malloc(sizeof(double) * md);
    int rc = -1;
    if (op < 0 || op > 4) rc = -2;
    else if (u && qkv && att && x1 && hid && mlp && sa && xhat) {
        rs_oracle_layernorm(x, ln1_g, ln1_b, ln_eps, M, D, u);
        rs_oracle_linear(u, w_qkv, b_qkv, M, D, 3 * D, qkv);
        rs_oracle_attention(qkv, qkv + D, qkv + 2 * D, att, B, H, N, dh,
                            N * 3 * D, 3 * D, dh, N * D, D, dh, attn_scale);
        rs_oracle_linear(att, w_proj, b_proj, M, D, D, sa);
        for (size_t t = 0; t < md; ++t) x1[t] = sa[t] + x[t];
        rs_oracle_layernorm(x1, ln2_g, ln2_b, ln_eps, M, D, u);
        rs_oracle_linear(u, w_fc1, b_fc1, M, D, Dm, hid);
        for (size_t t = 0; t < (size_t)M * (size_t)Dm; ++t) hid[t] = rs_oracle_gelu(hid[t]);
        rs_oracle_linear(hid, w_fc2, b_fc2, M, Dm, D, mlp);
        for (size_t t = 0; t < md; ++t) xhat[t] = mlp[t] + x1[t];
        if (scores) {
            const double *f_out = op == 0 ? mlp : op == 1 ? sa : op == 2 ? xhat : op == 3 ? xhat : mlp;
            const double *f_in = op == 0 ? x1 : op == 1 ? x : op == 2 ? x : op == 3 ? x1 : u;
            rs_oracle_shift_scores(f_out, f_in, M, D, dist, scores);   /* u still holds LN(x1) */
        }
        if (sa_out) memcpy(sa_out, sa, sizeof(double) * md);
        if (x1_out) memcpy(x1_out, x1, sizeof(double) * md);
        if (mlp_out) memcpy(mlp_out, mlp, sizeof(double) * md);
        if (xhat_out) memcpy(xhat_out, xhat, sizeof(double) * md);
        rc = 0;
    }
    free(u); free(qkv); free(att); free(x1); free(hid); free(mlp); free(sa); free(xhat);
    return rc;
}
