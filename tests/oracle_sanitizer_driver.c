/*
 * TEST INFRASTRUCTURE ONLY.  Driver for a sanitizer build of the CPU checker (oracle/rs_oracle.c):
 * compiled together with it under -fsanitize=address,undefined by tests/test_oracle_sanitizers.py
 * and run as a process of its own.  Exactly sized heap buffers, so that any access past an end or
 * any undefined arithmetic aborts the run; a few closed forms (Sec. 3.1 Eq. (1): V = 1 gives O = 1;
 * Sec. 3.2 Eq. (4): an identity sub-layer gives zero shift; all-equal scores keep the lowest
 * indices) are checked on the way.  Prints "ok" and exits 0.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void rs_oracle_layernorm(const double *x, const double *gamma, const double *beta, double eps, int64_t M,
                         int64_t D, double *out);
void rs_oracle_linear(const double *a, const double *w, const double *bias, int64_t M, int64_t K, int64_t N,
                      double *out);
void rs_oracle_attention(const double *q, const double *k, const double *v, double *o, int64_t B, int64_t H,
                         int64_t N, int64_t dh, int64_t sb, int64_t sn, int64_t sh, int64_t osb, int64_t osn,
                         int64_t osh, double scale);
void rs_oracle_shift_scores(const double *f_out, const double *f_in, int64_t M, int64_t D, int dist, double *scores);
void rs_oracle_topk(const double *scores, int64_t B, int64_t N, int64_t n_prefix, int64_t n_keep, int32_t *kept_idx);
void rs_oracle_gather(const double *src, const int32_t *kept_idx, int64_t B, int64_t N, int64_t K, int64_t D,
                      double *out);
int rs_oracle_block(int64_t B, int64_t N, int64_t D, int64_t H, int64_t Dm, double ln_eps, double attn_scale,
                    int dist, int op, const double *x, const double *ln1_g, const double *ln1_b,
                    const double *w_qkv, const double *b_qkv, const double *w_proj, const double *b_proj,
                    const double *ln2_g, const double *ln2_b, const double *w_fc1, const double *b_fc1,
                    const double *w_fc2, const double *b_fc2, double *sa_out, double *x1_out, double *mlp_out,
                    double *xhat_out, double *scores);

static uint64_t state = 0x9E3779B97F4A7C15ull;
static double rnd(void) {  /* xorshift, uniform in (-1, 1) */
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (double)(state >> 11) / 9007199254740992.0 * 2.0 - 1.0;
}
static double *vec(int64_t n, int fill_random, double value) {
    double *p = (double *)malloc((size_t)(n > 0 ? n : 1) * sizeof(double));
    if (!p) { fprintf(stderr, "out of memory\n"); exit(2); }
    for (int64_t i = 0; i < n; ++i) p[i] = fill_random ? rnd() : value;
    return p;
}
#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "check failed: %s (line %d)\n", #cond, __LINE__); exit(1); } } while (0)

int main(void) {
    /* ragged sizes on purpose: nothing is a multiple of anything */
    const int64_t B = 2, N = 13, H = 3, dh = 5, D = H * dh, Dm = 7;
    double *x = vec(B * N * D, 1, 0), *out = vec(B * N * D, 0, 0);
    double *g = vec(D, 1, 0), *bt = vec(D, 1, 0);
    rs_oracle_layernorm(x, g, bt, 1e-6, B * N, D, out);
    rs_oracle_layernorm(x, NULL, NULL, 1e-6, B * N, D, out);
    for (int64_t i = 0; i < B * N * D; ++i) CHECK(isfinite(out[i]));

    double *w = vec(D * Dm, 1, 0), *bias = vec(Dm, 1, 0), *lo = vec(B * N * Dm, 0, 0);
    rs_oracle_linear(x, w, bias, B * N, D, Dm, lo);
    rs_oracle_linear(x, w, NULL, B * N, D, Dm, lo);

    /* attention on strided views of a packed [B, N, 3, H, dh] buffer; V = 1 gives O = 1 */
    double *qkv = vec(B * N * 3 * D, 1, 0), *o = vec(B * N * D, 0, 0);
    for (int64_t b = 0; b < B; ++b)
        for (int64_t n = 0; n < N; ++n)
            for (int64_t d = 0; d < D; ++d) qkv[((b * N + n) * 3 + 2) * D + d] = 1.0;
    rs_oracle_attention(qkv, qkv + D, qkv + 2 * D, o, B, H, N, dh, N * 3 * D, 3 * D, dh, N * D, D, dh, 0.4);
    for (int64_t i = 0; i < B * N * D; ++i) CHECK(fabs(o[i] - 1.0) < 1e-12);
    rs_oracle_attention(qkv, qkv + D, qkv + 2 * D, o, B, H, 1, dh, N * 3 * D, 3 * D, dh, N * D, D, dh, 0.4); /* N = 1 */

    /* shift scores: identity gives zero under L2 and L1; all three distances run */
    double *s = vec(B * N, 0, 0);
    for (int dist = 0; dist < 3; ++dist) rs_oracle_shift_scores(out, x, B * N, D, dist, s);
    rs_oracle_shift_scores(x, x, B * N, D, 0, s);
    for (int64_t i = 0; i < B * N; ++i) CHECK(s[i] == 0.0);

    /* selection: every (n_prefix, n_keep) that fits, on all-equal scores -> the lowest indices */
    for (int64_t p = 0; p <= N; ++p)
        for (int64_t kk = 0; kk <= N - p; ++kk) {
            int32_t *kept = (int32_t *)malloc((size_t)(B * (p + kk) > 0 ? B * (p + kk) : 1) * sizeof(int32_t));
            rs_oracle_topk(s, B, N, p, kk, kept);
            for (int64_t b = 0; b < B; ++b)
                for (int64_t j = 0; j < p + kk; ++j) CHECK(kept[b * (p + kk) + j] == (int32_t)j);
            double *gt = vec(B * (p + kk) * D, 0, 0);
            rs_oracle_gather(x, kept, B, N, p + kk, D, gt);
            free(gt);
            free(kept);
        }
    /* random scores: ascending, distinct, in range */
    for (int64_t i = 0; i < B * N; ++i) s[i] = rnd();
    {
        int32_t kept[2 * 6];
        rs_oracle_topk(s, B, N, 1, 5, kept);
        for (int64_t b = 0; b < B; ++b) {
            CHECK(kept[b * 6] == 0);
            for (int j = 1; j < 6; ++j) CHECK(kept[b * 6 + j] > kept[b * 6 + j - 1] && kept[b * 6 + j] < N);
        }
    }

    /* whole block, every operation choice and distance, with and without biases */
    double *wq = vec(D * 3 * D, 1, 0), *bq = vec(3 * D, 1, 0), *wp = vec(D * D, 1, 0), *bp = vec(D, 1, 0);
    double *w1 = vec(D * Dm, 1, 0), *b1 = vec(Dm, 1, 0), *w2 = vec(Dm * D, 1, 0), *b2 = vec(D, 1, 0);
    double *sa = vec(B * N * D, 0, 0), *x1 = vec(B * N * D, 0, 0), *mlp = vec(B * N * D, 0, 0), *xh = vec(B * N * D, 0, 0);
    for (int op = 0; op < 5; ++op)
        for (int dist = 0; dist < 3; ++dist) {
            CHECK(rs_oracle_block(B, N, D, H, Dm, 1e-6, 0.3, dist, op, x, g, bt, wq, bq, wp, bp, g, bt, w1, b1, w2, b2,
                                  sa, x1, mlp, xh, s) == 0);
            for (int64_t i = 0; i < B * N; ++i) CHECK(isfinite(s[i]));
        }
    CHECK(rs_oracle_block(B, N, D, H, Dm, 1e-6, 0.3, 0, 0, x, NULL, NULL, wq, NULL, wp, NULL, NULL, NULL, w1, NULL, w2,
                          NULL, sa, x1, mlp, xh, s) == 0);
    CHECK(rs_oracle_block(B, N, D, H, Dm, 1e-6, 0.3, 0, 9, x, g, bt, wq, bq, wp, bp, g, bt, w1, b1, w2, b2, sa, x1, mlp,
                          xh, s) != 0);  /* unknown operation: an error code, nothing else */
    free(x); free(out); free(g); free(bt); free(w); free(bias); free(lo); free(qkv); free(o); free(s);
    free(wq); free(bq); free(wp); free(bp); free(w1); free(b1); free(w2); free(b2); free(sa); free(x1); free(mlp); free(xh);
    printf("ok\n");
    return 0;
}
