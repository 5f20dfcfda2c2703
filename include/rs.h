/*
 * rs.h -- C ABI of the representation-shift hot path for MI355X (gfx950).
 *
 * The library runs, on one GPU, a pre-LayerNorm ViT encoder block with fused
 * multi-head attention (the attention map is never written to memory), scores
 * every token by its representation shift around the MLP, keeps the highest
 * scoring tokens (plus a protected prefix such as the class token) and compacts
 * the survivors for the next block.
 *
 * Conventions shared by every call
 *   - Every data pointer is a DEVICE pointer owned by the caller, unless a
 *     comment says "host".  The library never allocates, frees or keeps device
 *     memory; scratch space comes in through the `workspace` argument.
 *   - Tensors are dense row-major.  B images, N tokens per image entering the
 *     call, D channels, H heads of dh = D/H = 64 channels, Dm MLP width.
 *     Linear weights are [in, out] ("[Q,K,V] = xW, W in R^{C x 3C}", Sec. 3.1).
 *   - dtype selects storage AND arithmetic of activations and weights:
 *     RS_F32 = fp32 storage, fp32 multiply-accumulate; RS_BF16 = bf16 storage,
 *     bf16 matrix-core products accumulated in fp32.  Scores are always fp32,
 *     indices int32.
 *   - All work is enqueued on the caller's stream (`hip_stream` is a
 *     hipStream_t, NULL = the default stream).  No call synchronises with the
 *     host or copies to the host; outputs are valid once the stream reaches
 *     that point.  Output shapes depend only on host-known integers.
 *   - Every call returns an rs_status.  Argument errors are found before any
 *     kernel is launched and leave the device untouched; rs_last_error() gives
 *     a message for the calling thread's most recent failure.
 *   - Same inputs give bit-identical outputs (no floating-point atomics).
 *   - Alignment: every tensor pointer must be 16-byte aligned.
 */
#ifndef RS_H
#define RS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RS_API __attribute__((visibility("default")))

typedef enum {
    RS_OK = 0,
    RS_ERR_INVALID_ARG = 1,        /* NULL pointer, non-positive size, misaligned pointer ... */
    RS_ERR_UNSUPPORTED = 2,        /* valid request outside what the kernels cover            */
    RS_ERR_WORKSPACE_TOO_SMALL = 3,
    RS_ERR_DEVICE = 4              /* a HIP call or kernel launch failed                      */
} rs_status;

typedef enum { RS_F32 = 0, RS_BF16 = 1 } rs_dtype;

/* Distance D of the representation shift ("Distance metrics", Sec. 3.3).
 * L2 is the paper's default. */
typedef enum { RS_DIST_L2 = 0, RS_DIST_L1 = 1, RS_DIST_COS = 2 } rs_dist;

/* Which pair (f_out, f_in) the shift s = D(f_out, f_in) of rs_block_fwd is taken over
 * ("Operation choice", Sec. 3.3).  With x' = SA(LN(x)) + x and xhat = MLP(LN(x')) + x':
 *   RS_SHIFT_MLP         case (ii), the paper's default:  D(MLP(LN(x')), x')
 *   RS_SHIFT_ATTN        case (i):                        D(SA(LN(x)), x)
 *   RS_SHIFT_BLOCK       case (iii):                      D(xhat, x)
 * and the two other ways "the shift before and after the MLP" can be read:
 *   RS_SHIFT_MLP_STREAM  residual stream around the MLP:  D(xhat, x')
 *   RS_SHIFT_MLP_NORMED  the MLP's own input and output:  D(MLP(v), v), v = LN(x')
 * Every choice is computed in the epilogue of the GEMM that produces f_out; pruning always
 * happens after the whole block. */
typedef enum {
    RS_SHIFT_MLP = 0, RS_SHIFT_ATTN = 1, RS_SHIFT_BLOCK = 2, RS_SHIFT_MLP_STREAM = 3,
    RS_SHIFT_MLP_NORMED = 4
} rs_shift_op;

/* Weights of one encoder block, Eqs. (5),(6) of Sec. 3.3.  Element type follows
 * cfg->dtype.  Any bias pointer may be NULL (= zero); LayerNorm gamma NULL = 1,
 * beta NULL = 0.  W_qkv columns are ordered [Q | K | V], each H heads of dh. */
typedef struct {
    const void *ln1_g, *ln1_b;     /* [D]                 */
    const void *w_qkv, *b_qkv;     /* [D, 3D], [3D]       */
    const void *w_proj, *b_proj;   /* [D, D], [D]         */
    const void *ln2_g, *ln2_b;     /* [D]                 */
    const void *w_fc1, *b_fc1;     /* [D, Dm], [Dm]       */
    const void *w_fc2, *b_fc2;     /* [Dm, D], [D]        */
    /* Optional: buffer of rs_packed_weights_size() bytes filled by rs_pack_weights()
     * from the tensors above: the four matrices as [out, in], with the LayerNorm scales
     * folded into W_qkv and W_fc1 (rounded to bf16), plus the fp32 column sums and the
     * biases beta W + b those two GEMMs need to apply the normalisation in their
     * epilogues.  It depends on every pointer above except b_proj and b_fc2: re-pack when
     * any of them changes.  NULL = the library re-packs into the workspace on every
     * rs_block_fwd call (RS_BF16 only; RS_F32 needs no packing). */
    const void *packed;
} rs_block_weights;

typedef struct {
    int32_t B, N, D, H, Dm;        /* D/H must be 64, D % 64 == 0, Dm % 64 == 0            */
    int32_t n_prefix;              /* tokens [0, n_prefix) are always kept (1 = class token) */
    int32_t n_keep;                /* non-prefix tokens kept; K = n_prefix + n_keep;        */
                                   /* n_keep == N - n_prefix keeps every token              */
    float ln_eps;                  /* LayerNorm epsilon (> 0)                               */
    float attn_scale;              /* softmax scale; <= 0 selects 1/sqrt(dh)                */
    rs_dtype dtype;
    rs_dist dist;
    rs_shift_op op;
} rs_block_cfg;

/* Thread-local message of the calling thread's most recent failing call
 * (static storage, never NULL). */
RS_API const char *rs_last_error(void);

/* Library version as major*10000 + minor*100 + patch. */
RS_API int32_t rs_version(void);

/* Host string (static storage): the tile configurations the matrix kernels were built with.
 * Counter readings carried from one profiling run to another are valid only for the same string. */
RS_API const char *rs_build_info(void);

/* Tuning aid (process-wide, not part of the method): which tile variant the bf16 matrix kernels
 * use.  0 = chosen by shape (the default), 1 = 256 x 256 persistent workgroups, 2 = 256 x 128 and
 * 3 = 128 x 128 tiles with two workgroups per compute unit.  Every variant gives the same bits;
 * only the speed differs.  The environment variable RS_GEMM_FORCE sets the initial value. */
RS_API rs_status rs_tune_gemm_variant(int32_t variant);

/*
 * Measurement aid (not part of the method): while enabled, every kernel the library
 * launches is bracketed by two HIP events on the caller's stream.  rs_profile_read waits
 * for the recorded events (host synchronisation), adds the elapsed milliseconds and the
 * launch counts per kernel class into ms_out[RS_PROFILE_CLASSES] and
 * launches_out[RS_PROFILE_CLASSES] (host arrays), and forgets the records.
 * Classes, by index: see rs_profile_class_name (host string, static storage).
 */
#define RS_PROFILE_CLASSES 11
RS_API rs_status rs_profile_enable(int32_t enable);
RS_API rs_status rs_profile_read(double *ms_out, int64_t *launches_out);
RS_API const char *rs_profile_class_name(int32_t cls);

/*
 * Fused multi-head self-attention, Eq. (1) of Sec. 3.1:
 *     O = Softmax(Q K^T * scale) V     per image and head,
 * computed tile by tile with a running row maximum and row sum so that the
 * N x N attention map never leaves the chip.
 *   q, k, v : element (b, n, h, d) at  b*stride_b + n*stride_n + h*stride_h + d
 *             (strides in ELEMENTS, shared by q, k and v; d is contiguous);
 *             strides must be multiples of 8 elements (16 bytes in bf16); bf16 needs
 *             (N + 256) * stride_n * 2 bytes < 2 GiB (RS_ERR_UNSUPPORTED otherwise).
 *   o       : same addressing with the o_stride_* values; must not alias q, k, v.
 *   dh      : must be 64.   scale: the caller's (1/sqrt(dh) for ViT heads; the
 *             paper prints 1/sqrt(C)).   Needs no workspace.
 */
RS_API rs_status rs_attention_fwd(const void *q, const void *k, const void *v, void *o,
                           int32_t B, int32_t H, int32_t N, int32_t dh,
                           int64_t stride_b, int64_t stride_n, int64_t stride_h,
                           int64_t o_stride_b, int64_t o_stride_n, int64_t o_stride_h,
                           float scale, rs_dtype dtype, void *hip_stream);

/*
 * Standard (unfused) attention with the attention map written to memory, and the attention-based
 * token importance that needs it (Sec. 3.1, Eqs. (2), (3); the "Self-Attention" row of Table 1).
 * This is the comparison system the method is measured against, kept out of the hot path: the
 * fused call above never has the map.
 *     A = Softmax(Q K^T * scale)            per image and head, written to attn_map
 *     O = A V
 *     s_cls[b, j]  = mean over heads of A[b, h, cls_index, j]                  Eq. (2)
 *     s_mean[b, j] = mean over heads of (1/N) sum_i A[b, h, i, j]              Eq. (3)
 *   (the paper writes both scores for one head; with H heads the mean over heads is taken)
 *   q, k, v, o, strides, dh, scale : as in rs_attention_fwd.   dtype : RS_BF16 only.
 *   attn_map : bf16 [B, H, N, Np] out, Np = N rounded up to a multiple of 64 (columns past N are
 *              zero), rs_attention_map_size bytes.
 *   s_cls, s_mean : float [B, N] out, either may be NULL.    cls_index in [0, N).
 *   workspace : rs_attention_map_workspace_size bytes, 256-byte aligned (packed heads, column sums).
 *   B * H <= 65535.  Deterministic.
 */
RS_API size_t rs_attention_map_size(int32_t B, int32_t H, int32_t N);
RS_API size_t rs_attention_map_workspace_size(int32_t B, int32_t H, int32_t N);
RS_API rs_status rs_attention_map_fwd(const void *q, const void *k, const void *v, void *o,
                               int32_t B, int32_t H, int32_t N, int32_t dh,
                               int64_t stride_b, int64_t stride_n, int64_t stride_h,
                               int64_t o_stride_b, int64_t o_stride_n, int64_t o_stride_h,
                               float scale, rs_dtype dtype, int32_t cls_index,
                               void *attn_map, float *s_cls, float *s_mean,
                               void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Representation shift score, selection and compaction (Eq. (4) of Sec. 3.2;
 * pruning of the lowest-score tokens, Secs. 3.1 and 3.2):
 *     scores[b, i] = D(f_out[b, i, :], f_in[b, i, :])
 *     per image, among tokens i >= n_prefix, the n_keep highest scores survive
 *     (equal scores: the lower index wins); kept_idx[b, :] lists the prefix and
 *     the survivors in ascending index order (K = n_prefix + n_keep entries);
 *     gathered[b, j, :] = src[b, kept_idx[b, j], :].
 *   f_out, f_in : [B, N, D]  F(x) and x.            src : [B, N, D] or NULL (= f_in).
 *   scores      : float [B, N], required.           kept_idx : int32 [B, K], required.
 *   gathered    : [B, K, D] or NULL (no gather); must not alias src.
 *   D % 8 == 0.  NaN scores order above +inf.  workspace: rs_shift_topk_workspace_size bytes.
 */
RS_API size_t rs_shift_topk_workspace_size(int32_t B, int32_t N, int32_t D, rs_dtype dtype);
RS_API rs_status rs_shift_topk(const void *f_out, const void *f_in, const void *src,
                        int32_t B, int32_t N, int32_t D, int32_t n_prefix, int32_t n_keep,
                        rs_dist dist, rs_dtype dtype,
                        float *scores, int32_t *kept_idx, void *gathered,
                        void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * One-off re-layout of a block's four weight matrices for the matrix-core
 * GEMMs (weights are static at inference; the method is training-free).
 * `packed_out` must hold rs_packed_weights_size(cfg) bytes and is then passed
 * as rs_block_weights.packed.  Only cfg->D, Dm, dtype are read.
 */
RS_API size_t rs_packed_weights_size(const rs_block_cfg *cfg);
RS_API rs_status rs_pack_weights(const rs_block_cfg *cfg, const rs_block_weights *w,
                          void *packed_out, void *hip_stream);

/*
 * Line-wise pruning of a 2-D token grid (Sec. 4.2, "CNN and SSM", variant (ii)): for feature maps
 * without a token sequence the shift s[b,h,w] = D(f_out[b,h,w,:], f_in[b,h,w,:]) (Eq. (4)) is
 * averaged along every row and every column, and whole lines with the lowest averages are
 * removed so that the grid stays rectangular.
 *   f_out, f_in : [B, H, W, C] channel-last, same shape (which two maps of a stage to compare
 *                 is the caller's choice: the paper compares a stage's input and output).
 *   src         : [B, H, W, C] map to cut down, NULL = f_out (the stage output).
 *   keep_rows, keep_cols : lines kept per image (ties: lower index kept; order ascending).
 *   scores [B,H,W], row_scores [B,H], col_scores [B,W] : fp32 outputs, all required.
 *   kept_rows [B, keep_rows], kept_cols [B, keep_cols] : int32 outputs.
 *   gathered [B, keep_rows, keep_cols, C] or NULL; must not alias src.
 * C % 8 == 0.  No workspace.  Deterministic.
 */
RS_API rs_status rs_grid_line_prune(const void *f_out, const void *f_in, const void *src, int32_t B,
                                    int32_t H, int32_t W, int32_t C, int32_t keep_rows,
                                    int32_t keep_cols, rs_dist dist, rs_dtype dtype, float *scores,
                                    float *row_scores, float *col_scores, int32_t *kept_rows,
                                    int32_t *kept_cols, void *gathered, void *hip_stream);

/*
 * Token-wise pruning of a 2-D token grid (Sec. 4.2, "CNN and SSM", variant (i): "removing the least
 * important tokens from each row and column").  The passage does not say how the grid stays
 * rectangular; the reading built here: every ROW first loses its W - keep_cols lowest-shift positions
 * and closes up (position j of row h is then that row's j-th survivor), after which every COLUMN of
 * the compacted H x keep_cols grid loses its H - keep_rows lowest-shift positions and closes up.
 * Ties: the lower index survives; survivors keep their order.
 *   f_out, f_in, src : as in rs_grid_line_prune ([B, H, W, C], src NULL = f_out).
 *   scores     [B, H, W]                 fp32 out: shift per position.
 *   kept_cols  [B, H, keep_cols]         int32 out: per row, the surviving column indices, ascending.
 *   col_scores [B, keep_cols, H]         fp32 out: shift of the row-compacted grid, column by column.
 *   kept_rows  [B, keep_cols, keep_rows] int32 out: per compacted column, surviving row indices, ascending.
 *   gathered   [B, keep_rows, keep_cols, C] or NULL:
 *              gathered[b, i, j, :] = src[b, r, kept_cols[b, r, j], :] with r = kept_rows[b, j, i].
 * C % 8 == 0, B*H <= 2^31 - 1 grid rows.  No workspace.  Deterministic.
 */
RS_API rs_status rs_grid_token_prune(const void *f_out, const void *f_in, const void *src, int32_t B,
                                     int32_t H, int32_t W, int32_t C, int32_t keep_rows,
                                     int32_t keep_cols, rs_dist dist, rs_dtype dtype, float *scores,
                                     int32_t *kept_cols, float *col_scores, int32_t *kept_rows,
                                     void *gathered, void *hip_stream);

/*
 * One linear layer of the block with its fused elementwise tail (the four contractions of
 * Eqs. (5),(6): QKV, output projection, fc1, fc2; the O(N C^2) term of Sec. 3.1):
 *     out = epilogue(a @ W + bias)
 *   RS_EPI_BIAS       out = a W + bias
 *   RS_EPI_BIAS_GELU  out = GELU(a W + bias)          (exact-erf GELU)
 *   RS_EPI_BIAS_RES   out = a W + bias + res
 *   a : [M, K].   out, res : [M, N]; out must not alias a.   bias : [N] or NULL.
 *   w : RS_F32: the [K, N] matrix as is.  RS_BF16: the [N, K] re-layout written by
 *       rs_pack_linear (wt must hold N*K elements).
 *   K % 64 == 0, N % 64 == 0.
 */
typedef enum { RS_EPI_BIAS = 0, RS_EPI_BIAS_GELU = 1, RS_EPI_BIAS_RES = 2 } rs_epilogue;
RS_API rs_status rs_pack_linear(const void *w, void *wt, int32_t K, int32_t N, rs_dtype dtype,
                                void *hip_stream);
RS_API rs_status rs_linear_fwd(const void *a, const void *w, const void *bias, const void *res,
                               void *out, int64_t M, int32_t N, int32_t K, rs_epilogue epi,
                               rs_dtype dtype, void *hip_stream);

/*
 * One pre-LN encoder block followed by representation-shift pruning
 * (Eqs. (5),(6) and case (ii) of "Operation choice", Sec. 3.3):
 *     x1   = SA(LN(x)) + x             SA = fused attention + output projection
 *     mlp  = W2 GELU(W1 LN(x1) + b1) + b2        (exact-erf GELU)
 *     xhat = mlp + x1
 *     scores[b, i] = D(f_out[b, i, :], f_in[b, i, :])   pair by cfg->op (default: mlp, x1),
 *                                                        distance by cfg->dist (default L2)
 *     kept_idx, y  = selection and gather of xhat as in rs_shift_topk.
 *   RS_BF16: the two LayerNorms are applied inside the GEMMs that follow them (their scale is
 *   folded into the packed weights, mean and variance come from a row-statistics pass), so the
 *   normalised rows are never written; results agree with the definition above to bf16 rounding.
 *   x        : [B, N, D] in.            y : [B, K, D] out, must not alias x.
 *   kept_idx : int32 [B, K] out.        scores : float [B, N] out, or NULL.
 *   workspace: rs_block_workspace_size(cfg) bytes, 256-byte aligned.
 * Restrictions: D/H == 64, D % 64 == 0, Dm % 64 == 0, D <= 4096, B*N < 2^31 and, in bf16,
 *   (N + 256) * 3 D * 2 bytes < 2 GiB; else RS_ERR_UNSUPPORTED.
 */
RS_API size_t rs_block_workspace_size(const rs_block_cfg *cfg);
RS_API rs_status rs_block_fwd(const rs_block_cfg *cfg, const rs_block_weights *w,
                       const void *x, void *y, int32_t *kept_idx, float *scores,
                       void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * rs_block_fwd for a caller that runs a stack of blocks: the LayerNorm in front of a block's
 * attention (Eq. (5)) needs the mean and variance of every input row, and the previous block has
 * those rows in registers when it writes them.  Same computation and bit-identical y, kept_idx and
 * scores as rs_block_fwd; the only difference is where the row statistics of x come from.
 *   x_stats : float [B * N, 2] in, or NULL: (mean, 1 / sqrt(variance + ln_eps)) of every row of x,
 *             population variance, exactly as a previous call wrote them to its y_stats with the
 *             same D and ln_eps.  NULL: computed here, as rs_block_fwd does.  RS_F32 ignores it.
 *   y_stats : float [B * K, 2] out, or NULL: the same statistics of every row of y.  With pruning
 *             (bf16, D <= 4096) the gather writes them on its way; otherwise a statistics pass over
 *             y runs at the end of the call.  May be the buffer x_stats points to.
 *   x_stats and y_stats must be 8-byte aligned and lie outside the workspace; y_stats must not
 *   overlap x, y, kept_idx or scores.  Everything else as in rs_block_fwd.
 */
RS_API rs_status rs_block_fwd_chained(const rs_block_cfg *cfg, const rs_block_weights *w,
                                      const void *x, const float *x_stats, void *y, float *y_stats,
                                      int32_t *kept_idx, float *scores, void *workspace,
                                      size_t workspace_bytes, void *hip_stream);

/*
 * rs_block_fwd for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * computation, same kernels and bit-identical outputs as rs_block_fwd; the scratch tensors live
 * in a buffer of rs_block_static_scratch_size() bytes (64 MiB) that is part of the library's
 * device code: every GPU the library runs on holds its own copy from the first use until the
 * process ends.  The call allocates nothing and frees nothing.
 *   - cfg must satisfy rs_block_workspace_size(cfg) <= rs_block_static_scratch_size(), else
 *     RS_ERR_UNSUPPORTED (a ViT-B/16 block in bf16 fits up to 16 images of 197 tokens; larger
 *     batches go through rs_block_fwd).
 *   - x, y, kept_idx, scores: as in rs_block_fwd, caller-owned.
 *   - All calls on one GPU share that GPU's buffer: calls that overlap in time on one GPU (two
 *     streams, two host threads) race on it and give undefined results; calls on one stream are
 *     ordered and safe.  Nothing in the buffer has to start at zero, so a call leaves nothing
 *     behind that the next one depends on.
 */
RS_API size_t rs_block_static_scratch_size(void);
RS_API rs_status rs_block_fwd_static(const rs_block_cfg *cfg, const rs_block_weights *w,
                                     const void *x, void *y, int32_t *kept_idx, float *scores,
                                     void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* RS_H */
