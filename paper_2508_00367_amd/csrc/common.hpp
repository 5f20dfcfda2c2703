// Shared device/host helpers of the representation-shift HIP library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rs.h"

namespace rs {

constexpr int kWave = 64;  // CDNA wavefront width

typedef uint16_t bf16raw;  // bf16 storage: upper half of an fp32
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// ---- bf16 <-> fp32 -------------------------------------------------------
__device__ __forceinline__ float bf2f(bf16raw b) { return __uint_as_float(((uint32_t)b) << 16); }

// round-to-nearest-even, NaN stays NaN: the hardware conversion (v_cvt_pk_bf16_f32)
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ bf16raw f2bf(float f) { return __builtin_bit_cast(bf16raw, (__bf16)f); }

__device__ __forceinline__ uint32_t pack2bf(float lo, float hi) {
    bf16x2 v;
    v[0] = (__bf16)lo;
    v[1] = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, v);
}

// Storage-type traits: load/store 8 consecutive elements as fp32.
template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr rs_dtype dtype = RS_F32;
    __device__ static __forceinline__ void load8(const float* p, float (&v)[8]) {
        float4 a = *reinterpret_cast<const float4*>(p);
        float4 b = *reinterpret_cast<const float4*>(p + 4);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
        v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    }
    __device__ static __forceinline__ void store8(float* p, const float (&v)[8]) {
        *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
        *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
    }
    __device__ static __forceinline__ float ld(const float* p) { return *p; }
    __device__ static __forceinline__ void st(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16raw> {
    static constexpr rs_dtype dtype = RS_BF16;
    __device__ static __forceinline__ void load8(const bf16raw* p, float (&v)[8]) {
        uint4 a = *reinterpret_cast<const uint4*>(p);
        uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    __device__ static __forceinline__ void store8(bf16raw* p, const float (&v)[8]) {
        uint4 a;
        a.x = pack2bf(v[0], v[1]); a.y = pack2bf(v[2], v[3]);
        a.z = pack2bf(v[4], v[5]); a.w = pack2bf(v[6], v[7]);
        *reinterpret_cast<uint4*>(p) = a;
    }
    __device__ static __forceinline__ float ld(const bf16raw* p) { return bf2f(*p); }
    __device__ static __forceinline__ void st(bf16raw* p, float v) { *p = f2bf(v); }
};

// ---- wave reductions (fixed butterfly order: deterministic) ---------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// Statistics of a row a wave holds as MAXC chunks of 8 values per lane (lane l: chunks l, l + 64,
// ...; chunks at or past nchunk are not read): (mean, 1 / sqrt(population variance + eps)), the
// variance taken over the deviations from the mean.  One fixed order of additions, shared by
// every kernel that produces LayerNorm statistics, so that they all give the same bits.
template <int MAXC>
__device__ __forceinline__ float2 wave_row_stats(const float (&v)[MAXC][8], int nchunk, int lane, int D, float eps) {
    float sum = 0.f;
#pragma unroll
    for (int c = 0; c < MAXC; ++c)
        if (lane + c * 64 < nchunk) {
#pragma unroll
            for (int i = 0; i < 8; ++i) sum += v[c][i];
        }
    const float mean = wave_sum(sum) / (float)D;
    float sq = 0.f;
#pragma unroll
    for (int c = 0; c < MAXC; ++c)
        if (lane + c * 64 < nchunk) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float d = v[c][i] - mean;
                sq += d * d;
            }
        }
    return make_float2(mean, rsqrtf(wave_sum(sq) / (float)D + eps));
}

// exact GELU: x * Phi(x)
__device__ __forceinline__ float gelu_erf(float x) {
    return 0.5f * x * (1.0f + erff(x * 0.70710678118654752440f));
}

// ---- host-side error plumbing ---------------------------------------------
void set_error(const char* fmt, ...);
rs_status device_error(const char* what, hipError_t e);

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline size_t elem_size(rs_dtype t) { return t == RS_F32 ? 4 : 2; }

// ---- kernel launchers (one per .hip file) -----------------------------------
// LayerNorm over the last axis of x[M, D]; gamma/beta may be null.
hipError_t launch_layernorm(rs_dtype dt, const void* x, const void* gamma, const void* beta,
                            void* out, int64_t M, int D, float eps, hipStream_t s);

// stats[M] = (mean, 1 / sqrt(population variance + eps)) of each row of x[M, D], as float pairs.
// iota_out (optional): int32 [M], receives row % iota_n (the kept_idx of a block that keeps every token).
hipError_t launch_rowstats(rs_dtype dt, const void* x, float* stats, int64_t M, int D, float eps,
                           hipStream_t s, int32_t* iota_out = nullptr, int iota_n = 1);

enum GemmEpilogue {
    EPI_BIAS = 0,            // out = acc + bias
    EPI_BIAS_GELU = 1,       // out = gelu(acc + bias)
    EPI_BIAS_RES = 2,        // out = acc + bias + res
    EPI_BIAS_RES_SHIFT = 3,  // out = acc + bias + res; partial sums of D(f_out, f_in) per row, with
                             // f_out = acc + bias (or out, if `post`) and f_in = res (or `ref`, if given)
    // bf16 only: the A operand is the raw input x of a LayerNorm whose scale is folded into the
    // packed weights, acc = x (gamma * W);  LN(x) W + b = rstd * (acc - mean * colsum) + bias'
    // with per-row (mean, rstd) and per-column colsum = sum_k gamma_k W_kn, bias' = beta W + b.
    EPI_LN_BIAS = 4,         // out = rstd * (acc - mean * colsum) + bias'
    EPI_LN_BIAS_GELU = 5     // out = gelu(rstd * (acc - mean * colsum) + bias')
};

// Per-row and per-column vectors of the EPI_LN_* epilogues (all fp32, device memory).
struct GemmLnFold {
    const float* stats;   // [M][2]  (mean, rstd)
    const float* colsum;  // [N]
    const float* bias;    // [N]
};

// Largest K and N of a GEMM: a workgroup addresses the (at most 256) rows of its tile with 32-bit
// byte offsets from the tile's first row, 256 * K * 2 bytes, and the copies of a K slice that does
// not exist are aimed at byte 0x7ff00000 of a resource that ends with the tile's last row.
constexpr int kGemmMaxK = 1 << 20;
constexpr int kGemmMaxN = 1 << 20;

// Tile configurations the bf16 GEMM was built with (measurements carried from one run to another
// are only valid for the same string).
const char* gemm_build_info();
// bf16 tile variant switch (0 = by shape, 1 = 256 x 256 persistent, 2 = 256 x 128 ring, 3 = 128 x 128 ring)
int gemm_variant();
void set_gemm_variant(int v);

// Number of per-row partial slots the SHIFT epilogue writes for an output width N.
int gemm_shift_slots(rs_dtype dt, int N);
constexpr int kShiftLanes = 3;  // floats per slot (L2/L1 use the first, cosine all three)

// out[M, N] = epilogue(a[M, K] @ W).  bf16: `w` is the packed [N, K] matrix; fp32: `w` is the
// caller's [K, N] matrix.  partials: float [M, slots, kShiftLanes] for EPI_BIAS_RES_SHIFT.
hipError_t launch_gemm(rs_dtype dt, GemmEpilogue epi, rs_dist dist, const void* a, const void* w,
                       const void* bias, const void* res, void* out, float* partials,
                       const void* ref, bool post, int64_t M, int N, int K, hipStream_t s);
// bf16 GEMM behind a LayerNorm (EPI_LN_BIAS / EPI_LN_BIAS_GELU).
hipError_t launch_gemm_ln(GemmEpilogue epi, const void* x, const void* w_folded, GemmLnFold ln, void* out,
                          int64_t M, int N, int K, hipStream_t s);

// `count` independent bf16 products out_p[M, N] = a_p[M, K] @ wt_p[N, K]^T, problem p at element offset
// p * stride from each base pointer (K % 32 == 0, N % 64 == 0; rows of wt_p past N must exist as zeros)
hipError_t launch_gemm_batched(const void* a, const void* wt, void* out, int count, int64_t stride_a,
                               int64_t stride_w, int64_t stride_out, int M, int N, int K, hipStream_t s);

// Standard (unfused) attention with the map written to memory, the comparison system of Sec. 3.1:
// pack q, k (zero-padded to Np rows) and v^T per head; softmax rows of the [N, Np] score matrices in
// place; column sums of the map; output rows back to the caller's layout.
hipError_t launch_attn_pack(const void* q, const void* k, const void* v, void* qh, void* kh, void* vt, int B, int H,
                            int N, int Np, int64_t sb, int64_t sn, int64_t sh, hipStream_t s);
hipError_t launch_attn_softmax_rows(void* map, int64_t rows, int N, int Np, float scale_log2e, hipStream_t s);
hipError_t launch_attn_map_scores(const void* map, float* partial, float* s_cls, float* s_mean, int B, int H, int N,
                                  int Np, int cls_index, hipStream_t s);
hipError_t launch_attn_unpack(const void* oh, void* o, int B, int H, int N, int64_t osb, int64_t osn, int64_t osh,
                              hipStream_t s);

// bf16 [K, N] row-major -> [N, K] row-major; with `gamma` ([K] bf16) row k is scaled by gamma[k]
// (product rounded to bf16).
hipError_t launch_pack_transpose(const void* w, const void* gamma, void* wt, int K, int N, hipStream_t s);
// colsum[n] = sum_k bf16(gamma[k] * w[k][n]),  bias_out[n] = sum_k beta[k] * w[k][n] + bias[n]
// (w [K, N] bf16; gamma, beta, bias bf16 or null = 1, 0, 0; outputs fp32).
hipError_t launch_pack_ln_fold(const void* w, const void* gamma, const void* beta, const void* bias,
                               float* colsum, float* bias_out, int K, int N, hipStream_t s);

hipError_t launch_attention(rs_dtype dt, const void* q, const void* k, const void* v, void* o,
                            int B, int H, int N, int64_t sb, int64_t sn, int64_t sh,
                            int64_t osb, int64_t osn, int64_t osh, float scale, hipStream_t s);

// scores[M] = D(f_out[M, D], f_in[M, D])
hipError_t launch_shift_scores(rs_dtype dt, rs_dist dist, const void* f_out, const void* f_in,
                               float* scores, int64_t M, int D, hipStream_t s);
// scores[M] from the GEMM epilogue's partial slots
hipError_t launch_finalize_scores(rs_dist dist, const float* partials, int slots, float* scores,
                                  int64_t M, hipStream_t s);
// per image: the n_keep highest scores among tokens >= n_prefix, ascending kept_idx[B, K]
// the two steps above in one launch (a real selection only: n_keep < N - n_prefix, n_keep > 0;
// N must pass select_from_partials_fits)
bool select_from_partials_fits(int N);
hipError_t launch_select_from_partials(rs_dist dist, const float* partials, int slots, float* scores,
                                       int32_t* kept_idx, int B, int N, int n_prefix, int n_keep,
                                       hipStream_t s);
hipError_t launch_select(const float* scores, int32_t* kept_idx, int B, int N, int n_prefix,
                         int n_keep, hipStream_t s);
// out[b, j, :] = src[b, kept_idx[b, j], :]
hipError_t launch_gather(rs_dtype dt, const void* src, const int32_t* kept_idx, void* out, int B,
                         int N, int K, int D, hipStream_t s);
// The gather for bf16 rows of at most 4096 elements that also writes stats[B * K] = (mean,
// 1 / sqrt(variance + eps)) of every gathered row, bit-identical to launch_rowstats on `out`.
bool gather_stats_fits(rs_dtype dt, int D);
hipError_t launch_gather_stats(const void* src, const int32_t* kept_idx, void* out, float* stats, int B, int N,
                               int K, int D, float eps, hipStream_t s);

// scores, kept_idx and gathered = f_in[kept_idx] of every image in one launch that reads f_out and
// f_in once (images whose f_in rows fit a compute unit's registers: shift_topk_resident_fits)
bool shift_topk_resident_fits(rs_dtype dt, int N, int D);
hipError_t launch_shift_topk_resident(rs_dtype dt, rs_dist dist, const void* f_out, const void* f_in,
                                      float* scores, int32_t* kept_idx, void* gathered, int B, int N, int D,
                                      int n_prefix, int n_keep, hipStream_t s);

// 2-D grid: row_scores[b, h] = mean_w scores[b, h, w], col_scores[b, w] = mean_h scores[b, h, w]
hipError_t launch_grid_line_scores(const float* scores, float* row_scores, float* col_scores, int B, int H,
                                   int W, hipStream_t s);
// out[b, i, j, :] = src[b, kept_rows[b, i], kept_cols[b, j], :]   (src [B, H, W, C], out [B, R, Q, C])
hipError_t launch_grid_gather(rs_dtype dt, const void* src, const int32_t* kept_rows, const int32_t* kept_cols,
                              void* out, int B, int H, int W, int R, int Q, int C, hipStream_t s);

// token-wise grid pruning: col_scores[b, j, h] = scores[b, h, kept_cols[b, h, j]]
hipError_t launch_grid_compact_scores(const float* scores, const int32_t* kept_cols, float* col_scores, int B, int H,
                                      int W, int Q, hipStream_t s);
// out[b, i, j, :] = src[b, r, kept_cols[b, r, j], :], r = kept_rows[b, j, i]
hipError_t launch_grid_token_gather(rs_dtype dt, const void* src, const int32_t* kept_cols, const int32_t* kept_rows,
                                    void* out, int B, int H, int W, int R, int Q, int C, hipStream_t s);

}  // namespace rs
