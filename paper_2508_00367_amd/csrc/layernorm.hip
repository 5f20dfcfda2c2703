// LayerNorm of Eqs. (5),(6), Sec. 3.3: one wavefront per token row, the row held in
// registers, mean then variance of the deviations (population variance), fp32 statistics.
// HBM-bound: one read and one write of the row.
#include "common.hpp"

namespace rs {

// MAXC = 8-element chunks a lane may hold: D <= MAXC * 64 * 8.
template <typename T, int MAXC>
__global__ __launch_bounds__(256) void layernorm_kernel(const T* __restrict__ x,
                                                        const T* __restrict__ gamma,
                                                        const T* __restrict__ beta,
                                                        T* __restrict__ out, int64_t M, int D,
                                                        float eps) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= M) return;
    const int nchunk = D >> 3;
    const T* xr = x + row * D;
    float v[MAXC][8];
    float sum = 0.f;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        const int ch = lane + c * 64;
        if (ch < nchunk) {
            Elem<T>::load8(xr + ch * 8, v[c]);
#pragma unroll
            for (int i = 0; i < 8; ++i) sum += v[c][i];
        }
    }
    const float mean = wave_sum(sum) / (float)D;
    float sq = 0.f;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        const int ch = lane + c * 64;
        if (ch < nchunk) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                v[c][i] -= mean;
                sq += v[c][i] * v[c][i];
            }
        }
    }
    const float inv = rsqrtf(wave_sum(sq) / (float)D + eps);
    T* orow = out + row * D;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        const int ch = lane + c * 64;
        if (ch < nchunk) {
            float g[8], b[8], r[8];
            if (gamma) Elem<T>::load8(gamma + ch * 8, g);
            if (beta) Elem<T>::load8(beta + ch * 8, b);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                float t = v[c][i] * inv;
                if (gamma) t *= g[i];
                if (beta) t += b[i];
                r[i] = t;
            }
            Elem<T>::store8(orow + ch * 8, r);
        }
    }
}

// Row statistics only: stats[row] = (mean, 1 / sqrt(var + eps)), same two-pass arithmetic as above.
// The bf16 block feeds them to the GEMM that follows the LayerNorm, which applies the
// normalisation in its epilogue (the normalised rows are never written).
template <typename T, int MAXC>
__global__ __launch_bounds__(256) void rowstats_kernel(const T* __restrict__ x, float2* __restrict__ stats,
                                                       int64_t M, int D, float eps,
                                                       int32_t* __restrict__ iota_out, int iota_n) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= M) return;
    const int nchunk = D >> 3;
    const T* xr = x + row * D;
    float v[MAXC][8];
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        const int ch = lane + c * 64;
        if (ch < nchunk) Elem<T>::load8(xr + ch * 8, v[c]);
    }
    const float2 st = wave_row_stats<MAXC>(v, nchunk, lane, D, eps);
    if (lane == 0) {
        stats[row] = st;
        if (iota_out) iota_out[row] = (int32_t)(row % iota_n);
    }
}

// Narrow rows (D <= 8 G, G = 16 or 32 lanes): 64 / G rows per wave, so that the lanes of a wave
// cover whole 16-byte chunks of consecutive rows instead of leaving most of them idle.  The sums
// run over the same lanes in the same butterfly order as above (the missing partners there
// hold zeros), so the statistics are the same bits.
template <typename T, int G>
__global__ __launch_bounds__(256) void rowstats_narrow_kernel(const T* __restrict__ x, float2* __restrict__ stats,
                                                              int64_t M, int D, float eps,
                                                              int32_t* __restrict__ iota_out, int iota_n) {
    constexpr int RPW = 64 / G;  // rows per wave
    const int lane = threadIdx.x & 63, sub = lane % G;
    const int64_t row = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * RPW + lane / G;
    const bool on = row < M && sub < (D >> 3);  // whole waves stay in the shuffles below
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = 0.f;
    if (on) Elem<T>::load8(x + row * D + sub * 8, v);
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) sum += v[i];
#pragma unroll
    for (int off = G / 2; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, kWave);
    const float mean = sum / (float)D;
    float sq = 0.f;
    if (on) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float d = v[i] - mean;
            sq += d * d;
        }
    }
#pragma unroll
    for (int off = G / 2; off >= 1; off >>= 1) sq += __shfl_xor(sq, off, kWave);
    if (sub == 0 && row < M) {
        stats[row] = make_float2(mean, rsqrtf(sq / (float)D + eps));
        if (iota_out) iota_out[row] = (int32_t)(row % iota_n);
    }
}

hipError_t launch_rowstats(rs_dtype dt, const void* x, float* stats, int64_t M, int D, float eps,
                           hipStream_t s, int32_t* iota_out, int iota_n) {
    if (M == 0) return hipSuccess;
    dim3 grid((unsigned)((M + 3) / 4)), block(256);
    float2* st = reinterpret_cast<float2*>(stats);
    if (dt == RS_BF16 && D <= 256) {
        const bf16raw* xb = (const bf16raw*)x;
        if (D <= 128) hipLaunchKernelGGL((rowstats_narrow_kernel<bf16raw, 16>), dim3((unsigned)((M + 15) / 16)), block, 0, s, xb, st, M, D, eps, iota_out, iota_n);
        else hipLaunchKernelGGL((rowstats_narrow_kernel<bf16raw, 32>), dim3((unsigned)((M + 7) / 8)), block, 0, s, xb, st, M, D, eps, iota_out, iota_n);
        return hipGetLastError();
    }
    if (dt == RS_F32) {
        if (D <= 2 * 512) hipLaunchKernelGGL((rowstats_kernel<float, 2>), grid, block, 0, s, (const float*)x, st, M, D, eps, iota_out, iota_n);
        else hipLaunchKernelGGL((rowstats_kernel<float, 8>), grid, block, 0, s, (const float*)x, st, M, D, eps, iota_out, iota_n);
    } else {
        if (D <= 2 * 512) hipLaunchKernelGGL((rowstats_kernel<bf16raw, 2>), grid, block, 0, s, (const bf16raw*)x, st, M, D, eps, iota_out, iota_n);
        else hipLaunchKernelGGL((rowstats_kernel<bf16raw, 8>), grid, block, 0, s, (const bf16raw*)x, st, M, D, eps, iota_out, iota_n);
    }
    return hipGetLastError();
}

template <typename T>
static hipError_t launch_ln_t(const void* x, const void* g, const void* b, void* out, int64_t M,
                              int D, float eps, hipStream_t s) {
    if (M == 0) return hipSuccess;
    dim3 grid((unsigned)((M + 3) / 4)), block(256);
    const T* xp = (const T*)x;
    const T* gp = (const T*)g;
    const T* bp = (const T*)b;
    T* op = (T*)out;
    if (D <= 2 * 512)
        hipLaunchKernelGGL((layernorm_kernel<T, 2>), grid, block, 0, s, xp, gp, bp, op, M, D, eps);
    else
        hipLaunchKernelGGL((layernorm_kernel<T, 8>), grid, block, 0, s, xp, gp, bp, op, M, D, eps);
    return hipGetLastError();
}

hipError_t launch_layernorm(rs_dtype dt, const void* x, const void* gamma, const void* beta,
                            void* out, int64_t M, int D, float eps, hipStream_t s) {
    // host-checked by the caller: D % 8 == 0 and D <= 4096
    return dt == RS_F32 ? launch_ln_t<float>(x, gamma, beta, out, M, D, eps, s)
                        : launch_ln_t<bf16raw>(x, gamma, beta, out, M, D, eps, s);
}

}  // namespace rs
