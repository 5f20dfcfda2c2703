// Linear layers of the encoder block (QKV, output projection, fc1, fc2; the O(N C^2)
// term of Sec. 3.1) with the block's elementwise work fused into the epilogue:
// bias, exact GELU, residual add (Eqs. (5),(6)) and the per-row partial sums of the
// representation shift D(MLP(LN(x')), x') (Eq. (4); case (ii) of "Operation choice").
//
// bf16 path: v_mfma_f32_32x32x16_bf16, fp32 accumulation.  The weight matrix is the
// A operand (rows = output features n) and the activations are the B operand
// (columns = token rows m), so that in the accumulator layout a lane owns ONE token
// row and 4 consecutive output features per register quad: row-wise epilogue work
// (residual, shift partial sums) stays inside a lane, and stores are 8-byte vectors.
//
// fp32 path: plain FMA tiles (parity configuration, true fp32 products).
#include "common.hpp"

namespace rs {

// ---------------------------------------------------------------------------
// bf16 MFMA GEMM:  out[m, n] = epi( sum_k a[m, k] * wt[n, k] )
//   a  : [M, K] bf16 (token rows),  wt : [N, K] bf16 (packed weights),  K % 64 == 0.
// Workgroup tile BM x BN, K step 64, WGM x WGN waves, LDS double buffered.
// LDS rows are 64 bf16 = 8 chunks of 16 B; chunk c of row r sits at c ^ (r & 7) so that
// the 32 rows a half-wave reads for one MFMA operand spread over all banks.
// ---------------------------------------------------------------------------
constexpr int BK = 64;

__device__ __forceinline__ int swz(int row, int chunk) { return row * 128 + ((chunk ^ (row & 7)) << 4); }

template <int BM, int BN, int WGM, int WGN, int EPI, int DIST>
__global__ __launch_bounds__(WGM* WGN * 64) void gemm_bf16_kernel(
    const bf16raw* __restrict__ a, const bf16raw* __restrict__ wt, const bf16raw* __restrict__ bias,
    const bf16raw* __restrict__ res, bf16raw* __restrict__ out, float* __restrict__ partials,
    int M, int N, int K, int tiles_m, int tiles_n, int slots) {
    constexpr int NT = WGM * WGN * 64;
    constexpr int WM = BM / WGM, WN = BN / WGN;  // wave tile
    constexpr int TM = WM / 32, TN = WN / 32;    // MFMA tiles per wave
    constexpr int A_LOADS = BM * 8 / NT, W_LOADS = BN * 8 / NT;
    static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "tile/threads mismatch");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    // stage s: activations at s*STAGE, weights after them
    constexpr int STAGE = (BM + BN) * 128;

    // XCD-aware tile order: consecutive workgroup ids go round-robin to the 8 XCDs, so give
    // each XCD a contiguous range of tiles; inside a range the n index runs fastest, so the
    // workgroups of one XCD share an activation row block in that XCD's L2.
    const int nblk = tiles_m * tiles_n;
    int bid = blockIdx.x;
    {
        const int x = bid & 7, j = bid >> 3;
        const int q = nblk >> 3, r = nblk & 7;  // XCD x owns q (+1 if x < r) tiles
        bid = x * q + (x < r ? x : r) + j;
    }
    const int tile_m = bid / tiles_n, tile_n = bid % tiles_n;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WGM, wn = wave / WGM;
    const int l32 = lane & 31, g = lane >> 5;

    // global -> LDS assignment: thread handles chunk (tid & 7) of rows (tid >> 3) + i * (NT/8)
    const int ld_chunk = tid & 7, ld_row = tid >> 3;
    const bf16raw* a_src[A_LOADS];
    const bf16raw* w_src[W_LOADS];
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) {
        int r = m0 + ld_row + i * (NT / 8);
        r = r < M ? r : M - 1;  // clamp: rows past the end are computed but never stored
        a_src[i] = a + (int64_t)r * K + ld_chunk * 8;
    }
#pragma unroll
    for (int i = 0; i < W_LOADS; ++i) {
        int r = n0 + ld_row + i * (NT / 8);
        r = r < N ? r : N - 1;
        w_src[i] = wt + (int64_t)r * K + ld_chunk * 8;
    }

    f32x16 acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    uint4 a_reg[A_LOADS], w_reg[W_LOADS];
    const int KT = K / BK;

    auto load_global = [&](int kt) {
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i) a_reg[i] = *reinterpret_cast<const uint4*>(a_src[i] + kt * BK);
#pragma unroll
        for (int i = 0; i < W_LOADS; ++i) w_reg[i] = *reinterpret_cast<const uint4*>(w_src[i] + kt * BK);
    };
    auto store_lds = [&](int stage) {
        unsigned char* sa = smem + stage * STAGE;
        unsigned char* sw = sa + BM * 128;
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i)
            *reinterpret_cast<uint4*>(sa + swz(ld_row + i * (NT / 8), ld_chunk)) = a_reg[i];
#pragma unroll
        for (int i = 0; i < W_LOADS; ++i)
            *reinterpret_cast<uint4*>(sw + swz(ld_row + i * (NT / 8), ld_chunk)) = w_reg[i];
    };

    load_global(0);
    store_lds(0);
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        if (kt + 1 < KT) load_global(kt + 1);
        const unsigned char* sa = smem + (kt & 1) * STAGE;
        const unsigned char* sw = sa + BM * 128;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8 wf[TN], af[TM];
#pragma unroll
            for (int i = 0; i < TN; ++i)
                wf[i] = *reinterpret_cast<const bf16x8*>(sw + swz(wn * WN + i * 32 + l32, kk * 2 + g));
#pragma unroll
            for (int j = 0; j < TM; ++j)
                af[j] = *reinterpret_cast<const bf16x8*>(sa + swz(wm * WM + j * 32 + l32, kk * 2 + g));
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int j = 0; j < TM; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[i], af[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < KT) store_lds((kt + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue: lane owns token row m = .. + l32; register r = 4*q + i of tile (tn, tm)
    //      is output feature n = .. + 8*q + 4*g + i.
#pragma unroll
    for (int j = 0; j < TM; ++j) {
        const int m = m0 + wm * WM + j * 32 + l32;
        const bool m_ok = m < M;
        float p0 = 0.f, p1 = 0.f, p2 = 0.f;  // shift partial sums of this row over the wave's columns
#pragma unroll
        for (int i = 0; i < TN; ++i) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = n0 + wn * WN + i * 32 + q * 8 + g * 4;
                if (n < N) {  // N % 4 == 0: a quad is either fully inside or fully outside
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = acc[i][j][q * 4 + e];
                    if (bias) {
                        uint2 b = *reinterpret_cast<const uint2*>(bias + n);
                        v[0] += __uint_as_float(b.x << 16); v[1] += __uint_as_float(b.x & 0xffff0000u);
                        v[2] += __uint_as_float(b.y << 16); v[3] += __uint_as_float(b.y & 0xffff0000u);
                    }
                    if (EPI == EPI_BIAS_GELU) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = gelu_erf(v[e]);
                    }
                    if (EPI == EPI_BIAS_RES || EPI == EPI_BIAS_RES_SHIFT) {
                        float r[4] = {0.f, 0.f, 0.f, 0.f};
                        if (m_ok) {
                            uint2 rr = *reinterpret_cast<const uint2*>(res + (int64_t)m * N + n);
                            r[0] = __uint_as_float(rr.x << 16); r[1] = __uint_as_float(rr.x & 0xffff0000u);
                            r[2] = __uint_as_float(rr.y << 16); r[3] = __uint_as_float(rr.y & 0xffff0000u);
                        }
                        if (EPI == EPI_BIAS_RES_SHIFT) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                if (DIST == RS_DIST_L2) { float d = v[e] - r[e]; p0 += d * d; }
                                else if (DIST == RS_DIST_L1) { p0 += fabsf(v[e] - r[e]); }
                                else { p0 += v[e] * r[e]; p1 += v[e] * v[e]; p2 += r[e] * r[e]; }
                            }
                        }
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] += r[e];
                    }
                    if (m_ok) {
                        uint2 o;
                        o.x = pack2bf(v[0], v[1]);
                        o.y = pack2bf(v[2], v[3]);
                        *reinterpret_cast<uint2*>(out + (int64_t)m * N + n) = o;
                    }
                }
            }
        }
        if (EPI == EPI_BIAS_RES_SHIFT) {
            // the two half-waves hold interleaved column quads of the same rows
            p0 += __shfl_xor(p0, 32, 64);
            if (DIST == RS_DIST_COS) {
                p1 += __shfl_xor(p1, 32, 64);
                p2 += __shfl_xor(p2, 32, 64);
            }
            if (g == 0 && m_ok) {
                const int slot = (n0 + wn * WN) / WN;
                float* dst = partials + ((int64_t)m * slots + slot) * kShiftLanes;
                dst[0] = p0;
                if (DIST == RS_DIST_COS) { dst[1] = p1; dst[2] = p2; }
            }
        }
    }
}

// Tile configuration of the bf16 GEMM.
struct GemmCfg {
    static constexpr int BM = 128, BN = 128, WGM = 2, WGN = 2;
    static constexpr int WN = BN / WGN;
};

template <int EPI, int DIST>
static hipError_t launch_bf16(const void* a, const void* wt, const void* bias, const void* res,
                              void* out, float* partials, int64_t M, int N, int K, hipStream_t s) {
    using C = GemmCfg;
    const int tiles_m = (int)((M + C::BM - 1) / C::BM), tiles_n = (N + C::BN - 1) / C::BN;
    const int slots = (tiles_n * C::BN) / C::WN;
    const size_t lds = 2 * (C::BM + C::BN) * 128;
    auto kern = gemm_bf16_kernel<C::BM, C::BN, C::WGM, C::WGN, EPI, DIST>;
    static bool attr_done = false;  // raise the dynamic LDS limit once per instantiation
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(C::WGM * C::WGN * 64), lds, s,
                       (const bf16raw*)a, (const bf16raw*)wt, (const bf16raw*)bias, (const bf16raw*)res,
                       (bf16raw*)out, partials, (int)M, N, K, tiles_m, tiles_n, slots);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// fp32 GEMM: out[m, n] = epi( sum_k a[m, k] * w[k, n] ), w as given by the caller ([K, N]).
// 64 x 64 tile, 256 threads, each a 4 x 4 micro tile; K % 16 == 0, N % 4 == 0.
// The shift partial sums are reduced over the 16 threads that share a row.
// ---------------------------------------------------------------------------
template <int EPI, int DIST>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ a,
                                                       const float* __restrict__ w,
                                                       const float* __restrict__ bias,
                                                       const float* __restrict__ res,
                                                       float* __restrict__ out,
                                                       float* __restrict__ partials, int M, int N,
                                                       int K, int slots) {
    constexpr int T = 64, KS = 16;
    __shared__ float sa[KS][T + 4];  // a tile transposed: sa[k][m]
    __shared__ float sw[KS][T + 4];  // sw[k][n]
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;  // tx: column quad, ty: row quad
    const int m0 = blockIdx.y * T, n0 = blockIdx.x * T;
    float acc[4][4] = {};
    // loaders: a tile 64 rows x 16 k = 256 float4 -> one per thread; w tile 16 k x 64 n = 256 float4
    const int a_row = tid >> 2, a_k4 = (tid & 3) * 4;
    const int w_k = tid >> 4, w_n4 = (tid & 15) * 4;
    for (int k0 = 0; k0 < K; k0 += KS) {
        {
            int r = m0 + a_row;
            r = r < M ? r : M - 1;
            float4 v = *reinterpret_cast<const float4*>(a + (int64_t)r * K + k0 + a_k4);
            sa[a_k4 + 0][a_row] = v.x; sa[a_k4 + 1][a_row] = v.y;
            sa[a_k4 + 2][a_row] = v.z; sa[a_k4 + 3][a_row] = v.w;
            int n = n0 + w_n4;
            float4 u = make_float4(0.f, 0.f, 0.f, 0.f);
            if (n < N) u = *reinterpret_cast<const float4*>(w + (int64_t)(k0 + w_k) * N + n);
            *reinterpret_cast<float4*>(&sw[w_k][w_n4]) = u;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < KS; ++k) {
            float4 av = *reinterpret_cast<const float4*>(&sa[k][ty * 4]);
            float4 wv = *reinterpret_cast<const float4*>(&sw[k][tx * 4]);
            float ar[4] = {av.x, av.y, av.z, av.w}, wr[4] = {wv.x, wv.y, wv.z, wv.w};
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(ar[i], wr[j], acc[i][j]);
        }
        __syncthreads();
    }
    const int n = n0 + tx * 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        const bool m_ok = m < M;
        float p0 = 0.f, p1 = 0.f, p2 = 0.f;
        if (n < N) {
            float v[4] = {acc[i][0], acc[i][1], acc[i][2], acc[i][3]};
            if (bias) {
                float4 b = *reinterpret_cast<const float4*>(bias + n);
                v[0] += b.x; v[1] += b.y; v[2] += b.z; v[3] += b.w;
            }
            if (EPI == EPI_BIAS_GELU) {
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = gelu_erf(v[e]);
            }
            if (EPI == EPI_BIAS_RES || EPI == EPI_BIAS_RES_SHIFT) {
                float r[4] = {0.f, 0.f, 0.f, 0.f};
                if (m_ok) {
                    float4 rr = *reinterpret_cast<const float4*>(res + (int64_t)m * N + n);
                    r[0] = rr.x; r[1] = rr.y; r[2] = rr.z; r[3] = rr.w;
                }
                if (EPI == EPI_BIAS_RES_SHIFT) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (DIST == RS_DIST_L2) { float d = v[e] - r[e]; p0 += d * d; }
                        else if (DIST == RS_DIST_L1) { p0 += fabsf(v[e] - r[e]); }
                        else { p0 += v[e] * r[e]; p1 += v[e] * v[e]; p2 += r[e] * r[e]; }
                    }
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] += r[e];
            }
            if (m_ok) *reinterpret_cast<float4*>(out + (int64_t)m * N + n) = make_float4(v[0], v[1], v[2], v[3]);
        }
        if (EPI == EPI_BIAS_RES_SHIFT) {
            // threads tx = 0..15 of one ty share row m: they are 16 consecutive lanes
#pragma unroll
            for (int off = 8; off >= 1; off >>= 1) {
                p0 += __shfl_xor(p0, off, 64);
                if (DIST == RS_DIST_COS) { p1 += __shfl_xor(p1, off, 64); p2 += __shfl_xor(p2, off, 64); }
            }
            if (tx == 0 && m_ok) {
                float* dst = partials + ((int64_t)m * slots + blockIdx.x) * kShiftLanes;
                dst[0] = p0;
                if (DIST == RS_DIST_COS) { dst[1] = p1; dst[2] = p2; }
            }
        }
    }
}

template <int EPI, int DIST>
static hipError_t launch_f32(const void* a, const void* w, const void* bias, const void* res,
                             void* out, float* partials, int64_t M, int N, int K, hipStream_t s) {
    dim3 grid((N + 63) / 64, (unsigned)((M + 63) / 64));
    hipLaunchKernelGGL((gemm_f32_kernel<EPI, DIST>), grid, dim3(256), 0, s, (const float*)a,
                       (const float*)w, (const float*)bias, (const float*)res, (float*)out, partials,
                       (int)M, N, K, (N + 63) / 64);
    return hipGetLastError();
}

int gemm_shift_slots(rs_dtype dt, int N) {
    if (dt == RS_F32) return (N + 63) / 64;
    return ((N + GemmCfg::BN - 1) / GemmCfg::BN) * GemmCfg::BN / GemmCfg::WN;
}

template <int EPI, int DIST>
static hipError_t launch_any(rs_dtype dt, const void* a, const void* w, const void* bias,
                             const void* res, void* out, float* partials, int64_t M, int N, int K,
                             hipStream_t s) {
    return dt == RS_F32 ? launch_f32<EPI, DIST>(a, w, bias, res, out, partials, M, N, K, s)
                        : launch_bf16<EPI, DIST>(a, w, bias, res, out, partials, M, N, K, s);
}

hipError_t launch_gemm(rs_dtype dt, GemmEpilogue epi, rs_dist dist, const void* a, const void* w,
                       const void* bias, const void* res, void* out, float* partials, int64_t M,
                       int N, int K, hipStream_t s) {
    if (M == 0) return hipSuccess;
    switch (epi) {
        case EPI_BIAS: return launch_any<EPI_BIAS, 0>(dt, a, w, bias, res, out, partials, M, N, K, s);
        case EPI_BIAS_GELU: return launch_any<EPI_BIAS_GELU, 0>(dt, a, w, bias, res, out, partials, M, N, K, s);
        case EPI_BIAS_RES: return launch_any<EPI_BIAS_RES, 0>(dt, a, w, bias, res, out, partials, M, N, K, s);
        case EPI_BIAS_RES_SHIFT:
            if (dist == RS_DIST_L2) return launch_any<EPI_BIAS_RES_SHIFT, RS_DIST_L2>(dt, a, w, bias, res, out, partials, M, N, K, s);
            if (dist == RS_DIST_L1) return launch_any<EPI_BIAS_RES_SHIFT, RS_DIST_L1>(dt, a, w, bias, res, out, partials, M, N, K, s);
            return launch_any<EPI_BIAS_RES_SHIFT, RS_DIST_COS>(dt, a, w, bias, res, out, partials, M, N, K, s);
    }
    return hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------
// Weight re-layout for the bf16 path: [K, N] row-major -> [N, K] row-major.
// 64 x 64 tiles through LDS, coalesced on both sides.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void transpose_bf16_kernel(const bf16raw* __restrict__ w,
                                                             bf16raw* __restrict__ wt, int K, int N) {
    __shared__ bf16raw tile[64][66];
    const int k0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int r = ty; r < 64; r += 4) {
        const int k = k0 + r, n = n0 + tx;
        tile[r][tx] = (k < K && n < N) ? w[(int64_t)k * N + n] : (bf16raw)0;
    }
    __syncthreads();
    for (int r = ty; r < 64; r += 4) {
        const int n = n0 + r, k = k0 + tx;
        if (n < N && k < K) wt[(int64_t)n * K + k] = tile[tx][r];
    }
}

hipError_t launch_pack_transpose(const void* w, void* wt, int K, int N, hipStream_t s) {
    dim3 grid((N + 63) / 64, (K + 63) / 64);
    hipLaunchKernelGGL(transpose_bf16_kernel, grid, dim3(256), 0, s, (const bf16raw*)w, (bf16raw*)wt, K, N);
    return hipGetLastError();
}

}  // namespace rs
