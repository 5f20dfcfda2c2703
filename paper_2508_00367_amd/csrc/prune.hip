// Representation-shift score, token selection and compaction
// (Eq. (4) of Sec. 3.2; "Distance metrics", Sec. 3.3; pruning of the lowest-score
// tokens, Secs. 3.1 and 3.2).  All of it is HBM-bound: the score pass streams F(x)
// and x once, the selection works on N floats per image, the gather copies K rows.
#include "common.hpp"

namespace rs {

// ---------------------------------------------------------------------------
// scores[row] = D(f_out[row, :], f_in[row, :]); one wavefront per row, 8 elements per
// lane per step, butterfly reduction in a fixed order (bit-reproducible).
// ---------------------------------------------------------------------------
template <typename T, int DIST>
__global__ __launch_bounds__(256) void shift_scores_kernel(const T* __restrict__ f_out,
                                                           const T* __restrict__ f_in,
                                                           float* __restrict__ scores, int64_t M,
                                                           int D) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= M) return;
    const T* a = f_out + row * D;
    const T* b = f_in + row * D;
    float p0 = 0.f, p1 = 0.f, p2 = 0.f;
    for (int c = lane * 8; c < D; c += 64 * 8) {
        float x[8], y[8];
        Elem<T>::load8(a + c, x);
        Elem<T>::load8(b + c, y);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (DIST == RS_DIST_L2) { float d = x[i] - y[i]; p0 = fmaf(d, d, p0); }
            else if (DIST == RS_DIST_L1) { p0 += fabsf(x[i] - y[i]); }
            else { p0 = fmaf(x[i], y[i], p0); p1 = fmaf(x[i], x[i], p1); p2 = fmaf(y[i], y[i], p2); }
        }
    }
    p0 = wave_sum(p0);
    if (DIST == RS_DIST_COS) { p1 = wave_sum(p1); p2 = wave_sum(p2); }
    if (lane == 0) {
        float s;
        if (DIST == RS_DIST_L2) s = sqrtf(p0);
        else if (DIST == RS_DIST_L1) s = p0;
        else s = 1.0f - p0 / (sqrtf(p1) * sqrtf(p2));
        scores[row] = s;
    }
}

template <typename T>
static hipError_t launch_scores_t(rs_dist dist, const void* f_out, const void* f_in, float* scores,
                                  int64_t M, int D, hipStream_t s) {
    dim3 grid((unsigned)((M + 3) / 4)), block(256);
    const T* a = (const T*)f_out;
    const T* b = (const T*)f_in;
    if (dist == RS_DIST_L2)
        hipLaunchKernelGGL((shift_scores_kernel<T, RS_DIST_L2>), grid, block, 0, s, a, b, scores, M, D);
    else if (dist == RS_DIST_L1)
        hipLaunchKernelGGL((shift_scores_kernel<T, RS_DIST_L1>), grid, block, 0, s, a, b, scores, M, D);
    else
        hipLaunchKernelGGL((shift_scores_kernel<T, RS_DIST_COS>), grid, block, 0, s, a, b, scores, M, D);
    return hipGetLastError();
}

hipError_t launch_shift_scores(rs_dtype dt, rs_dist dist, const void* f_out, const void* f_in,
                               float* scores, int64_t M, int D, hipStream_t s) {
    if (M == 0) return hipSuccess;
    return dt == RS_F32 ? launch_scores_t<float>(dist, f_out, f_in, scores, M, D, s)
                        : launch_scores_t<bf16raw>(dist, f_out, f_in, scores, M, D, s);
}

// ---------------------------------------------------------------------------
// scores from the fc2 epilogue's per-row partial slots, summed in slot order.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void finalize_scores_kernel(const float* __restrict__ partials,
                                                              int slots, int dist,
                                                              float* __restrict__ scores, int64_t M) {
    const int64_t row = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (row >= M) return;
    const float* p = partials + row * slots * kShiftLanes;
    float p0 = 0.f, p1 = 0.f, p2 = 0.f;
    for (int s = 0; s < slots; ++s) {
        p0 += p[s * kShiftLanes];
        if (dist == RS_DIST_COS) { p1 += p[s * kShiftLanes + 1]; p2 += p[s * kShiftLanes + 2]; }
    }
    float r;
    if (dist == RS_DIST_L2) r = sqrtf(p0);
    else if (dist == RS_DIST_L1) r = p0;
    else r = 1.0f - p0 / (sqrtf(p1) * sqrtf(p2));
    scores[row] = r;
}

hipError_t launch_finalize_scores(rs_dist dist, const float* partials, int slots, float* scores,
                                  int64_t M, hipStream_t s) {
    if (M == 0) return hipSuccess;
    hipLaunchKernelGGL(finalize_scores_kernel, dim3((unsigned)((M + 255) / 256)), dim3(256), 0, s,
                       partials, slots, (int)dist, scores, M);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Selection: one workgroup per image.  Scores become order-preserving uint32 keys
// (sign flip trick; NaN above +inf); a 4-pass, 8-bit, most-significant-first radix
// select over an LDS histogram finds the key of the n_keep-th largest candidate and
// how many candidates equal to it survive (lowest indices first); one ordered
// compaction pass then writes the prefix and the survivors in ascending index order.
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint32_t score_key(float s) {
    const uint32_t u = __float_as_uint(s);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// inclusive scan over the 256 threads of a workgroup (4 waves), values in thread order
__device__ __forceinline__ int block_scan_incl(int v, int* s_wave /*[4]*/, int tid) {
    const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        int t = __shfl_up(v, off, 64);
        if (lane >= off) v += t;
    }
    __syncthreads();  // protects s_wave against the previous use
    if (lane == 63) s_wave[wave] = v;
    __syncthreads();
    int add = 0;
    for (int w = 0; w < wave; ++w) add += s_wave[w];
    return v + add;
}

// With `partials` the scores are first formed from the GEMM epilogue's per-row slots (added in
// slot order, as finalize_scores_kernel does), kept in LDS for the selection and written to
// `scores`: the block's prune pass needs no separate score launch.  N * 4 bytes of dynamic LDS.
__global__ __launch_bounds__(256) void select_kernel(float* __restrict__ scores,
                                                     int32_t* __restrict__ kept_idx, int N,
                                                     int n_prefix, int n_keep,
                                                     const float* __restrict__ partials, int slots, int dist) {
    __shared__ int hist[256];
    __shared__ int s_wave[4];
    __shared__ uint32_t s_prefix;
    __shared__ int s_remaining;
    extern __shared__ float s_scores[];
    const int tid = threadIdx.x;
    const float* sc = scores + (int64_t)blockIdx.x * N;
    int32_t* out = kept_idx + (int64_t)blockIdx.x * (n_prefix + n_keep);
    if (partials) {
        for (int i = tid; i < N; i += 256) {
            const float* p = partials + ((int64_t)blockIdx.x * N + i) * slots * kShiftLanes;
            float p0 = 0.f, p1 = 0.f, p2 = 0.f;
            for (int sl = 0; sl < slots; ++sl) {
                p0 += p[sl * kShiftLanes];
                if (dist == RS_DIST_COS) { p1 += p[sl * kShiftLanes + 1]; p2 += p[sl * kShiftLanes + 2]; }
            }
            float r;
            if (dist == RS_DIST_L2) r = sqrtf(p0);
            else if (dist == RS_DIST_L1) r = p0;
            else r = 1.0f - p0 / (sqrtf(p1) * sqrtf(p2));
            s_scores[i] = r;
            scores[(int64_t)blockIdx.x * N + i] = r;
        }
        sc = s_scores;
        __syncthreads();
    }

    for (int i = tid; i < n_prefix; i += 256) out[i] = i;
    if (n_keep == 0) return;

    uint32_t prefix = 0, mask = 0;
    int remaining = n_keep;  // how many of the candidates matching `prefix` still to take
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        hist[tid] = 0;
        __syncthreads();
        for (int i = n_prefix + tid; i < N; i += 256) {
            const uint32_t key = score_key(sc[i]);
            if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255], 1);
        }
        __syncthreads();
        // suffix sums over the bins: thread t looks at bin 255 - t, so an inclusive scan in
        // thread order counts the candidates in bins >= bin.
        const int bin = 255 - tid;
        const int cnt = hist[bin];
        const int incl = block_scan_incl(cnt, s_wave, tid);
        // the wanted key's digit is the first bin (from the top) whose suffix count reaches `remaining`
        if (incl >= remaining && incl - cnt < remaining) {
            s_prefix = prefix | ((uint32_t)bin << shift);
            s_remaining = remaining - (incl - cnt);
        }
        __syncthreads();
        prefix = s_prefix;
        remaining = s_remaining;
        mask |= 255u << shift;
        __syncthreads();
    }
    // `prefix` = key of the n_keep-th largest candidate; `remaining` = how many candidates with
    // exactly that key are kept (those with the lowest indices).
    const uint32_t thr = prefix;
    const int n = N - n_prefix;
    const int seg = (n + 255) / 256;
    const int lo = n_prefix + tid * seg;
    const int hi = min(lo + seg, N);
    int gt = 0, eq = 0;
    for (int i = lo; i < hi; ++i) {
        const uint32_t key = score_key(sc[i]);
        gt += key > thr;
        eq += key == thr;
    }
    const int gt_before = block_scan_incl(gt, s_wave, tid) - gt;
    const int eq_before = block_scan_incl(eq, s_wave, tid) - eq;
    int pos = n_prefix + gt_before + min(eq_before, remaining);
    int eq_rank = eq_before;
    for (int i = lo; i < hi; ++i) {
        const uint32_t key = score_key(sc[i]);
        bool keep = key > thr;
        if (key == thr) { keep = eq_rank < remaining; ++eq_rank; }
        if (keep) out[pos++] = i;
    }
}

// kept_idx[b, j] = j when every token survives
__global__ __launch_bounds__(256) void iota_kernel(int32_t* __restrict__ kept_idx, int B, int K) {
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t < (int64_t)B * K) kept_idx[t] = (int32_t)(t % K);
}

hipError_t launch_select(const float* scores, int32_t* kept_idx, int B, int N, int n_prefix,
                         int n_keep, hipStream_t s) {
    if (B == 0 || n_prefix + n_keep == 0) return hipSuccess;
    if (n_keep == N - n_prefix) {
        const int64_t tot = (int64_t)B * N;
        hipLaunchKernelGGL(iota_kernel, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, s, kept_idx, B, N);
    } else {
        hipLaunchKernelGGL(select_kernel, dim3(B), dim3(256), 0, s, const_cast<float*>(scores), kept_idx, N,
                           n_prefix, n_keep, (const float*)nullptr, 0, 0);
    }
    return hipGetLastError();
}

bool select_from_partials_fits(int N) { return N <= 12288; }  // scores of one image in LDS

hipError_t launch_select_from_partials(rs_dist dist, const float* partials, int slots, float* scores,
                                       int32_t* kept_idx, int B, int N, int n_prefix, int n_keep,
                                       hipStream_t s) {
    if (B == 0) return hipSuccess;
    hipLaunchKernelGGL(select_kernel, dim3(B), dim3(256), (size_t)N * sizeof(float), s, scores, kept_idx, N,
                       n_prefix, n_keep, partials, slots, (int)dist);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Gather: out[b, j, :] = src[b, kept_idx[b, j], :]; one wavefront per row, 16 bytes per
// lane per step (rows are D * e bytes, a multiple of 16).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void gather_rows_kernel(const uint4* __restrict__ src,
                                                          const int32_t* __restrict__ kept_idx,
                                                          uint4* __restrict__ out, int64_t rows,
                                                          int N, int K, int row_vec) {
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= rows) return;
    const int64_t b = r / K;
    const int32_t idx = kept_idx[r];
    const uint4* s = src + (b * N + idx) * row_vec;
    uint4* d = out + r * row_vec;
    for (int c = lane; c < row_vec; c += 64) d[c] = s[c];
}

hipError_t launch_gather(rs_dtype dt, const void* src, const int32_t* kept_idx, void* out, int B,
                         int N, int K, int D, hipStream_t s) {
    const int64_t rows = (int64_t)B * K;
    if (rows == 0) return hipSuccess;
    const int row_vec = (int)((size_t)D * elem_size(dt) / 16);
    hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s,
                       (const uint4*)src, kept_idx, (uint4*)out, rows, N, K, row_vec);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Line-wise pruning of a 2-D token grid (Sec. 4.2, "CNN and SSM", variant (ii)).
// Line scores: the per-position shift averaged along each row and along each column; one
// workgroup per image, thread h sums row h over w in index order and thread w sums column w
// over h in index order (fixed order: bit-reproducible).  The rows and columns to keep are then
// picked by select_kernel, and the grid gather copies the surviving positions.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void grid_line_scores_kernel(const float* __restrict__ scores,
                                                               float* __restrict__ row_scores,
                                                               float* __restrict__ col_scores, int H, int W) {
    const float* s = scores + (int64_t)blockIdx.x * H * W;
    for (int h = threadIdx.x; h < H; h += 256) {
        float a = 0.f;
        for (int w = 0; w < W; ++w) a += s[h * W + w];
        row_scores[(int64_t)blockIdx.x * H + h] = a / (float)W;
    }
    for (int w = threadIdx.x; w < W; w += 256) {
        float a = 0.f;
        for (int h = 0; h < H; ++h) a += s[h * W + w];
        col_scores[(int64_t)blockIdx.x * W + w] = a / (float)H;
    }
}

hipError_t launch_grid_line_scores(const float* scores, float* row_scores, float* col_scores, int B, int H,
                                   int W, hipStream_t s) {
    if (B == 0) return hipSuccess;
    hipLaunchKernelGGL(grid_line_scores_kernel, dim3(B), dim3(256), 0, s, scores, row_scores, col_scores, H, W);
    return hipGetLastError();
}

// out[b, i, j, :] = src[b, kept_rows[b, i], kept_cols[b, j], :]; one wavefront per output position
__global__ __launch_bounds__(256) void grid_gather_kernel(const uint4* __restrict__ src,
                                                          const int32_t* __restrict__ kept_rows,
                                                          const int32_t* __restrict__ kept_cols,
                                                          uint4* __restrict__ out, int64_t positions, int H, int W,
                                                          int R, int Q, int vec) {
    const int lane = threadIdx.x & 63;
    const int64_t p = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (p >= positions) return;
    const int64_t b = p / ((int64_t)R * Q);
    const int ij = (int)(p - b * R * Q);
    const int i = ij / Q, j = ij - i * Q;
    const int64_t sp = (b * H + kept_rows[b * R + i]) * W + kept_cols[b * Q + j];
    for (int c = lane; c < vec; c += 64) out[p * vec + c] = src[sp * vec + c];
}

hipError_t launch_grid_gather(rs_dtype dt, const void* src, const int32_t* kept_rows, const int32_t* kept_cols,
                              void* out, int B, int H, int W, int R, int Q, int C, hipStream_t s) {
    const int64_t positions = (int64_t)B * R * Q;
    if (positions == 0) return hipSuccess;
    const int vec = (int)((size_t)C * elem_size(dt) / 16);
    hipLaunchKernelGGL(grid_gather_kernel, dim3((unsigned)((positions + 3) / 4)), dim3(256), 0, s, (const uint4*)src,
                       kept_rows, kept_cols, (uint4*)out, positions, H, W, R, Q, vec);
    return hipGetLastError();
}

}  // namespace rs
