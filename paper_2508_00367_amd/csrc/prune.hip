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

// inclusive scan over the NT threads of a workgroup (NT / 64 waves), values in thread order
template <int NT>
__device__ __forceinline__ int block_scan_incl(int v, int* s_wave /*[NT / 64]*/, int tid) {
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

struct SelectShared {
    int hist[256];
    int wave[16];
    uint32_t prefix;
    int remaining;
};

// Selection of one image by the NT threads of a workgroup (all of them must call it): among
// the tokens i >= n_prefix of sc[0 .. N) the n_keep highest keys survive, equal keys by lower
// index; out[0 .. n_prefix + n_keep) lists the prefix and the survivors in ascending order.
// With `slot` (N ints, workgroup-visible) slot[i] becomes the position of token i in `out`, or
// -1 for a dropped token.  `sc` may be LDS or global memory written before a barrier.
template <int NT>
__device__ __forceinline__ void block_select(const float* sc, int N, int n_prefix, int n_keep,
                                             int32_t* __restrict__ out, int* slot, SelectShared& sh, int tid) {
    for (int i = tid; i < n_prefix; i += NT) out[i] = i;
    if (slot)
        for (int i = tid; i < N; i += NT) slot[i] = i < n_prefix ? i : -1;
    if (n_keep == 0) return;  // uniform over the workgroup

    uint32_t prefix = 0, mask = 0;
    int remaining = n_keep;  // how many of the candidates matching `prefix` still to take
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        if (tid < 256) sh.hist[tid] = 0;
        __syncthreads();
        for (int i = n_prefix + tid; i < N; i += NT) {
            const uint32_t key = score_key(sc[i]);
            if ((key & mask) == prefix) atomicAdd(&sh.hist[(key >> shift) & 255], 1);
        }
        __syncthreads();
        // suffix sums over the bins: thread t < 256 looks at bin 255 - t, so an inclusive scan in
        // thread order counts the candidates in bins >= bin (threads beyond 255 add nothing).
        const int bin = 255 - tid;
        const int cnt = tid < 256 ? sh.hist[bin] : 0;
        const int incl = block_scan_incl<NT>(cnt, sh.wave, tid);
        // the wanted key's digit is the first bin (from the top) whose suffix count reaches `remaining`
        if (tid < 256 && incl >= remaining && incl - cnt < remaining) {
            sh.prefix = prefix | ((uint32_t)bin << shift);
            sh.remaining = remaining - (incl - cnt);
        }
        __syncthreads();
        prefix = sh.prefix;
        remaining = sh.remaining;
        mask |= 255u << shift;
        __syncthreads();
    }
    // `prefix` = key of the n_keep-th largest candidate; `remaining` = how many candidates with
    // exactly that key are kept (those with the lowest indices).
    const uint32_t thr = prefix;
    const int n = N - n_prefix;
    const int seg = (n + NT - 1) / NT;
    const int lo = n_prefix + tid * seg;
    const int hi = min(lo + seg, N);
    int gt = 0, eq = 0;
    for (int i = lo; i < hi; ++i) {
        const uint32_t key = score_key(sc[i]);
        gt += key > thr;
        eq += key == thr;
    }
    const int gt_before = block_scan_incl<NT>(gt, sh.wave, tid) - gt;
    const int eq_before = block_scan_incl<NT>(eq, sh.wave, tid) - eq;
    int pos = n_prefix + gt_before + min(eq_before, remaining);
    int eq_rank = eq_before;
    for (int i = lo; i < hi; ++i) {
        const uint32_t key = score_key(sc[i]);
        bool keep = key > thr;
        if (key == thr) { keep = eq_rank < remaining; ++eq_rank; }
        if (keep) {
            if (slot) slot[i] = pos;
            out[pos++] = i;
        }
    }
}

// The same selection for N <= 256 tokens by counting: token i's rank among the candidates is the
// number of candidates with a larger key, or an equal key and a lower index; ranks below n_keep
// survive.  NT / 256 threads share a token's count, a ballot scan over the survival flags gives the
// output positions: three barriers instead of the radix passes' thirty.  Identical results.
template <int NT>
__device__ __forceinline__ void block_select_rank(const float* sc /* LDS */, int N, int n_prefix, int n_keep,
                                                  int32_t* __restrict__ out, int* slot, SelectShared& sh, int tid) {
    constexpr int TPT = NT / 256;  // threads per token
    const int i = tid / TPT, part = tid % TPT;
    int cnt = 0;
    if (i >= n_prefix && i < N) {
        const uint32_t ki = score_key(sc[i]);
        const int n = N - n_prefix, seg = (n + TPT - 1) / TPT;
        const int lo = n_prefix + part * seg, hi = min(lo + seg, N);
        for (int j = lo; j < hi; ++j) {
            const uint32_t kj = score_key(sc[j]);
            cnt += (kj > ki) || (kj == ki && j < i);
        }
    }
#pragma unroll
    for (int off = 1; off < TPT; off <<= 1) cnt += __shfl_xor(cnt, off, 64);
    // (a caller that loops has a barrier between this write and the previous round's reads of sh)
    if (part == 0 && i < N) sh.hist[i] = (i < n_prefix || cnt < n_keep) ? 1 : 0;
    __syncthreads();
    const int lane = tid & 63, wave = tid >> 6;
    const int f = (tid < N) ? sh.hist[tid] : 0;        // thread t now stands for token t
    const unsigned long long mask = __ballot(f);
    const int before = __popcll(mask & ((1ull << lane) - 1ull));
    if (wave < 4 && lane == 0) sh.wave[wave] = __popcll(mask);
    __syncthreads();
    if (tid < N) {
        int pos = before;
        for (int w = 0; w < wave; ++w) pos += sh.wave[w];
        if (f) out[pos] = tid;
        if (slot) slot[tid] = f ? pos : -1;
    }
}

// With `partials` the scores are first formed from the GEMM epilogue's per-row slots (added in
// slot order, as finalize_scores_kernel does), kept in LDS for the selection and written to
// `scores`: the block's prune pass needs no separate score launch.  N * 4 bytes of dynamic LDS.
template <int NT>
__global__ __launch_bounds__(NT) void select_kernel(float* __restrict__ scores,
                                                     int32_t* __restrict__ kept_idx, int N,
                                                     int n_prefix, int n_keep,
                                                     const float* __restrict__ partials, int slots, int dist) {
    __shared__ SelectShared sh;
    extern __shared__ float s_scores[];
    const int tid = threadIdx.x;
    const float* sc = scores + (int64_t)blockIdx.x * N;
    int32_t* out = kept_idx + (int64_t)blockIdx.x * (n_prefix + n_keep);
    if (partials) {
        for (int i = tid; i < N; i += NT) {
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
        if (NT > 256) {  // short sequences: launched with NT / 256 threads per token (N <= 256)
            block_select_rank<NT>(sc, N, n_prefix, n_keep, out, nullptr, sh, tid);
            return;
        }
    }
    block_select<NT>(sc, N, n_prefix, n_keep, out, nullptr, sh, tid);
}

// ---------------------------------------------------------------------------
// Score, selection and gather of one image in ONE pass over memory, for images whose f_in rows
// fit the register file of a compute unit (N <= 16 NR rows of at most 512 CH bytes: every
// image-classification shape).  One workgroup of 16 waves per image at a time: wave w holds rows
// w, w + 16, ... of f_in in registers (8 bytes per lane and chunk), streams the same rows of f_out
// past them for the scores, the workgroup selects, and every wave then writes its surviving rows
// to their places in `gathered` straight from registers.  Against the three-launch path the
// kept rows are not read a second time: memory traffic is the algorithmic minimum
// (2 N D e read, K D e written per image).  Workgroups loop over images (persistent grid).
// ---------------------------------------------------------------------------
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
template <typename T> __device__ __forceinline__ void unpack8(u32x2 v, float (&f)[4]);
template <> __device__ __forceinline__ void unpack8<bf16raw>(u32x2 v, float (&f)[4]) {
    f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
    f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
}
template <> __device__ __forceinline__ void unpack8<float>(u32x2 v, float (&f)[4]) {
    f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y); f[2] = 0.f; f[3] = 0.f;
}

#ifndef RS_RES_WAVES
#define RS_RES_WAVES 16
#endif
#ifndef RS_RES_G
#define RS_RES_G 4
#endif
constexpr int RES_WAVES = RS_RES_WAVES;   // waves per workgroup: between them they own the CU's registers
constexpr int RES_MAXN = 208;             // longest sequence the kernel takes
constexpr int RES_NR = (RES_MAXN + RES_WAVES - 1) / RES_WAVES;  // rows per wave

template <typename T, int DIST, int CH, int NR>
__global__ __launch_bounds__(RES_WAVES * 64) void shift_topk_resident_kernel(
    const T* __restrict__ f_out, const T* __restrict__ f_in, float* __restrict__ scores,
    int32_t* __restrict__ kept_idx, T* __restrict__ gathered, int B, int N, int D, int n_prefix, int n_keep) {
    constexpr int NT = RES_WAVES * 64;
    __shared__ SelectShared sh;
    __shared__ float s_scores[NR * RES_WAVES];
    __shared__ int s_slot[NR * RES_WAVES];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: row addresses stay scalar
    const int row_u = D * (int)sizeof(T) / 8;  // 8-byte units per row
    const int K = n_prefix + n_keep;
    // Rows are addressed through buffer resources over one image: the row offset is a scalar, the
    // lane offset one register per chunk, and whatever lies outside (rows past N, lanes past the
    // row's end, which are aimed far outside) reads as zero and is dropped on stores.
    const int row_bytes = D * (int)sizeof(T);
    int voff[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) voff[c] = (lane + 64 * c) < row_u ? (lane + 64 * c) * 8 : 0x7fff0000;
    // The resident rows of the first image; those of every later image are requested row by row
    // while the previous image's surviving rows are being written out of the same registers, so
    // their latency passes under that image's stores and the next image's f_out stream.
    u32x2 keep[NR][CH];
    {
        const __amdgpu_buffer_rsrc_t r_in0 = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<T*>(f_in + (int64_t)blockIdx.x * N * D), 0, (int)blockIdx.x < B ? N * row_bytes : 0, 0x00020000);
#pragma unroll
        for (int k = 0; k < NR; ++k)
#pragma unroll
            for (int c = 0; c < CH; ++c)
                keep[k][c] = __builtin_amdgcn_raw_buffer_load_b64(r_in0, voff[c], (wave + RES_WAVES * k) * row_bytes, 0);
    }
    for (int b = blockIdx.x; b < B; b += gridDim.x) {
        const __amdgpu_buffer_rsrc_t r_fo = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<T*>(f_out + (int64_t)b * N * D), 0, N * row_bytes, 0x00020000);
        __builtin_amdgcn_sched_barrier(0);
        constexpr int G = RS_RES_G;  // rows of f_out in flight per wave (next to the resident rows)
#pragma unroll
        for (int k0 = 0; k0 < NR; k0 += G) {
            u32x2 t[G][CH];
#pragma unroll
            for (int kk = 0; kk < G; ++kk)
#pragma unroll
                for (int c = 0; c < CH; ++c)
                    if (k0 + kk < NR)
                        t[kk][c] = __builtin_amdgcn_raw_buffer_load_b64(r_fo, voff[c], (wave + RES_WAVES * (k0 + kk)) * row_bytes, 0);
#pragma unroll
            for (int kk = 0; kk < G; ++kk) {
                if (k0 + kk >= NR) break;
                const int i = wave + RES_WAVES * (k0 + kk);
                float p0 = 0.f, p1 = 0.f, p2 = 0.f;
#pragma unroll
                for (int c = 0; c < CH; ++c) {
                    float x[4], y[4];
                    unpack8<T>(t[kk][c], x);
                    unpack8<T>(keep[k0 + kk][c], y);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (DIST == RS_DIST_L2) { float d = x[e] - y[e]; p0 = fmaf(d, d, p0); }
                        else if (DIST == RS_DIST_L1) { p0 += fabsf(x[e] - y[e]); }
                        else { p0 = fmaf(x[e], y[e], p0); p1 = fmaf(x[e], x[e], p1); p2 = fmaf(y[e], y[e], p2); }
                    }
                }
                p0 = wave_sum(p0);
                if (DIST == RS_DIST_COS) { p1 = wave_sum(p1); p2 = wave_sum(p2); }
                if (lane == 0 && i < N) {
                    float sc;
                    if (DIST == RS_DIST_L2) sc = sqrtf(p0);
                    else if (DIST == RS_DIST_L1) sc = p0;
                    else sc = 1.0f - p0 / (sqrtf(p1) * sqrtf(p2));
                    s_scores[i] = sc;
                    scores[(int64_t)b * N + i] = sc;
                }
            }
            __builtin_amdgcn_sched_barrier(0);  // the next group's loads stay behind this group's sums
        }
        __syncthreads();
        block_select_rank<NT>(s_scores, N, n_prefix, n_keep, kept_idx + (int64_t)b * K, s_slot, sh, tid);
        __syncthreads();
        // (no barrier at the end of the loop: s_scores is next written before the barrier above, which
        // no wave passes before all have left the selection; s_slot and sh are next written two barriers on)
        const __amdgpu_buffer_rsrc_t r_out = __builtin_amdgcn_make_buffer_rsrc(
            gathered + (int64_t)b * K * D, 0, K * row_bytes, 0x00020000);
        const int b_next = b + gridDim.x;
        const __amdgpu_buffer_rsrc_t r_in = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<T*>(f_in + (int64_t)(b_next < B ? b_next : 0) * N * D), 0, b_next < B ? N * row_bytes : 0, 0x00020000);
#pragma unroll
        for (int k = 0; k < NR; ++k) {
            const int i = wave + RES_WAVES * k;
            const int j = i < N ? s_slot[i] : -1;  // wave-uniform
            if (j >= 0) {
#pragma unroll
                for (int c = 0; c < CH; ++c)
                    __builtin_amdgcn_raw_buffer_store_b64(keep[k][c], r_out, voff[c], __builtin_amdgcn_readfirstlane(j) * row_bytes, 0);
            }
#pragma unroll
            for (int c = 0; c < CH; ++c)
                keep[k][c] = __builtin_amdgcn_raw_buffer_load_b64(r_in, voff[c], i * row_bytes, 0);
        }
    }
}

bool shift_topk_resident_fits(rs_dtype dt, int N, int D) {
    return N <= RES_MAXN && (size_t)D * elem_size(dt) <= 512 * 3;
}

template <typename T, int CH>
static hipError_t launch_resident_t(rs_dist dist, const void* f_out, const void* f_in, float* scores,
                                    int32_t* kept_idx, void* gathered, int B, int N, int D, int n_prefix,
                                    int n_keep, int grid, hipStream_t s) {
#define RS_RES_LAUNCH(DIST_)                                                                                  \
    hipLaunchKernelGGL((shift_topk_resident_kernel<T, DIST_, CH, RES_NR>), dim3(grid), dim3(RES_WAVES * 64), 0, s, \
                       (const T*)f_out, (const T*)f_in, scores, kept_idx, (T*)gathered, B, N, D, n_prefix, n_keep)
    if (dist == RS_DIST_L2) RS_RES_LAUNCH(RS_DIST_L2);
    else if (dist == RS_DIST_L1) RS_RES_LAUNCH(RS_DIST_L1);
    else RS_RES_LAUNCH(RS_DIST_COS);
#undef RS_RES_LAUNCH
    return hipGetLastError();
}

hipError_t launch_shift_topk_resident(rs_dtype dt, rs_dist dist, const void* f_out, const void* f_in,
                                      float* scores, int32_t* kept_idx, void* gathered, int B, int N, int D,
                                      int n_prefix, int n_keep, hipStream_t s) {
    if (B == 0 || N == 0) return hipSuccess;
    static const int cus = [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 256;
        return n;
    }();
    const int grid = B < cus ? B : cus;  // one workgroup fills a compute unit's register file
    const int ch = (int)(((size_t)D * elem_size(dt) + 511) / 512);
#define RS_RES_CH(T_)                                                                                                   \
    (ch == 1 ? launch_resident_t<T_, 1>(dist, f_out, f_in, scores, kept_idx, gathered, B, N, D, n_prefix, n_keep, grid, s) \
     : ch == 2 ? launch_resident_t<T_, 2>(dist, f_out, f_in, scores, kept_idx, gathered, B, N, D, n_prefix, n_keep, grid, s) \
               : launch_resident_t<T_, 3>(dist, f_out, f_in, scores, kept_idx, gathered, B, N, D, n_prefix, n_keep, grid, s))
    return dt == RS_F32 ? RS_RES_CH(float) : RS_RES_CH(bf16raw);
#undef RS_RES_CH
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
        if (N > 1024)
            hipLaunchKernelGGL(select_kernel<1024>, dim3(B), dim3(1024), 0, s, const_cast<float*>(scores), kept_idx, N,
                               n_prefix, n_keep, (const float*)nullptr, 0, 0);
        else
            hipLaunchKernelGGL(select_kernel<256>, dim3(B), dim3(256), 0, s, const_cast<float*>(scores), kept_idx, N,
                               n_prefix, n_keep, (const float*)nullptr, 0, 0);
    }
    return hipGetLastError();
}

bool select_from_partials_fits(int N) { return N <= 12288; }  // scores of one image in LDS

hipError_t launch_select_from_partials(rs_dist dist, const float* partials, int slots, float* scores,
                                       int32_t* kept_idx, int B, int N, int n_prefix, int n_keep,
                                       hipStream_t s) {
    if (B == 0) return hipSuccess;
    if (N <= 256) {
        hipLaunchKernelGGL(select_kernel<1024>, dim3(B), dim3(1024), (size_t)N * sizeof(float), s, scores, kept_idx, N,
                           n_prefix, n_keep, partials, slots, (int)dist);
    } else if (B < 64) {
        // a few long sequences (video clips): one workgroup per image would walk its image's slots
        // alone, one cache line per thread and slot, and spend more time there than selecting.
        // The scores are formed by a grid over all rows instead (the same additions in the same
        // order), and the selection reads them back.
        if (hipError_t e = launch_finalize_scores(dist, partials, slots, scores, (int64_t)B * N, s); e != hipSuccess)
            return e;
        return launch_select(scores, kept_idx, B, N, n_prefix, n_keep, s);
    } else {
        hipLaunchKernelGGL(select_kernel<256>, dim3(B), dim3(256), (size_t)N * sizeof(float), s, scores, kept_idx, N,
                           n_prefix, n_keep, partials, slots, (int)dist);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Gather: out[b, j, :] = src[b, kept_idx[b, j], :]; one wavefront per row, 16 bytes per
// lane per step (rows are D * e bytes, a multiple of 16).  (A variant over the flat output, four
// vectors per thread whatever the row length, measured 50 % slower at 1536-byte rows.)
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

// The same gather for bf16 rows that also leaves the LayerNorm statistics of every row it writes
// (mean, 1 / sqrt(variance + eps)): the wave has the row in registers anyway, and the block that
// consumes the gathered rows then needs no statistics pass of its own.  Same arithmetic as the
// statistics kernel (wave_row_stats), hence the same bits.
template <int MAXC>
__global__ __launch_bounds__(256) void gather_rows_stats_kernel(const bf16raw* __restrict__ src,
                                                                const int32_t* __restrict__ kept_idx,
                                                                bf16raw* __restrict__ out,
                                                                float2* __restrict__ stats, int64_t rows, int N,
                                                                int K, int D, float eps) {
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= rows) return;
    const int64_t b = r / K;
    const bf16raw* s = src + (b * N + kept_idx[r]) * D;
    bf16raw* d = out + r * D;
    const int nchunk = D >> 3;
    float v[MAXC][8];
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        const int ch = lane + c * 64;
        if (ch < nchunk) {
            const uint4 raw = *reinterpret_cast<const uint4*>(s + ch * 8);
            *reinterpret_cast<uint4*>(d + ch * 8) = raw;
            const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                v[c][2 * i] = __uint_as_float(w[i] << 16);
                v[c][2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
            }
        }
    }
    const float2 st = wave_row_stats<MAXC>(v, nchunk, lane, D, eps);
    if (lane == 0) stats[r] = st;
}

bool gather_stats_fits(rs_dtype dt, int D) { return dt == RS_BF16 && D <= 8 * 64 * 8; }

hipError_t launch_gather_stats(const void* src, const int32_t* kept_idx, void* out, float* stats, int B, int N,
                               int K, int D, float eps, hipStream_t s) {
    const int64_t rows = (int64_t)B * K;
    if (rows == 0) return hipSuccess;
    const dim3 grid((unsigned)((rows + 3) / 4)), block(256);
    if (D <= 2 * 512)
        hipLaunchKernelGGL(gather_rows_stats_kernel<2>, grid, block, 0, s, (const bf16raw*)src, kept_idx, (bf16raw*)out,
                           reinterpret_cast<float2*>(stats), rows, N, K, D, eps);
    else
        hipLaunchKernelGGL(gather_rows_stats_kernel<8>, grid, block, 0, s, (const bf16raw*)src, kept_idx, (bf16raw*)out,
                           reinterpret_cast<float2*>(stats), rows, N, K, D, eps);
    return hipGetLastError();
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

// ---------------------------------------------------------------------------
// Token-wise pruning of a 2-D token grid (Sec. 4.2, "CNN and SSM", variant (i)): every row first
// keeps its Q highest-shift positions (select_kernel, one grid row as one "image"), the rows close
// up, and every column of the compacted H x Q grid then keeps its R highest-shift positions.
// col_scores[b, j, h] = scores[b, h, kept_cols[b, h, j]] feeds the second selection.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void grid_compact_scores_kernel(const float* __restrict__ scores,
                                                                  const int32_t* __restrict__ kept_cols,
                                                                  float* __restrict__ col_scores, int64_t total,
                                                                  int H, int W, int Q) {
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;  // index into [B, Q, H]
    if (t >= total) return;
    const int h = (int)(t % H);
    const int64_t bj = t / H;
    const int j = (int)(bj % Q);
    const int64_t b = bj / Q;
    col_scores[t] = scores[(b * H + h) * W + kept_cols[(b * H + h) * Q + j]];
}

// out[b, i, j, :] = src[b, r, kept_cols[b, r, j], :] with r = kept_rows[b, j, i]; one wavefront per position
__global__ __launch_bounds__(256) void grid_token_gather_kernel(const uint4* __restrict__ src,
                                                                const int32_t* __restrict__ kept_cols,
                                                                const int32_t* __restrict__ kept_rows,
                                                                uint4* __restrict__ out, int64_t positions, int H,
                                                                int W, int R, int Q, int vec) {
    const int lane = threadIdx.x & 63;
    const int64_t p = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (p >= positions) return;
    const int64_t b = p / ((int64_t)R * Q);
    const int ij = (int)(p - b * R * Q);
    const int i = ij / Q, j = ij - i * Q;
    const int r = kept_rows[(b * Q + j) * R + i];
    const int c = kept_cols[(b * H + r) * Q + j];
    const int64_t sp = (b * H + r) * W + c;
    for (int v = lane; v < vec; v += 64) out[p * vec + v] = src[sp * vec + v];
}

hipError_t launch_grid_compact_scores(const float* scores, const int32_t* kept_cols, float* col_scores, int B, int H,
                                      int W, int Q, hipStream_t s) {
    const int64_t total = (int64_t)B * Q * H;
    if (total == 0) return hipSuccess;
    hipLaunchKernelGGL(grid_compact_scores_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, scores,
                       kept_cols, col_scores, total, H, W, Q);
    return hipGetLastError();
}

hipError_t launch_grid_token_gather(rs_dtype dt, const void* src, const int32_t* kept_cols, const int32_t* kept_rows,
                                    void* out, int B, int H, int W, int R, int Q, int C, hipStream_t s) {
    const int64_t positions = (int64_t)B * R * Q;
    if (positions == 0) return hipSuccess;
    const int vec = (int)((size_t)C * elem_size(dt) / 16);
    hipLaunchKernelGGL(grid_token_gather_kernel, dim3((unsigned)((positions + 3) / 4)), dim3(256), 0, s,
                       (const uint4*)src, kept_cols, kept_rows, (uint4*)out, positions, H, W, R, Q, vec);
    return hipGetLastError();
}

}  // namespace rs
