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
#include <stdlib.h>

#include <atomic>

#include "common.hpp"

namespace rs {

// ---------------------------------------------------------------------------
// bf16 MFMA GEMM:  out[m, n] = epi( sum_k a[m, k] * wt[n, k] )
//   a  : [M, K] bf16 (token rows),  wt : [N, K] bf16 (packed weights),  K % 64 == 0.
// Workgroup tile BM x BN, K slices of BK, WGM x WGN waves, a ring of LDS stages.
// LDS rows are 64 bf16 = 8 slots of 16 B; chunk c of row r sits in slot c ^ ((r ^ (r >> 3)) & 7).
// The LDS has 64 banks of 4 bytes and serves a 16-byte-per-lane read 16 lanes at a time, so the
// 16 consecutive rows those lanes read for one MFMA operand must fall into 16 different
// 16-byte bank groups: the row parity picks the 128-byte half, the XOR makes the slots of rows
// r and r + 8 differ (measured: zero SQ_LDS_BANK_CONFLICT, against every second cycle with
// the plain c ^ (r & 7)).
// ---------------------------------------------------------------------------

// Exact-erf GELU x * Phi(x) for the bf16 epilogue: Phi(x) = sigmoid(x (a + b x^2 + c x^4)) with
// (a, b, c) fitted (minimax over [-9, 9]) to the erf form; max |error| of x * Phi(x) is 2.5e-5,
// below half a bf16 ulp of every output larger than 6e-3.  7 plain + 2 transcendental ops per
// element (libm erff: ~40) -- it matters: the fc1 epilogue runs M * Dm of them and plain ALU
// work does not overlap with the matrix cores on this chip.  The polynomial argument is
// clamped to [-10, 10] (it changes sign near |x| = 11); beyond that the sigmoid is 0 or 1 in
// fp32 anyway.  Constants carry the factor -log2(e) for v_exp_f32.
__device__ __forceinline__ float gelu_sp(float x) {
    const float xc = __builtin_amdgcn_fmed3f(x, -10.0f, 10.0f);
    const float x2 = xc * xc;
    float p = fmaf(1.0142687e-3f, x2, -0.10677576f);
    p = fmaf(p, x2, -2.3011212f);
    const float e = __builtin_amdgcn_exp2f(p * xc);  // exp(-x (a + b x^2 + c x^4))
    return x * __builtin_amdgcn_rcpf(1.0f + e);
}

// One element's contribution to the per-row sums of the shift: the same operations, in the same
// order per 8-feature chunk and over the chunks of a 64-feature slot, in every GEMM variant, so that
// the scores do not depend on which tile shape ran.
template <int DIST>
__device__ __forceinline__ void shift_term(float fo, float fi, float& p0, float& p1, float& p2) {
    if (DIST == RS_DIST_L2) { const float d = fo - fi; p0 = fmaf(d, d, p0); }
    else if (DIST == RS_DIST_L1) { p0 += fabsf(fo - fi); }
    else { p0 = fmaf(fo, fi, p0); p1 = fmaf(fo, fo, p1); p2 = fmaf(fi, fi, p2); }
}

// element strides between the problems of a batched launch (0 = one problem)
struct GemmBatch {
    int64_t a, w, out;
};

template <int TN, int TM>
struct Frags {
    bf16x8 w[TN], a[TM];
};

typedef __attribute__((address_space(3))) void* lds_ptr;

// One wave-wide 16-byte-per-lane copy from a buffer resource straight into LDS
// (buffer_load_dwordx4 ... lds): lane l lands at lds_base + 16 * l; reads past the
// resource's size return zeros.  `voff` is the lane's byte offset, `soff` a uniform one.
__device__ __forceinline__ void dma16(__amdgpu_buffer_rsrc_t rsrc, unsigned char* lds_base, int voff, int soff) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr)lds_base, 16, voff, soff, 0, 0);
}

// Buffer resource over the rows of ONE tile (at most 256 rows of K <= kGemmMaxK elements: under
// 2^29 bytes), so that every offset from kPastEnd upwards lies outside it and reads as zero.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, int64_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}
constexpr int kPastEnd = 0x7ff00000;

// s_waitcnt immediate for "at most n vector-memory operations outstanding" (gfx9 encoding,
// other counters left at their maximum).
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0F70; }

// WGM x WGN waves; workgroup tile BM x BN, wave tile BM/WGM x BN/WGN, K slice BK (32 or 64).
// A ring of LDS stages of (BM + BN) rows x 2*BK bytes (NSTAGE = 2), or three stages for the
// activation rows and two for the weight rows (NSTAGE = 3, long K): K slices stream from global
// memory directly into LDS (buffer_load ... lds, no register staging), one slice ahead of the
// one the matrix cores work on (activation rows with NSTAGE = 3: two).  Loads return in order,
// so "slice t has landed" is s_waitcnt vmcnt(<loads issued after it>); one workgroup barrier per
// slice.  The slice count is padded to a multiple of the unrolled trip (2 or 6 slices) with copies
// aimed past the end of the buffer resource (they deliver zeros), which keeps the loop free of
// tail branches.  Operand fragments are double buffered in registers and each LDS read is
// interleaved with its share of the previous K step's MFMAs (sched_group_barrier).  One
// workgroup per CU; the register budget is that of NW / 4 waves per SIMD.
template <int BM, int BN, int BK, int NSTAGE, int WGM, int WGN, int EPI, int DIST>
__global__ __launch_bounds__(WGM* WGN * 64, WGM* WGN / 4) void gemm_bf16_kernel(
    const bf16raw* __restrict__ a, const bf16raw* __restrict__ wt, const bf16raw* __restrict__ bias,
    const bf16raw* __restrict__ res, bf16raw* __restrict__ out, float* __restrict__ partials,
    const bf16raw* __restrict__ ref, int post, GemmLnFold ln, int M, int N, int K, int tiles_m,
    int tiles_n, int slots, int gm) {
    constexpr int NW = WGM * WGN;               // waves: WGM along tokens x WGN along features
    constexpr int WM = BM / WGM, WN = BN / WGN; // wave tile
    constexpr int TM = WM / 32, TN = WN / 32;   // MFMA tiles per wave
    constexpr int RB = BK * 2;                  // bytes per LDS row
    constexpr int SPR = BK / 8;                 // 16-byte slots per row (4 or 8)
    constexpr int RPI = 64 / SPR;               // rows one wave copy (1 KiB) covers
    constexpr int A_LOADS = BM / RPI / NW, W_LOADS = BN / RPI / NW;  // wave copies per slice and wave
    constexpr int LPW = A_LOADS + W_LOADS;
    constexpr int KK = BK / 16;                 // MFMA K steps per slice
    constexpr int STAGE = (BM + BN) * RB;
    static_assert(WM % 64 == 0 && WN % 64 == 0, "wave tiles must be multiples of 64 rows");
    static_assert(NW == 4 || NW == 8, "4 or 8 waves");
    static_assert(BM % (RPI * NW) == 0 && BN % (RPI * NW) == 0, "tile rows must split evenly over the wave copies");
    static_assert(BK == 32 || BK == 64, "K slice of 32 or 64");
    static_assert(NSTAGE == 2 || NSTAGE == 3, "two stages, or three for the activation rows (deeper rings of narrower slices measured no better)");

    // LDS, NSTAGE = 2: two stages of (BM + BN) rows.  Epilogue staging (32 fp32 rows of the wave tile
    // + the wave's row statistics per wave) lives in the array of stage 1, which is made large
    // enough for all waves: stage 0 receives the next tile's first K slice meanwhile, and being a
    // different array the compiler knows that the epilogue's LDS traffic need not wait for those
    // copies.
    // NSTAGE = 3 (long K): the activation rows of a slice and its weight rows live in arrays of
    // their own, THREE for the activations (requested two slices ahead: they are the rows that
    // come from HBM, and under load a CU's 64 KB request takes longer than one slice of matrix
    // work) and two for the weights (shared by every row panel, they come from the L2): all 160
    // KB.  Epilogue staging in activation stages 1, 2 and weight stage 1.
    constexpr int EPW = (32 * (WN * 4 + 16) + WM * 8 + 255) / 256 * 256;  // bytes per wave
    constexpr int SA = BM * RB, SW = BN * RB;
    constexpr bool DEEP = NSTAGE == 3;
    static_assert(!DEEP || (NW == 8 && 3 * EPW <= SA && 2 * EPW <= SW), "staging of waves 0-2, 3-5, 6-7 in three stage arrays");
    __shared__ __attribute__((aligned(1024))) unsigned char stage0[DEEP ? 16 : STAGE];
    __shared__ __attribute__((aligned(1024))) unsigned char stage1[DEEP ? 16 : (STAGE > NW * EPW ? STAGE : NW * EPW)];
    __shared__ __attribute__((aligned(1024))) unsigned char sa0[DEEP ? SA : 16];
    __shared__ __attribute__((aligned(1024))) unsigned char sa1[DEEP ? SA : 16];
    __shared__ __attribute__((aligned(1024))) unsigned char sa2[DEEP ? SA : 16];
    __shared__ __attribute__((aligned(1024))) unsigned char sw0[DEEP ? SW : 16];
    __shared__ __attribute__((aligned(1024))) unsigned char sw1[DEEP ? SW : 16];

    // Tile order.  Consecutive workgroup ids go round-robin to the 8 XCDs, each with its own
    // 4 MB L2, so XCD x takes a contiguous range of the tile sequence.  The sequence walks the tile
    // grid in groups of `gm` row panels, n-major inside a group (m fastest): the ~32 tiles an XCD
    // runs at a time then share gm activation panels, which stay in its L2 while the weight
    // panels stream past, instead of re-reading the whole weight matrix for every row panel.
    //
    // Persistent workgroups: the grid is one workgroup per CU; workgroup (x, j) of XCD x walks
    // positions j, j + per_xcd, ... of that XCD's range, so the tiles an XCD runs at a time are the
    // same as with one workgroup per tile, but the first K slice of the next tile is fetched while
    // the epilogue of the current one runs.
    const int nblk = tiles_m * tiles_n;
    const int xcd = blockIdx.x & 7, per_xcd = gridDim.x >> 3;
    const int xq = nblk >> 3, xr = nblk & 7;  // XCD x owns xq (+1 if x < xr) tiles
    const int x_cnt = xq + (xcd < xr ? 1 : 0), x_start = xcd * xq + (xcd < xr ? xcd : xr);
    int seq = blockIdx.x >> 3;
    if (seq >= x_cnt) return;  // whole workgroup, before any barrier
#define RS_GEMM_DECODE(seq_, m0_, n0_)                                                                    \
    {                                                                                                     \
        const int bid_ = x_start + (seq_);                                                                \
        const int per_group_ = gm * tiles_n;                                                              \
        const int grp_ = bid_ / per_group_, rem_ = bid_ - grp_ * per_group_;                              \
        const int first_m_ = grp_ * gm;                                                                   \
        const int gsz_ = min(tiles_m - first_m_, gm);                                                     \
        const int tn_ = rem_ / gsz_;                                                                      \
        (n0_) = tn_ * BN;                                                                                 \
        (m0_) = (first_m_ + rem_ - tn_ * gsz_) * BM;                                                      \
    }
    int m0, n0;
    RS_GEMM_DECODE(seq, m0, n0)

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: LDS copy targets go to M0
    const int wm = wave % WGM, wn = wave / WGM;
    const int l32 = lane & 31, g = lane >> 5;

    // LDS layout.  Chunk c (16 bytes = 8 k values) of row r sits in slot c ^ f(r).  gfx950's LDS has
    // 64 banks of 4 bytes and serves a 16-byte-per-lane read 16 lanes at a time, so the 16
    // consecutive rows those lanes read for one MFMA operand must fall into 16 different 16-byte
    // bank groups of a 256-byte line:
    //   128-byte rows (BK 64): f(r) = (r & 7) ^ ((r >> 3) & 1)   (row parity picks the half line, the
    //                          XOR makes rows r and r + 8 differ; the plain r & 7 conflicts every
    //                          second cycle.  f has period 16 in r, so one set of lane offsets
    //                          serves every 32-row MFMA tile of the wave)
    //    64-byte rows (BK 32): f(r) = (r >> 2) & 3         (r & 3 picks the quarter line)
    // global -> LDS: wave copy i of wave w fills rows (NW*i + w)*RPI .. +RPI-1 (lane l: row l / SPR,
    // slot l % SPR), so the lane fetches chunk (l % SPR) ^ f(row).
    __amdgpu_buffer_rsrc_t rs_a = make_rsrc(a + (int64_t)m0 * K, (int64_t)min(M - m0, BM) * K * 2);
    __amdgpu_buffer_rsrc_t rs_w = make_rsrc(wt + (int64_t)n0 * K, (int64_t)min(N - n0, BN) * K * 2);
    const int ld_r = lane / SPR, ld_p = lane % SPR;
    // lane byte offset inside a wave copy (NW is even, so row >> 3 = NW*i + w has the parity of w)
    const int voff = SPR == 8 ? ((wave * RPI + ld_r) * K + ((ld_p ^ ld_r ^ (wave & 1)) << 3)) * 2
                              : ((wave * RPI + ld_r) * K + ((ld_p ^ ((ld_r >> 2) & 3)) << 3)) * 2;
    const int pass_bytes = NW * RPI * K * 2;

    const int S = K / BK;                                   // real slices
    constexpr int PERIOD = DEEP ? 6 : 2;                    // slices per trip of the unrolled ring
    const int S_pad = (S + PERIOD - 1) / PERIOD * PERIOD;   // loop trip count (zero slices at the end)
    const int a_row0 = wm * WM + l32, w_row0 = wn * WN + l32;
    // slot XOR of operand row 32*t + l32 (the same for every MFMA tile t of the wave tile)
    const int sw = SPR == 8 ? ((l32 & 7) ^ ((l32 >> 3) & 1)) : ((l32 >> 2) & 3);

// copies of K slice t_ into stage_; slices past the end are aimed beyond the resource (which covers
// this tile's rows only, so the aim is past its end whatever the size of the whole matrix)
#define RS_GEMM_DMA_A(sa_, t_)                                                                            \
    {                                                                                                     \
        const bool real_ = (t_) < S;                                                                      \
        const int kb_ = (t_) * RB;                                                                        \
        _Pragma("unroll") for (int i = 0; i < A_LOADS; ++i)                                               \
            dma16(rs_a, (sa_) + (i * NW + wave) * 1024, voff, real_ ? i * pass_bytes + kb_ : kPastEnd);   \
    }
#define RS_GEMM_DMA_W(sw_, t_)                                                                            \
    {                                                                                                     \
        const bool real_ = (t_) < S;                                                                      \
        const int kb_ = (t_) * RB;                                                                        \
        _Pragma("unroll") for (int i = 0; i < W_LOADS; ++i)                                               \
            dma16(rs_w, (sw_) + (i * NW + wave) * 1024, voff, real_ ? i * pass_bytes + kb_ : kPastEnd);   \
    }
#define RS_GEMM_DMA(stage_, t_)                                                                           \
    {                                                                                                     \
        RS_GEMM_DMA_A(stage_, t_)                                                                         \
        RS_GEMM_DMA_W((stage_) + BM * RB, t_)                                                             \
    }
#define RS_GEMM_LOAD_FRAGS2(f_, sa_, sw_, kk_)                                                            \
    {                                                                                                     \
        const int c_ = ((((kk_) * 2 + g) ^ sw) << 4);                                                     \
        _Pragma("unroll") for (int i = 0; i < TN; ++i)                                                    \
            (f_).w[i] = *reinterpret_cast<const bf16x8*>((sw_) + (w_row0 + i * 32) * RB + c_);            \
        _Pragma("unroll") for (int j = 0; j < TM; ++j)                                                    \
            (f_).a[j] = *reinterpret_cast<const bf16x8*>((sa_) + (a_row0 + j * 32) * RB + c_);            \
    }
#define RS_GEMM_LOAD_FRAGS(f_, stage_, kk_) RS_GEMM_LOAD_FRAGS2(f_, stage_, (stage_) + BM * RB, kk_)
#define RS_GEMM_MFMA(f_)                                                                                  \
    {                                                                                                     \
        _Pragma("unroll") for (int i = 0; i < TN; ++i)                                                    \
            _Pragma("unroll") for (int j = 0; j < TM; ++j)                                                \
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16((f_).w[i], (f_).a[j], acc[i][j], 0, 0, 0); \
    }
// Scheduling recipe for one K step (one scheduling region): every LDS fragment read of the
// next step is followed by its share of global->LDS copies (vm_) and of this step's MFMAs.
#define RS_GEMM_INTERLEAVE(vm_)                                                                           \
    {                                                                                                     \
        _Pragma("unroll") for (int s_ = 0; s_ < TN + TM; ++s_) {                                          \
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                            \
            if (vm_) __builtin_amdgcn_sched_group_barrier(0x020, (LPW + TN + TM - 1) / (TN + TM), 0);     \
            __builtin_amdgcn_sched_group_barrier(0x008, (TN * TM) / (TN + TM), 0);                        \
        }                                                                                                 \
        __builtin_amdgcn_sched_barrier(0);                                                                \
    }
// One K slice from cur_ (its first fragments are already in f0).  Three of the four K steps run
// with the LDS reads of the following step between their MFMAs; then the wave waits for slice
// t+1 (in nxt_) to land, meets the others at the slice's one barrier -- after it every wave has
// finished reading cur_, so the copies of slice t+2 may overwrite it -- and the last K step's
// MFMAs cover those copies and the first fragment reads of slice t+1: the matrix cores have
// work on both sides of the barrier.
#define RS_GEMM_SLICE(cur_, nxt_, t_)                                                                     \
    {                                                                                                     \
        RS_GEMM_LOAD_FRAGS(f1, cur_, 1)                                                                   \
        RS_GEMM_MFMA(f0)                                                                                  \
        RS_GEMM_INTERLEAVE(0)                                                                             \
        RS_GEMM_LOAD_FRAGS(f0, cur_, 2)                                                                   \
        RS_GEMM_MFMA(f1)                                                                                  \
        RS_GEMM_INTERLEAVE(0)                                                                             \
        RS_GEMM_LOAD_FRAGS(f1, cur_, 3)                                                                   \
        RS_GEMM_MFMA(f0)                                                                                  \
        RS_GEMM_INTERLEAVE(0)                                                                             \
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));                                                         \
        __syncthreads();                                                                                  \
        RS_GEMM_DMA(cur_, (t_) + 2)                                                                       \
        RS_GEMM_LOAD_FRAGS(f0, nxt_, 0)                                                                   \
        RS_GEMM_MFMA(f1)                                                                                  \
        RS_GEMM_INTERLEAVE(1)                                                                             \
    }

// The same slice with three activation stages (sa_ / sw_: this slice, san_ / swn_: the next): the
// wave waits for slice t+1 only -- the activation rows of slice t+2, requested last, may still be
// on their way: loads complete in order, and no global store is in flight inside the K loop --
// and after the barrier requests the weights of slice t+2, then the activation rows of slice t+3.
#define RS_GEMM_SLICE3(sa_, sw_, san_, swn_, t_)                                                          \
    {                                                                                                     \
        RS_GEMM_LOAD_FRAGS2(f1, sa_, sw_, 1)                                                              \
        RS_GEMM_MFMA(f0)                                                                                  \
        RS_GEMM_INTERLEAVE(0)                                                                             \
        RS_GEMM_LOAD_FRAGS2(f0, sa_, sw_, 2)                                                              \
        RS_GEMM_MFMA(f1)                                                                                  \
        RS_GEMM_INTERLEAVE(0)                                                                             \
        RS_GEMM_LOAD_FRAGS2(f1, sa_, sw_, 3)                                                              \
        RS_GEMM_MFMA(f0)                                                                                  \
        RS_GEMM_INTERLEAVE(0)                                                                             \
        __builtin_amdgcn_s_waitcnt(((A_LOADS) & 15) | (((A_LOADS) >> 4) << 14) | 0x0070);                 \
        __builtin_amdgcn_s_barrier();                                                                     \
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup"); /* LDS reads stay below the barrier */     \
        __builtin_amdgcn_sched_barrier(0);                                                                \
        RS_GEMM_DMA_W(sw_, (t_) + 2)                                                                      \
        RS_GEMM_DMA_A(sa_, (t_) + 3)                                                                      \
        RS_GEMM_LOAD_FRAGS2(f0, san_, swn_, 0)                                                            \
        RS_GEMM_MFMA(f1)                                                                                  \
        RS_GEMM_INTERLEAVE(1)                                                                             \
    }

    static_assert(KK == 4, "the slice schedules are written for 64-wide slices");
    static_assert(A_LOADS <= 15, "copies in flight across a barrier must fit the counter");
    // first K slice of the first tile
    if constexpr (DEEP) {
        RS_GEMM_DMA_A(sa0, 0)
        RS_GEMM_DMA_W(sw0, 0)
    } else {
        RS_GEMM_DMA(stage0, 0)
    }

    for (;;) {  // one tile per iteration
    // LayerNorm-folded epilogues: fetch the (mean, rstd) of this wave's WM rows now (lane l: rows
    // l, l + 64, ...), so that the loads are long done when the epilogue wants them
    constexpr bool LN_EPI = EPI == EPI_LN_BIAS || EPI == EPI_LN_BIAS_GELU;
    float2 row_st[LN_EPI ? WM / 64 : 1];
    if (LN_EPI) {
#pragma unroll
        for (int h = 0; h < WM / 64; ++h) {
            const int m = m0 + wm * WM + h * 64 + lane;
            row_st[h] = m < M ? reinterpret_cast<const float2*>(ln.stats)[m] : make_float2(0.f, 0.f);
        }
    }

    // Likewise the per-column epilogue vectors of the lane's 8 output features (on the way out a
    // row of the wave tile is covered by WN / 8 lanes, 8 consecutive features each).
    const int ep_oc = (lane % (WN / 8)) * 8;
    const int ep_n = n0 + wn * WN + ep_oc;
    const bool ep_n_ok = ep_n < N;  // N % 8 == 0
    uint4 bias_raw = make_uint4(0u, 0u, 0u, 0u);
    float ln_bv[LN_EPI ? 8 : 1], ln_cs[LN_EPI ? 8 : 1];
    if (LN_EPI) {
#pragma unroll
        for (int e = 0; e < 8; ++e) { ln_bv[e] = 0.f; ln_cs[e] = 0.f; }
        if (ep_n_ok) {
            Elem<float>::load8(ln.bias + ep_n, reinterpret_cast<float(&)[8]>(ln_bv));
            Elem<float>::load8(ln.colsum + ep_n, reinterpret_cast<float(&)[8]>(ln_cs));
        }
    } else if (bias && ep_n_ok) {
        bias_raw = *reinterpret_cast<const uint4*>(bias + ep_n);
    }

    f32x16 acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // slice 0 has been requested (before the loop, or under the previous tile's epilogue); when it
    // has landed and every wave is past that epilogue, slice 1 goes on its way and the first
    // fragments into registers
    Frags<TN, TM> f0, f1;
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __syncthreads();
    if constexpr (DEEP) {
        // slices 1 and 2 go on their way, the activation rows of slice 2 last (they may stay in
        // flight across the first barrier).  Three activation stages and two weight stages: six
        // slices per trip, no way out in between (an exit inside the trip would make the
        // compiler keep copies of the accumulators for each way out)
        RS_GEMM_DMA_W(sw1, 1)
        RS_GEMM_DMA_A(sa1, 1)
        RS_GEMM_DMA_A(sa2, 2)
        RS_GEMM_LOAD_FRAGS2(f0, sa0, sw0, 0)
        __builtin_amdgcn_sched_barrier(0);
        for (int t = 0; t < S_pad; t += 6) {
            RS_GEMM_SLICE3(sa0, sw0, sa1, sw1, t)
            RS_GEMM_SLICE3(sa1, sw1, sa2, sw0, t + 1)
            RS_GEMM_SLICE3(sa2, sw0, sa0, sw1, t + 2)
            RS_GEMM_SLICE3(sa0, sw1, sa1, sw0, t + 3)
            RS_GEMM_SLICE3(sa1, sw0, sa2, sw1, t + 4)
            RS_GEMM_SLICE3(sa2, sw1, sa0, sw0, t + 5)
        }
    } else {
        RS_GEMM_DMA(stage1, 1)
        RS_GEMM_LOAD_FRAGS(f0, stage0, 0)
        __builtin_amdgcn_sched_barrier(0);
        for (int t = 0; t < S_pad; t += 2) {
            RS_GEMM_SLICE(stage0, stage1, t)
            RS_GEMM_SLICE(stage1, stage0, t + 1)
        }
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));  // the trailing (empty) copies too: the stages get reused
    __syncthreads();  // every wave is done with the K-loop stages


    // next tile: its first K slice streams into stage0 while the epilogue runs (past the last tile
    // the copies are aimed outside the resource and deliver zeros nobody reads).  The copies are
    // issued inside the epilogue, right after its first residual loads: loads return in order,
    // and those must not queue up behind 64 KB of copies.
    const int m0_cur = m0, n0_cur = n0;
    seq += per_xcd;
    const bool more = seq < x_cnt;
    if (more) {
        RS_GEMM_DECODE(seq, m0, n0)
        rs_a = make_rsrc(a + (int64_t)m0 * K, (int64_t)min(M - m0, BM) * K * 2);
        rs_w = make_rsrc(wt + (int64_t)n0 * K, (int64_t)min(N - n0, BN) * K * 2);
    }

    // ---- epilogue, staged through LDS so that global traffic is row-contiguous.
    // Accumulator layout: lane (l32, g) owns token row l32 of each 32-row group; register
    // 4*q + e of tile (i, j) is feature 32*i + 8*q + 4*g + e.  Per 32-row group j the wave writes
    // its 32 x WN fp32 block into a private LDS region (row pitch WN*4 + 16 bytes: conflict
    // free), then re-reads it with 16 lanes per row, 8 consecutive features per lane; bias,
    // GELU, residual, the shift partial sums and the bf16 rounding happen on that layout, and
    // every global load/store instruction covers whole 16 * WN / 8-byte row segments.
    {
        constexpr int PITCH = WN * 4 + 16;         // bytes per staged row
        constexpr int LPR = WN / 8;                // lanes per row on the way out (16 for WN = 128)
        constexpr int RPS = 64 / LPR;              // rows per step
        static_assert(32 * PITCH + WM * 8 <= EPW, "epilogue staging does not fit");
        unsigned char* ep = !DEEP ? stage1 + wave * EPW
                            : wave < 3 ? sa1 + wave * EPW : wave < 6 ? sa2 + (wave - 3) * EPW : sw1 + (wave - 6) * EPW;
        float2* ep_st = reinterpret_cast<float2*>(ep + 32 * PITCH);  // the wave's row statistics
        if (LN_EPI) {
#pragma unroll
            for (int h = 0; h < WM / 64; ++h) ep_st[h * 64 + lane] = row_st[h];
        }
        const int oc = ep_oc;                      // this lane's first feature inside the wave tile
        const int orow = lane / LPR;
        const int n = ep_n;
        const bool n_ok = ep_n_ok;
        constexpr bool LN = LN_EPI;
        float bv[8], cs[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            bv[e] = LN ? ln_bv[LN ? e : 0] : 0.f;
            cs[e] = LN ? ln_cs[LN ? e : 0] : 0.f;
        }
        if (!LN) {
            const uint32_t w4[4] = {bias_raw.x, bias_raw.y, bias_raw.z, bias_raw.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                bv[2 * e] = __uint_as_float(w4[e] << 16);
                bv[2 * e + 1] = __uint_as_float(w4[e] & 0xffff0000u);
            }
        }
        // The residual rows of a 32-row group are requested one group ahead (those of group 0 before
        // the loop): a group's staging round trip through LDS is far shorter than a trip to memory.
        constexpr bool RES = EPI == EPI_BIAS_RES || EPI == EPI_BIAS_RES_SHIFT;
        uint4 res_all[RES ? TM : 1][RES ? 32 / RPS : 1];
#define RS_GEMM_LOAD_RES(j_)                                                                              \
    if (RES) {                                                                                            \
        _Pragma("unroll") for (int st = 0; st < 32 / RPS; ++st) {                                         \
            const int m = m0_cur + wm * WM + (j_) * 32 + st * RPS + orow;                                 \
            res_all[RES ? (j_) : 0][st] = (m < M && n_ok) ? *reinterpret_cast<const uint4*>(res + (int64_t)m * N + n) \
                                                           : make_uint4(0u, 0u, 0u, 0u);                  \
        }                                                                                                 \
    }
        RS_GEMM_LOAD_RES(0)
#pragma unroll
        for (int j = 0; j < TM; ++j) {
            if (j + 1 < TM) RS_GEMM_LOAD_RES(j + 1)
            const uint4 (&res_raw)[RES ? 32 / RPS : 1] = res_all[RES ? j : 0];
            if (j == 0) {
                if constexpr (DEEP) {
                    RS_GEMM_DMA_A(sa0, more ? 0 : S)
                    RS_GEMM_DMA_W(sw0, more ? 0 : S)
                } else {
                    RS_GEMM_DMA(stage0, more ? 0 : S)
                }
            }
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    f32x4 v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                    *reinterpret_cast<f32x4*>(ep + l32 * PITCH + (i * 32 + q * 8 + g * 4) * 4) = v;
                }
#pragma unroll
            for (int st = 0; st < 32 / RPS; ++st) {
                const int r = st * RPS + orow;
                const int m = m0_cur + wm * WM + j * 32 + r;
                const bool ok = m < M && n_ok;
                float v[8];
                {
                    const f32x4 lo = *reinterpret_cast<const f32x4*>(ep + r * PITCH + oc * 4);
                    const f32x4 hi = *reinterpret_cast<const f32x4*>(ep + r * PITCH + oc * 4 + 16);
                    if (LN) {
                        const float2 st = ep_st[j * 32 + r];
                        const float nm = -st.x;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            v[e] = fmaf(st.y, fmaf(nm, cs[e], lo[e]), bv[e]);
                            v[4 + e] = fmaf(st.y, fmaf(nm, cs[4 + e], hi[e]), bv[4 + e]);
                        }
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) { v[e] = lo[e] + bv[e]; v[4 + e] = hi[e] + bv[4 + e]; }
                    }
                }
                if (EPI == EPI_BIAS_GELU || EPI == EPI_LN_BIAS_GELU) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[e] = gelu_sp(v[e]);
                }
                float p0 = 0.f, p1 = 0.f, p2 = 0.f;
                if (EPI == EPI_BIAS_RES || EPI == EPI_BIAS_RES_SHIFT) {
                    float rr[8];
                    {
                        const uint4 q4 = res_raw[RES ? st : 0];
                        const uint32_t w4[4] = {q4.x, q4.y, q4.z, q4.w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            rr[2 * e] = __uint_as_float(w4[e] << 16);
                            rr[2 * e + 1] = __uint_as_float(w4[e] & 0xffff0000u);
                        }
                    }
                    if (EPI == EPI_BIAS_RES_SHIFT && ok) {
                        // D(f_out, f_in): f_out is the branch output, or (post) the residual stream
                        // after the add; f_in is the residual operand, or `ref` when one is given
                        float fi[8];
#pragma unroll
                        for (int e = 0; e < 8; ++e) fi[e] = rr[e];
                        if (ref) Elem<bf16raw>::load8(ref + (int64_t)m * N + n, fi);
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const float fo = post ? v[e] + rr[e] : v[e];
                            shift_term<DIST>(fo, fi[e], p0, p1, p2);
                        }
                    }
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[e] += rr[e];
                }
                if (ok) Elem<bf16raw>::store8(out + (int64_t)m * N + n, v);
                if (EPI == EPI_BIAS_RES_SHIFT) {
                    // sum over the LPR lanes that share the row (fixed butterfly order)
#pragma unroll
                    for (int off = LPR / 2; off >= 1; off >>= 1) {
                        p0 += __shfl_xor(p0, off, 64);
                        if (DIST == RS_DIST_COS) { p1 += __shfl_xor(p1, off, 64); p2 += __shfl_xor(p2, off, 64); }
                    }
                    const int slot = (n0_cur + wn * WN) / WN;
                    if ((lane % LPR) == 0 && m < M && slot < slots) {
                        float* dst = partials + ((int64_t)m * slots + slot) * kShiftLanes;
                        dst[0] = p0;
                        if (DIST == RS_DIST_COS) { dst[1] = p1; dst[2] = p2; }
                    }
                }
            }
        }
    }
        if (!more) break;
    }  // tiles
#undef RS_GEMM_DMA
#undef RS_GEMM_DMA_A
#undef RS_GEMM_DMA_W
#undef RS_GEMM_LOAD_RES
#undef RS_GEMM_LOAD_FRAGS2
#undef RS_GEMM_SLICE3
#undef RS_GEMM_DECODE
#undef RS_GEMM_LOAD_FRAGS
#undef RS_GEMM_MFMA
#undef RS_GEMM_INTERLEAVE
#undef RS_GEMM_SLICE
}

// ---------------------------------------------------------------------------
// Epilogue in the accumulator layout (ring kernels below).
//
// A wave owns WM = 32 TM token rows x 64 features; lane (l32, g) holds, for row 32 j + l32 of
// every 32-row group j, features 32 i + 8 q + 4 g + e in register 4 q + e of acc[i][j].  All the
// arithmetic of the epilogue -- LayerNorm fold, bias, GELU, residual add, the per-row partial sums
// of the shift -- runs on that layout: per-row quantities (mean, rstd, the shift sums) are lane
// private, per-column vectors are the same for the 32 lanes of a half-wave.  Only the traffic with
// global memory goes through LDS, in bf16, one 4 KB region (32 rows x 128 bytes) per 32-row group:
// the residual rows arrive there by direct copies (8 lanes per 128-byte row segment), a lane picks
// up its 4 features at a time (8 bytes), puts the result back IN PLACE, and the group then leaves
// as 16 bytes per lane, 8 lanes per row segment.  An element is rounded to bf16 once, after all
// arithmetic in fp32, whatever the epilogue.
// All residual copies of the tile are requested before anything else and awaited once: vector
// memory loads and stores complete out of order with respect to each other, so "all but the
// newest n operations have completed" says nothing about a copy once output stores are in flight.
// 16-byte chunk c of row r sits in slot c ^ ((r ^ (r >> 3)) & 7).
// ---------------------------------------------------------------------------
__device__ __forceinline__ int epi_swz(int r) { return (r ^ (r >> 3)) & 7; }

template <int TM>
struct EpiRegions {
    unsigned char* r[TM];  // one 4 KB LDS region per 32-row group of this wave
};

template <int TM, int EPI, int DIST>
__device__ __forceinline__ void gemm_epilogue_acc_layout(
    f32x16 (&acc)[2][TM], const EpiRegions<TM>& reg,
    const bf16raw* __restrict__ bias, const bf16raw* __restrict__ res, bf16raw* __restrict__ out,
    float* __restrict__ partials, const bf16raw* __restrict__ ref, int post, const GemmLnFold& ln,
    int M, int N, int slots, int m_base /* first row of the wave tile */, int n_base /* first feature */,
    int lane) {
    constexpr bool LN = EPI == EPI_LN_BIAS || EPI == EPI_LN_BIAS_GELU;
    constexpr bool GELU = EPI == EPI_BIAS_GELU || EPI == EPI_LN_BIAS_GELU;
    constexpr bool RES = EPI == EPI_BIAS_RES || EPI == EPI_BIAS_RES_SHIFT;
    constexpr bool SHIFT = EPI == EPI_BIAS_RES_SHIFT;
    if (n_base >= N) return;  // a wave's 64 features are all inside N or all outside (N % 64 == 0)
    const int l32 = lane & 31, g = lane >> 5;
    const int rows_valid = min(max(M - m_base, 0), 32 * TM);
    if (rows_valid == 0) return;

    // residual rows: per group 4 copies of 8 rows x 128 bytes (lane l: row l / 8, slot l % 8 holds
    // chunk (l % 8) ^ swz(row)); rows past M read as zeros through the resource
    if (RES) {
        const __amdgpu_buffer_rsrc_t rs_res =
            make_rsrc(res + (int64_t)m_base * N + n_base, ((int64_t)(rows_valid - 1) * N + 64) * 2);
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int r = p * 8 + (lane >> 3);
            const int voff = (r * N + (((lane & 7) ^ epi_swz(r)) << 3)) * 2;
#pragma unroll
            for (int j = 0; j < TM; ++j) dma16(rs_res, reg.r[j] + p * 1024, voff, j * 32 * N * 2);
        }
    }

    // per-column vectors of this lane's 32 features
    float bv[2][4][4], cs[LN ? 2 : 1][4][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int n = n_base + i * 32 + q * 8 + g * 4;
            if (LN) {
                const f32x4 b4 = *reinterpret_cast<const f32x4*>(ln.bias + n);
                const f32x4 c4 = *reinterpret_cast<const f32x4*>(ln.colsum + n);
#pragma unroll
                for (int e = 0; e < 4; ++e) { bv[i][q][e] = b4[e]; cs[LN ? i : 0][q][e] = c4[e]; }
            } else if (bias) {
                const uint2 b2 = *reinterpret_cast<const uint2*>(bias + n);
                bv[i][q][0] = __uint_as_float(b2.x << 16); bv[i][q][1] = __uint_as_float(b2.x & 0xffff0000u);
                bv[i][q][2] = __uint_as_float(b2.y << 16); bv[i][q][3] = __uint_as_float(b2.y & 0xffff0000u);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) bv[i][q][e] = 0.f;
            }
        }
    // per-row LayerNorm statistics of this lane's TM rows
    float2 stats[LN ? TM : 1];
    if (LN) {
#pragma unroll
        for (int j = 0; j < TM; ++j) {
            const int m = m_base + j * 32 + l32;
            stats[LN ? j : 0] = m < M ? reinterpret_cast<const float2*>(ln.stats)[m] : make_float2(0.f, 0.f);
        }
    }
    if (RES) __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));  // every residual row of the tile has landed

    const int sw = epi_swz(l32);
#pragma unroll
    for (int j = 0; j < TM; ++j) {
        const int m = m_base + j * 32 + l32;
        const bool m_ok = m < M;
        const float2 st = stats[LN ? j : 0];
        unsigned char* buf = reg.r[j];
        // Shift sums of the row's 64 features: per chunk of 8 features a running sum in feature order
        // (half-wave g = 0 holds the first four terms and hands its sum to g = 1, which goes on with
        // the other four), then the 8 chunk sums pairwise (c, c ^ 4), (.., c ^ 2), (.., c ^ 1).
        float pc0[8], pc1[DIST == RS_DIST_COS ? 8 : 1], pc2[DIST == RS_DIST_COS ? 8 : 1];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                unsigned char* at = buf + l32 * 128 + (((i * 4 + q) ^ sw) << 4) + g * 8;
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float a_ = acc[i][j][4 * q + e];
                    v[e] = LN ? fmaf(st.y, fmaf(-st.x, cs[LN ? i : 0][q][e], a_), bv[i][q][e]) : a_ + bv[i][q][e];
                    if (GELU) v[e] = gelu_sp(v[e]);
                }
                if (RES) {
                    const uint2 r2 = *reinterpret_cast<const uint2*>(at);
                    float rr[4] = {__uint_as_float(r2.x << 16), __uint_as_float(r2.x & 0xffff0000u),
                                   __uint_as_float(r2.y << 16), __uint_as_float(r2.y & 0xffff0000u)};
                    if (SHIFT) {
                        // D(f_out, f_in): f_out is the branch output, or (post) the residual stream after
                        // the add; f_in is the residual operand, or `ref` when one is given
                        float fi[4] = {rr[0], rr[1], rr[2], rr[3]};
                        if (ref && m_ok) {
                            const uint2 f2 = *reinterpret_cast<const uint2*>(ref + (int64_t)m * N + n_base + i * 32 + q * 8 + g * 4);
                            fi[0] = __uint_as_float(f2.x << 16); fi[1] = __uint_as_float(f2.x & 0xffff0000u);
                            fi[2] = __uint_as_float(f2.y << 16); fi[3] = __uint_as_float(f2.y & 0xffff0000u);
                        }
                        float s0 = 0.f, s1 = 0.f, s2 = 0.f;
                        if (m_ok) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) shift_term<DIST>(post ? v[e] + rr[e] : v[e], fi[e], s0, s1, s2);
                        }
                        // g = 1 restarts from the sum of g = 0 (its own first pass is discarded)
                        const float h0 = __shfl_xor(s0, 32, 64);
                        float t0 = h0, t1 = 0.f, t2 = 0.f;
                        if (DIST == RS_DIST_COS) { t1 = __shfl_xor(s1, 32, 64); t2 = __shfl_xor(s2, 32, 64); }
                        if (m_ok) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) shift_term<DIST>(post ? v[e] + rr[e] : v[e], fi[e], t0, t1, t2);
                        }
                        pc0[i * 4 + q] = t0;
                        if (DIST == RS_DIST_COS) { pc1[DIST == RS_DIST_COS ? i * 4 + q : 0] = t1; pc2[DIST == RS_DIST_COS ? i * 4 + q : 0] = t2; }
                    }
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] += rr[e];
                }
                uint2 w2;
                w2.x = pack2bf(v[0], v[1]);
                w2.y = pack2bf(v[2], v[3]);
                *reinterpret_cast<uint2*>(at) = w2;  // in place: this lane alone reads and writes these 8 bytes
            }
        if (SHIFT) {
            if (g == 1 && m_ok) {  // the half-wave that holds the complete chunk sums
                float* dst = partials + ((int64_t)m * slots + (n_base >> 6)) * kShiftLanes;
                dst[0] = ((pc0[0] + pc0[4]) + (pc0[2] + pc0[6])) + ((pc0[1] + pc0[5]) + (pc0[3] + pc0[7]));
                if (DIST == RS_DIST_COS) {
                    constexpr int C = DIST == RS_DIST_COS ? 1 : 0;
                    dst[1] = ((pc1[0] + pc1[4 * C]) + (pc1[2 * C] + pc1[6 * C])) + ((pc1[1 * C] + pc1[5 * C]) + (pc1[3 * C] + pc1[7 * C]));
                    dst[2] = ((pc2[0] + pc2[4 * C]) + (pc2[2 * C] + pc2[6 * C])) + ((pc2[1 * C] + pc2[5 * C]) + (pc2[3 * C] + pc2[7 * C]));
                }
            }
        }
        // the group leaves as 16 bytes per lane (LDS accesses of one wave are served in order)
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int r = p * 8 + (lane >> 3), cc = lane & 7;
            const uint4 o4 = *reinterpret_cast<const uint4*>(buf + r * 128 + ((cc ^ epi_swz(r)) << 4));
            const int mo = m_base + j * 32 + r;
            if (mo < M) *reinterpret_cast<uint4*>(out + (int64_t)mo * N + n_base + cc * 8) = o4;
        }
    }
}

// ---------------------------------------------------------------------------
// Ring kernel: workgroup tile BM x BN (BM token rows, BN features), four waves (WGM x WGN, wave
// tile BM / WGM x 64), K slices of 32 in a ring of three LDS stages, one tile per workgroup and TWO
// workgroups per compute unit (at most 72 KB of LDS and 256 registers each).  The two run out of
// step: while one is in its epilogue, or waits at its per-slice barrier for a late copy, the
// other's K loop keeps the matrix cores busy, and the hardware hands a finished workgroup's slot
// to the next tile, so the tail of a launch is balanced at half-tile granularity.  Copies run two
// slices ahead of the matrix work.
// Slice schedule (one barrier per slice, matrix work on both sides of it): the second K step's
// fragments are read under the first step's MFMAs; then the wave waits for the next slice's
// copies, meets the barrier (now every wave has read this slice: its stage is free), requests the
// slice three ahead into the freed stage and reads the next slice's first fragments under the
// second step's MFMAs.
// ---------------------------------------------------------------------------
template <int BM, int BN, int WGM, int WGN, int EPI, int DIST>
__global__ __launch_bounds__(256, 2) void gemm_bf16_ring_kernel(
    const bf16raw* __restrict__ a, const bf16raw* __restrict__ wt, const bf16raw* __restrict__ bias,
    const bf16raw* __restrict__ res, bf16raw* __restrict__ out, float* __restrict__ partials,
    const bf16raw* __restrict__ ref, int post, GemmLnFold ln, int M, int N, int K, int tiles_m,
    int tiles_n, int slots, int gm, GemmBatch batch) {
    constexpr int NW = WGM * WGN;
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int BK = 32, RB = BK * 2, RPI = 16;   // 64-byte LDS rows, 16 rows per wave copy
    // batched use (blockIdx.y = problem): the same shape at other addresses, plain epilogues only
    a += (int64_t)blockIdx.y * batch.a;
    wt += (int64_t)blockIdx.y * batch.w;
    out += (int64_t)blockIdx.y * batch.out;
    constexpr int A_LOADS = BM / RPI / NW, W_LOADS = BN / RPI / NW, LPW = A_LOADS + W_LOADS;
    constexpr int STAGE = (BM + BN) * RB;
    static_assert(NW == 4 && WN == 64 && TN == 2, "four waves, wave tiles 64 features wide");
    static_assert(BM % (RPI * NW) == 0 && BN % (RPI * NW) == 0, "tile rows must split evenly over the wave copies");
    static_assert(3 * (STAGE / 4096) >= NW * TM, "the three stages must hold TM 4 KB epilogue regions per wave");
    __shared__ __attribute__((aligned(1024))) unsigned char st0[STAGE];
    __shared__ __attribute__((aligned(1024))) unsigned char st1[STAGE];
    __shared__ __attribute__((aligned(1024))) unsigned char st2[STAGE];

    // tile of this workgroup: ids go round-robin to the 8 XCDs, XCD x takes a contiguous range of a
    // sequence that walks the grid in groups of gm row panels, m fastest (see gemm_bf16_kernel)
    const int nblk = tiles_m * tiles_n;
    const int xcd = blockIdx.x & 7;
    const int xq = nblk >> 3, xr = nblk & 7;
    const int x_cnt = xq + (xcd < xr ? 1 : 0), x_start = xcd * xq + (xcd < xr ? xcd : xr);
    const int seq = blockIdx.x >> 3;
    if (seq >= x_cnt) return;  // whole workgroup, before any barrier
    int m0, n0;
    {
        const int bid = x_start + seq;
        const int per_group = gm * tiles_n;
        const int grp = bid / per_group, rem = bid - grp * per_group;
        const int first_m = grp * gm;
        const int gsz = min(tiles_m - first_m, gm);
        const int tn = rem / gsz;
        n0 = tn * BN;
        m0 = (first_m + rem - tn * gsz) * BM;
    }

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WGM, wn = wave / WGM;
    const int l32 = lane & 31, g = lane >> 5;

    // global -> LDS: wave copy i of wave w fills rows (NW i + w) 16 .. + 15 (lane l: row l / 4, slot
    // l % 4 holds chunk (l % 4) ^ f(row), f(r) = (r >> 2) & 3: the 16 rows an operand read touches
    // fall into 16 different 16-byte bank groups)
    const __amdgpu_buffer_rsrc_t rs_a = make_rsrc(a + (int64_t)m0 * K, (int64_t)min(M - m0, BM) * K * 2);
    const __amdgpu_buffer_rsrc_t rs_w = make_rsrc(wt + (int64_t)n0 * K, (int64_t)min(N - n0, BN) * K * 2);
    const int ld_r = lane >> 2, ld_p = lane & 3;
    const int voff = ((wave * RPI + ld_r) * K + ((ld_p ^ ((ld_r >> 2) & 3)) << 3)) * 2;
    const int pass_bytes = NW * RPI * K * 2;
    const int S = K / BK;
    const int S_pad = (S + 2) / 3 * 3;
    const int a_row0 = wm * WM + l32, w_row0 = wn * WN + l32;
    const int sw = (l32 >> 2) & 3;

#define RS_RING_DMA(stage_, t_)                                                                           \
    {                                                                                                     \
        const bool real_ = (t_) < S;                                                                      \
        const int kb_ = (t_) * RB;                                                                        \
        _Pragma("unroll") for (int i = 0; i < A_LOADS; ++i)                                               \
            dma16(rs_a, (stage_) + (i * NW + wave) * 1024, voff, real_ ? i * pass_bytes + kb_ : kPastEnd); \
        _Pragma("unroll") for (int i = 0; i < W_LOADS; ++i)                                               \
            dma16(rs_w, (stage_) + BM * RB + (i * NW + wave) * 1024, voff, real_ ? i * pass_bytes + kb_ : kPastEnd); \
    }
#define RS_RING_FRAGS(f_, stage_, kk_)                                                                    \
    {                                                                                                     \
        const int co_ = ((((kk_) * 2 + g) ^ sw) << 4);                                                    \
        _Pragma("unroll") for (int i = 0; i < TN; ++i)                                                    \
            (f_).w[i] = *reinterpret_cast<const bf16x8*>((stage_) + (BM + w_row0 + i * 32) * RB + co_);   \
        _Pragma("unroll") for (int j = 0; j < TM; ++j)                                                    \
            (f_).a[j] = *reinterpret_cast<const bf16x8*>((stage_) + (a_row0 + j * 32) * RB + co_);        \
    }
#define RS_RING_MFMA(f_)                                                                                  \
    {                                                                                                     \
        _Pragma("unroll") for (int i = 0; i < TN; ++i)                                                    \
            _Pragma("unroll") for (int j = 0; j < TM; ++j)                                                \
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16((f_).w[i], (f_).a[j], acc[i][j], 0, 0, 0); \
    }
// every LDS fragment read is followed by its share of copies and of the running step's MFMAs
#define RS_RING_INTERLEAVE(vm_)                                                                           \
    {                                                                                                     \
        _Pragma("unroll") for (int s_ = 0; s_ < TN + TM; ++s_) {                                          \
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                            \
            if (vm_) __builtin_amdgcn_sched_group_barrier(0x020, (LPW + TN + TM - 1) / (TN + TM), 0);     \
            __builtin_amdgcn_sched_group_barrier(0x008, (TN * TM + TN + TM - 1) / (TN + TM), 0);          \
        }                                                                                                 \
        __builtin_amdgcn_sched_barrier(0);                                                                \
    }
// vmcnt <= LPW: the copies of the slice after next may be in flight; LDS reads all answered
#define RS_RING_SLICE(cur_, nxt_, t_)                                                                     \
    {                                                                                                     \
        RS_RING_FRAGS(f1, cur_, 1)                                                                        \
        RS_RING_MFMA(f0)                                                                                  \
        RS_RING_INTERLEAVE(0)                                                                             \
        __builtin_amdgcn_s_waitcnt(((LPW) & 15) | (((LPW) >> 4) << 14) | 0x0070);                         \
        __builtin_amdgcn_s_barrier();                                                                     \
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup"); /* LDS reads stay below the barrier */     \
        __builtin_amdgcn_sched_barrier(0);                                                                \
        RS_RING_DMA(cur_, (t_) + 3)                                                                       \
        RS_RING_FRAGS(f0, nxt_, 0)                                                                        \
        RS_RING_MFMA(f1)                                                                                  \
        RS_RING_INTERLEAVE(1)                                                                             \
    }

    f32x16 acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    RS_RING_DMA(st0, 0)
    RS_RING_DMA(st1, 1)
    RS_RING_DMA(st2, 2)
    Frags<TN, TM> f0, f1;
    __builtin_amdgcn_s_waitcnt(((2 * LPW) & 15) | (((2 * LPW) >> 4) << 14) | 0x0070);  // slice 0 has landed
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    __builtin_amdgcn_sched_barrier(0);
    RS_RING_FRAGS(f0, st0, 0)
    for (int t = 0; t < S_pad; t += 3) {
        RS_RING_SLICE(st0, st1, t)
        RS_RING_SLICE(st1, st2, t + 1)
        RS_RING_SLICE(st2, st0, t + 2)
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0) & 0xC07F);  // trailing (empty) copies and LDS reads: the stages get reused
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    __builtin_amdgcn_sched_barrier(0);
#undef RS_RING_DMA
#undef RS_RING_FRAGS
#undef RS_RING_MFMA
#undef RS_RING_INTERLEAVE
#undef RS_RING_SLICE

    // epilogue regions: TM x 4 KB per wave, numbered through the three stage arrays
    EpiRegions<TM> reg;
    {
        constexpr int PER = STAGE / 4096;  // regions per stage array
#pragma unroll
        for (int j = 0; j < TM; ++j) {
            const int gi = wave * TM + j;
            reg.r[j] = (gi / PER == 0 ? st0 : gi / PER == 1 ? st1 : st2) + (gi % PER) * 4096;
        }
    }
    gemm_epilogue_acc_layout<TM, EPI, DIST>(acc, reg, bias, res, out, partials, ref, post, ln, M, N, slots,
                                            m0 + wm * WM, n0 + wn * WN, lane);
}

// Tile configuration of the bf16 GEMM: BM, BN, BK, NSTAGE, waves along tokens, waves along features.
#ifndef RS_GEMM_GM
#define RS_GEMM_GM 8
#endif
struct GemmCfg {
#ifndef RS_GEMM_CFG
#define RS_GEMM_CFG 256, 256, 64, 2, 2, 4
#endif
    static constexpr int P[6] = {RS_GEMM_CFG};
    static constexpr int BM = P[0], BN = P[1], BK = P[2], NSTAGE = P[3], WGM = P[4], WGN = P[5];
    static constexpr int WN = BN / WGN;
};

static int device_cus() {
    static const int cus = [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 8) n = 256;
        return n;
    }();
    return cus;
}

// Which bf16 tile variant runs: 0 = chosen by shape (below), 1 = 256 x 256 persistent kernel,
// 2 = 256 x 128 ring kernel, 3 = 128 x 128 ring kernel.  Every variant gives the same bits; the
// switch exists for tuning and for the test that checks exactly that.  Initial value from the
// environment variable RS_GEMM_FORCE.
static std::atomic<int> g_gemm_variant{-1};

int gemm_variant() {
    int v = g_gemm_variant.load(std::memory_order_relaxed);
    if (v < 0) {
        const char* e = getenv("RS_GEMM_FORCE");
        v = e ? atoi(e) : 0;
        if (v < 0 || v > 4) v = 0;
        g_gemm_variant.store(v);
    }
    return v;
}

void set_gemm_variant(int v) { g_gemm_variant.store(v >= 0 && v <= 4 ? v : 0); }

struct GemmArgs {
    const bf16raw *a, *wt, *bias, *res, *ref;
    bf16raw* out;
    float* partials;
    int post;
    GemmLnFold ln;
    int64_t M;
    int N, K;
    // the same problem restricted to rows [r0, r1)
    GemmArgs rows(int64_t r0, int64_t r1) const {
        GemmArgs g = *this;
        const int slots = (N + 63) / 64;
        g.a = a + r0 * K;
        g.res = res ? res + r0 * N : nullptr;
        g.ref = ref ? ref + r0 * N : nullptr;
        g.out = out + r0 * N;
        g.partials = partials ? partials + r0 * slots * kShiftLanes : nullptr;
        g.ln.stats = ln.stats ? ln.stats + r0 * 2 : nullptr;
        g.M = r1 - r0;
        return g;
    }
};

template <int BM, int BN, int EPI, int DIST>
static void launch_ring(const GemmArgs& g, hipStream_t s) {
    const int tiles_m = (int)((g.M + BM - 1) / BM), tiles_n = (g.N + BN - 1) / BN;
    const int nblk = tiles_m * tiles_n;
    constexpr int WGN = BN / 64, WGM = 4 / WGN;  // four waves, each 64 features wide
    hipLaunchKernelGGL((gemm_bf16_ring_kernel<BM, BN, WGM, WGN, EPI, DIST>), dim3(8 * ((nblk + 7) / 8)), dim3(256), 0, s,
                       g.a, g.wt, g.bias, g.res, g.out, g.partials, g.ref, g.post, g.ln, (int)g.M, g.N, g.K, tiles_m,
                       tiles_n, (g.N + 63) / 64, RS_GEMM_GM, GemmBatch{0, 0, 0});
}

// The ring kernel with the tile width that suits the grid.  128 x 128 tiles unless they would leave
// some CUs two workgroups and others one (more than one workgroup per CU, at most two): then the
// 128 x 256 tiles, half as many, give every CU one workgroup of the same length (fc2 at 6280 rows:
// 58 -> 48 us); and for large grids, where the wider tile moves fewer bytes per flop.
template <int EPI, int DIST>
static void launch_ring_auto(const GemmArgs& g, hipStream_t s) {
    const int cus = device_cus();
    const int64_t n128 = ((g.M + 127) / 128) * ((g.N + 127) / 128);  // workgroups of the 128 x 128 tiling
    if ((n128 > cus && n128 <= 2 * cus) || n128 >= 4 * cus) launch_ring<128, 256, EPI, DIST>(g, s);
    else launch_ring<128, 128, EPI, DIST>(g, s);
}

// With a long K (at least 2048, and a slice count that the six-slice trip of the deeper ring pads
// by under 5 %) the kernel runs with three activation stages: its copies, not its matrix work,
// set the pace there (fc2 of ViT-B: -5 %); with a short K the tile is mostly prologue and
// epilogue and the third stage's extra requests cost more than they hide (+2..5 %).
static bool gemm_deep_stages(int K) {
    static const int force = [] { const char* e = getenv("RS_GEMM_STAGES"); return e ? atoi(e) : 0; }();  // tuning aid: 2 or 3
    if (force == 2 || force == 3) return force == 3;
    const int S = K / 64, pad = (S + 5) / 6 * 6 - S;
    return K >= 2048 && 20 * pad <= S;
}

template <int EPI, int DIST>
static void launch_persistent(const GemmArgs& g, hipStream_t s) {
    using C = GemmCfg;
    const int tiles_m = (int)((g.M + C::BM - 1) / C::BM), tiles_n = (g.N + C::BN - 1) / C::BN;
    // one workgroup per CU (8 XCDs x CUs / 8), fewer when an XCD's share of the tiles is smaller
    const int cus = device_cus();
    const int share = (tiles_m * tiles_n + 7) / 8;
    const int per_xcd = share < cus / 8 ? share : cus / 8;
    if (gemm_deep_stages(g.K))
        hipLaunchKernelGGL((gemm_bf16_kernel<C::BM, C::BN, C::BK, 3, C::WGM, C::WGN, EPI, DIST>),
                           dim3(8 * per_xcd), dim3(C::WGM * C::WGN * 64), 0, s, g.a, g.wt, g.bias, g.res, g.out, g.partials,
                           g.ref, g.post, g.ln, (int)g.M, g.N, g.K, tiles_m, tiles_n, (g.N + 63) / 64, RS_GEMM_GM);
    else
        hipLaunchKernelGGL((gemm_bf16_kernel<C::BM, C::BN, C::BK, 2, C::WGM, C::WGN, EPI, DIST>),
                           dim3(8 * per_xcd), dim3(C::WGM * C::WGN * 64), 0, s, g.a, g.wt, g.bias, g.res, g.out, g.partials,
                           g.ref, g.post, g.ln, (int)g.M, g.N, g.K, tiles_m, tiles_n, (g.N + 63) / 64, RS_GEMM_GM);
}

// Choice by shape.  The persistent 256 x 256 kernel has the best matrix-core rate while most CUs
// have a tile, but its last round costs a whole round however few tiles it holds, and well below
// one round it leaves CUs empty; the ring kernels (two smaller workgroups per CU, tiles handed out
// as slots free up, epilogues under the other workgroup's matrix work) keep the chip busy on
// small and ragged problems at a lower peak rate.  Measured crossovers on MI355X: the ring kernels
// win up to half a round of 256 x 256 tiles, and up to a round and a half when K is short
// (K <= 512: a tile is mostly epilogue).  Beyond that: the rows that make up whole rounds go to the
// persistent kernel and the rows behind them to a ring kernel in a second launch -- when a round
// is long (K at least RS_GEMM_TAIL_MINK: a second launch costs a few microseconds) and the last
// one is at most RS_GEMM_TAIL_FRAC full.
#ifndef RS_GEMM_TAIL_FRAC
#define RS_GEMM_TAIL_FRAC 0.5
#endif
#ifndef RS_GEMM_TAIL_MINK
#define RS_GEMM_TAIL_MINK 2048
#endif
// (tuning aids: the environment variables of the same names override the two thresholds)
static double gemm_tail_frac() {
    static const double v = [] { const char* e = getenv("RS_GEMM_TAIL_FRAC"); return e ? atof(e) : (double)RS_GEMM_TAIL_FRAC; }();
    return v;
}
static int gemm_tail_mink() {
    static const int v = [] { const char* e = getenv("RS_GEMM_TAIL_MINK"); return e ? atoi(e) : (int)RS_GEMM_TAIL_MINK; }();
    return v;
}
template <int EPI, int DIST>
static hipError_t launch_bf16(const void* a, const void* wt, const void* bias, const void* res,
                              void* out, float* partials, const void* ref, bool post, GemmLnFold ln,
                              int64_t M, int N, int K, hipStream_t s) {
    const GemmArgs g{(const bf16raw*)a, (const bf16raw*)wt, (const bf16raw*)bias, (const bf16raw*)res,
                     (const bf16raw*)ref, (bf16raw*)out, partials, post ? 1 : 0, ln, M, N, K};
    const int variant = gemm_variant();
    if (variant == 1) launch_persistent<EPI, DIST>(g, s);
    else if (variant == 2) launch_ring<256, 128, EPI, DIST>(g, s);
    else if (variant == 3) launch_ring<128, 128, EPI, DIST>(g, s);
    else if (variant == 4) launch_ring<128, 256, EPI, DIST>(g, s);
    else {
        const int cus = device_cus();
        const int64_t tiles_n = (N + 255) / 256, panels = (M + 255) / 256;
        const int64_t tiles = panels * tiles_n, rounds = tiles / cus, rem = tiles - rounds * cus;
        const bool small = 2 * tiles <= cus || (K <= 512 && 2 * tiles <= 3 * cus);
        if (small) launch_ring_auto<EPI, DIST>(g, s);
        else if (rounds == 0) launch_persistent<EPI, DIST>(g, s);
        else if (rem == 0 || K < gemm_tail_mink() || (double)rem > gemm_tail_frac() * cus) launch_persistent<EPI, DIST>(g, s);
        else {
            const int64_t m1 = (rounds * cus / tiles_n) * 256;  // row panels that fill whole rounds
            launch_persistent<EPI, DIST>(g.rows(0, m1), s);
            launch_ring_auto<EPI, DIST>(g.rows(m1, M), s);
        }
    }
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
                                                       float* __restrict__ partials,
                                                       const float* __restrict__ ref, int post, int M,
                                                       int N, int K, int slots) {
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
                if (EPI == EPI_BIAS_RES_SHIFT && m_ok) {
                    float fi[4] = {r[0], r[1], r[2], r[3]};
                    if (ref) {
                        float4 q = *reinterpret_cast<const float4*>(ref + (int64_t)m * N + n);
                        fi[0] = q.x; fi[1] = q.y; fi[2] = q.z; fi[3] = q.w;
                    }
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float fo = post ? v[e] + r[e] : v[e];
                        if (DIST == RS_DIST_L2) { float d = fo - fi[e]; p0 += d * d; }
                        else if (DIST == RS_DIST_L1) { p0 += fabsf(fo - fi[e]); }
                        else { p0 += fo * fi[e]; p1 += fo * fo; p2 += fi[e] * fi[e]; }
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
                             void* out, float* partials, const void* ref, bool post, int64_t M, int N,
                             int K, hipStream_t s) {
    dim3 grid((N + 63) / 64, (unsigned)((M + 63) / 64));
    hipLaunchKernelGGL((gemm_f32_kernel<EPI, DIST>), grid, dim3(256), 0, s, (const float*)a,
                       (const float*)w, (const float*)bias, (const float*)res, (float*)out, partials,
                       (const float*)ref, post ? 1 : 0, (int)M, N, K, (N + 63) / 64);
    return hipGetLastError();
}

#define RS_STR2(...) #__VA_ARGS__
#define RS_STR(...) RS_STR2(__VA_ARGS__)
const char* gemm_build_info() {
    return "bf16 gemm: persistent tiles (BM,BN,BK,stages,waves m,waves n) " RS_STR(RS_GEMM_CFG)
           ", three activation stages when K >= 2048"
           "; ring tiles 128x256x32 and 128x128x32, 3 stages, 4 waves, 2 workgroups per CU, up to 0.5 rounds (1.5 if K <= 512)"
           "; rows behind whole rounds go to a ring kernel when K >= " RS_STR(RS_GEMM_TAIL_MINK) " and the last round is under " RS_STR(RS_GEMM_TAIL_FRAC) " full";
}

// `count` independent products out_p[M, N] = a_p[M, K] @ wt_p[N, K]^T (bf16, no bias), problem p at
// element offsets p * stride from the base pointers; 128 x 128 tiles, grid.y = problem.
hipError_t launch_gemm_batched(const void* a, const void* wt, void* out, int count, int64_t stride_a,
                               int64_t stride_w, int64_t stride_out, int M, int N, int K, hipStream_t s) {
    if (count == 0 || M == 0) return hipSuccess;
    const GemmBatch gb{stride_a, stride_w, stride_out};
    if (N <= 64) {  // one 64-wide wave column: 256 x 64 tiles, four waves along the rows
        const int tiles_m = (M + 255) / 256;
        hipLaunchKernelGGL((gemm_bf16_ring_kernel<256, 64, 4, 1, EPI_BIAS, 0>), dim3(8 * ((tiles_m + 7) / 8), count), dim3(256), 0, s,
                           (const bf16raw*)a, (const bf16raw*)wt, (const bf16raw*)nullptr, (const bf16raw*)nullptr,
                           (bf16raw*)out, (float*)nullptr, (const bf16raw*)nullptr, 0, GemmLnFold{}, M, N, K, tiles_m, 1,
                           1, RS_GEMM_GM, gb);
    } else {
        const int tiles_m = (M + 127) / 128, tiles_n = (N + 127) / 128;
        const int nblk = tiles_m * tiles_n;
        hipLaunchKernelGGL((gemm_bf16_ring_kernel<128, 128, 2, 2, EPI_BIAS, 0>), dim3(8 * ((nblk + 7) / 8), count), dim3(256), 0, s,
                           (const bf16raw*)a, (const bf16raw*)wt, (const bf16raw*)nullptr, (const bf16raw*)nullptr,
                           (bf16raw*)out, (float*)nullptr, (const bf16raw*)nullptr, 0, GemmLnFold{}, M, N, K, tiles_m,
                           tiles_n, (N + 63) / 64, RS_GEMM_GM, gb);
    }
    return hipGetLastError();
}

int gemm_shift_slots(rs_dtype dt, int N) {
    if (dt == RS_F32) return (N + 63) / 64;
    return (N + 63) / 64;  // one slot per 64 features, whatever the tile variant
}

template <int EPI, int DIST>
static hipError_t launch_any(rs_dtype dt, const void* a, const void* w, const void* bias,
                             const void* res, void* out, float* partials, const void* ref, bool post,
                             int64_t M, int N, int K, hipStream_t s) {
    return dt == RS_F32 ? launch_f32<EPI, DIST>(a, w, bias, res, out, partials, ref, post, M, N, K, s)
                        : launch_bf16<EPI, DIST>(a, w, bias, res, out, partials, ref, post, GemmLnFold{}, M, N, K, s);
}

hipError_t launch_gemm(rs_dtype dt, GemmEpilogue epi, rs_dist dist, const void* a, const void* w,
                       const void* bias, const void* res, void* out, float* partials, const void* ref,
                       bool post, int64_t M, int N, int K, hipStream_t s) {
    if (M == 0) return hipSuccess;
    switch (epi) {
        case EPI_BIAS: return launch_any<EPI_BIAS, 0>(dt, a, w, bias, res, out, partials, ref, post, M, N, K, s);
        case EPI_BIAS_GELU: return launch_any<EPI_BIAS_GELU, 0>(dt, a, w, bias, res, out, partials, ref, post, M, N, K, s);
        case EPI_BIAS_RES: return launch_any<EPI_BIAS_RES, 0>(dt, a, w, bias, res, out, partials, ref, post, M, N, K, s);
        case EPI_BIAS_RES_SHIFT:
            if (dist == RS_DIST_L2) return launch_any<EPI_BIAS_RES_SHIFT, RS_DIST_L2>(dt, a, w, bias, res, out, partials, ref, post, M, N, K, s);
            if (dist == RS_DIST_L1) return launch_any<EPI_BIAS_RES_SHIFT, RS_DIST_L1>(dt, a, w, bias, res, out, partials, ref, post, M, N, K, s);
            return launch_any<EPI_BIAS_RES_SHIFT, RS_DIST_COS>(dt, a, w, bias, res, out, partials, ref, post, M, N, K, s);
        default: break;  // the LayerNorm-folded epilogues go through launch_gemm_ln
    }
    return hipErrorInvalidValue;
}

hipError_t launch_gemm_ln(GemmEpilogue epi, const void* x, const void* w_folded, GemmLnFold ln, void* out,
                          int64_t M, int N, int K, hipStream_t s) {
    if (M == 0) return hipSuccess;
    if (epi == EPI_LN_BIAS)
        return launch_bf16<EPI_LN_BIAS, 0>(x, w_folded, nullptr, nullptr, out, nullptr, nullptr, false, ln, M, N, K, s);
    if (epi == EPI_LN_BIAS_GELU)
        return launch_bf16<EPI_LN_BIAS_GELU, 0>(x, w_folded, nullptr, nullptr, out, nullptr, nullptr, false, ln, M, N, K, s);
    return hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------
// Weight re-layout for the bf16 path: [K, N] row-major -> [N, K] row-major, optionally with
// row k scaled by gamma[k] (a LayerNorm scale folded into the weights; the product is rounded
// to bf16).  64 x 64 tiles through LDS, coalesced on both sides.
// ---------------------------------------------------------------------------
__device__ __forceinline__ bf16raw fold_gamma(bf16raw w, const bf16raw* gamma, int k) {
    return gamma ? f2bf(bf2f(gamma[k]) * bf2f(w)) : w;
}

__global__ __launch_bounds__(256) void transpose_bf16_kernel(const bf16raw* __restrict__ w,
                                                             const bf16raw* __restrict__ gamma,
                                                             bf16raw* __restrict__ wt, int K, int N) {
    __shared__ bf16raw tile[64][66];
    const int k0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int r = ty; r < 64; r += 4) {
        const int k = k0 + r, n = n0 + tx;
        tile[r][tx] = (k < K && n < N) ? fold_gamma(w[(int64_t)k * N + n], gamma, k) : (bf16raw)0;
    }
    __syncthreads();
    for (int r = ty; r < 64; r += 4) {
        const int n = n0 + r, k = k0 + tx;
        if (n < N && k < K) wt[(int64_t)n * K + k] = tile[tx][r];
    }
}

hipError_t launch_pack_transpose(const void* w, const void* gamma, void* wt, int K, int N, hipStream_t s) {
    dim3 grid((N + 63) / 64, (K + 63) / 64);
    hipLaunchKernelGGL(transpose_bf16_kernel, grid, dim3(256), 0, s, (const bf16raw*)w, (const bf16raw*)gamma,
                       (bf16raw*)wt, K, N);
    return hipGetLastError();
}

// Column vectors of a LayerNorm folded into the linear layer behind it:
//   colsum[n] = sum_k bf16(gamma_k w_kn)   -- over exactly the values transpose_bf16_kernel stores,
//                                             so that mean * colsum cancels the mean's share of acc
//   bias_out[n] = sum_k beta_k w_kn + bias[n]
// One thread per column, 4 row groups per workgroup reduced through LDS; fp64 sums (one-off work).
__global__ __launch_bounds__(256) void ln_fold_kernel(const bf16raw* __restrict__ w, const bf16raw* __restrict__ gamma,
                                                      const bf16raw* __restrict__ beta, const bf16raw* __restrict__ bias,
                                                      float* __restrict__ colsum, float* __restrict__ bias_out,
                                                      int K, int N) {
    __shared__ double s_cs[4][64], s_bb[4][64];
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int n = blockIdx.x * 64 + tx;
    double cs = 0.0, bb = 0.0;
    if (n < N)
        for (int k = ty; k < K; k += 4) {
            const bf16raw wv = w[(int64_t)k * N + n];
            cs += (double)bf2f(fold_gamma(wv, gamma, k));
            if (beta) bb += (double)bf2f(beta[k]) * (double)bf2f(wv);
        }
    s_cs[ty][tx] = cs;
    s_bb[ty][tx] = bb;
    __syncthreads();
    if (ty == 0 && n < N) {
        cs = ((s_cs[0][tx] + s_cs[1][tx]) + s_cs[2][tx]) + s_cs[3][tx];
        bb = ((s_bb[0][tx] + s_bb[1][tx]) + s_bb[2][tx]) + s_bb[3][tx];
        if (bias) bb += (double)bf2f(bias[n]);
        colsum[n] = (float)cs;
        bias_out[n] = (float)bb;
    }
}

hipError_t launch_pack_ln_fold(const void* w, const void* gamma, const void* beta, const void* bias,
                               float* colsum, float* bias_out, int K, int N, hipStream_t s) {
    hipLaunchKernelGGL(ln_fold_kernel, dim3((N + 63) / 64), dim3(256), 0, s, (const bf16raw*)w,
                       (const bf16raw*)gamma, (const bf16raw*)beta, (const bf16raw*)bias, colsum, bias_out, K, N);
    return hipGetLastError();
}

}  // namespace rs
