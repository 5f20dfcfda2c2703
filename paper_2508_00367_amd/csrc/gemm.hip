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
// A ring of NSTAGE LDS stages of (BM + BN) rows x 2*BK bytes: K slices stream from global
// memory directly into LDS (buffer_load ... lds, no register staging), NSTAGE-1 slices ahead of
// the one the matrix cores work on.  Loads return in order, so "slice t has landed" is
// s_waitcnt vmcnt(<loads issued after it>); one workgroup barrier per slice.  The slice count is
// padded to a multiple of NSTAGE with copies aimed past the end of the buffer resource (they
// deliver zeros), which keeps the loop free of tail branches.  Operand fragments are double
// buffered in registers and each LDS read is interleaved with its share of the previous K step's
// MFMAs (sched_group_barrier).  One workgroup per CU; the register budget is that of NW / 4 waves
// per SIMD.
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
    static_assert(NSTAGE == 2, "two stages (deeper rings of narrower slices measured no better)");

    // Epilogue staging: 32 fp32 rows of the wave tile + the wave's row statistics per wave.  It lives
    // in the array of stage 1, which is made large enough for all waves: stage 0 receives the next
    // tile's first K slice meanwhile, and being a different array the compiler knows that the
    // epilogue's LDS traffic need not wait for those copies.
    constexpr int EPW = (32 * (WN * 4 + 16) + WM * 8 + 255) / 256 * 256;  // bytes per wave
    __shared__ __attribute__((aligned(1024))) unsigned char stage0[STAGE];
    __shared__ __attribute__((aligned(1024))) unsigned char stage1[STAGE > NW * EPW ? STAGE : NW * EPW];

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
    //   128-byte rows (BK 64): f(r) = (r ^ (r >> 3)) & 7   (row parity picks the half line, the XOR
    //                          makes rows r and r + 8 differ; measured 0 SQ_LDS_BANK_CONFLICT,
    //                          against every second cycle with the plain r & 7)
    //    64-byte rows (BK 32): f(r) = (r >> 2) & 3         (r & 3 picks the quarter line)
    // global -> LDS: wave copy i of wave w fills rows (NW*i + w)*RPI .. +RPI-1 (lane l: row l / SPR,
    // slot l % SPR), so the lane fetches chunk (l % SPR) ^ f(row).
    __amdgpu_buffer_rsrc_t rs_a = make_rsrc(a + (int64_t)m0 * K, (int64_t)min(M - m0, BM) * K * 2);
    __amdgpu_buffer_rsrc_t rs_w = make_rsrc(wt + (int64_t)n0 * K, (int64_t)min(N - n0, BN) * K * 2);
    const int ld_r = lane / SPR, ld_p = lane % SPR;
    int voff_e, voff_o;  // lane byte offset for even / odd copy index i
    if (SPR == 8) {  // row >> 3 = NW*i + w
        voff_e = ((wave * RPI + ld_r) * K + ((ld_p ^ ld_r ^ (wave & 7)) << 3)) * 2;
        voff_o = ((wave * RPI + ld_r) * K + ((ld_p ^ ld_r ^ ((wave + NW) & 7)) << 3)) * 2;
    } else {
        voff_e = voff_o = ((wave * RPI + ld_r) * K + ((ld_p ^ ((ld_r >> 2) & 3)) << 3)) * 2;
    }
    const int pass_bytes = NW * RPI * K * 2;

    const int S = K / BK;                                   // real slices
    const int S_pad = (S + NSTAGE - 1) / NSTAGE * NSTAGE;   // loop trip count (zero slices at the end)
    const int a_row0 = wm * WM + l32, w_row0 = wn * WN + l32;
    // slot XOR of operand row 32*t + l32 (t = MFMA tile index inside the wave tile)
    const int sw_e = SPR == 8 ? ((l32 ^ (l32 >> 3)) & 7) : ((l32 >> 2) & 3);
    const int sw_o = SPR == 8 ? (sw_e ^ 4) : sw_e;

// copies of K slice t_ into stage_; slices past the end are aimed beyond the resource (which covers
// this tile's rows only, so the aim is past its end whatever the size of the whole matrix)
#define RS_GEMM_DMA(stage_, t_)                                                                           \
    {                                                                                                     \
        const bool real_ = (t_) < S;                                                                      \
        const int kb_ = (t_) * RB;                                                                        \
        _Pragma("unroll") for (int i = 0; i < A_LOADS; ++i)                                               \
            dma16(rs_a, (stage_) + (i * NW + wave) * 1024, (i & 1) ? voff_o : voff_e, real_ ? i * pass_bytes + kb_ : kPastEnd); \
        _Pragma("unroll") for (int i = 0; i < W_LOADS; ++i)                                               \
            dma16(rs_w, (stage_) + BM * RB + (i * NW + wave) * 1024, (i & 1) ? voff_o : voff_e, real_ ? i * pass_bytes + kb_ : kPastEnd); \
    }
#define RS_GEMM_LOAD_FRAGS(f_, stage_, kk_)                                                               \
    {                                                                                                     \
        const int ce_ = ((((kk_) * 2 + g) ^ sw_e) << 4), co_ = ((((kk_) * 2 + g) ^ sw_o) << 4);           \
        _Pragma("unroll") for (int i = 0; i < TN; ++i)                                                    \
            (f_).w[i] = *reinterpret_cast<const bf16x8*>((stage_) + (BM + w_row0 + i * 32) * RB + ((i & 1) ? co_ : ce_)); \
        _Pragma("unroll") for (int j = 0; j < TM; ++j)                                                    \
            (f_).a[j] = *reinterpret_cast<const bf16x8*>((stage_) + (a_row0 + j * 32) * RB + ((j & 1) ? co_ : ce_)); \
    }
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

    static_assert(NSTAGE == 2 && KK == 4, "the slice schedule below is written for two stages of 64-wide slices");
    RS_GEMM_DMA(stage0, 0)  // first K slice of the first tile

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
    RS_GEMM_DMA(stage1, 1)
    RS_GEMM_LOAD_FRAGS(f0, stage0, 0)
    __builtin_amdgcn_sched_barrier(0);
    for (int t = 0; t < S_pad; t += 2) {
        RS_GEMM_SLICE(stage0, stage1, t)
        RS_GEMM_SLICE(stage1, stage0, t + 1)
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
        unsigned char* ep = stage1 + wave * EPW;
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
#pragma unroll
        for (int j = 0; j < TM; ++j) {
            // the residual rows of this 32-row group: issued before the staging round trip
            constexpr bool RES = EPI == EPI_BIAS_RES || EPI == EPI_BIAS_RES_SHIFT;
            uint4 res_raw[RES ? 32 / RPS : 1];
            if (RES) {
#pragma unroll
                for (int st = 0; st < 32 / RPS; ++st) {
                    const int m = m0_cur + wm * WM + j * 32 + st * RPS + orow;
                    res_raw[st] = (m < M && n_ok) ? *reinterpret_cast<const uint4*>(res + (int64_t)m * N + n)
                                                  : make_uint4(0u, 0u, 0u, 0u);
                }
            }
            if (j == 0) RS_GEMM_DMA(stage0, more ? 0 : S)
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
                            if (DIST == RS_DIST_L2) { float d = fo - fi[e]; p0 += d * d; }
                            else if (DIST == RS_DIST_L1) { p0 += fabsf(fo - fi[e]); }
                            else { p0 += fo * fi[e]; p1 += fo * fo; p2 += fi[e] * fi[e]; }
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
                    if ((lane % LPR) == 0 && m < M) {
                        const int slot = (n0_cur + wn * WN) / WN;
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
#undef RS_GEMM_DECODE
#undef RS_GEMM_LOAD_FRAGS
#undef RS_GEMM_MFMA
#undef RS_GEMM_INTERLEAVE
#undef RS_GEMM_SLICE
}

// Tile configuration of the bf16 GEMM: BM, BN, BK, NSTAGE, waves along tokens, waves along features.
struct GemmCfg {
#ifndef RS_GEMM_CFG
#define RS_GEMM_CFG 256, 256, 64, 2, 2, 4
#endif
    static constexpr int P[6] = {RS_GEMM_CFG};
    static constexpr int BM = P[0], BN = P[1], BK = P[2], NSTAGE = P[3], WGM = P[4], WGN = P[5];
    static constexpr int WN = BN / WGN;
};

template <int EPI, int DIST>
static hipError_t launch_bf16(const void* a, const void* wt, const void* bias, const void* res,
                              void* out, float* partials, const void* ref, bool post, GemmLnFold ln,
                              int64_t M, int N, int K, hipStream_t s) {
    using C = GemmCfg;
    const int tiles_m = (int)((M + C::BM - 1) / C::BM), tiles_n = (N + C::BN - 1) / C::BN;
    const int slots = (tiles_n * C::BN) / C::WN;
#ifndef RS_GEMM_GM
#define RS_GEMM_GM 8
#endif
    const int gm = RS_GEMM_GM;  // row panels per tile group: their activations stay in an XCD's L2 during a sweep over n
    // one workgroup per CU (8 XCDs x CUs / 8), fewer when an XCD's share of the tiles is smaller
    static const int cus = [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 8) n = 256;
        return n;
    }();
    const int share = (tiles_m * tiles_n + 7) / 8;
    const int per_xcd = share < cus / 8 ? share : cus / 8;
    hipLaunchKernelGGL((gemm_bf16_kernel<C::BM, C::BN, C::BK, C::NSTAGE, C::WGM, C::WGN, EPI, DIST>),
                       dim3(8 * per_xcd), dim3(C::WGM * C::WGN * 64), 0, s, (const bf16raw*)a,
                       (const bf16raw*)wt, (const bf16raw*)bias, (const bf16raw*)res, (bf16raw*)out, partials,
                       (const bf16raw*)ref, post ? 1 : 0, ln, (int)M, N, K, tiles_m, tiles_n, slots, gm);
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
const char* gemm_build_info() { return "bf16 gemm tiles (BM,BN,BK,stages,waves m,waves n): " RS_STR(RS_GEMM_CFG); }

int gemm_shift_slots(rs_dtype dt, int N) {
    if (dt == RS_F32) return (N + 63) / 64;
    return ((N + GemmCfg::BN - 1) / GemmCfg::BN) * GemmCfg::BN / GemmCfg::WN;
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
