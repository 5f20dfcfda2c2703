// Fused multi-head self-attention, Eq. (1) of Sec. 3.1:  O = Softmax(Q K^T * scale) V
// per (image, head), head width 64.  The N x N attention map is never stored: K/V
// stream through LDS in tiles of 64 keys while each wavefront keeps a running row
// maximum, row sum and output accumulator in registers (online softmax).
//
// bf16 path (v_mfma_f32_32x32x16_bf16).  Everything is computed transposed so that the
// softmax state of a query row lives in ONE lane:
//     S^T = K Q^T     A operand = K rows from LDS, B operand = Q rows held in registers;
//                     accumulator: lane (q = lane%32, g = lane/32) holds, for its query q,
//                     keys 8j + 4g + i  (register 4j + i)  of each 32-key block.
//     O^T = V^T P^T   B operand = P taken straight from the S^T accumulator registers
//                     (8 registers = the lane's 8 keys of a 16-key group), A operand = V^T.
//                     V sits in LDS as it sits in memory, one row per key; the transposing
//                     LDS read of gfx950 (ds_read_b64_tr_b16) hands a lane one channel at 4
//                     keys, and two of them fetch the 8 keys in the order the accumulator
//                     layout yields them (slot 4u + i  <->  key 8u + 4g + i of the group).
// Row max / row sum need one exchange between the two half-waves per tile.
//
// fp32 path: one query row per thread, true fp32 products (parity configuration).
#include "common.hpp"

namespace rs {

constexpr int ATT_BM = 256;  // query rows per workgroup (8 waves x 32)
constexpr int ATT_BN = 64;   // keys per tile
constexpr int DH = 64;

// 16-byte chunk `c` (0..7) of 128-byte LDS row `r` of a K tile; the XOR spreads the 16-lane
// operand reads over the 64 banks.
__device__ __forceinline__ int att_swz(int r, int c) { return r * 128 + (((c ^ r ^ (r >> 3)) & 7) << 4); }

typedef __attribute__((address_space(3))) void* att_lds_ptr;
typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) v4i16* lds_v4i16;

// Row-major V tile [64 keys][128 B]: 16-byte chunk c of key row r sits in slot c ^ att_vswz(r).  A
// transposing read touches 4 consecutive key rows x 64 bytes per 32 lanes; flipping the 64-byte
// half on every second pair of rows keeps those four rows on different banks.
__device__ __forceinline__ int att_vswz(int r) { return ((r >> 1) & 1) << 2; }

// One block of 32 query rows against one resident tile of 64 keys: S^T = K Q^T, online softmax
// in registers (one lane = one query row, half of the tile's keys), O^T += V^T P^T.
// `sk`: K tile [64 keys][128 B] (att_swz); `sv`: V tile [64 keys][128 B] (att_vswz).
template <bool MASK>
__device__ __forceinline__ void att_tile(const unsigned char* sk, const unsigned char* sv,
                                         const bf16x8 (&qf)[4], f32x16 (&oacc)[2], float& m_run,
                                         float& l_run, int key0, int N, float scale_log2e, int l32, int g) {
    // In the padded last tile only the 32-key blocks and 16-key groups that hold real keys are
    // worked on (wave-uniform conditions): N = 197 leaves 5 keys in its fourth tile.
    const int valid = MASK ? N - key0 : ATT_BN;  // real keys in this tile, 1 .. 64
    f32x16 sacc[2];
#pragma unroll
    for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[kb2][r] = 0.f;
    if (!MASK || valid > 32) {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
#pragma unroll
            for (int kb2 = 0; kb2 < 2; ++kb2) {  // independent accumulator chains alternate
                const bf16x8 kf = *reinterpret_cast<const bf16x8*>(sk + att_swz(kb2 * 32 + l32, kk * 2 + g));
                sacc[kb2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], sacc[kb2], 0, 0, 0);
            }
    } else {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const bf16x8 kf = *reinterpret_cast<const bf16x8*>(sk + att_swz(l32, kk * 2 + g));
            sacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], sacc[0], 0, 0, 0);
        }
    }
    if (MASK) {  // keys past the end
#pragma unroll
        for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = key0 + kb2 * 32 + (r >> 2) * 8 + g * 4 + (r & 3);
                if (key >= N) sacc[kb2][r] = -INFINITY;
            }
    }
    float mx = fmaxf(sacc[0][0], sacc[1][0]);
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(fmaxf(mx, sacc[0][r]), sacc[1][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);  // finite: every tile holds at least one real key
    const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * scale_log2e);
    const float mb = m_new * scale_log2e;
    m_run = m_new;
    if (!MASK || valid > 32) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            sacc[0][r] = __builtin_amdgcn_exp2f(fmaf(sacc[0][r], scale_log2e, -mb));
            sacc[1][r] = __builtin_amdgcn_exp2f(fmaf(sacc[1][r], scale_log2e, -mb));
        }
    } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[0][r] = __builtin_amdgcn_exp2f(fmaf(sacc[0][r], scale_log2e, -mb));
    }
    if (__ballot(alpha != 1.0f)) {  // the running maximum moved for some row of this block
        // in-place multiplies: with plain C++ the compiler renames the 32 accumulators on this
        // rarely taken path and pays 32 register copies on EVERY tile to merge the two paths
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float t = oacc[i][r];
                asm volatile("v_mul_f32 %0, %0, %1" : "+v"(t) : "v"(alpha));
                oacc[i][r] = t;
            }
    }
    // P goes to bf16 once; the row sum is taken over the same rounded values (v_dot2 with ones)
    float psum = 0.f;
    const bf16x2 ones = __builtin_bit_cast(bf16x2, 0x3f803f80u);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        if (MASK && 16 * t >= valid) break;  // groups of padding keys only: P = 0
        const int kb2 = t >> 1, r0 = (t & 1) * 8;
        union { uint32_t u[4]; bf16x8 v; } pf;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            pf.u[e] = pack2bf(sacc[kb2][r0 + 2 * e], sacc[kb2][r0 + 2 * e + 1]);
            psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pf.u[e]), ones, psum, false);
        }
#pragma unroll
        for (int db = 0; db < 2; ++db) {
            // V tile as it sits in memory, [64 keys][64 channels]: two transposing LDS reads
            // (ds_read_b64_tr_b16) hand this lane its channel's values at 4 keys each.  Within a
            // group of 16 lanes, lane s = 4 j + a points at key j, channels 4 a .. 4 a + 3, and
            // lane L receives channel L of keys j = 0 .. 3.  The keys are taken in the order of
            // the P operand: slot 4 u + j of this lane is key 16 t + 8 u + 4 g + j.
            const int s16 = l32 & 15;
            const int chunk = db * 4 + 2 * (l32 >> 4) + ((s16 & 3) >> 1);
            union { v4i16 h[2]; bf16x8 v; } tr;
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int key = 16 * t + 8 * u + 4 * g + (s16 >> 2);
                tr.h[u] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (lds_v4i16)(sv + key * 128 + ((chunk ^ att_vswz(key)) << 4) + (s16 & 1) * 8));
            }
            oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tr.v, pf.v, oacc[db], 0, 0, 0);
        }
    }
    l_run = l_run * alpha + psum;
}

// Long sequences: workgroup = 256 query rows (8 waves x 32 rows) of one (image, head); two
// workgroups share a CU (at most 128 registers), four waves per SIMD.  K and V tiles stream
// global -> LDS directly (buffer_load ... lds, rows past N read as zero through the buffer
// resource).  Two stages each; the copies of tile t+1 are issued before the MFMAs of tile t, one barrier per tile.
__global__ __launch_bounds__(512, 4) void attention_bf16_kernel(
    const bf16raw* __restrict__ q, const bf16raw* __restrict__ k, const bf16raw* __restrict__ v,
    bf16raw* __restrict__ o, int N, int64_t sb, int64_t sn, int64_t sh, int64_t osb, int64_t osn,
    int64_t osh, float scale_log2e, int H, int BH, int q_tiles) {
    __shared__ __attribute__((aligned(1024))) unsigned char sk0[ATT_BN * 128];
    __shared__ __attribute__((aligned(1024))) unsigned char sk1[ATT_BN * 128];
    __shared__ __attribute__((aligned(16))) unsigned char sv0[DH * 128];
    __shared__ __attribute__((aligned(16))) unsigned char sv1[DH * 128];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, g = lane >> 5;
    // Workgroup ids go round-robin to the 8 XCDs; all query tiles of one (image, head) are given
    // to the same XCD so that its K/V tiles are fetched into that XCD's L2 once and hit afterwards.
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int head = xcd + 8 * (local / q_tiles);
    if (head >= BH) return;  // whole workgroup, before any barrier
    const int b = head / H, h = head - b * H;
    const int q0 = (local % q_tiles) * ATT_BM + wave * 32;
    const int64_t base = (int64_t)b * sb + (int64_t)h * sh;

    // Q fragments: B operand, column = query row q0 + l32, k-slots = 8 channels 16*kk + 8*g ..
    bf16x8 qf[4];
    {
        int qr = q0 + l32;
        qr = qr < N ? qr : N - 1;  // rows past the end are computed on a copy and never stored
        const bf16raw* qp = q + base + (int64_t)qr * sn;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) qf[kk] = *reinterpret_cast<const bf16x8*>(qp + kk * 16 + g * 8);
    }

    // K copies: wave w fills LDS rows 8w .. 8w+7 of the tile (lane l: row l/8, slot l%8 holds
    // chunk (l%8) ^ f(row)); the resource ends with key N-1, so later rows arrive as zeros.
    const int64_t k_bytes = ((int64_t)(N - 1) * sn + DH) * 2;
    const __amdgpu_buffer_rsrc_t rs_k = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16raw*>(k + base), 0, (int)(k_bytes < 0xffffffffll ? k_bytes : 0xffffffffll), 0x00020000);
    const int k_lr = lane >> 3;
    const int k_voff = (int)(((int64_t)(wave * 8 + k_lr) * sn + (((lane & 7) ^ k_lr ^ wave) << 3)) * 2);
    const int k_tile_bytes = (int)(ATT_BN * sn * 2);

    // V copies: the same rows and lanes as K, chunk (l%8) ^ att_vswz(row) in slot l%8.
    const __amdgpu_buffer_rsrc_t rs_v = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16raw*>(v + base), 0, (int)(k_bytes < 0xffffffffll ? k_bytes : 0xffffffffll), 0x00020000);
    const int v_voff = (int)(((int64_t)(wave * 8 + k_lr) * sn + (((lane & 7) ^ att_vswz(k_lr)) << 3)) * 2);

#define ATT_LOAD_NEXT(SKn, SVn, kt_)                                                                     \
    {                                                                                                    \
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_k, (att_lds_ptr)((SKn) + wave * 1024), 16, k_voff,    \
                                                 (kt_) * k_tile_bytes, 0, 0);                            \
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_v, (att_lds_ptr)((SVn) + wave * 1024), 16, v_voff,    \
                                                 (kt_) * k_tile_bytes, 0, 0);                            \
    }
// tile kt_ is resident in (SKc, SVc); tile kt_+1 is fetched into (SKn, SVn) meanwhile
#define ATT_STEP(SKc, SVc, SKn, SVn, kt_, MASK_)                                                              \
    {                                                                                                    \
        ATT_LOAD_NEXT(SKn, SVn, (kt_) + 1)                                                               \
        if (active)                                                                                      \
            att_tile<MASK_>(SKc, SVc, qf, oacc, m_run, l_run, (kt_) * ATT_BN, N, scale_log2e, l32, g);   \
        __builtin_amdgcn_s_waitcnt(0x0F70); /* this wave's K and V copies have landed */                 \
        __syncthreads();                                                                                 \
    }

    f32x16 oacc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[i][r] = 0.f;
    float m_run = -INFINITY;  // running max of the raw logits of this lane's query row
    float l_run = 0.f;        // this lane's share of the running row sum

    // A wave whose query rows all lie past N (last query tile of a head) copies its share of the
    // K/V tiles and meets the barriers but computes nothing: the wave it shares a SIMD with then
    // has that SIMD to itself.
    const bool active = q0 < N;
    const int KT = (N + ATT_BN - 1) / ATT_BN;
    ATT_LOAD_NEXT(sk0, sv0, 0)
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    const int KF = N / ATT_BN;  // tiles without padding keys
    int kt = 0;
    for (; kt + 2 <= KF; kt += 2) {
        ATT_STEP(sk0, sv0, sk1, sv1, kt, false)
        ATT_STEP(sk1, sv1, sk0, sv0, kt + 1, false)
    }
    if (kt < KT) {  // one or two tiles left, the last one possibly padded
        ATT_STEP(sk0, sv0, sk1, sv1, kt, true)
        if (kt + 1 < KT) ATT_STEP(sk1, sv1, sk0, sv0, kt + 1, true)
    }
#undef ATT_LOAD_NEXT
#undef ATT_STEP

    // ---- normalise and store: lane holds O[q][db*32 + 8j + 4g + i] in oacc[db][4j + i]
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    const float inv = 1.0f / l_tot;
    const int qr = q0 + l32;
    if (qr < N) {
        bf16raw* op = o + (int64_t)b * osb + (int64_t)qr * osn + (int64_t)h * osh;
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint2 w;
                w.x = pack2bf(oacc[db][4 * j] * inv, oacc[db][4 * j + 1] * inv);
                w.y = pack2bf(oacc[db][4 * j + 2] * inv, oacc[db][4 * j + 3] * inv);
                *reinterpret_cast<uint2*>(op + db * 32 + j * 8 + g * 4) = w;
            }
    }
}

// ---------------------------------------------------------------------------
// Last rows of a long sequence.  When N leaves a few rows (at most 64) beyond the last full
// query tile, a whole workgroup of the kernel above would stream every K/V tile for them with
// one or two of its eight waves working.  Here one workgroup per (image, head) takes those rows
// and its eight waves split the KEY tiles instead (wave w: tiles w, w + 8, ...), each with its
// own K / V tile in LDS and no workgroup barrier inside the loop; the eight partial results
// (running maximum, row sum, unnormalised output) are merged through LDS in wave order, so the
// result does not depend on timing.
// ---------------------------------------------------------------------------
constexpr int ATT_TAIL_ROWS = 64;

__global__ __launch_bounds__(512, 2) void attention_bf16_tail_kernel(
    const bf16raw* __restrict__ q, const bf16raw* __restrict__ k, const bf16raw* __restrict__ v,
    bf16raw* __restrict__ o, int N, int64_t sb, int64_t sn, int64_t sh, int64_t osb, int64_t osn,
    int64_t osh, float scale_log2e, int H, int q_begin) {
    // per wave: K tile (8 KB) + V tile (8 KB); after the loop the same 16 KB hold the wave's
    // output partial [2 blocks][32 rows][64 channels] fp32
    __shared__ __attribute__((aligned(1024))) unsigned char s_tiles[8][16384];
    __shared__ float s_m[8][2][32];
    __shared__ float s_l[8][2][32];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, g = lane >> 5;
    const int b = blockIdx.x / H, h = blockIdx.x - b * H;
    const int64_t base = (int64_t)b * sb + (int64_t)h * sh;
    unsigned char* sk = s_tiles[wave];
    unsigned char* svt = sk + ATT_BN * 128;

    bf16x8 qf[2][4];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        int qr = q_begin + qb * 32 + l32;
        qr = qr < N ? qr : N - 1;  // rows past the end are computed on a copy and never stored
        const bf16raw* qp = q + base + (int64_t)qr * sn;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) qf[qb][kk] = *reinterpret_cast<const bf16x8*>(qp + kk * 16 + g * 8);
    }
    const int64_t k_bytes = ((int64_t)(N - 1) * sn + DH) * 2;
    const __amdgpu_buffer_rsrc_t rs_k = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16raw*>(k + base), 0, (int)(k_bytes < 0xffffffffll ? k_bytes : 0xffffffffll), 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_v = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16raw*>(v + base), 0, (int)(k_bytes < 0xffffffffll ? k_bytes : 0xffffffffll), 0x00020000);
    const int k_lr = lane >> 3;
    const int k_tile_bytes = (int)(ATT_BN * sn * 2);

    f32x16 oacc[2][2];
    float m_run[2], l_run[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[qb][i][r] = 0.f;
        m_run[qb] = -INFINITY;
        l_run[qb] = 0.f;
    }

    const bool second = N - q_begin > 32;  // rows in the second block of 32
    const int KT = (N + ATT_BN - 1) / ATT_BN;
    for (int kt = wave; kt < KT; kt += 8) {
        // K tile: copy i fills rows 8i .. 8i+7 (lane l: row l/8, slot l%8 holds chunk (l%8) ^ f(row))
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int voff = (int)(((int64_t)(i * 8 + k_lr) * sn + (((lane & 7) ^ k_lr ^ i) << 3)) * 2);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_k, (att_lds_ptr)(sk + i * 1024), 16, voff, kt * k_tile_bytes, 0, 0);
        }
        // V tile: the same rows and lanes, chunk (l%8) ^ att_vswz(row) in slot l%8
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int voff = (int)(((int64_t)(i * 8 + k_lr) * sn + (((lane & 7) ^ att_vswz(k_lr)) << 3)) * 2);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_v, (att_lds_ptr)(svt + i * 1024), 16, voff, kt * k_tile_bytes, 0, 0);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wave's K and V copies have landed
        // one block of 32 rows at a time: fewer live registers than both at once, and LDS
        // bandwidth is not what limits this kernel
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            if (qb == 1 && !second) break;  // at most 32 rows left: the second block has none
            if (kt == KT - 1 && (N & (ATT_BN - 1)))
                att_tile<true>(sk, svt, qf[qb], oacc[qb], m_run[qb], l_run[qb], kt * ATT_BN, N, scale_log2e, l32, g);
            else
                att_tile<false>(sk, svt, qf[qb], oacc[qb], m_run[qb], l_run[qb], kt * ATT_BN, N, scale_log2e, l32, g);
        }
    }

    // ---- merge the eight partials
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const float l_tot = l_run[qb] + __shfl_xor(l_run[qb], 32, 64);
        if (g == 0) {
            s_m[wave][qb][l32] = m_run[qb];
            s_l[wave][qb][l32] = l_tot;
        }
    }
    __syncthreads();  // every wave has left its tiles: the partials may overwrite them
    float* part = reinterpret_cast<float*>(s_tiles[wave]);
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        if (qb == 1 && !second) break;  // its rows are never stored
        float m_tot = s_m[0][qb][l32];
#pragma unroll
        for (int w = 1; w < 8; ++w) m_tot = fmaxf(m_tot, s_m[w][qb][l32]);
        float L = 0.f;
#pragma unroll
        for (int w = 0; w < 8; ++w)
            L += s_l[w][qb][l32] * __builtin_amdgcn_exp2f((s_m[w][qb][l32] - m_tot) * scale_log2e);
        const float f = __builtin_amdgcn_exp2f((m_run[qb] - m_tot) * scale_log2e) / L;  // 0 for a wave without tiles
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int slot = db * 8 + 2 * j + g;  // 4 channels db*32 + 8j + 4g ..
                const f32x4 val = {oacc[qb][db][4 * j] * f, oacc[qb][db][4 * j + 1] * f,
                                   oacc[qb][db][4 * j + 2] * f, oacc[qb][db][4 * j + 3] * f};
                *reinterpret_cast<f32x4*>(part + (qb * 32 + l32) * 64 + ((slot ^ (l32 & 15)) << 2)) = val;
            }
    }
    __syncthreads();
    {
        const int r = tid >> 3, c8 = tid & 7;  // row of the 64, channels 8 c8 .. 8 c8 + 7
        float acc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = 0.f;
#pragma unroll
        for (int w = 0; w < 8; ++w) {
            const float* pw = reinterpret_cast<const float*>(s_tiles[w]) + r * 64;
            const f32x4 lo = *reinterpret_cast<const f32x4*>(pw + (((2 * c8) ^ (r & 15)) << 2));
            const f32x4 hi = *reinterpret_cast<const f32x4*>(pw + (((2 * c8 + 1) ^ (r & 15)) << 2));
#pragma unroll
            for (int e = 0; e < 4; ++e) { acc[e] += lo[e]; acc[4 + e] += hi[e]; }
        }
        const int qr = q_begin + r;
        if (qr < N) Elem<bf16raw>::store8(o + (int64_t)b * osb + (int64_t)qr * osn + (int64_t)h * osh + c8 * 8, acc);
    }
}

// ---------------------------------------------------------------------------
// Short sequences (N <= 256, every image-classification block): one workgroup of 8 waves per
// (image, head).  K and V (N x 64 each) of the head are copied into LDS once; wave w runs query
// rows 32w .. 32w+31 against all key tiles.  The copies are requested in tile order and the
// first two tiles are used as soon as they have landed, while the other two still stream in:
// two barriers in all.  Against the tiled kernel this reads K and V once instead of once per
// query tile and has no per-tile barrier; two workgroups share a CU, so one's load phase runs
// under the other's tile loop.  The tile loop itself is bound by instruction issue (plain ALU
// and matrix instructions of a SIMD's waves do not overlap), so it carries no masking work
// outside the last key tile.
// LDS: K and V rows of 128 bytes in the tiled kernel's two slot orders (att_swz, att_vswz).
// ---------------------------------------------------------------------------
constexpr int SM_MAXN = 256;

__global__ __launch_bounds__(512, 4) void attention_bf16_small_kernel(
    const bf16raw* __restrict__ q, const bf16raw* __restrict__ k, const bf16raw* __restrict__ v,
    bf16raw* __restrict__ o, int N, int64_t sb, int64_t sn, int64_t sh, int64_t osb, int64_t osn,
    int64_t osh, float scale_log2e) {
    // one array per half and operand: the compiler then knows which copies a half's LDS reads wait for
    __shared__ __attribute__((aligned(1024))) unsigned char s_ka[2 * ATT_BN * 128], s_kb[2 * ATT_BN * 128];
    __shared__ __attribute__((aligned(1024))) unsigned char s_va[2 * ATT_BN * 128], s_vb[2 * ATT_BN * 128];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, g = lane >> 5;
    const int b = blockIdx.y, h = blockIdx.x;
    const int64_t base = (int64_t)b * sb + (int64_t)h * sh;
    const int KT = (N + ATT_BN - 1) / ATT_BN;   // key tiles of 64
    const int KF = N / ATT_BN;                  // tiles without padding keys: no masking work in them

    const int q0 = wave * 32;
    // Q fragments (B operand): column = query row q0 + l32, k-slots = channels 16 kk + 8 g ..
    bf16x8 qf[4];
    {
        int qr = q0 + l32;
        qr = qr < N ? qr : N - 1;
        const bf16raw* qp = q + base + (int64_t)qr * sn;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) qf[kk] = *reinterpret_cast<const bf16x8*>(qp + kk * 16 + g * 8);
    }
    // K and V of the head go from memory straight into LDS: per tile of 64 keys, wave w copies
    // rows 8w .. 8w+7 (lane l: row l/8, 16-byte slot l%8).  Both resources end with key N-1, so
    // rows past the end arrive as zeros without touching memory: zero V rows add nothing, and
    // the padded keys' logits are masked in the last tile.  All four tiles are always requested,
    // in tile order, so that "all but the newest 2 (3 - i) copies" means "tile i has landed".
    const int64_t k_bytes = ((int64_t)(N - 1) * sn + DH) * 2;
    const __amdgpu_buffer_rsrc_t rs_k = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16raw*>(k + base), 0, (int)(k_bytes < 0xffffffffll ? k_bytes : 0xffffffffll), 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_v = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16raw*>(v + base), 0, (int)(k_bytes < 0xffffffffll ? k_bytes : 0xffffffffll), 0x00020000);
    const int k_lr = lane >> 3;
    const int k_voff = (int)(((int64_t)(wave * 8 + k_lr) * sn + (((lane & 7) ^ k_lr ^ wave) << 3)) * 2);
    const int v_voff = (int)(((int64_t)(wave * 8 + k_lr) * sn + (((lane & 7) ^ att_vswz(k_lr)) << 3)) * 2);
    const int k_tile_bytes = (int)(ATT_BN * sn * 2);
#define SM_COPY(SK, SV, i_)                                                                                       \
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_k, (att_lds_ptr)((SK) + wave * 1024), 16, k_voff, (i_) * k_tile_bytes, 0, 0); \
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_v, (att_lds_ptr)((SV) + wave * 1024), 16, v_voff, (i_) * k_tile_bytes, 0, 0);
    SM_COPY(s_ka, s_va, 0)
    SM_COPY(s_ka + ATT_BN * 128, s_va + ATT_BN * 128, 1)
    SM_COPY(s_kb, s_vb, 2)
    SM_COPY(s_kb + ATT_BN * 128, s_vb + ATT_BN * 128, 3)
#undef SM_COPY

    f32x16 oacc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[i][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    // The first two tiles are used as soon as every wave's share of them has landed; the other
    // two keep streaming in meanwhile.  Waves without query rows (q0 >= N) still wait and meet
    // the barriers: the others read the rows they copied.
#define SM_HALF(SK, SV, t0_, WAIT)                                                                                \
    if ((t0_) < KT) {                                                                                             \
        __builtin_amdgcn_s_waitcnt(WAIT);                                                                         \
        __builtin_amdgcn_s_barrier();                                                                             \
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup"); /* the LDS reads stay below the barrier */         \
        if (q0 < N) {                                                                                             \
            const int t1 = KF < (t0_) + 2 ? KF : (t0_) + 2;                                                       \
            int t = (t0_);                                                                                        \
            for (; t < t1; ++t)                                                                                   \
                att_tile<false>((SK) + (t - (t0_)) * (ATT_BN * 128), (SV) + (t - (t0_)) * (ATT_BN * 128), qf, oacc, \
                                   m_run, l_run, t * ATT_BN, N, scale_log2e, l32, g);                             \
            if (t < KT && t < (t0_) + 2)                                                                          \
                att_tile<true>((SK) + (t - (t0_)) * (ATT_BN * 128), (SV) + (t - (t0_)) * (ATT_BN * 128), qf, oacc, \
                                  m_run, l_run, t * ATT_BN, N, scale_log2e, l32, g);                              \
        }                                                                                                         \
    }
    SM_HALF(s_ka, s_va, 0, 0x0F74)  // vmcnt(4): all but the newest four copies
    SM_HALF(s_kb, s_vb, 2, 0x0F70)
#undef SM_HALF
    __builtin_amdgcn_s_waitcnt(0x0F70);  // no copy is in flight when the wave ends
    if (q0 >= N) return;

    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    const float inv = 1.0f / l_tot;
    const int qr = q0 + l32;
    if (qr < N) {
        bf16raw* op = o + (int64_t)b * osb + (int64_t)qr * osn + (int64_t)h * osh;
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint2 w;
                w.x = pack2bf(oacc[db][4 * j] * inv, oacc[db][4 * j + 1] * inv);
                w.y = pack2bf(oacc[db][4 * j + 2] * inv, oacc[db][4 * j + 3] * inv);
                *reinterpret_cast<uint2*>(op + db * 32 + j * 8 + g * 4) = w;
            }
    }
}

// ---------------------------------------------------------------------------
// fp32 path: workgroup = 64 query rows of one (image, head), one row per thread;
// K/V tiles of 32 keys in LDS, broadcast reads.
// ---------------------------------------------------------------------------
constexpr int F32_BN = 32;

__global__ __launch_bounds__(64) void attention_f32_kernel(
    const float* __restrict__ q, const float* __restrict__ k, const float* __restrict__ v,
    float* __restrict__ o, int N, int64_t sb, int64_t sn, int64_t sh, int64_t osb, int64_t osn,
    int64_t osh, float scale_log2e) {
    __shared__ __attribute__((aligned(16))) float s_k[F32_BN][DH];
    __shared__ __attribute__((aligned(16))) float s_v[F32_BN][DH];
    const int tid = threadIdx.x;
    const int b = blockIdx.z, h = blockIdx.y;
    const int64_t base = (int64_t)b * sb + (int64_t)h * sh;
    const int qi = blockIdx.x * 64 + tid;
    const int qr = qi < N ? qi : N - 1;
    float qv[DH], acc[DH];
    {
        const float* qp = q + base + (int64_t)qr * sn;
#pragma unroll
        for (int d = 0; d < DH; d += 4) {
            float4 t = *reinterpret_cast<const float4*>(qp + d);
            qv[d] = t.x; qv[d + 1] = t.y; qv[d + 2] = t.z; qv[d + 3] = t.w;
        }
#pragma unroll
        for (int d = 0; d < DH; ++d) acc[d] = 0.f;
    }
    float m_run = -INFINITY, l_run = 0.f;
    for (int key0 = 0; key0 < N; key0 += F32_BN) {
        __syncthreads();
        // 32 keys x 16 float4 = 512 float4 per tensor, 8 per thread
        for (int t = tid; t < F32_BN * 16; t += 64) {
            const int r = t >> 4, c = (t & 15) * 4;
            const int kr = key0 + r;
            float4 kk = make_float4(0.f, 0.f, 0.f, 0.f), vv = kk;
            if (kr < N) {
                kk = *reinterpret_cast<const float4*>(k + base + (int64_t)kr * sn + c);
                vv = *reinterpret_cast<const float4*>(v + base + (int64_t)kr * sn + c);
            }
            *reinterpret_cast<float4*>(&s_k[r][c]) = kk;
            *reinterpret_cast<float4*>(&s_v[r][c]) = vv;
        }
        __syncthreads();
        float s[F32_BN];
        float mx = -INFINITY;
#pragma unroll
        for (int j = 0; j < F32_BN; ++j) {
            float t = 0.f;
#pragma unroll
            for (int d = 0; d < DH; d += 4) {
                float4 kk = *reinterpret_cast<const float4*>(&s_k[j][d]);
                t = fmaf(qv[d], kk.x, t); t = fmaf(qv[d + 1], kk.y, t);
                t = fmaf(qv[d + 2], kk.z, t); t = fmaf(qv[d + 3], kk.w, t);
            }
            s[j] = (key0 + j < N) ? t : -INFINITY;
            mx = fmaxf(mx, s[j]);
        }
        const float m_new = fmaxf(m_run, mx);
        const float alpha = exp2f((m_run - m_new) * scale_log2e);
        const float mb = m_new * scale_log2e;
        m_run = m_new;
        l_run *= alpha;
#pragma unroll
        for (int d = 0; d < DH; ++d) acc[d] *= alpha;
#pragma unroll
        for (int j = 0; j < F32_BN; ++j) {
            const float p = exp2f(fmaf(s[j], scale_log2e, -mb));
            l_run += p;
#pragma unroll
            for (int d = 0; d < DH; d += 4) {
                float4 vv = *reinterpret_cast<const float4*>(&s_v[j][d]);
                acc[d] = fmaf(p, vv.x, acc[d]); acc[d + 1] = fmaf(p, vv.y, acc[d + 1]);
                acc[d + 2] = fmaf(p, vv.z, acc[d + 2]); acc[d + 3] = fmaf(p, vv.w, acc[d + 3]);
            }
        }
    }
    if (qi < N) {
        const float inv = 1.0f / l_run;
        float* op = o + (int64_t)b * osb + (int64_t)qi * osn + (int64_t)h * osh;
#pragma unroll
        for (int d = 0; d < DH; d += 4)
            *reinterpret_cast<float4*>(op + d) =
                make_float4(acc[d] * inv, acc[d + 1] * inv, acc[d + 2] * inv, acc[d + 3] * inv);
    }
}

hipError_t launch_attention(rs_dtype dt, const void* q, const void* k, const void* v, void* o, int B,
                            int H, int N, int64_t sb, int64_t sn, int64_t sh, int64_t osb,
                            int64_t osn, int64_t osh, float scale, hipStream_t s) {
    if (B == 0 || H == 0 || N == 0) return hipSuccess;
    const float scale_log2e = scale * 1.44269504088896340736f;
    if (dt == RS_BF16 && N <= SM_MAXN) {
        hipLaunchKernelGGL(attention_bf16_small_kernel, dim3(H, B), dim3(512), 0, s, (const bf16raw*)q,
                           (const bf16raw*)k, (const bf16raw*)v, (bf16raw*)o, N, sb, sn, sh, osb, osn, osh,
                           scale_log2e);
    } else if (dt == RS_BF16) {
        // Whether the rows beyond the last full query tile of 256 go to the tail kernel: a CU holds
        // two workgroups, so a round is 512 of them; the tail kernel costs about a fifth of a round.
        const int BH = B * H;
        const int rem = N % ATT_BM;
        const bool tail_ok = rem > 0 && rem <= ATT_TAIL_ROWS && N > ATT_BM;
        const float cost_plain = (float)(((int64_t)BH * ((N + ATT_BM - 1) / ATT_BM) + 511) / 512);
        const float cost_tail = (float)(((int64_t)BH * (N / ATT_BM) + 511) / 512) + 0.22f * (float)((BH + 255) / 256);
        const bool best_tail = tail_ok && cost_tail < cost_plain;
        const int bm = ATT_BM;
        const int q_tiles = best_tail ? N / bm : (N + bm - 1) / bm;
        dim3 grid(8 * ((BH + 7) / 8) * q_tiles);
        hipLaunchKernelGGL(attention_bf16_kernel, grid, dim3(512), 0, s, (const bf16raw*)q, (const bf16raw*)k,
                           (const bf16raw*)v, (bf16raw*)o, N, sb, sn, sh, osb, osn, osh, scale_log2e, H, BH,
                           q_tiles);
        if (best_tail)
            hipLaunchKernelGGL(attention_bf16_tail_kernel, dim3(BH), dim3(512), 0, s, (const bf16raw*)q,
                               (const bf16raw*)k, (const bf16raw*)v, (bf16raw*)o, N, sb, sn, sh, osb, osn,
                               osh, scale_log2e, H, q_tiles * bm);
    } else {
        dim3 grid((N + 63) / 64, H, B);
        hipLaunchKernelGGL(attention_f32_kernel, grid, dim3(64), 0, s, (const float*)q,
                           (const float*)k, (const float*)v, (float*)o, N, sb, sn, sh, osb, osn, osh,
                           scale_log2e);
    }
    return hipGetLastError();
}

}  // namespace rs

// ---------------------------------------------------------------------------
// Standard (unfused) attention, the comparison system of Sec. 3.1 / Table 1: the attention map
// A = Softmax(Q K^T * scale) is written to memory, which is what the attention-based importance
// scores of Eqs. (2), (3) need and what the fused kernels above avoid.  Steps: pack the heads
// (q, k as [B H, Np, 64] with zero rows up to Np = N rounded up to 64, v transposed to
// [B H, 64, Np]); S = Q K^T as a batched matrix-core GEMM; softmax over every row in place;
// O = A V as a second batched GEMM; rows back to the caller's layout; column sums of the map.
// ---------------------------------------------------------------------------
namespace rs {

// one workgroup per (image * head, 64-token tile)
__global__ __launch_bounds__(256) void attn_pack_kernel(const bf16raw* __restrict__ q, const bf16raw* __restrict__ k,
                                                        const bf16raw* __restrict__ v, bf16raw* __restrict__ qh,
                                                        bf16raw* __restrict__ kh, bf16raw* __restrict__ vt, int H, int N,
                                                        int Np, int64_t sb, int64_t sn, int64_t sh) {
    __shared__ bf16raw tile[64][72];  // v rows of this tile, padded against bank conflicts
    const int bh = blockIdx.y, b = bh / H, h = bh - b * H;
    const int n0 = blockIdx.x * 64;
    const int64_t base = (int64_t)b * sb + (int64_t)h * sh;
    // 64 rows x 8 chunks of 16 bytes: two chunks per thread
    for (int t = threadIdx.x; t < 512; t += 256) {
        const int r = t >> 3, c = (t & 7) * 8;
        const int n = n0 + r;
        uint4 zq = make_uint4(0u, 0u, 0u, 0u), zk = zq, zv = zq;
        if (n < N) {
            zq = *reinterpret_cast<const uint4*>(q + base + (int64_t)n * sn + c);
            zk = *reinterpret_cast<const uint4*>(k + base + (int64_t)n * sn + c);
            zv = *reinterpret_cast<const uint4*>(v + base + (int64_t)n * sn + c);
        }
        *reinterpret_cast<uint4*>(qh + ((int64_t)bh * Np + n) * 64 + c) = zq;
        *reinterpret_cast<uint4*>(kh + ((int64_t)bh * Np + n) * 64 + c) = zk;
        *reinterpret_cast<uint4*>(&tile[r][c]) = zv;
    }
    __syncthreads();
    // vt[bh][d][n0 + r]: thread (d, r-chunk of 8)
    for (int t = threadIdx.x; t < 512; t += 256) {
        const int d = t >> 3, r0 = (t & 7) * 8;
        union { bf16raw e[8]; uint4 u; } w;
#pragma unroll
        for (int i = 0; i < 8; ++i) w.e[i] = tile[r0 + i][d];
        *reinterpret_cast<uint4*>(vt + ((int64_t)bh * 64 + d) * Np + n0 + r0) = w.u;
    }
}

hipError_t launch_attn_pack(const void* q, const void* k, const void* v, void* qh, void* kh, void* vt, int B, int H,
                            int N, int Np, int64_t sb, int64_t sn, int64_t sh, hipStream_t s) {
    hipLaunchKernelGGL(attn_pack_kernel, dim3(Np / 64, B * H), dim3(256), 0, s, (const bf16raw*)q, (const bf16raw*)k,
                       (const bf16raw*)v, (bf16raw*)qh, (bf16raw*)kh, (bf16raw*)vt, H, N, Np, sb, sn, sh);
    return hipGetLastError();
}

// one wavefront per row of the [rows, Np] score matrices: three passes over the row (maximum, sum,
// normalised write), the columns past N become zero
__global__ __launch_bounds__(256) void attn_softmax_rows_kernel(bf16raw* __restrict__ map, int64_t rows, int N, int Np,
                                                                float scale_log2e) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    bf16raw* p = map + row * Np;
    float mx = -INFINITY;
    for (int c = lane * 8; c < Np; c += 512) {
        float x[8];
        Elem<bf16raw>::load8(p + c, x);
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (c + i < N) mx = fmaxf(mx, x[i]);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    const float mb = mx * scale_log2e;
    float sum = 0.f;
    for (int c = lane * 8; c < Np; c += 512) {
        float x[8];
        Elem<bf16raw>::load8(p + c, x);
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (c + i < N) sum += __builtin_amdgcn_exp2f(fmaf(x[i], scale_log2e, -mb));
    }
    sum = wave_sum(sum);
    const float inv = 1.0f / sum;
    for (int c = lane * 8; c < Np; c += 512) {
        float x[8];
        Elem<bf16raw>::load8(p + c, x);
#pragma unroll
        for (int i = 0; i < 8; ++i) x[i] = c + i < N ? __builtin_amdgcn_exp2f(fmaf(x[i], scale_log2e, -mb)) * inv : 0.f;
        Elem<bf16raw>::store8(p + c, x);
    }
}

hipError_t launch_attn_softmax_rows(void* map, int64_t rows, int N, int Np, float scale_log2e, hipStream_t s) {
    if (rows == 0) return hipSuccess;
    hipLaunchKernelGGL(attn_softmax_rows_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, (bf16raw*)map, rows,
                       N, Np, scale_log2e);
    return hipGetLastError();
}

// partial[bh][j] = sum_i A[bh][i][j]  (thread j walks the rows in order: fixed order, coalesced)
__global__ __launch_bounds__(256) void attn_colsum_kernel(const bf16raw* __restrict__ map, float* __restrict__ partial,
                                                          int N, int Np) {
    const int j = blockIdx.x * 256 + threadIdx.x;
    const int bh = blockIdx.y;
    if (j >= N) return;
    const bf16raw* p = map + (int64_t)bh * N * Np + j;
    float acc = 0.f;
    for (int i = 0; i < N; ++i) acc += bf2f(p[(int64_t)i * Np]);
    partial[(int64_t)bh * N + j] = acc;
}

// Eq. (2): s_cls[b][j] = mean_h A[b,h,cls,j];  Eq. (3): s_mean[b][j] = mean_h (1/N) sum_i A[b,h,i,j]
__global__ __launch_bounds__(256) void attn_scores_kernel(const bf16raw* __restrict__ map, const float* __restrict__ partial,
                                                          float* __restrict__ s_cls, float* __restrict__ s_mean, int H,
                                                          int N, int Np, int cls_index) {
    const int j = blockIdx.x * 256 + threadIdx.x;
    const int b = blockIdx.y;
    if (j >= N) return;
    float c = 0.f, m = 0.f;
    for (int h = 0; h < H; ++h) {
        const int64_t bh = (int64_t)b * H + h;
        c += bf2f(map[(bh * N + cls_index) * Np + j]);
        m += partial[bh * N + j];
    }
    if (s_cls) s_cls[(int64_t)b * N + j] = c / (float)H;
    if (s_mean) s_mean[(int64_t)b * N + j] = m / ((float)H * (float)N);
}

hipError_t launch_attn_map_scores(const void* map, float* partial, float* s_cls, float* s_mean, int B, int H, int N,
                                  int Np, int cls_index, hipStream_t s) {
    if (!s_cls && !s_mean) return hipSuccess;
    if (s_mean)
        hipLaunchKernelGGL(attn_colsum_kernel, dim3((N + 255) / 256, B * H), dim3(256), 0, s, (const bf16raw*)map, partial, N, Np);
    hipLaunchKernelGGL(attn_scores_kernel, dim3((N + 255) / 256, B), dim3(256), 0, s, (const bf16raw*)map, partial,
                       s_cls, s_mean, H, N, Np, cls_index);
    return hipGetLastError();
}

// o[b, n, h, :] = oh[b h][n][:]; 8 lanes per 128-byte row
__global__ __launch_bounds__(256) void attn_unpack_kernel(const bf16raw* __restrict__ oh, bf16raw* __restrict__ o, int H,
                                                          int N, int64_t rows, int64_t osb, int64_t osn, int64_t osh) {
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t r = t >> 3;  // row index into [B H, N]
    if (r >= rows) return;
    const int c = (int)(t & 7) * 8;
    const int64_t bh = r / N;
    const int n = (int)(r - bh * N);
    const int64_t b = bh / H;
    const int h = (int)(bh - b * H);
    *reinterpret_cast<uint4*>(o + b * osb + (int64_t)n * osn + (int64_t)h * osh + c) =
        *reinterpret_cast<const uint4*>(oh + r * 64 + c);
}

hipError_t launch_attn_unpack(const void* oh, void* o, int B, int H, int N, int64_t osb, int64_t osn, int64_t osh,
                              hipStream_t s) {
    const int64_t rows = (int64_t)B * H * N;
    if (rows == 0) return hipSuccess;
    hipLaunchKernelGGL(attn_unpack_kernel, dim3((unsigned)((rows * 8 + 255) / 256)), dim3(256), 0, s, (const bf16raw*)oh,
                       (bf16raw*)o, H, N, rows, osb, osn, osh);
    return hipGetLastError();
}

}  // namespace rs
