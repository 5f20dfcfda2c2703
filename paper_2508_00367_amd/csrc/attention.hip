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
//                     (8 registers = the lane's 8 keys of a 16-key group), A operand = V^T
//                     from LDS.  V is transposed on its way into LDS, with the keys of each
//                     16-key group stored in the order the accumulator layout yields them
//                     (position 8g + 4u + i  <->  key 8u + 4g + i), so a lane reads its 8
//                     keys as one 16-byte vector.
// Row max / row sum need one exchange between the two half-waves per tile.
//
// fp32 path: one query row per thread, true fp32 products (parity configuration).
#include "common.hpp"

namespace rs {

constexpr int ATT_BM = 128;  // query rows per workgroup (4 waves x 32)
constexpr int ATT_BN = 64;   // keys per tile
constexpr int DH = 64;

// 16-byte chunk `c` (0..7) of 128-byte LDS row `r`; the XOR spreads both the row-wise
// operand reads and the transposed V writes over the banks.
__device__ __forceinline__ int att_swz(int r, int c) { return r * 128 + (((c ^ r ^ (r >> 3)) & 7) << 4); }

__global__ __launch_bounds__(256) void attention_bf16_kernel(
    const bf16raw* __restrict__ q, const bf16raw* __restrict__ k, const bf16raw* __restrict__ v,
    bf16raw* __restrict__ o, int N, int64_t sb, int64_t sn, int64_t sh, int64_t osb, int64_t osn,
    int64_t osh, float scale_log2e) {
    __shared__ __attribute__((aligned(16))) unsigned char s_k[2][ATT_BN * 128];
    __shared__ __attribute__((aligned(16))) unsigned char s_vt[2][DH * 128];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, g = lane >> 5;
    const int b = blockIdx.z, h = blockIdx.y;
    const int q0 = blockIdx.x * ATT_BM + wave * 32;
    const int64_t base = (int64_t)b * sb + (int64_t)h * sh;
    const bf16raw* kb = k + base;
    const bf16raw* vb = v + base;

    // Q fragments: B operand, column = query row q0 + l32, k-slots = 8 channels 16*kk + 8*g ..
    bf16x8 qf[4];
    {
        int qr = q0 + l32;
        qr = qr < N ? qr : N - 1;  // rows past the end are computed on a copy and never stored
        const bf16raw* qp = q + base + (int64_t)qr * sn;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) qf[kk] = *reinterpret_cast<const bf16x8*>(qp + kk * 16 + g * 8);
    }

    // K tile loader: thread -> chunk (tid & 7) of key rows (tid >> 3) and (tid >> 3) + 32.
    const int ld_chunk = tid & 7, ld_row = tid >> 3;
    // V tile loader: thread -> channel chunk (tid & 7), key pair at positions 2a, 2a+1 (a = tid >> 3).
    // position p = 16T + 8g' + 4u + i  <->  key 16T + 8u + 4g' + i
    const int va = tid >> 3;
    const int vpos = 2 * va;
    const int vkey = (vpos & ~15) | (((vpos >> 2) & 1) << 3) | (((vpos >> 3) & 1) << 2) | (vpos & 3);

    uint4 k_reg[2], v_reg[2];
    auto load_global = [&](int kt) {
        const int key0 = kt * ATT_BN;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            int kr = key0 + ld_row + i * 32;
            kr = kr < N ? kr : N - 1;  // masked to -inf below
            k_reg[i] = *reinterpret_cast<const uint4*>(kb + (int64_t)kr * sn + ld_chunk * 8);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int kr = key0 + vkey + i;
            uint4 t = make_uint4(0u, 0u, 0u, 0u);  // keys past the end contribute exact zeros
            if (kr < N) t = *reinterpret_cast<const uint4*>(vb + (int64_t)kr * sn + ld_chunk * 8);
            v_reg[i] = t;
        }
    };
    auto store_lds = [&](int stage) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
            *reinterpret_cast<uint4*>(&s_k[stage][att_swz(ld_row + i * 32, ld_chunk)]) = k_reg[i];
        // transpose: channel d = 8*ld_chunk + e gets the pair (key, key+1) at positions vpos, vpos+1
        const uint32_t w0[4] = {v_reg[0].x, v_reg[0].y, v_reg[0].z, v_reg[0].w};
        const uint32_t w1[4] = {v_reg[1].x, v_reg[1].y, v_reg[1].z, v_reg[1].w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t lo = (e & 1) ? (w0[e >> 1] >> 16) : (w0[e >> 1] & 0xffffu);
            const uint32_t hi = (e & 1) ? (w1[e >> 1] & 0xffff0000u) : (w1[e >> 1] << 16);
            const int d = ld_chunk * 8 + e;
            *reinterpret_cast<uint32_t*>(&s_vt[stage][att_swz(d, vpos >> 3) + (vpos & 7) * 2]) = lo | hi;
        }
    };

    f32x16 oacc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[i][r] = 0.f;
    float m_run = -INFINITY;  // running max of the raw logits of this lane's query row
    float l_run = 0.f;        // this lane's share of the running row sum

    const int KT = (N + ATT_BN - 1) / ATT_BN;
    load_global(0);
    store_lds(0);
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        if (kt + 1 < KT) load_global(kt + 1);
        const unsigned char* sk = s_k[kt & 1];
        const unsigned char* sv = s_vt[kt & 1];

        // ---- S^T = K Q^T for the 64 keys of this tile
        f32x16 sacc[2];
#pragma unroll
        for (int kb2 = 0; kb2 < 2; ++kb2) {
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[kb2][r] = 0.f;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                bf16x8 kf = *reinterpret_cast<const bf16x8*>(sk + att_swz(kb2 * 32 + l32, kk * 2 + g));
                sacc[kb2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], sacc[kb2], 0, 0, 0);
            }
        }
        // ---- mask keys past the end (last tile only)
        if ((kt + 1) * ATT_BN > N) {
#pragma unroll
            for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = kt * ATT_BN + kb2 * 32 + (r >> 2) * 8 + g * 4 + (r & 3);
                    if (key >= N) sacc[kb2][r] = -INFINITY;
                }
        }
        // ---- online softmax: row max over this lane's 32 keys, then across the half-waves
        float mx = sacc[0][0];
#pragma unroll
        for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[kb2][r]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m_run, mx);  // finite: every tile holds at least one real key
        const float alpha = exp2f((m_run - m_new) * scale_log2e);
        const float mb = m_new * scale_log2e;
        m_run = m_new;
        float psum = 0.f;
#pragma unroll
        for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = exp2f(fmaf(sacc[kb2][r], scale_log2e, -mb));
                sacc[kb2][r] = p;
                psum += p;
            }
        l_run = l_run * alpha + psum;
        if (__ballot(alpha != 1.0f)) {  // the running maximum moved for some row of this wave
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[i][r] *= alpha;
        }

        // ---- O^T += V^T P^T, 16 keys per MFMA
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int kb2 = t >> 1, r0 = (t & 1) * 8;
            union { uint32_t u[4]; bf16x8 v; } pf;
#pragma unroll
            for (int e = 0; e < 4; ++e) pf.u[e] = pack2bf(sacc[kb2][r0 + 2 * e], sacc[kb2][r0 + 2 * e + 1]);
#pragma unroll
            for (int db = 0; db < 2; ++db) {
                bf16x8 vf = *reinterpret_cast<const bf16x8*>(sv + att_swz(db * 32 + l32, 2 * t + g));
                oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf.v, oacc[db], 0, 0, 0);
            }
        }

        if (kt + 1 < KT) store_lds((kt + 1) & 1);
        __syncthreads();
    }

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
// Short sequences (N <= 256, every image-classification block): one workgroup of 8 waves per
// (image, head).  K (N x 64) and V^T (64 x N) of the head are copied into LDS once, one
// barrier, then wave w runs query rows 32w .. 32w+31 against all key tiles without further
// synchronisation.  Against the tiled kernel this reads K and V once instead of once per
// query tile and has no per-tile barrier or staging latency; two workgroups share a CU, so
// one wave's exp/max/sum work runs under another's MFMAs.
// LDS: K rows of 128 bytes, chunk c of row r in slot c ^ ((r ^ r>>3) & 7); V^T rows of 512
// bytes (256 key positions), 16-byte chunk c of channel row d in slot c ^ ((d ^ d>>3) & 15):
// both the 16-lane operand reads and the transposing 4-byte writes are bank-conflict free.
// ---------------------------------------------------------------------------
constexpr int SM_MAXN = 256;

__device__ __forceinline__ int vt_off(int d, int chunk) { return d * 512 + ((chunk ^ ((d ^ (d >> 3)) & 15)) << 4); }

__global__ __launch_bounds__(512) void attention_bf16_small_kernel(
    const bf16raw* __restrict__ q, const bf16raw* __restrict__ k, const bf16raw* __restrict__ v,
    bf16raw* __restrict__ o, int N, int64_t sb, int64_t sn, int64_t sh, int64_t osb, int64_t osn,
    int64_t osh, float scale_log2e) {
    __shared__ __attribute__((aligned(16))) unsigned char s_k[SM_MAXN * 128];
    __shared__ __attribute__((aligned(16))) unsigned char s_vt[DH * 512];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, g = lane >> 5;
    const int b = blockIdx.y, h = blockIdx.x;
    const int64_t base = (int64_t)b * sb + (int64_t)h * sh;
    const bf16raw* kb = k + base;
    const bf16raw* vb = v + base;
    const int KT = (N + ATT_BN - 1) / ATT_BN;   // key tiles of 64
    const int NP = KT * ATT_BN;                 // keys including the padding of the last tile

    // ---- K -> LDS: 16-byte chunk (tid & 7) of key rows (tid >> 3) + 64 i
    {
        const int ld_chunk = tid & 7, ld_row = tid >> 3;
        for (int r = ld_row; r < NP; r += 64) {
            const int kr = r < N ? r : N - 1;  // padded keys are masked to -inf below
            const uint4 t = *reinterpret_cast<const uint4*>(kb + (int64_t)kr * sn + ld_chunk * 8);
            *reinterpret_cast<uint4*>(&s_k[att_swz(r, ld_chunk)]) = t;
        }
    }
    // ---- V -> LDS transposed.  Thread: channel chunk (tid & 7), key positions 2a, 2a+1 with
    //      a = (tid >> 3) + 64 i; position p = 16T + 8g' + 4u + i  <->  key 16T + 8u + 4g' + i
    {
        const int dc = tid & 7;
        for (int a2 = tid >> 3; 2 * a2 < NP; a2 += 64) {
            const int vpos = 2 * a2;
            const int vkey = (vpos & ~15) | (((vpos >> 2) & 1) << 3) | (((vpos >> 3) & 1) << 2) | (vpos & 3);
            uint4 r0 = make_uint4(0u, 0u, 0u, 0u), r1 = r0;  // keys past the end contribute exact zeros
            if (vkey < N) r0 = *reinterpret_cast<const uint4*>(vb + (int64_t)vkey * sn + dc * 8);
            if (vkey + 1 < N) r1 = *reinterpret_cast<const uint4*>(vb + (int64_t)(vkey + 1) * sn + dc * 8);
            const uint32_t w0[4] = {r0.x, r0.y, r0.z, r0.w};
            const uint32_t w1[4] = {r1.x, r1.y, r1.z, r1.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t lo = (e & 1) ? (w0[e >> 1] >> 16) : (w0[e >> 1] & 0xffffu);
                const uint32_t hi = (e & 1) ? (w1[e >> 1] & 0xffff0000u) : (w1[e >> 1] << 16);
                const int d = dc * 8 + e;
                *reinterpret_cast<uint32_t*>(&s_vt[vt_off(d, vpos >> 3) + (vpos & 7) * 2]) = lo | hi;
            }
        }
    }
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
    __syncthreads();
    if (q0 >= N) return;  // whole-wave exit after the only barrier

    f32x16 oacc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[i][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    for (int kt = 0; kt < KT; ++kt) {
        f32x16 sacc[2];
#pragma unroll
        for (int kb2 = 0; kb2 < 2; ++kb2) {
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[kb2][r] = 0.f;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                bf16x8 kf = *reinterpret_cast<const bf16x8*>(&s_k[att_swz(kt * 64 + kb2 * 32 + l32, kk * 2 + g)]);
                sacc[kb2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], sacc[kb2], 0, 0, 0);
            }
        }
        if ((kt + 1) * ATT_BN > N) {
#pragma unroll
            for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = kt * ATT_BN + kb2 * 32 + (r >> 2) * 8 + g * 4 + (r & 3);
                    if (key >= N) sacc[kb2][r] = -INFINITY;
                }
        }
        float mx = sacc[0][0];
#pragma unroll
        for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[kb2][r]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m_run, mx);
        const float alpha = exp2f((m_run - m_new) * scale_log2e);
        const float mb = m_new * scale_log2e;
        m_run = m_new;
        float psum = 0.f;
#pragma unroll
        for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = __builtin_amdgcn_exp2f(fmaf(sacc[kb2][r], scale_log2e, -mb));
                sacc[kb2][r] = p;
                psum += p;
            }
        l_run = l_run * alpha + psum;
        if (__ballot(alpha != 1.0f)) {  // the running maximum moved for some row of this wave
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[i][r] *= alpha;
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int kb2 = t >> 1, r0 = (t & 1) * 8;
            union { uint32_t u[4]; bf16x8 v; } pf;
#pragma unroll
            for (int e = 0; e < 4; ++e) pf.u[e] = pack2bf(sacc[kb2][r0 + 2 * e], sacc[kb2][r0 + 2 * e + 1]);
#pragma unroll
            for (int db = 0; db < 2; ++db) {
                bf16x8 vf = *reinterpret_cast<const bf16x8*>(&s_vt[vt_off(db * 32 + l32, 2 * (kt * 4 + t) + g)]);
                oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf.v, oacc[db], 0, 0, 0);
            }
        }
    }
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
        dim3 grid((N + ATT_BM - 1) / ATT_BM, H, B);
        hipLaunchKernelGGL(attention_bf16_kernel, grid, dim3(256), 0, s, (const bf16raw*)q,
                           (const bf16raw*)k, (const bf16raw*)v, (bf16raw*)o, N, sb, sn, sh, osb, osn,
                           osh, scale_log2e);
    } else {
        dim3 grid((N + 63) / 64, H, B);
        hipLaunchKernelGGL(attention_f32_kernel, grid, dim3(64), 0, s, (const float*)q,
                           (const float*)k, (const float*)v, (float*)o, N, sb, sn, sh, osb, osn, osh,
                           scale_log2e);
    }
    return hipGetLastError();
}

}  // namespace rs
