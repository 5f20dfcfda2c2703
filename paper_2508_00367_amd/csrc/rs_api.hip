// C ABI of the representation-shift library: argument validation, workspace carving
// and the launch sequence of the block (Eqs. (5),(6), Sec. 3.3) on the caller's stream.
// Every argument check happens before the first HIP call, so the error paths run
// (and are tested) without a GPU.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <atomic>
#include <mutex>
#include <vector>

#include "common.hpp"

namespace rs {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

rs_status device_error(const char* what, hipError_t e) {
    set_error("%s: %s", what, hipGetErrorString(e));
    return RS_ERR_DEVICE;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// [a, a + na) and [b, b + nb) share a byte (NULL or empty ranges never do)
static bool overlaps(const void* a, size_t na, const void* b, size_t nb) {
    if (!a || !b || na == 0 || nb == 0) return false;
    const uintptr_t pa = reinterpret_cast<uintptr_t>(a), pb = reinterpret_cast<uintptr_t>(b);
    return pa < pb + nb && pb < pa + na;
}

#define RS_REQUIRE(cond, status, ...)  \
    do {                               \
        if (!(cond)) {                 \
            rs::set_error(__VA_ARGS__); \
            return (status);           \
        }                              \
    } while (0)

#define RS_LAUNCH(expr)                                          \
    do {                                                         \
        hipError_t e_ = (expr);                                  \
        if (e_ != hipSuccess) return rs::device_error(#expr, e_); \
    } while (0)

// ---- optional per-kernel timing with HIP events on the caller's stream ---------
enum KernelClass { K_PACK = 0, K_LN, K_GEMM_QKV, K_ATTN, K_GEMM_PROJ, K_GEMM_FC1, K_GEMM_FC2, K_SCORE,
                   K_SELECT, K_GATHER, K_LINEAR, K_COUNT };
static_assert(K_COUNT == RS_PROFILE_CLASSES, "header and library disagree on the class count");
static const char* const kClassNames[K_COUNT] = {"pack_weights", "layernorm", "gemm_qkv", "attention",
                                                 "gemm_proj", "gemm_fc1", "gemm_fc2", "shift_score",
                                                 "select", "gather", "linear"};
struct ProfRec { int cls; hipEvent_t start, stop; };
static struct {
    std::mutex mu;
    std::atomic<bool> on{false};  // read on every launch without the mutex
    std::vector<ProfRec> recs;
    std::vector<hipEvent_t> pool;
} g_prof;

static hipEvent_t prof_event() {
    if (!g_prof.pool.empty()) {
        hipEvent_t e = g_prof.pool.back();
        g_prof.pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

// Runs `launch` and, when profiling is on, brackets it with two events on `s`.
template <typename F>
static hipError_t timed(int cls, hipStream_t s, F launch) {
    if (!g_prof.on.load(std::memory_order_relaxed)) return launch();
    std::lock_guard<std::mutex> lk(g_prof.mu);
    hipEvent_t a = prof_event(), b = prof_event();
    hipError_t e = (a && b) ? hipEventRecord(a, s) : hipErrorOutOfMemory;
    if (e == hipSuccess) e = launch();
    if (e == hipSuccess) e = hipEventRecord(b, s);
    if (e != hipSuccess) {  // nothing recorded: the events go back to the pool
        if (a) g_prof.pool.push_back(a);
        if (b) g_prof.pool.push_back(b);
        return e;
    }
    g_prof.recs.push_back({cls, a, b});
    return hipSuccess;
}

#define RS_LAUNCH_K(cls, stream, expr)                                         \
    do {                                                                       \
        hipError_t e_ = rs::timed((cls), (stream), [&]() { return (expr); });  \
        if (e_ != hipSuccess) return rs::device_error(#expr, e_);              \
    } while (0)

// ---- workspace layout of rs_block_fwd ---------------------------------------
struct BlockLayout {
    size_t packed, u, qkv, att, x1, hid, partials, scores, stats, total;
    int slots;
};

// Packed bf16 weights: the four matrices as [out, in] (LayerNorm scales folded into W_qkv and
// W_fc1), then the fp32 column vectors of the two folded LayerNorms.
struct PackedLayout {
    size_t w_qkv, w_proj, w_fc1, w_fc2, cs_qkv, b_qkv, cs_fc1, b_fc1, total;
};

static PackedLayout packed_layout(const rs_block_cfg* c) {
    PackedLayout P;
    const size_t D = c->D, Dm = c->Dm;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes, 256); return o; };
    P.w_qkv = take(3 * D * D * 2);
    P.w_proj = take(D * D * 2);
    P.w_fc1 = take(D * Dm * 2);
    P.w_fc2 = take(D * Dm * 2);
    P.cs_qkv = take(3 * D * sizeof(float));
    P.b_qkv = take(3 * D * sizeof(float));
    P.cs_fc1 = take(Dm * sizeof(float));
    P.b_fc1 = take(Dm * sizeof(float));
    P.total = off;
    return P;
}

static size_t packed_bytes(const rs_block_cfg* c) {
    return c->dtype == RS_BF16 ? packed_layout(c).total : 0;
}

static BlockLayout block_layout(const rs_block_cfg* c) {
    BlockLayout L;
    const size_t e = elem_size(c->dtype);
    const size_t M = (size_t)c->B * (size_t)c->N, D = c->D, Dm = c->Dm;
    L.slots = gemm_shift_slots(c->dtype, c->D);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes, 256); return o; };
    L.packed = take(packed_bytes(c));
    L.u = take(M * D * e);
    L.qkv = take(M * 3 * D * e);
    L.att = take(M * D * e);
    L.x1 = take(M * D * e);
    L.hid = take(M * Dm * e);
    L.partials = take(M * (size_t)L.slots * kShiftLanes * sizeof(float));
    L.scores = take(M * sizeof(float));
    L.stats = take(M * 2 * sizeof(float));
    L.total = off;
    return L;
}

static rs_status check_cfg(const rs_block_cfg* c) {
    RS_REQUIRE(c != nullptr, RS_ERR_INVALID_ARG, "cfg is NULL");
    RS_REQUIRE(c->dtype == RS_F32 || c->dtype == RS_BF16, RS_ERR_INVALID_ARG, "unknown dtype %d", (int)c->dtype);
    RS_REQUIRE(c->dist == RS_DIST_L2 || c->dist == RS_DIST_L1 || c->dist == RS_DIST_COS, RS_ERR_INVALID_ARG,
               "unknown distance %d", (int)c->dist);
    RS_REQUIRE(c->op >= RS_SHIFT_MLP && c->op <= RS_SHIFT_MLP_NORMED, RS_ERR_INVALID_ARG,
               "unknown shift operation %d", (int)c->op);
    RS_REQUIRE(c->B >= 0 && c->N >= 0, RS_ERR_INVALID_ARG, "negative B or N");
    RS_REQUIRE(c->B <= 65535, RS_ERR_UNSUPPORTED, "B %d > 65535 (one launch-grid axis of the attention kernels)", c->B);
    RS_REQUIRE(c->D > 0 && c->H > 0 && c->Dm > 0, RS_ERR_INVALID_ARG, "D, H, Dm must be positive");
    RS_REQUIRE(c->D % c->H == 0, RS_ERR_INVALID_ARG, "D %d not divisible by H %d", c->D, c->H);
    RS_REQUIRE(c->D / c->H == 64, RS_ERR_UNSUPPORTED, "head width D/H = %d, only 64 is built", c->D / c->H);
    RS_REQUIRE(c->Dm % 64 == 0, RS_ERR_UNSUPPORTED, "Dm %d is not a multiple of 64", c->Dm);
    RS_REQUIRE(c->D <= 4096, RS_ERR_UNSUPPORTED, "D %d > 4096", c->D);
    RS_REQUIRE(c->Dm <= kGemmMaxK, RS_ERR_UNSUPPORTED, "Dm %d > %d", c->Dm, kGemmMaxK);
    RS_REQUIRE((int64_t)c->B * c->N < (int64_t)1 << 31, RS_ERR_UNSUPPORTED, "B*N does not fit 31 bits");
    // bf16 attention addresses one image's rows of the [N, 3D] QKV buffer with 32-bit byte offsets
    RS_REQUIRE(c->dtype != RS_BF16 || ((int64_t)c->N + 256) * 3 * c->D * 2 < (int64_t)0x7fffffff, RS_ERR_UNSUPPORTED,
               "(N + 256) * 3 D * 2 bytes must stay below 2 GiB in bf16");
    RS_REQUIRE(c->n_prefix >= 0 && c->n_keep >= 0, RS_ERR_INVALID_ARG, "negative n_prefix or n_keep");
    RS_REQUIRE((int64_t)c->n_prefix + c->n_keep <= c->N, RS_ERR_INVALID_ARG,
               "n_prefix %d + n_keep %d exceeds N %d", c->n_prefix, c->n_keep, c->N);
    RS_REQUIRE(c->ln_eps > 0.f, RS_ERR_INVALID_ARG, "ln_eps must be positive");
    return RS_OK;
}

}  // namespace rs

using namespace rs;

static rs_status block_fwd(const rs_block_cfg* cfg, const rs_block_weights* w, const void* x, void* y,
                           int32_t* kept_idx, float* scores, void* workspace, size_t workspace_bytes,
                           void* hip_stream, const float* x_stats = nullptr, float* y_stats = nullptr);

// ---- scratch of rs_block_fwd_static ------------------------------------------------------
// One buffer per GPU, part of the loaded code object: it exists from the moment the library's
// device code is loaded on a GPU until the process ends, and no call ever allocates it.  The
// name below is a host-side handle, not a device address; the address on the current device comes
// from hipGetSymbolAddress, once per device, and only that pointer is handed to kernels.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

static rs_status static_scratch(void** out) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void* ptrs[kMaxDevices] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return device_error("hipGetDevice", e);
    RS_REQUIRE(dev >= 0 && dev < kMaxDevices, RS_ERR_UNSUPPORTED, "device index %d beyond %d", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lk(mu);
    if (!ptrs[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return device_error("hipGetSymbolAddress(scratch)", e);
        RS_REQUIRE(p != nullptr && (reinterpret_cast<uintptr_t>(p) & 255u) == 0, RS_ERR_DEVICE,
                   "static scratch buffer has no usable device address");
        ptrs[dev] = p;
    }
    *out = ptrs[dev];
    return RS_OK;
}

extern "C" {

const char* rs_last_error(void) { return g_err; }

int32_t rs_version(void) { return 200; }

const char* rs_build_info(void) { return gemm_build_info(); }

rs_status rs_tune_gemm_variant(int32_t variant) {
    RS_REQUIRE(variant >= 0 && variant <= 4, RS_ERR_INVALID_ARG, "variant %d outside 0..4", (int)variant);
    set_gemm_variant(variant);
    return RS_OK;
}

rs_status rs_profile_enable(int32_t enable) {
    std::lock_guard<std::mutex> lk(g_prof.mu);
    g_prof.on.store(enable != 0);
    return RS_OK;
}

const char* rs_profile_class_name(int32_t cls) {
    return (cls >= 0 && cls < K_COUNT) ? kClassNames[cls] : "";
}

rs_status rs_profile_read(double* ms_out, int64_t* launches_out) {
    RS_REQUIRE(ms_out && launches_out, RS_ERR_INVALID_ARG, "ms_out and launches_out must not be NULL");
    std::lock_guard<std::mutex> lk(g_prof.mu);
    for (int i = 0; i < K_COUNT; ++i) { ms_out[i] = 0.0; launches_out[i] = 0; }
    rs_status st = RS_OK;
    for (const ProfRec& r : g_prof.recs) {
        float ms = 0.f;
        hipError_t e = hipEventSynchronize(r.stop);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.start, r.stop);
        if (e != hipSuccess) st = device_error("profile event", e);
        ms_out[r.cls] += ms;
        launches_out[r.cls] += 1;
        g_prof.pool.push_back(r.start);
        g_prof.pool.push_back(r.stop);
    }
    g_prof.recs.clear();
    return st;
}

rs_status rs_attention_fwd(const void* q, const void* k, const void* v, void* o, int32_t B, int32_t H,
                           int32_t N, int32_t dh, int64_t stride_b, int64_t stride_n, int64_t stride_h,
                           int64_t o_stride_b, int64_t o_stride_n, int64_t o_stride_h, float scale,
                           rs_dtype dtype, void* hip_stream) {
    RS_REQUIRE(dtype == RS_F32 || dtype == RS_BF16, RS_ERR_INVALID_ARG, "unknown dtype %d", (int)dtype);
    RS_REQUIRE(B >= 0 && H >= 0 && N >= 0, RS_ERR_INVALID_ARG, "negative B, H or N");
    RS_REQUIRE(dh > 0, RS_ERR_INVALID_ARG, "dh must be positive");
    RS_REQUIRE(dh == 64, RS_ERR_UNSUPPORTED, "head width %d, only 64 is built", dh);
    RS_REQUIRE(B <= 65535 && H <= 65535, RS_ERR_UNSUPPORTED, "B and H are limited to 65535");
    RS_REQUIRE(scale > 0.f && scale < INFINITY, RS_ERR_INVALID_ARG, "scale must be positive and finite");
    if (B == 0 || H == 0 || N == 0) return RS_OK;
    RS_REQUIRE(q && k && v && o, RS_ERR_INVALID_ARG, "q, k, v and o must not be NULL");
    RS_REQUIRE(aligned16(q) && aligned16(k) && aligned16(v) && aligned16(o), RS_ERR_INVALID_ARG,
               "q, k, v and o must be 16-byte aligned");
    RS_REQUIRE(o != q && o != k && o != v, RS_ERR_INVALID_ARG, "o must not alias q, k or v");
    const int64_t st[6] = {stride_b, stride_n, stride_h, o_stride_b, o_stride_n, o_stride_h};
    for (int i = 0; i < 6; ++i)
        RS_REQUIRE(st[i] >= 0 && st[i] % 8 == 0, RS_ERR_INVALID_ARG,
                   "strides must be non-negative multiples of 8 elements");
    RS_REQUIRE(stride_n >= dh && o_stride_n >= dh, RS_ERR_INVALID_ARG, "token stride smaller than dh");
    // the bf16 kernels address the K and V rows of one (image, head) with 32-bit byte offsets,
    // up to 256 rows past the last one (those read as zeros)
    RS_REQUIRE(dtype != RS_BF16 || ((int64_t)N + 256) * stride_n * 2 < (int64_t)0x7fffffff, RS_ERR_UNSUPPORTED,
               "(N + 256) * stride_n * 2 bytes must stay below 2 GiB for bf16 attention");
    RS_LAUNCH_K(K_ATTN, (hipStream_t)hip_stream, launch_attention(dtype, q, k, v, o, B, H, N, stride_b, stride_n, stride_h, o_stride_b,
                               o_stride_n, o_stride_h, scale, (hipStream_t)hip_stream));
    return RS_OK;
}

// workspace of rs_attention_map_fwd: packed q, k [B H, Np, 64], v^T [B H, 64, Np], o [B H, N, 64], column sums
struct AttnMapLayout {
    size_t qh, kh, vt, oh, partial, total;
    int Np;
};

static AttnMapLayout attn_map_layout(int64_t B, int64_t H, int64_t N) {
    AttnMapLayout L;
    L.Np = (int)((N + 63) / 64 * 64);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes, 256); return o; };
    const size_t BH = (size_t)(B * H);
    L.qh = take(BH * L.Np * 64 * 2);
    L.kh = take(BH * L.Np * 64 * 2);
    L.vt = take(BH * 64 * L.Np * 2);
    L.oh = take(BH * N * 64 * 2);
    L.partial = take(BH * N * sizeof(float));
    L.total = off;
    return L;
}

size_t rs_attention_map_workspace_size(int32_t B, int32_t H, int32_t N) {
    if (B <= 0 || H <= 0 || N <= 0) return 0;
    return attn_map_layout(B, H, N).total;
}

size_t rs_attention_map_size(int32_t B, int32_t H, int32_t N) {
    if (B <= 0 || H <= 0 || N <= 0) return 0;
    return (size_t)B * H * N * ((N + 63) / 64 * 64) * 2;
}

rs_status rs_attention_map_fwd(const void* q, const void* k, const void* v, void* o, int32_t B, int32_t H, int32_t N,
                               int32_t dh, int64_t stride_b, int64_t stride_n, int64_t stride_h, int64_t o_stride_b,
                               int64_t o_stride_n, int64_t o_stride_h, float scale, rs_dtype dtype, int32_t cls_index,
                               void* attn_map, float* s_cls, float* s_mean, void* workspace, size_t workspace_bytes,
                               void* hip_stream) {
    RS_REQUIRE(dtype == RS_F32 || dtype == RS_BF16, RS_ERR_INVALID_ARG, "unknown dtype %d", (int)dtype);
    RS_REQUIRE(dtype == RS_BF16, RS_ERR_UNSUPPORTED, "the materialised-map attention is built for bf16 only");
    RS_REQUIRE(B >= 0 && H >= 0 && N >= 0, RS_ERR_INVALID_ARG, "negative B, H or N");
    RS_REQUIRE(dh > 0, RS_ERR_INVALID_ARG, "dh must be positive");
    RS_REQUIRE(dh == 64, RS_ERR_UNSUPPORTED, "head width %d, only 64 is built", dh);
    RS_REQUIRE((int64_t)B * H <= 65535, RS_ERR_UNSUPPORTED, "B * H is limited to 65535");
    RS_REQUIRE(N <= (1 << 20), RS_ERR_UNSUPPORTED, "N is limited to 2^20");
    RS_REQUIRE(scale > 0.f && scale < INFINITY, RS_ERR_INVALID_ARG, "scale must be positive and finite");
    if (B == 0 || H == 0 || N == 0) return RS_OK;
    RS_REQUIRE(cls_index >= 0 && cls_index < N, RS_ERR_INVALID_ARG, "cls_index %d outside [0, N)", (int)cls_index);
    RS_REQUIRE(q && k && v && o && attn_map, RS_ERR_INVALID_ARG, "q, k, v, o and attn_map must not be NULL");
    RS_REQUIRE(aligned16(q) && aligned16(k) && aligned16(v) && aligned16(o) && aligned16(attn_map), RS_ERR_INVALID_ARG,
               "q, k, v, o and attn_map must be 16-byte aligned");
    RS_REQUIRE(o != q && o != k && o != v, RS_ERR_INVALID_ARG, "o must not alias q, k or v");
    const int64_t st6[6] = {stride_b, stride_n, stride_h, o_stride_b, o_stride_n, o_stride_h};
    for (int i = 0; i < 6; ++i)
        RS_REQUIRE(st6[i] >= 0 && st6[i] % 8 == 0, RS_ERR_INVALID_ARG, "strides must be non-negative multiples of 8 elements");
    RS_REQUIRE(stride_n >= dh && o_stride_n >= dh, RS_ERR_INVALID_ARG, "token stride smaller than dh");
    const AttnMapLayout L = attn_map_layout(B, H, N);
    RS_REQUIRE(workspace_bytes >= L.total, RS_ERR_WORKSPACE_TOO_SMALL,
               "workspace has %zu bytes, rs_attention_map_workspace_size needs %zu", workspace_bytes, L.total);
    RS_REQUIRE(workspace != nullptr && (reinterpret_cast<uintptr_t>(workspace) & 255u) == 0, RS_ERR_INVALID_ARG,
               "workspace must be a 256-byte aligned buffer");
    hipStream_t s = (hipStream_t)hip_stream;
    char* ws = (char*)workspace;
    const int BH = B * H, Np = L.Np;
    RS_LAUNCH_K(K_ATTN, s, launch_attn_pack(q, k, v, ws + L.qh, ws + L.kh, ws + L.vt, B, H, N, Np, stride_b, stride_n, stride_h, s));
    // S = Q K^T per head, written out; then the row softmax in place: the map
    RS_LAUNCH_K(K_ATTN, s, launch_gemm_batched(ws + L.qh, ws + L.kh, attn_map, BH, (int64_t)Np * 64, (int64_t)Np * 64,
                                             (int64_t)N * Np, N, Np, 64, s));
    RS_LAUNCH_K(K_ATTN, s, launch_attn_softmax_rows(attn_map, (int64_t)BH * N, N, Np, scale * 1.44269504088896340736f, s));
    // O = A V per head
    RS_LAUNCH_K(K_ATTN, s, launch_gemm_batched(attn_map, ws + L.vt, ws + L.oh, BH, (int64_t)N * Np, (int64_t)64 * Np,
                                             (int64_t)N * 64, N, 64, Np, s));
    RS_LAUNCH_K(K_ATTN, s, launch_attn_unpack(ws + L.oh, o, B, H, N, o_stride_b, o_stride_n, o_stride_h, s));
    RS_LAUNCH_K(K_SCORE, s, launch_attn_map_scores(attn_map, (float*)(ws + L.partial), s_cls, s_mean, B, H, N, Np, cls_index, s));
    return RS_OK;
}

size_t rs_shift_topk_workspace_size(int32_t B, int32_t N, int32_t D, rs_dtype dtype) {
    (void)B; (void)N; (void)D; (void)dtype;
    return 0;
}

rs_status rs_shift_topk(const void* f_out, const void* f_in, const void* src, int32_t B, int32_t N,
                        int32_t D, int32_t n_prefix, int32_t n_keep, rs_dist dist, rs_dtype dtype,
                        float* scores, int32_t* kept_idx, void* gathered, void* workspace,
                        size_t workspace_bytes, void* hip_stream) {
    (void)workspace;
    RS_REQUIRE(dtype == RS_F32 || dtype == RS_BF16, RS_ERR_INVALID_ARG, "unknown dtype %d", (int)dtype);
    RS_REQUIRE(dist == RS_DIST_L2 || dist == RS_DIST_L1 || dist == RS_DIST_COS, RS_ERR_INVALID_ARG,
               "unknown distance %d", (int)dist);
    RS_REQUIRE(B >= 0 && N >= 0, RS_ERR_INVALID_ARG, "negative B or N");
    RS_REQUIRE(D > 0 && D % 8 == 0, RS_ERR_INVALID_ARG, "D must be a positive multiple of 8");
    RS_REQUIRE(n_prefix >= 0 && n_keep >= 0 && (int64_t)n_prefix + n_keep <= N, RS_ERR_INVALID_ARG,
               "need 0 <= n_prefix, 0 <= n_keep, n_prefix + n_keep <= N");
    RS_REQUIRE((int64_t)B * N < (int64_t)1 << 31, RS_ERR_UNSUPPORTED, "B*N does not fit 31 bits");
    RS_REQUIRE(workspace_bytes >= rs_shift_topk_workspace_size(B, N, D, dtype), RS_ERR_WORKSPACE_TOO_SMALL,
               "workspace too small");
    if (B == 0 || N == 0) return RS_OK;
    RS_REQUIRE(f_out && f_in && scores, RS_ERR_INVALID_ARG, "f_out, f_in and scores must not be NULL");
    RS_REQUIRE(kept_idx || n_prefix + n_keep == 0, RS_ERR_INVALID_ARG, "kept_idx must not be NULL");
    const void* s = src ? src : f_in;
    RS_REQUIRE(aligned16(f_out) && aligned16(f_in) && aligned16(s) && aligned16(gathered), RS_ERR_INVALID_ARG,
               "tensors must be 16-byte aligned");
    RS_REQUIRE(gathered == nullptr || gathered != s, RS_ERR_INVALID_ARG, "gathered must not alias src");
    hipStream_t st = (hipStream_t)hip_stream;
    const int K = n_prefix + n_keep;
    if (gathered && s == f_in && K > 0 && shift_topk_resident_fits(dtype, N, D)) {
        // small images: one pass over memory, the rows to keep never leave the registers
        RS_LAUNCH_K(K_SCORE, st, launch_shift_topk_resident(dtype, dist, f_out, f_in, scores, kept_idx, gathered, B, N, D,
                                                          n_prefix, n_keep, st));
        return RS_OK;
    }
    RS_LAUNCH_K(K_SCORE, st, launch_shift_scores(dtype, dist, f_out, f_in, scores, (int64_t)B * N, D, st));
    RS_LAUNCH_K(K_SELECT, st, launch_select(scores, kept_idx, B, N, n_prefix, n_keep, st));
    if (gathered) RS_LAUNCH_K(K_GATHER, st, launch_gather(dtype, s, kept_idx, gathered, B, N, K, D, st));
    return RS_OK;
}

rs_status rs_grid_line_prune(const void* f_out, const void* f_in, const void* src, int32_t B, int32_t H,
                             int32_t W, int32_t C, int32_t keep_rows, int32_t keep_cols, rs_dist dist,
                             rs_dtype dtype, float* scores, float* row_scores, float* col_scores,
                             int32_t* kept_rows, int32_t* kept_cols, void* gathered, void* hip_stream) {
    RS_REQUIRE(dtype == RS_F32 || dtype == RS_BF16, RS_ERR_INVALID_ARG, "unknown dtype %d", (int)dtype);
    RS_REQUIRE(dist == RS_DIST_L2 || dist == RS_DIST_L1 || dist == RS_DIST_COS, RS_ERR_INVALID_ARG,
               "unknown distance %d", (int)dist);
    RS_REQUIRE(B >= 0 && H >= 0 && W >= 0, RS_ERR_INVALID_ARG, "negative B, H or W");
    RS_REQUIRE(C > 0 && C % 8 == 0, RS_ERR_INVALID_ARG, "C must be a positive multiple of 8");
    RS_REQUIRE(keep_rows >= 0 && keep_rows <= H && keep_cols >= 0 && keep_cols <= W, RS_ERR_INVALID_ARG,
               "need 0 <= keep_rows <= H and 0 <= keep_cols <= W");
    RS_REQUIRE((int64_t)B * H * W < (int64_t)1 << 31, RS_ERR_UNSUPPORTED, "B*H*W does not fit 31 bits");
    if (B == 0 || H == 0 || W == 0) return RS_OK;
    RS_REQUIRE(f_out && f_in && scores && row_scores && col_scores, RS_ERR_INVALID_ARG,
               "f_out, f_in, scores, row_scores and col_scores must not be NULL");
    RS_REQUIRE((kept_rows || keep_rows == 0) && (kept_cols || keep_cols == 0), RS_ERR_INVALID_ARG,
               "kept_rows and kept_cols must not be NULL");
    const void* s = src ? src : f_out;
    RS_REQUIRE(aligned16(f_out) && aligned16(f_in) && aligned16(s) && aligned16(gathered), RS_ERR_INVALID_ARG,
               "tensors must be 16-byte aligned");
    RS_REQUIRE(gathered == nullptr || gathered != s, RS_ERR_INVALID_ARG, "gathered must not alias src");
    hipStream_t st = (hipStream_t)hip_stream;
    RS_LAUNCH_K(K_SCORE, st, launch_shift_scores(dtype, dist, f_out, f_in, scores, (int64_t)B * H * W, C, st));
    RS_LAUNCH_K(K_SCORE, st, launch_grid_line_scores(scores, row_scores, col_scores, B, H, W, st));
    RS_LAUNCH_K(K_SELECT, st, launch_select(row_scores, kept_rows, B, H, 0, keep_rows, st));
    RS_LAUNCH_K(K_SELECT, st, launch_select(col_scores, kept_cols, B, W, 0, keep_cols, st));
    if (gathered)
        RS_LAUNCH_K(K_GATHER, st, launch_grid_gather(dtype, s, kept_rows, kept_cols, gathered, B, H, W, keep_rows,
                                                   keep_cols, C, st));
    return RS_OK;
}

rs_status rs_grid_token_prune(const void* f_out, const void* f_in, const void* src, int32_t B, int32_t H,
                              int32_t W, int32_t C, int32_t keep_rows, int32_t keep_cols, rs_dist dist,
                              rs_dtype dtype, float* scores, int32_t* kept_cols, float* col_scores,
                              int32_t* kept_rows, void* gathered, void* hip_stream) {
    RS_REQUIRE(dtype == RS_F32 || dtype == RS_BF16, RS_ERR_INVALID_ARG, "unknown dtype %d", (int)dtype);
    RS_REQUIRE(dist == RS_DIST_L2 || dist == RS_DIST_L1 || dist == RS_DIST_COS, RS_ERR_INVALID_ARG,
               "unknown distance %d", (int)dist);
    RS_REQUIRE(B >= 0 && H >= 0 && W >= 0, RS_ERR_INVALID_ARG, "negative B, H or W");
    RS_REQUIRE(C > 0 && C % 8 == 0, RS_ERR_INVALID_ARG, "C must be a positive multiple of 8");
    RS_REQUIRE(keep_rows >= 0 && keep_rows <= H && keep_cols >= 0 && keep_cols <= W, RS_ERR_INVALID_ARG,
               "need 0 <= keep_rows <= H and 0 <= keep_cols <= W");
    RS_REQUIRE((int64_t)B * H * W < (int64_t)1 << 31, RS_ERR_UNSUPPORTED, "B*H*W does not fit 31 bits");
    if (B == 0 || H == 0 || W == 0) return RS_OK;
    RS_REQUIRE(f_out && f_in && scores, RS_ERR_INVALID_ARG, "f_out, f_in and scores must not be NULL");
    RS_REQUIRE(kept_cols || keep_cols == 0, RS_ERR_INVALID_ARG, "kept_cols must not be NULL");
    RS_REQUIRE((col_scores && kept_rows) || keep_cols == 0 || keep_rows == 0, RS_ERR_INVALID_ARG,
               "col_scores and kept_rows must not be NULL");
    const void* s = src ? src : f_out;
    RS_REQUIRE(aligned16(f_out) && aligned16(f_in) && aligned16(s) && aligned16(gathered), RS_ERR_INVALID_ARG,
               "tensors must be 16-byte aligned");
    RS_REQUIRE(gathered == nullptr || gathered != s, RS_ERR_INVALID_ARG, "gathered must not alias src");
    hipStream_t st = (hipStream_t)hip_stream;
    RS_LAUNCH_K(K_SCORE, st, launch_shift_scores(dtype, dist, f_out, f_in, scores, (int64_t)B * H * W, C, st));
    if (keep_cols == 0) return RS_OK;
    // step 1: every grid row is one selection problem over its W positions
    RS_LAUNCH_K(K_SELECT, st, launch_select(scores, kept_cols, B * H, W, 0, keep_cols, st));
    if (keep_rows == 0) return RS_OK;
    // step 2: every column of the row-compacted grid is one selection problem over H positions
    RS_LAUNCH_K(K_SCORE, st, launch_grid_compact_scores(scores, kept_cols, col_scores, B, H, W, keep_cols, st));
    RS_LAUNCH_K(K_SELECT, st, launch_select(col_scores, kept_rows, B * keep_cols, H, 0, keep_rows, st));
    if (gathered)
        RS_LAUNCH_K(K_GATHER, st, launch_grid_token_gather(dtype, s, kept_cols, kept_rows, gathered, B, H, W, keep_rows,
                                                         keep_cols, C, st));
    return RS_OK;
}

size_t rs_packed_weights_size(const rs_block_cfg* cfg) {
    if (!cfg || cfg->D <= 0 || cfg->Dm <= 0) return 0;
    return packed_bytes(cfg);
}

static rs_status pack_into(const rs_block_cfg* c, const rs_block_weights* w, void* dst, hipStream_t st) {
    const PackedLayout P = packed_layout(c);
    char* p = (char*)dst;
    const int D = c->D, Dm = c->Dm;
    RS_LAUNCH_K(K_PACK, st, launch_pack_transpose(w->w_qkv, w->ln1_g, p + P.w_qkv, D, 3 * D, st));
    RS_LAUNCH_K(K_PACK, st, launch_pack_transpose(w->w_proj, nullptr, p + P.w_proj, D, D, st));
    RS_LAUNCH_K(K_PACK, st, launch_pack_transpose(w->w_fc1, w->ln2_g, p + P.w_fc1, D, Dm, st));
    RS_LAUNCH_K(K_PACK, st, launch_pack_transpose(w->w_fc2, nullptr, p + P.w_fc2, Dm, D, st));
    RS_LAUNCH_K(K_PACK, st, launch_pack_ln_fold(w->w_qkv, w->ln1_g, w->ln1_b, w->b_qkv, (float*)(p + P.cs_qkv),
                                              (float*)(p + P.b_qkv), D, 3 * D, st));
    RS_LAUNCH_K(K_PACK, st, launch_pack_ln_fold(w->w_fc1, w->ln2_g, w->ln2_b, w->b_fc1, (float*)(p + P.cs_fc1),
                                              (float*)(p + P.b_fc1), D, Dm, st));
    return RS_OK;
}

static rs_status check_weights(const rs_block_weights* w) {
    RS_REQUIRE(w != nullptr, RS_ERR_INVALID_ARG, "weights is NULL");
    RS_REQUIRE(w->w_qkv && w->w_proj && w->w_fc1 && w->w_fc2, RS_ERR_INVALID_ARG,
               "w_qkv, w_proj, w_fc1 and w_fc2 must not be NULL");
    const void* all[] = {w->ln1_g, w->ln1_b, w->w_qkv, w->b_qkv, w->w_proj, w->b_proj, w->ln2_g,
                         w->ln2_b, w->w_fc1, w->b_fc1, w->w_fc2, w->b_fc2, w->packed};
    for (const void* p : all) RS_REQUIRE(aligned16(p), RS_ERR_INVALID_ARG, "weight pointers must be 16-byte aligned");
    return RS_OK;
}

rs_status rs_pack_weights(const rs_block_cfg* cfg, const rs_block_weights* w, void* packed_out,
                          void* hip_stream) {
    RS_REQUIRE(cfg != nullptr, RS_ERR_INVALID_ARG, "cfg is NULL");
    RS_REQUIRE(cfg->D > 0 && cfg->Dm > 0 && cfg->D % 64 == 0 && cfg->Dm % 64 == 0, RS_ERR_INVALID_ARG,
               "D and Dm must be positive multiples of 64");
    RS_REQUIRE(cfg->dtype == RS_F32 || cfg->dtype == RS_BF16, RS_ERR_INVALID_ARG, "unknown dtype");
    rs_status s = check_weights(w);
    if (s != RS_OK) return s;
    if (cfg->dtype == RS_F32) return RS_OK;  // the fp32 path reads the caller's layout
    RS_REQUIRE(packed_out != nullptr && aligned16(packed_out), RS_ERR_INVALID_ARG,
               "packed_out must be a 16-byte aligned buffer");
    return pack_into(cfg, w, packed_out, (hipStream_t)hip_stream);
}

rs_status rs_pack_linear(const void* w, void* wt, int32_t K, int32_t N, rs_dtype dtype, void* hip_stream) {
    RS_REQUIRE(dtype == RS_F32 || dtype == RS_BF16, RS_ERR_INVALID_ARG, "unknown dtype %d", (int)dtype);
    RS_REQUIRE(K > 0 && N > 0, RS_ERR_INVALID_ARG, "K and N must be positive");
    if (dtype == RS_F32) return RS_OK;  // the fp32 path reads the caller's layout
    RS_REQUIRE(w && wt && w != wt, RS_ERR_INVALID_ARG, "w and wt must be distinct non-NULL buffers");
    hipStream_t st = (hipStream_t)hip_stream;
    RS_LAUNCH_K(K_PACK, st, launch_pack_transpose(w, nullptr, wt, K, N, st));
    return RS_OK;
}

rs_status rs_linear_fwd(const void* a, const void* w, const void* bias, const void* res, void* out, int64_t M,
                        int32_t N, int32_t K, rs_epilogue epi, rs_dtype dtype, void* hip_stream) {
    RS_REQUIRE(dtype == RS_F32 || dtype == RS_BF16, RS_ERR_INVALID_ARG, "unknown dtype %d", (int)dtype);
    RS_REQUIRE(epi == RS_EPI_BIAS || epi == RS_EPI_BIAS_GELU || epi == RS_EPI_BIAS_RES, RS_ERR_INVALID_ARG,
               "unknown epilogue %d", (int)epi);
    RS_REQUIRE(M >= 0 && M < ((int64_t)1 << 31), RS_ERR_INVALID_ARG, "M out of range");
    RS_REQUIRE(N > 0 && K > 0, RS_ERR_INVALID_ARG, "N and K must be positive");
    RS_REQUIRE(N % 64 == 0 && K % 64 == 0, RS_ERR_UNSUPPORTED, "N and K must be multiples of 64");
    // a tile's rows are addressed with 32-bit byte offsets from the tile's first row
    RS_REQUIRE(K <= kGemmMaxK && N <= kGemmMaxN, RS_ERR_UNSUPPORTED, "K > %d or N > %d", kGemmMaxK, kGemmMaxN);
    if (M == 0) return RS_OK;
    RS_REQUIRE(a && w && out, RS_ERR_INVALID_ARG, "a, w and out must not be NULL");
    RS_REQUIRE(epi != RS_EPI_BIAS_RES || res, RS_ERR_INVALID_ARG, "res must not be NULL for RS_EPI_BIAS_RES");
    RS_REQUIRE(out != a, RS_ERR_INVALID_ARG, "out must not alias a");
    RS_REQUIRE(aligned16(a) && aligned16(w) && aligned16(bias) && aligned16(res) && aligned16(out),
               RS_ERR_INVALID_ARG, "tensors must be 16-byte aligned");
    hipStream_t st = (hipStream_t)hip_stream;
    const GemmEpilogue e = epi == RS_EPI_BIAS ? EPI_BIAS : epi == RS_EPI_BIAS_GELU ? EPI_BIAS_GELU : EPI_BIAS_RES;
    RS_LAUNCH_K(K_LINEAR, st, launch_gemm(dtype, e, RS_DIST_L2, a, w, bias, res, out, nullptr, nullptr, false, M, N, K, st));
    return RS_OK;
}

size_t rs_block_workspace_size(const rs_block_cfg* cfg) {
    if (check_cfg(cfg) != RS_OK) return 0;
    return block_layout(cfg).total;
}

rs_status rs_block_fwd(const rs_block_cfg* cfg, const rs_block_weights* w, const void* x, void* y,
                       int32_t* kept_idx, float* scores, void* workspace, size_t workspace_bytes,
                       void* hip_stream) {
    return block_fwd(cfg, w, x, y, kept_idx, scores, workspace, workspace_bytes, hip_stream);
}

rs_status rs_block_fwd_chained(const rs_block_cfg* cfg, const rs_block_weights* w, const void* x,
                               const float* x_stats, void* y, float* y_stats, int32_t* kept_idx, float* scores,
                               void* workspace, size_t workspace_bytes, void* hip_stream) {
    return block_fwd(cfg, w, x, y, kept_idx, scores, workspace, workspace_bytes, hip_stream, x_stats, y_stats);
}

rs_status rs_block_fwd_static(const rs_block_cfg* cfg, const rs_block_weights* w, const void* x, void* y,
                              int32_t* kept_idx, float* scores, void* hip_stream) {
    rs_status st = check_cfg(cfg);
    if (st != RS_OK) return st;
    const size_t need = block_layout(cfg).total;
    RS_REQUIRE(need <= kStaticScratchBytes, RS_ERR_UNSUPPORTED,
               "this block needs %zu bytes of scratch, the static buffer holds %zu: use rs_block_fwd with a workspace",
               need, kStaticScratchBytes);
    if (cfg->B == 0 || cfg->N == 0) return RS_OK;
    void* scratch_ptr = nullptr;
    st = static_scratch(&scratch_ptr);
    if (st != RS_OK) return st;
    return block_fwd(cfg, w, x, y, kept_idx, scores, scratch_ptr, kStaticScratchBytes, hip_stream);
}

size_t rs_block_static_scratch_size(void) { return kStaticScratchBytes; }

}  // extern "C"

static rs_status block_fwd(const rs_block_cfg* cfg, const rs_block_weights* w, const void* x, void* y,
                           int32_t* kept_idx, float* scores, void* workspace, size_t workspace_bytes,
                           void* hip_stream, const float* x_stats, float* y_stats) {
    rs_status st = check_cfg(cfg);
    if (st != RS_OK) return st;
    st = check_weights(w);
    if (st != RS_OK) return st;
    const rs_block_cfg& c = *cfg;
    if (c.B == 0 || c.N == 0) return RS_OK;  // nothing to do, nothing touched
    const BlockLayout L = block_layout(cfg);
    RS_REQUIRE(workspace_bytes >= L.total, RS_ERR_WORKSPACE_TOO_SMALL,
               "workspace has %zu bytes, rs_block_workspace_size needs %zu", workspace_bytes, L.total);
    const int K = c.n_prefix + c.n_keep;
    RS_REQUIRE(x != nullptr, RS_ERR_INVALID_ARG, "x is NULL");
    RS_REQUIRE(K == 0 || (y != nullptr && kept_idx != nullptr), RS_ERR_INVALID_ARG, "y and kept_idx must not be NULL");
    RS_REQUIRE(workspace != nullptr, RS_ERR_INVALID_ARG, "workspace is NULL");
    RS_REQUIRE((reinterpret_cast<uintptr_t>(workspace) & 255u) == 0, RS_ERR_INVALID_ARG,
               "workspace must be 256-byte aligned");
    RS_REQUIRE(aligned16(x) && aligned16(y), RS_ERR_INVALID_ARG, "x and y must be 16-byte aligned");
    RS_REQUIRE(x != y, RS_ERR_INVALID_ARG, "y must not alias x");
    {   // the kernels write y, kept_idx and scores while workspace tensors are still being read
        const size_t e = elem_size(c.dtype), M_ = (size_t)c.B * c.N;
        RS_REQUIRE(!overlaps(workspace, L.total, x, M_ * c.D * e) &&
                   !overlaps(workspace, L.total, y, (size_t)c.B * K * c.D * e) &&
                   !overlaps(workspace, L.total, kept_idx, (size_t)c.B * K * sizeof(int32_t)) &&
                   !overlaps(workspace, L.total, scores, M_ * sizeof(float)),
                   RS_ERR_INVALID_ARG, "x, y, kept_idx and scores must lie outside the workspace");
        const size_t ys = (size_t)c.B * K * 2 * sizeof(float);
        RS_REQUIRE(!overlaps(workspace, L.total, x_stats, M_ * 2 * sizeof(float)) && !overlaps(workspace, L.total, y_stats, ys),
                   RS_ERR_INVALID_ARG, "x_stats and y_stats must lie outside the workspace");
        RS_REQUIRE(!overlaps(y_stats, ys, x, M_ * c.D * e) && !overlaps(y_stats, ys, y, (size_t)c.B * K * c.D * e) &&
                   !overlaps(y_stats, ys, kept_idx, (size_t)c.B * K * sizeof(int32_t)) &&
                   !overlaps(y_stats, ys, scores, M_ * sizeof(float)),
                   RS_ERR_INVALID_ARG, "y_stats must not overlap x, y, kept_idx or scores");
        RS_REQUIRE((reinterpret_cast<uintptr_t>(x_stats) & 7u) == 0 && (reinterpret_cast<uintptr_t>(y_stats) & 7u) == 0,
                   RS_ERR_INVALID_ARG, "x_stats and y_stats must be 8-byte aligned");
    }

    hipStream_t s = (hipStream_t)hip_stream;
    char* ws = (char*)workspace;
    const rs_dtype dt = c.dtype;
    const int64_t M = (int64_t)c.B * c.N;
    const int D = c.D, Dm = c.Dm;
    void* u = ws + L.u;
    void* qkv = ws + L.qkv;
    void* att = ws + L.att;
    void* x1 = ws + L.x1;
    void* hid = ws + L.hid;
    float* partials = (float*)(ws + L.partials);
    const bool prune = c.n_keep < c.N - c.n_prefix;
    const bool want_scores = prune || scores != nullptr;
    float* sc = scores ? scores : (float*)(ws + L.scores);

    // weights as the GEMMs read them
    const void *wq = w->w_qkv, *wp = w->w_proj, *w1 = w->w_fc1, *w2 = w->w_fc2;
    GemmLnFold ln1{}, ln2{};
    if (dt == RS_BF16) {
        const char* pk = (const char*)w->packed;
        if (!pk) {
            st = pack_into(cfg, w, ws + L.packed, s);
            if (st != RS_OK) return st;
            pk = ws + L.packed;
        }
        const PackedLayout P = packed_layout(cfg);
        wq = pk + P.w_qkv;
        wp = pk + P.w_proj;
        w1 = pk + P.w_fc1;
        w2 = pk + P.w_fc2;
        float* stats = (float*)(ws + L.stats);
        ln1 = GemmLnFold{x_stats ? x_stats : stats, (const float*)(pk + P.cs_qkv), (const float*)(pk + P.b_qkv)};
        ln2 = GemmLnFold{stats, (const float*)(pk + P.cs_fc1), (const float*)(pk + P.b_fc1)};
    }
    const float scale = c.attn_scale > 0.f ? c.attn_scale : 0.125f;  // 1/sqrt(64)

    // x1 = SA(LN(x)) + x                                                     Eq. (5)
    // bf16: the LayerNorm in front of a GEMM is a pass for the row statistics only; the GEMM reads
    // the raw rows against weights that carry the LayerNorm scale and normalises in its epilogue
    // (a caller that chains blocks hands over the statistics the previous block left for its output)
    if (dt == RS_BF16) {
        if (!x_stats) RS_LAUNCH_K(K_LN, s, launch_rowstats(dt, x, (float*)(ws + L.stats), M, D, c.ln_eps, s));
        RS_LAUNCH_K(K_GEMM_QKV, s, launch_gemm_ln(EPI_LN_BIAS, x, wq, ln1, qkv, M, 3 * D, D, s));
    } else {
        RS_LAUNCH_K(K_LN, s, launch_layernorm(dt, x, w->ln1_g, w->ln1_b, u, M, D, c.ln_eps, s));
        RS_LAUNCH_K(K_GEMM_QKV, s, launch_gemm(dt, EPI_BIAS, RS_DIST_L2, u, wq, w->b_qkv, nullptr, qkv, nullptr, nullptr, false, M, 3 * D, D, s));
    }
    {
        const size_t e = elem_size(dt);
        const char* qp = (const char*)qkv;
        RS_LAUNCH_K(K_ATTN, s, launch_attention(dt, qp, qp + (size_t)D * e, qp + 2 * (size_t)D * e, att, c.B, c.H, c.N,
                                   (int64_t)c.N * 3 * D, 3 * D, 64, (int64_t)c.N * D, D, 64, scale, s));
    }
    // the shift around the attention layer, case (i), comes out of the projection's epilogue
    const bool attn_scores = want_scores && c.op == RS_SHIFT_ATTN;
    RS_LAUNCH_K(K_GEMM_PROJ, s, launch_gemm(dt, attn_scores ? EPI_BIAS_RES_SHIFT : EPI_BIAS_RES, c.dist, att, wp, w->b_proj, x, x1,
                            partials, nullptr, false, M, D, D, s));
    // xhat = MLP(LN(x1)) + x1, with the shift partial sums of D(MLP(LN(x1)), x1)   Eq. (6), Eq. (4)
    const bool need_v = want_scores && c.op == RS_SHIFT_MLP_NORMED;  // LN(x1) itself is an operand of the score
    // a block that keeps every token has kept_idx[b, j] = j: written by the statistics pass on its way
    const bool iota_folded = dt == RS_BF16 && !prune && K > 0;
    if (dt == RS_BF16) {
        RS_LAUNCH_K(K_LN, s, launch_rowstats(dt, x1, (float*)(ws + L.stats), M, D, c.ln_eps, s,
                                             iota_folded ? kept_idx : nullptr, c.N));
        if (need_v) RS_LAUNCH_K(K_LN, s, launch_layernorm(dt, x1, w->ln2_g, w->ln2_b, u, M, D, c.ln_eps, s));
        RS_LAUNCH_K(K_GEMM_FC1, s, launch_gemm_ln(EPI_LN_BIAS_GELU, x1, w1, ln2, hid, M, Dm, D, s));
    } else {
        RS_LAUNCH_K(K_LN, s, launch_layernorm(dt, x1, w->ln2_g, w->ln2_b, u, M, D, c.ln_eps, s));
        RS_LAUNCH_K(K_GEMM_FC1, s, launch_gemm(dt, EPI_BIAS_GELU, RS_DIST_L2, u, w1, w->b_fc1, nullptr, hid, nullptr, nullptr, false, M, Dm, D, s));
    }
    void* xhat = prune ? att : y;  // without pruning the block output goes straight to y
    // every other choice of (f_out, f_in) comes out of fc2's epilogue: f_out is the MLP output or
    // (post) xhat, f_in the residual operand x1 or another tensor still in memory (x, LN(x1))
    const bool fc2_scores = want_scores && !attn_scores;
    const bool post = c.op == RS_SHIFT_BLOCK || c.op == RS_SHIFT_MLP_STREAM;
    const void* ref = c.op == RS_SHIFT_BLOCK ? x : c.op == RS_SHIFT_MLP_NORMED ? (const void*)u : nullptr;
    RS_LAUNCH_K(K_GEMM_FC2, s, launch_gemm(dt, fc2_scores ? EPI_BIAS_RES_SHIFT : EPI_BIAS_RES, c.dist, hid, w2, w->b_fc2, x1,
                          xhat, partials, ref, post, M, D, Dm, s));
    // the survivors' rows, with the LayerNorm statistics the next block needs if the caller asks for them
    auto gather_out = [&]() -> rs_status {
        if (y_stats && gather_stats_fits(dt, D)) {
            RS_LAUNCH_K(K_GATHER, s, launch_gather_stats(xhat, kept_idx, y, y_stats, c.B, c.N, K, D, c.ln_eps, s));
        } else {
            RS_LAUNCH_K(K_GATHER, s, launch_gather(dt, xhat, kept_idx, y, c.B, c.N, K, D, s));
            if (y_stats) RS_LAUNCH_K(K_LN, s, launch_rowstats(dt, y, y_stats, (int64_t)c.B * K, D, c.ln_eps, s));
        }
        return RS_OK;
    };
    if (prune && c.n_keep > 0 && select_from_partials_fits(c.N)) {
        // scores straight from the epilogue's partial sums inside the selection kernel
        RS_LAUNCH_K(K_SELECT, s, launch_select_from_partials(c.dist, partials, L.slots, sc, kept_idx, c.B, c.N, c.n_prefix,
                                                           c.n_keep, s));
        return gather_out();
    }
    if (want_scores) RS_LAUNCH_K(K_SCORE, s, launch_finalize_scores(c.dist, partials, L.slots, sc, M, s));
    // keep the n_keep highest-shift tokens (plus the prefix) and compact them
    if (!iota_folded) RS_LAUNCH_K(K_SELECT, s, launch_select(sc, kept_idx, c.B, c.N, c.n_prefix, c.n_keep, s));
    if (prune) return gather_out();
    if (y_stats) RS_LAUNCH_K(K_LN, s, launch_rowstats(dt, y, y_stats, M, D, c.ln_eps, s));
    return RS_OK;
}
