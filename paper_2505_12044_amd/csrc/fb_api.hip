// C-ABI entry points: argument validation and kernel selection.  No device work happens
// here beyond enqueueing kernels on the caller's stream.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstring>

#include "../../include/flashbias.h"
#include "fb_launch.h"
#include "fb_params.h"

namespace {

std::atomic<int> g_fwd_qb{0};   // 0 = choose automatically
std::atomic<int> g_causal_up{1};

// Scratch of the allocation-free entry point: one copy per GPU, resident from module load.  In
// host code the array's name is only a handle for hipGetSymbolAddress; kernels get the device
// address obtained there.
}  // namespace
static __device__ __align__(256) unsigned char scratch[FB_STATIC_SCRATCH_BYTES];
namespace {
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device; resolved once per device (racing first
// calls store the same value).  Returns nullptr on failure.
void* static_scratch() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (ptr != nullptr) return ptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return nullptr;
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);
    return ptr;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int padded_rank(int R, fb_dtype dtype, fb_dtype phi_dtype) {
    if (R == 0) return 0;
    const int cols = (dtype == FB_BF16 && phi_dtype == FB_F32) ? 6 * R : R;
    return (cols + 15) / 16 * 16;
}

// What the kernels' indexing needs: every offset above the head level is 64-bit; row and
// work-unit counters (B H N rows, B H ceil(N / 128) tiles, launch grids) are 32-bit; byte
// offsets inside one head's rows (N C bf16 / fp32 elements, N R factor values) are 32-bit.
int check_common(int B, int H, int N, int C, int R) {
    if (B <= 0 || H <= 0 || N <= 0 || R < 0) return FB_ERR_SHAPE;
    if ((long long)B * H * N >= (1LL << 31)) return FB_ERR_SHAPE;
    if ((long long)N * C * 4 >= (1LL << 32)) return FB_ERR_SHAPE;
    if ((long long)N * R * 4 >= (1LL << 32)) return FB_ERR_SHAPE;
    if (C != 16 && C != 32 && C != 64 && C != 128) return FB_ERR_UNSUPPORTED;
    return FB_OK;
}

// Multiplicative bias: widest block of extra channels C (R - 1) the kernels are instantiated
// for.  C = 128 takes none beyond R = 1: its score operand already fills the registers that
// two waves per SIMD leave (C + 64 columns is the widest instantiation there).
int mulbias_max_rest(int C) { return C <= 64 ? 128 : 0; }

// Padded width of a block of `rest` bf16 extra channels: multiples of 16 up to 64, then 96, 128.
int mulbias_padded(int rest) { return rest <= 64 ? (rest + 15) / 16 * 16 : (rest <= 96 ? 96 : 128); }

int pick_qb(int B, int H, int N, int C, int rp, bool dense, bool causal) {
    const int forced = g_fwd_qb.load(std::memory_order_relaxed);
    if (forced == 1 || forced == 2 || forced == 8 || forced == 16) return forced;
    (void)rp;
    // (the eight-wave ping-pong kernel, fwd_qb = 8, was the choice for long non-causal C = 128
    // sequences until the four-wave kernel got compile-time ring slots and early K operand reads:
    // 2.00 ms against 2.14 ms on B 2, H 8, N 16384)
    // (the direct-to-LDS kernel, fwd_qb = 16, was the choice for short C = 32 sequences; the four-wave
    // kernel is now 6 % faster there: 0.070 ms against 0.074 ms on B 384, H 4, N 384)
    // Two query blocks per wave halve the LDS traffic per MFMA but double the accumulator
    // registers: they fit the 256-register budget (two waves per SIMD) only for C <= 64, and
    // only pay when 256-row tiles still leave every CU several workgroups.
    if (C == 128 || dense) return 1;
    if (N % 256 != 0 && N < 1024) return 1;
    // (measured: from four full rounds of 512 resident workgroups on; for full attention over
    // long sequences from two)
    const long long tiles256 = (long long)B * H * ((N + 255) / 256);
    if (tiles256 >= 2048) return 2;
    return (!causal && N >= 2048 && tiles256 >= 1000) ? 2 : 1;
}

}  // namespace

#pragma GCC visibility push(default)
extern "C" {

int fb_version(void) { return 100; }

const char* fb_status_string(int status) {
    switch (status) {
        case FB_OK: return "ok";
        case FB_ERR_NULL: return "required pointer is NULL";
        case FB_ERR_SHAPE: return "invalid shape";
        case FB_ERR_UNSUPPORTED: return "unsupported C / R / dtype combination";
        case FB_ERR_ALIGN: return "pointer not 16-byte aligned";
        case FB_ERR_WORKSPACE: return "workspace missing or too small";
        case FB_ERR_LAUNCH: return "kernel launch failed";
        case FB_ERR_TOO_LARGE: return "problem exceeds the static scratch of the allocation-free entry point";
        default: return "unknown status";
    }
}

int fb_tune_set(const char* name, int value) {
    if (name == nullptr) return FB_ERR_NULL;
    if (std::strcmp(name, "fwd_qb") == 0) {
        if (value != 0 && value != 1 && value != 2 && value != 8 && value != 16) return FB_ERR_SHAPE;
        g_fwd_qb.store(value, std::memory_order_relaxed);
        return FB_OK;
    }
    if (std::strcmp(name, "fwd_causal_up") == 0) {
        if (value != 0 && value != 1) return FB_ERR_SHAPE;
        g_causal_up.store(value, std::memory_order_relaxed);
        return FB_OK;
    }
    return FB_ERR_UNSUPPORTED;
}

// Shared by the self-attention (M = N) and cross-attention entry points.
static int lowrank_fwd_impl(const void* q, const void* k, const void* v,
                            const void* phi_q, const void* phi_k, void* out, float* lse,
                            int B, int H, int N, int M, int C, int R, int causal,
                            fb_dtype dtype, fb_dtype phi_dtype, int phi_batch_broadcast,
                            float scale, void* stream) {
    if (!q || !k || !v || !out || !lse) return FB_ERR_NULL;
    if (int st = check_common(B, H, N > M ? N : M, C, R)) return st;
    if (N <= 0 || M <= 0) return FB_ERR_SHAPE;
    if (R > 0 && (!phi_q || !phi_k)) return FB_ERR_NULL;
    if (dtype != FB_F32 && dtype != FB_BF16) return FB_ERR_UNSUPPORTED;
    if (phi_dtype != FB_F32 && phi_dtype != FB_BF16) return FB_ERR_UNSUPPORTED;
    if (dtype == FB_F32 && R > 0 && phi_dtype != FB_F32) return FB_ERR_UNSUPPORTED;
    if (N != M && causal) return FB_ERR_UNSUPPORTED;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(lse))
        return FB_ERR_ALIGN;
    if (R > 0 && (!aligned16(phi_q) || !aligned16(phi_k))) return FB_ERR_ALIGN;
    const int rp = padded_rank(R, dtype, phi_dtype);
    if (rp > 64) return FB_ERR_UNSUPPORTED;

    FwdParams p{};
    p.q = q; p.k = k; p.v = v; p.phi_q = phi_q; p.phi_k = phi_k; p.bias = nullptr;
    p.out = out; p.lse = lse;
    p.B = B; p.H = H; p.N = N; p.M = M; p.R = R; p.causal = causal != 0;
    p.phi_f32 = phi_dtype == FB_F32;
    p.phi_bstride = phi_batch_broadcast ? 0 : (long long)H * N * R;
    p.phik_bstride = phi_batch_broadcast ? 0 : (long long)H * M * R;
    p.bias_bstride = 0;
    p.causal_up = g_causal_up.load(std::memory_order_relaxed);
    p.scale = scale > 0.f ? scale : 1.0f / std::sqrt((float)C);
    p.inv_scale = 1.0f / p.scale;
    int rc;
    if (dtype == FB_F32) {
        rc = fb_launch_fwd_f32(p, C, false, (hipStream_t)stream);
    } else {
        int qb = pick_qb(B, H, N, C, rp, false, causal != 0);
        if (N != M && qb != 2) qb = 1;     // only the four-wave kernel takes N != M
        rc = fb_launch_fwd_bf16(p, C, rp, false, qb, (hipStream_t)stream);
    }
    return rc == 0 ? FB_OK : (rc < 0 ? FB_ERR_UNSUPPORTED : FB_ERR_LAUNCH);
}

int fb_lowrank_attn_fwd(const void* q, const void* k, const void* v,
                        const void* phi_q, const void* phi_k, void* out, float* lse,
                        int B, int H, int N, int C, int R, int causal,
                        fb_dtype dtype, fb_dtype phi_dtype, int phi_batch_broadcast,
                        float scale, void* stream) {
    return lowrank_fwd_impl(q, k, v, phi_q, phi_k, out, lse, B, H, N, N, C, R, causal, dtype, phi_dtype,
                            phi_batch_broadcast, scale, stream);
}

int fb_lowrank_xattn_fwd(const void* q, const void* k, const void* v,
                         const void* phi_q, const void* phi_k, void* out, float* lse,
                         int B, int H, int N, int M, int C, int R,
                         fb_dtype dtype, fb_dtype phi_dtype, int phi_batch_broadcast,
                         float scale, void* stream) {
    return lowrank_fwd_impl(q, k, v, phi_q, phi_k, out, lse, B, H, N, M, C, R, 0, dtype, phi_dtype,
                            phi_batch_broadcast, scale, stream);
}

int fb_dense_bias_attn_fwd(const void* q, const void* k, const void* v, const void* bias,
                           void* out, float* lse, int B, int H, int N, int C, int causal,
                           fb_dtype dtype, int bias_batch_broadcast, float scale, void* stream) {
    if (!q || !k || !v || !bias || !out || !lse) return FB_ERR_NULL;
    if (int st = check_common(B, H, N, C, 0)) return st;
    if (dtype != FB_F32 && dtype != FB_BF16) return FB_ERR_UNSUPPORTED;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(bias) || !aligned16(out) ||
        !aligned16(lse))
        return FB_ERR_ALIGN;

    FwdParams p{};
    p.q = q; p.k = k; p.v = v; p.phi_q = nullptr; p.phi_k = nullptr; p.bias = bias;
    p.out = out; p.lse = lse;
    p.B = B; p.H = H; p.N = N; p.M = N; p.R = 0; p.causal = causal != 0;
    p.phi_f32 = 0;
    p.phi_bstride = 0;
    p.phik_bstride = 0;
    p.bias_bstride = bias_batch_broadcast ? 0 : (long long)H * N * N;
    p.causal_up = g_causal_up.load(std::memory_order_relaxed);
    p.scale = scale > 0.f ? scale : 1.0f / std::sqrt((float)C);
    p.inv_scale = 1.0f / p.scale;
    int rc;
    if (dtype == FB_F32) rc = fb_launch_fwd_f32(p, C, true, (hipStream_t)stream);
    else rc = fb_launch_fwd_bf16(p, C, 0, true, pick_qb(B, H, N, C, 0, true, causal != 0), (hipStream_t)stream);
    return rc == 0 ? FB_OK : (rc < 0 ? FB_ERR_UNSUPPORTED : FB_ERR_LAUNCH);
}

int fb_alibi_attn_fwd(const void* q, const void* k, const void* v, const float* slopes,
                      void* out, float* lse, int B, int H, int N, int C, int causal,
                      fb_dtype dtype, float scale, void* stream) {
    if (!q || !k || !v || !slopes || !out || !lse) return FB_ERR_NULL;
    if (int st = check_common(B, H, N, C, 2)) return st;
    if (dtype != FB_BF16) return FB_ERR_UNSUPPORTED;
    if (N > (1 << 24)) return FB_ERR_UNSUPPORTED;          // positions are carried as fp32 integers
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(lse))
        return FB_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(slopes) & 3u) != 0) return FB_ERR_ALIGN;

    FwdParams p{};
    p.q = q; p.k = k; p.v = v; p.phi_q = nullptr; p.phi_k = nullptr; p.slopes = slopes;
    p.bias = nullptr; p.out = out; p.lse = lse;
    p.B = B; p.H = H; p.N = N; p.M = N; p.R = 2; p.causal = causal != 0;
    p.phi_f32 = 1;
    p.phi_bstride = 0;
    p.phik_bstride = 0;
    p.bias_bstride = 0;
    p.causal_up = g_causal_up.load(std::memory_order_relaxed);
    p.scale = scale > 0.f ? scale : 1.0f / std::sqrt((float)C);
    p.inv_scale = 1.0f / p.scale;
    int qb = pick_qb(B, H, N, C, 16, false, causal != 0);
    if (qb != 2) qb = 1;     // only the four-wave kernel generates factors
    const int rc = fb_launch_fwd_bf16_alibi(p, C, qb, (hipStream_t)stream);
    return rc == 0 ? FB_OK : (rc < 0 ? FB_ERR_UNSUPPORTED : FB_ERR_LAUNCH);
}

size_t fb_lowrank_mulbias_attn_fwd_workspace_bytes(int B, int H, int N, int C, int R, fb_dtype dtype) {
    (void)dtype;
    if (B <= 0 || H <= 0 || N <= 0 || C <= 0 || R <= 0) return 0;
    return (size_t)2 * B * H * N * C * R * 2;     // q' and k' rows of C R bf16 channels
}

int fb_lowrank_mulbias_attn_fwd(const void* q, const void* k, const void* v,
                                const void* phi_q, const void* phi_k, void* out, float* lse,
                                int B, int H, int N, int C, int R, int causal,
                                fb_dtype dtype, fb_dtype phi_dtype, int phi_batch_broadcast,
                                float scale, void* workspace, size_t workspace_bytes, void* stream) {
    if (!q || !k || !v || !phi_q || !phi_k || !out || !lse) return FB_ERR_NULL;
    if (R <= 0) return FB_ERR_SHAPE;
    if (int st = check_common(B, H, N, C, R)) return st;
    if ((long long)B * H * N * (long long)C * R >= (1LL << 38)) return FB_ERR_SHAPE;   // pre-pass grid: one thread per 8 channels
    if (dtype != FB_BF16) return FB_ERR_UNSUPPORTED;
    if (phi_dtype != FB_F32 && phi_dtype != FB_BF16) return FB_ERR_UNSUPPORTED;
    const int rest = C * (R - 1);                  // channels beyond the first repeat
    if (rest > mulbias_max_rest(C)) return FB_ERR_UNSUPPORTED;
    const void* ptrs[] = {q, k, v, out, lse};
    for (const void* ptr : ptrs) if (!aligned16(ptr)) return FB_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(phi_q) & 3u) != 0 || (reinterpret_cast<uintptr_t>(phi_k) & 3u) != 0)
        return FB_ERR_ALIGN;
    if (!workspace || workspace_bytes < fb_lowrank_mulbias_attn_fwd_workspace_bytes(B, H, N, C, R, dtype))
        return FB_ERR_WORKSPACE;
    if (!aligned16(workspace)) return FB_ERR_ALIGN;

    const size_t rows = (size_t)B * H * N;
    unsigned char* ws = (unsigned char*)workspace;
    void* qh = ws;                                  // [rows][C]
    void* kh = ws + rows * C * 2;                   // [rows][C]
    void* qr = ws + rows * C * 4;                   // [rows][C (R-1)]
    void* kr = ws + rows * C * 4 + rows * rest * 2;
    const float sc = scale > 0.f ? scale : 1.0f / std::sqrt((float)C);
    const long long pbs = phi_batch_broadcast ? 0 : (long long)H * N * R;
    const int f32 = phi_dtype == FB_F32;
    if (fb_launch_mulbias_prep(q, phi_q, qh, qr, B, (long long)H * N, C, R, f32, pbs, sc, (hipStream_t)stream) ||
        fb_launch_mulbias_prep(k, phi_k, kh, kr, B, (long long)H * N, C, R, f32, pbs, 1.0f, (hipStream_t)stream))
        return FB_ERR_LAUNCH;

    FwdParams p{};
    p.q = qh; p.k = kh; p.v = v; p.phi_q = rest ? qr : nullptr; p.phi_k = rest ? kr : nullptr; p.bias = nullptr;
    p.out = out; p.lse = lse;
    p.B = B; p.H = H; p.N = N; p.M = N; p.R = rest; p.causal = causal != 0;
    p.phi_f32 = 0;
    p.phi_bstride = (long long)H * N * rest;
    p.phik_bstride = (long long)H * N * rest;
    p.bias_bstride = 0;
    p.causal_up = g_causal_up.load(std::memory_order_relaxed);
    p.scale = 1.0f;                                 // already folded into q'
    p.inv_scale = 1.0f / p.scale;
    const int rp = mulbias_padded(rest);
    int qb = pick_qb(B, H, N, C, rp, false, causal != 0);
    if (rp > 64) qb = 1;                           // wide blocks: four-wave kernel, one query block per wave
    const int rc = fb_launch_fwd_bf16(p, C, rp, false, qb, (hipStream_t)stream);
    return rc == 0 ? FB_OK : (rc < 0 ? FB_ERR_UNSUPPORTED : FB_ERR_LAUNCH);
}

size_t fb_lowrank_mulbias_attn_bwd_workspace_bytes(int B, int H, int N, int C, int R, fb_dtype dtype) {
    (void)dtype;
    if (B <= 0 || H <= 0 || N <= 0 || C <= 0 || R <= 0) return 0;
    const long long rows = (long long)B * H * N;
    // q', k' (C R bf16 channels each), their gradients (float) and the additive backward's own scratch
    return (size_t)2 * rows * C * R * (2 + 4) + fb_bwd_workspace_bytes(rows, rows, C, C * (R - 1));
}

int fb_lowrank_mulbias_attn_bwd(const void* q, const void* k, const void* v,
                                const void* phi_q, const void* phi_k,
                                const void* out, const float* lse, const void* dout,
                                void* dq, void* dk, void* dv, void* dphi_q, void* dphi_k,
                                int B, int H, int N, int C, int R, int causal,
                                fb_dtype dtype, fb_dtype phi_dtype, int phi_batch_broadcast,
                                float scale, void* workspace, size_t workspace_bytes, void* stream) {
    if (!q || !k || !v || !phi_q || !phi_k || !out || !lse || !dout || !dq || !dk || !dv || !dphi_q || !dphi_k)
        return FB_ERR_NULL;
    if (R <= 0) return FB_ERR_SHAPE;
    if (int st = check_common(B, H, N, C, R)) return st;
    if ((long long)B * H * N * (long long)C * R >= (1LL << 38)) return FB_ERR_SHAPE;   // pre-pass grid: one thread per 8 channels
    if (dtype != FB_BF16) return FB_ERR_UNSUPPORTED;
    if (phi_dtype != FB_F32 && phi_dtype != FB_BF16) return FB_ERR_UNSUPPORTED;
    const int rest = C * (R - 1);
    if (rest > mulbias_max_rest(C)) return FB_ERR_UNSUPPORTED;
    const void* ptrs[] = {q, k, v, out, lse, dout, dq, dk, dv};
    for (const void* ptr : ptrs) if (!aligned16(ptr)) return FB_ERR_ALIGN;
    const void* p4[] = {phi_q, phi_k, dphi_q, dphi_k};
    for (const void* ptr : p4) if ((reinterpret_cast<uintptr_t>(ptr) & 3u) != 0) return FB_ERR_ALIGN;
    if (!workspace || workspace_bytes < fb_lowrank_mulbias_attn_bwd_workspace_bytes(B, H, N, C, R, dtype))
        return FB_ERR_WORKSPACE;
    if (!aligned16(workspace)) return FB_ERR_ALIGN;

    const size_t rows = (size_t)B * H * N;
    const size_t head_b = rows * C * 2, rest_b = rows * (size_t)rest * 2;
    unsigned char* ws = (unsigned char*)workspace;
    void* qh = ws;                 void* kh = ws + head_b;
    void* qr = ws + 2 * head_b;    void* kr = ws + 2 * head_b + rest_b;
    // gradients in the same order, as float: dq, dphi_q are sums over them, so the main kernels
    // must not round them to bf16 first
    unsigned char* g = ws + 2 * head_b + 2 * rest_b;
    void* dqh = g;                     void* dkh = g + 2 * head_b;
    void* dqr = g + 4 * head_b;        void* dkr = g + 4 * head_b + 2 * rest_b;
    void* inner = g + 4 * head_b + 4 * rest_b;
    const float sc = scale > 0.f ? scale : 1.0f / std::sqrt((float)C);
    const long long pbs = phi_batch_broadcast ? 0 : (long long)H * N * R;
    const int f32 = phi_dtype == FB_F32;
    hipStream_t st = (hipStream_t)stream;
    if (fb_launch_mulbias_prep(q, phi_q, qh, qr, B, (long long)H * N, C, R, f32, pbs, sc, st) ||
        fb_launch_mulbias_prep(k, phi_k, kh, kr, B, (long long)H * N, C, R, f32, pbs, 1.0f, st))
        return FB_ERR_LAUNCH;

    BwdParams p{};
    p.q = qh; p.k = kh; p.v = v; p.phi_q = rest ? qr : nullptr; p.phi_k = rest ? kr : nullptr;
    p.out = out; p.lse = lse; p.dout = dout;
    p.dq = dqh; p.dk = dkh; p.dv = dv; p.dphi_q = rest ? dqr : nullptr; p.dphi_k = rest ? dkr : nullptr;
    p.workspace = inner;
    p.B = B; p.H = H; p.N = N; p.M = N; p.R = rest; p.Cg = C; p.causal = causal != 0;
    p.phi_f32 = 0;
    p.grad_f32 = 1;
    p.phi_bstride = (long long)H * N * rest;
    p.phik_bstride = (long long)H * N * rest;
    p.scale = 1.0f;                // folded into q'
    const int rc = fb_launch_bwd_bf16(p, C, mulbias_padded(rest), st);
    if (rc != 0) return rc < 0 ? FB_ERR_UNSUPPORTED : FB_ERR_LAUNCH;
    if (fb_launch_mulbias_fold(q, phi_q, dqh, dqr, dq, dphi_q, B, (long long)H * N, C, R, f32, pbs, sc, st) ||
        fb_launch_mulbias_fold(k, phi_k, dkh, dkr, dk, dphi_k, B, (long long)H * N, C, R, f32, pbs, 1.0f, st))
        return FB_ERR_LAUNCH;
    return FB_OK;
}

static size_t bwd_ws_impl(int B, int H, int N, int M, int C, int R) {
    if (B <= 0 || H <= 0 || N <= 0 || M <= 0) return 0;
    // (lse * log2 e, D) per query row and the concatenated operand rows [q*scale | phi_q], [k | phi_k]
    return fb_bwd_workspace_bytes((long long)B * H * N, (long long)B * H * M, C, R);
}

static int lowrank_bwd_impl(const void* q, const void* k, const void* v,
                            const void* phi_q, const void* phi_k,
                            const void* out, const float* lse, const void* dout,
                            void* dq, void* dk, void* dv, void* dphi_q, void* dphi_k,
                            int B, int H, int N, int M, int C, int R, int causal,
                            fb_dtype dtype, fb_dtype phi_dtype, int phi_batch_broadcast,
                            float scale, void* workspace, size_t workspace_bytes, void* stream) {
    if (!q || !k || !v || !out || !lse || !dout || !dq || !dk || !dv) return FB_ERR_NULL;
    if (int st = check_common(B, H, N > M ? N : M, C, R)) return st;
    if (N <= 0 || M <= 0) return FB_ERR_SHAPE;
    if (R > 0 && (!phi_q || !phi_k)) return FB_ERR_NULL;       // dphi_q / dphi_k may be NULL: not wanted
    if (dtype != FB_BF16 && dtype != FB_F32) return FB_ERR_UNSUPPORTED;
    if (phi_dtype != FB_F32 && phi_dtype != FB_BF16) return FB_ERR_UNSUPPORTED;
    if (dtype == FB_F32 && R > 0 && phi_dtype != FB_F32) return FB_ERR_UNSUPPORTED;
    if (N != M && causal) return FB_ERR_UNSUPPORTED;
    const void* ptrs[] = {q, k, v, out, lse, dout, dq, dk, dv};
    for (const void* ptr : ptrs) if (!aligned16(ptr)) return FB_ERR_ALIGN;
    if (R > 0 && (!aligned16(phi_q) || !aligned16(phi_k) || !aligned16(dphi_q) || !aligned16(dphi_k)))
        return FB_ERR_ALIGN;                                    // a NULL gradient pointer counts as aligned
    const int rp = padded_rank(R, dtype, phi_dtype);
    if (rp > 64) return FB_ERR_UNSUPPORTED;
    if (!workspace || workspace_bytes < bwd_ws_impl(B, H, N, M, C, R)) return FB_ERR_WORKSPACE;
    if (!aligned16(workspace)) return FB_ERR_ALIGN;

    BwdParams p{};
    p.q = q; p.k = k; p.v = v; p.phi_q = phi_q; p.phi_k = phi_k;
    p.out = out; p.lse = lse; p.dout = dout;
    p.dq = dq; p.dk = dk; p.dv = dv; p.dphi_q = dphi_q; p.dphi_k = dphi_k;
    p.workspace = workspace;
    p.B = B; p.H = H; p.N = N; p.M = M; p.R = R; p.Cg = C; p.causal = causal != 0;
    p.phi_f32 = phi_dtype == FB_F32;
    p.phi_bstride = phi_batch_broadcast ? 0 : (long long)H * N * R;
    p.phik_bstride = phi_batch_broadcast ? 0 : (long long)H * M * R;
    p.scale = scale > 0.f ? scale : 1.0f / std::sqrt((float)C);
    const int rc = dtype == FB_F32 ? fb_launch_bwd_f32(p, C, (hipStream_t)stream)
                                   : fb_launch_bwd_bf16(p, C, rp, (hipStream_t)stream);
    return rc == 0 ? FB_OK : (rc < 0 ? FB_ERR_UNSUPPORTED : FB_ERR_LAUNCH);
}

size_t fb_alibi_attn_bwd_workspace_bytes(int B, int H, int N, int C, fb_dtype dtype) {
    (void)dtype;
    return bwd_ws_impl(B, H, N, N, C, 2);
}

int fb_alibi_attn_bwd(const void* q, const void* k, const void* v, const float* slopes,
                      const void* out, const float* lse, const void* dout,
                      void* dq, void* dk, void* dv, float* dslope_rows,
                      int B, int H, int N, int C, int causal, fb_dtype dtype, float scale,
                      void* workspace, size_t workspace_bytes, void* stream) {
    if (!q || !k || !v || !slopes || !out || !lse || !dout || !dq || !dk || !dv) return FB_ERR_NULL;
    if (int st = check_common(B, H, N, C, 2)) return st;
    if (dtype != FB_BF16) return FB_ERR_UNSUPPORTED;
    if (N > (1 << 24)) return FB_ERR_UNSUPPORTED;          // positions are carried as fp32 integers
    const void* ptrs[] = {q, k, v, out, lse, dout, dq, dk, dv};
    for (const void* ptr : ptrs) if (!aligned16(ptr)) return FB_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(slopes) & 3u) != 0) return FB_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(dslope_rows) & 3u) != 0) return FB_ERR_ALIGN;     // NULL: not wanted
    if (!workspace || workspace_bytes < bwd_ws_impl(B, H, N, N, C, 2)) return FB_ERR_WORKSPACE;
    if (!aligned16(workspace)) return FB_ERR_ALIGN;

    BwdParams p{};
    p.q = q; p.k = k; p.v = v; p.phi_q = nullptr; p.phi_k = nullptr; p.slopes = slopes;
    p.out = out; p.lse = lse; p.dout = dout;
    p.dq = dq; p.dk = dk; p.dv = dv; p.dphi_q = nullptr; p.dphi_k = nullptr;
    p.dslope = dslope_rows;
    p.workspace = workspace;
    p.B = B; p.H = H; p.N = N; p.M = N; p.R = 2; p.Cg = C; p.causal = causal != 0;
    p.phi_f32 = 1;
    p.phi_bstride = 0;
    p.phik_bstride = 0;
    p.scale = scale > 0.f ? scale : 1.0f / std::sqrt((float)C);
    const int rc = fb_launch_bwd_bf16(p, C, 16, (hipStream_t)stream);
    return rc == 0 ? FB_OK : (rc < 0 ? FB_ERR_UNSUPPORTED : FB_ERR_LAUNCH);
}

size_t fb_dense_bias_attn_bwd_workspace_bytes(int B, int H, int N, int C, fb_dtype dtype) {
    (void)dtype;
    return bwd_ws_impl(B, H, N, N, C, 0);
}

int fb_dense_bias_attn_bwd(const void* q, const void* k, const void* v, const void* bias,
                           const void* out, const float* lse, const void* dout,
                           void* dq, void* dk, void* dv, void* dbias,
                           int B, int H, int N, int C, int causal,
                           fb_dtype dtype, int bias_batch_broadcast, float scale,
                           void* workspace, size_t workspace_bytes, void* stream) {
    if (!q || !k || !v || !bias || !out || !lse || !dout || !dq || !dk || !dv || !dbias) return FB_ERR_NULL;
    if (int st = check_common(B, H, N, C, 0)) return st;
    if ((long long)B * H * N * (long long)N >= (1LL << 40)) return FB_ERR_SHAPE;
    if (dtype != FB_BF16 && dtype != FB_F32) return FB_ERR_UNSUPPORTED;
    if (dtype == FB_BF16 && (N % 8) != 0) return FB_ERR_UNSUPPORTED;      // bf16 bias rows are copied in 16-byte pieces
    const void* ptrs[] = {q, k, v, bias, out, lse, dout, dq, dk, dv, dbias};
    for (const void* ptr : ptrs) if (!aligned16(ptr)) return FB_ERR_ALIGN;
    if (!workspace || workspace_bytes < bwd_ws_impl(B, H, N, N, C, 0)) return FB_ERR_WORKSPACE;
    if (!aligned16(workspace)) return FB_ERR_ALIGN;

    BwdParams p{};
    p.q = q; p.k = k; p.v = v; p.phi_q = nullptr; p.phi_k = nullptr;
    p.out = out; p.lse = lse; p.dout = dout;
    p.dq = dq; p.dk = dk; p.dv = dv; p.dphi_q = nullptr; p.dphi_k = nullptr;
    p.bias = bias; p.dbias = dbias;
    p.bias_bstride = bias_batch_broadcast ? 0 : (long long)H * N * N;
    p.workspace = workspace;
    p.B = B; p.H = H; p.N = N; p.M = N; p.R = 0; p.Cg = C; p.causal = causal != 0;
    p.phi_f32 = 0;
    p.phi_bstride = 0;
    p.phik_bstride = 0;
    p.scale = scale > 0.f ? scale : 1.0f / std::sqrt((float)C);
    const int rc = dtype == FB_F32 ? fb_launch_bwd_dense_f32(p, C, (hipStream_t)stream)
                                   : fb_launch_bwd_dense_bf16(p, C, (hipStream_t)stream);
    return rc == 0 ? FB_OK : (rc < 0 ? FB_ERR_UNSUPPORTED : FB_ERR_LAUNCH);
}

size_t fb_lowrank_attn_bwd_workspace_bytes(int B, int H, int N, int C, int R, fb_dtype dtype) {
    (void)dtype;
    return bwd_ws_impl(B, H, N, N, C, R);
}

size_t fb_lowrank_xattn_bwd_workspace_bytes(int B, int H, int N, int M, int C, int R, fb_dtype dtype) {
    (void)dtype;
    return bwd_ws_impl(B, H, N, M, C, R);
}

int fb_lowrank_attn_bwd(const void* q, const void* k, const void* v,
                        const void* phi_q, const void* phi_k,
                        const void* out, const float* lse, const void* dout,
                        void* dq, void* dk, void* dv, void* dphi_q, void* dphi_k,
                        int B, int H, int N, int C, int R, int causal,
                        fb_dtype dtype, fb_dtype phi_dtype, int phi_batch_broadcast,
                        float scale, void* workspace, size_t workspace_bytes, void* stream) {
    return lowrank_bwd_impl(q, k, v, phi_q, phi_k, out, lse, dout, dq, dk, dv, dphi_q, dphi_k, B, H, N, N, C, R,
                            causal, dtype, phi_dtype, phi_batch_broadcast, scale, workspace, workspace_bytes,
                            stream);
}

int fb_lowrank_attn_bwd_noalloc(const void* q, const void* k, const void* v,
                                const void* phi_q, const void* phi_k,
                                const void* out, const float* lse, const void* dout,
                                void* dq, void* dk, void* dv, void* dphi_q, void* dphi_k,
                                int B, int H, int N, int C, int R, int causal,
                                fb_dtype dtype, fb_dtype phi_dtype, int phi_batch_broadcast,
                                float scale, void* stream) {
    // shape errors first (the size query is meaningless for them), then the size limit
    if (int st = check_common(B, H, N, C, R)) return st;
    const size_t need = bwd_ws_impl(B, H, N, N, C, R);
    if (need > FB_STATIC_SCRATCH_BYTES) return FB_ERR_TOO_LARGE;
    void* ws = static_scratch();
    if (ws == nullptr) return FB_ERR_LAUNCH;
    return lowrank_bwd_impl(q, k, v, phi_q, phi_k, out, lse, dout, dq, dk, dv, dphi_q, dphi_k, B, H, N, N, C, R,
                            causal, dtype, phi_dtype, phi_batch_broadcast, scale, ws, FB_STATIC_SCRATCH_BYTES,
                            stream);
}

int fb_lowrank_xattn_bwd(const void* q, const void* k, const void* v,
                         const void* phi_q, const void* phi_k,
                         const void* out, const float* lse, const void* dout,
                         void* dq, void* dk, void* dv, void* dphi_q, void* dphi_k,
                         int B, int H, int N, int M, int C, int R,
                         fb_dtype dtype, fb_dtype phi_dtype, int phi_batch_broadcast,
                         float scale, void* workspace, size_t workspace_bytes, void* stream) {
    return lowrank_bwd_impl(q, k, v, phi_q, phi_k, out, lse, dout, dq, dk, dv, dphi_q, dphi_k, B, H, N, M, C, R,
                            0, dtype, phi_dtype, phi_batch_broadcast, scale, workspace, workspace_bytes,
                            stream);
}

}  // extern "C"
#pragma GCC visibility pop
