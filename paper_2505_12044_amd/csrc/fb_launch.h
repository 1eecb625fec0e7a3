// Internal launchers (one per kernel family); defined in the matching .hip file.
// Each returns 0 on success, 1 when the HIP runtime rejected the launch, -1 when the
// requested shape has no instantiation.
#ifndef FB_LAUNCH_H_
#define FB_LAUNCH_H_

#include <hip/hip_runtime.h>

#include <atomic>

#include "fb_params.h"

int fb_launch_fwd_f32(const FwdParams& p, int C, bool dense, hipStream_t stream);
int fb_launch_fwd_bf16(const FwdParams& p, int C, int rp, bool dense, int qb, hipStream_t stream);
// ALiBi factors generated in the kernel from p.slopes (p.phi_q / p.phi_k unused); qb = 1 or 2.
int fb_launch_fwd_bf16_alibi(const FwdParams& p, int C, int qb, hipStream_t stream);
// p.workspace points at fb_bwd_workspace_bytes(B*H*N, B*H*M, C, R) bytes of device scratch.
int fb_launch_bwd_bf16(const BwdParams& p, int C, int rp, hipStream_t stream);
size_t fb_bwd_workspace_bytes(long long rows_q, long long rows_k, int C, int R);
// fp32 tensors and fp32 factors (N = M): p.workspace holds one float per query row (a prefix of the
// size above).
int fb_launch_bwd_f32(const BwdParams& p, int C, hipStream_t stream);
int fb_launch_bwd_dense_f32(const BwdParams& p, int C, hipStream_t stream);
// Dense-bias backward (p.bias, p.dbias, p.bias_bstride set; p.R = 0; workspace as above with R = 0).
int fb_launch_bwd_dense_bf16(const BwdParams& p, int C, hipStream_t stream);

// Multiplicative bias pre-pass: head[row][C] = x * phi[:, 0] * mul, rest[row][C (R-1)] = the other
// repeats, bf16, for the B * rows_per_batch rows of x (rows_per_batch = H * sequence length);
// phi is [Bp, rows_per_batch, R] with phi_bstride elements between batch items (0 when shared).
int fb_launch_mulbias_prep(const void* x, const void* phi, void* head, void* rest, int B, long long rows_per_batch,
                           int C, int R, int phi_f32, long long phi_bstride, float mul, hipStream_t stream);

// Multiplicative bias backward fold: dx[row][C] = mul * sum_r phi_r g_r, dphi[row][R] = mul * sum_c x_c g_r,c
// from g_head [rows][C], g_rest [rows][C (R-1)] (float gradients of the reweighted repeats); dphi is per batch element.
int fb_launch_mulbias_fold(const void* x, const void* phi, const void* g_head, const void* g_rest, void* dx,
                           void* dphi, int B, long long rows_per_batch, int C, int R, int phi_f32,
                           long long phi_bstride, float mul, hipStream_t stream);

// A kernel's dynamic-LDS limit is an attribute of the (kernel, device) pair: raise it on the
// first launch on each device.  Racing first launches all set the same value; the flag is
// published only after the attribute call has returned.
constexpr int kFbMaxDevices = 64;
struct FbLdsOnce { std::atomic<bool> done[kFbMaxDevices] = {}; };
inline bool fb_raise_lds_limit(const void* kern, size_t bytes, FbLdsOnce& once) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    const bool tracked = dev >= 0 && dev < kFbMaxDevices;
    if (tracked && once.done[dev].load(std::memory_order_acquire)) return true;
    if (hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess) return false;
    if (tracked) once.done[dev].store(true, std::memory_order_release);
    return true;
}

#endif
