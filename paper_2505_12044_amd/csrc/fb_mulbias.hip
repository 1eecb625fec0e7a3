// Multiplicative low-rank bias (FlashBias App. I): softmax((q k^T / sqrt(C)) o (phi_q phi_k^T)) v
// equals plain attention on the reweighted repeats
//   q' = [q o phi_q,1 | ... | q o phi_q,R],  k' = [k o phi_k,1 | ... | k o phi_k,R]   (C R channels)
// with the scale of the ORIGINAL C.  This file holds the pre-pass that writes q' (with the
// scale folded in) and k' as bf16 rows, split into the first C channels and the remaining
// C (R - 1): the forward kernels then take the first part as their q / k operand and the rest
// as "factor" columns of the same contraction, so no kernel of its own is needed.
#include <hip/hip_runtime.h>

#include "fb_device.h"
#include "fb_launch.h"

namespace {

// One thread per 16-byte piece (8 channels) of one repeat r of one row.
__global__ __launch_bounds__(256) void mulbias_prep_kernel(const bf16_t* __restrict__ x, const void* __restrict__ phi,
                                                           bf16_t* __restrict__ head, bf16_t* __restrict__ rest,
                                                           long long rows, long long rows_per_batch, int C, int R,
                                                           int phi_f32, long long phi_bstride, float mul) {
    const int cpr = C / 8;                                   // pieces per repeat
    const long long gid = (long long)blockIdx.x * 256 + threadIdx.x;
    const long long row = gid / (cpr * R);
    if (row >= rows) return;
    const int rem = (int)(gid - row * (cpr * R));
    const int r = rem / cpr, c8 = rem - r * cpr;
    const long long bb = row / rows_per_batch;
    const long long poff = bb * phi_bstride + (row - bb * rows_per_batch) * R + r;
    const float f = (phi_f32 ? ((const float*)phi)[poff] : (float)((const bf16_t*)phi)[poff]) * mul;
    const bf16x8 a = as_bf16x8(*(const u32x4*)(x + row * C + c8 * 8));
    bf16x8 o;
#pragma unroll
    for (int e = 0; e < 8; e++) o[e] = (bf16_t)((float)a[e] * f);
    bf16_t* dst = r == 0 ? head + row * C + c8 * 8 : rest + row * (long long)(C * (R - 1)) + (r - 1) * C + c8 * 8;
    *(u32x4*)dst = as_uint4(o);
}

// Backward fold.  g_head [rows][C] and g_rest [rows][C (R-1)] (float: the backward kernels leave
// them unrounded, because every output here is a sum over them) hold dL/dx' for the reweighted
// repeats x' = [x phi_1 mul | ... | x phi_R mul]; the chain rule gives
//   dx[c]     = mul * sum_r phi_r * g[r][c]        (one thread per 8 channels)
//   dphi[r]   = mul * sum_c x[c]  * g[r][c]        (thread c8 == 0 of each row, after a row-wide sum)
// Threads of one row are consecutive lanes (C / 8 <= 16 of them), so the channel sum of dphi is a
// shuffle reduction.
__global__ __launch_bounds__(256) void mulbias_fold_kernel(const bf16_t* __restrict__ x, const void* __restrict__ phi,
                                                           const float* __restrict__ g_head,
                                                           const float* __restrict__ g_rest,
                                                           bf16_t* __restrict__ dx, void* __restrict__ dphi,
                                                           long long rows, long long rows_per_batch, int C, int R,
                                                           int phi_f32, long long phi_bstride, float mul) {
    const int cpr = C / 8;                                   // threads per row: 2, 4, 8 or 16
    const long long gid = (long long)blockIdx.x * 256 + threadIdx.x;
    const long long row = gid / cpr;
    const int c8 = (int)(gid - row * cpr);
    const bool live = row < rows;
    const long long rw = live ? row : rows - 1;              // idle lanes shadow the last row (shuffles stay uniform)
    const long long bb = rw / rows_per_batch;
    const long long poff = bb * phi_bstride + (rw - bb * rows_per_batch) * R;
    const bf16x8 xv = as_bf16x8(*(const u32x4*)(x + rw * C + c8 * 8));
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; e++) acc[e] = 0.f;
    for (int r = 0; r < R; r++) {
        const float* gp = r == 0 ? g_head + rw * C + c8 * 8 : g_rest + rw * (long long)(C * (R - 1)) + (r - 1) * C + c8 * 8;
        const f32x4 g0 = *(const f32x4*)gp, g1 = *(const f32x4*)(gp + 4);
        const float gv[8] = {g0[0], g0[1], g0[2], g0[3], g1[0], g1[1], g1[2], g1[3]};
        const float f = phi_f32 ? ((const float*)phi)[poff + r] : (float)((const bf16_t*)phi)[poff + r];
        float dot = 0.f;
#pragma unroll
        for (int e = 0; e < 8; e++) {
            const float ge = gv[e];
            acc[e] = fmaf(f, ge, acc[e]);
            dot = fmaf((float)xv[e], ge, dot);
        }
        for (int off = cpr / 2; off > 0; off >>= 1) dot += __shfl_xor(dot, off);
        if (live && c8 == 0) {
            const long long o = row * R + r;                 // gradients are per batch element
            if (phi_f32) ((float*)dphi)[o] = dot * mul;
            else ((bf16_t*)dphi)[o] = (bf16_t)(dot * mul);
        }
    }
    if (live) {
        bf16x8 o;
#pragma unroll
        for (int e = 0; e < 8; e++) o[e] = (bf16_t)(acc[e] * mul);
        *(u32x4*)(dx + row * C + c8 * 8) = as_uint4(o);
    }
}

}  // namespace

int fb_launch_mulbias_fold(const void* x, const void* phi, const void* g_head, const void* g_rest, void* dx,
                           void* dphi, int B, long long rows_per_batch, int C, int R, int phi_f32,
                           long long phi_bstride, float mul, hipStream_t stream) {
    const long long rows = (long long)B * rows_per_batch;
    const long long threads = rows * (C / 8);
    hipLaunchKernelGGL(mulbias_fold_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, stream,
                       (const bf16_t*)x, phi, (const float*)g_head, (const float*)g_rest, (bf16_t*)dx, dphi, rows,
                       rows_per_batch, C, R, phi_f32, phi_bstride, mul);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int fb_launch_mulbias_prep(const void* x, const void* phi, void* head, void* rest, int B, long long rows_per_batch,
                           int C, int R, int phi_f32, long long phi_bstride, float mul, hipStream_t stream) {
    const long long rows = (long long)B * rows_per_batch;
    const long long threads = rows * (C / 8) * R;
    hipLaunchKernelGGL(mulbias_prep_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, stream,
                       (const bf16_t*)x, phi, (bf16_t*)head, (bf16_t*)rest, rows, rows_per_batch, C, R, phi_f32,
                       phi_bstride, mul);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}
