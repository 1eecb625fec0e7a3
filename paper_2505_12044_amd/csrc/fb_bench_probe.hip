// Bench-only probes, built into their own library (libfb_bench_probe.so): nothing in the product
// path links or calls them.  bench.py uses them to quote measured ceilings next to the vendor peaks.
//
//   fbp_mfma_loop : back-to-back v_mfma_f32_32x32x16_bf16 on every SIMD, no memory traffic; the
//                   rate it sustains is the practical ceiling of any bf16 MFMA kernel on this chip
//                   at the clock the chip holds under matrix load.
//   fbp_copy      : plain 16-byte-per-lane copy of a known size, the calibration kernel for the
//                   FETCH_SIZE / WRITE_SIZE counters (rocprofv3 --pmc) and a measured HBM stream rate.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kChains = 4;          // independent accumulation chains per wave
constexpr int kMfmaPerIter = 16;

__global__ __launch_bounds__(256) void mfma_loop_kernel(float* out, int iters) {
    bf16x8 a, b;
    for (int e = 0; e < 8; e++) {
        a[e] = (__bf16)(threadIdx.x * 0.001f + e);
        b[e] = (__bf16)(0.5f + e * 0.01f);
    }
    f32x16 acc[kChains];
    for (int c = 0; c < kChains; c++)
        for (int r = 0; r < 16; r++) acc[c][r] = 0.f;
    for (int i = 0; i < iters; i++) {
#pragma unroll
        for (int rep = 0; rep < kMfmaPerIter / kChains; rep++)
#pragma unroll
            for (int c = 0; c < kChains; c++) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[c], 0, 0, 0);
    }
    float s = 0.f;
    for (int c = 0; c < kChains; c++)
        for (int r = 0; r < 16; r++) s += acc[c][r];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n16) {
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace

#pragma GCC visibility push(default)
extern "C" {

// out: device buffer of blocks * 256 floats.  One workgroup = 4 waves = one per SIMD of a CU.
// Executes blocks * 4 * iters * 16 MFMAs of 32768 flop each.  Returns 0, or 1 on a bad argument /
// rejected launch.
int fbp_mfma_loop(float* out, int blocks, int iters, void* stream) {
    if (out == nullptr || blocks <= 0 || iters <= 0) return 1;
    hipLaunchKernelGGL(mfma_loop_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, out, iters);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

double fbp_mfma_loop_flop(int blocks, int iters) { return (double)blocks * 4.0 * iters * kMfmaPerIter * 32768.0; }

// Copies bytes (a multiple of 16) from src to dst, both 16-byte aligned device pointers.
int fbp_copy(const void* src, void* dst, size_t bytes, void* stream) {
    if (src == nullptr || dst == nullptr || bytes == 0 || (bytes & 15) != 0) return 1;
    if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15u) return 1;
    hipLaunchKernelGGL(copy_kernel, dim3(256 * 16), dim3(256), 0, (hipStream_t)stream, (const u32x4*)src, (u32x4*)dst,
                       bytes / 16);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

}  // extern "C"
#pragma GCC visibility pop
