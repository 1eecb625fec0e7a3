// fp32 forward: attention with a factorised or dense additive bias, all arithmetic in fp32
// FMA (gfx950's fp32 matrix rate equals its fp32 vector rate, so there is nothing to gain
// from MFMA here).  This is the full-precision path (tolerance 1e-4 against float64).
//
// One thread owns one query row: [q*scale | phi_q] and the output accumulator live in
// registers; key/value tiles are staged in LDS and read by all lanes at the same address
// (a broadcast, conflict-free).  Scores of a tile are [q*scale | phi_q] . [k | phi_k]
// (FlashBias Eq. 3) followed by an online softmax over tiles.
// Every global access is coalesced: the query rows, the output rows and the dense bias tile
// pass through LDS (consecutive lanes touch consecutive addresses in memory, and a thread
// then picks up or drops its own row in LDS), 32 rows at a time.
#include <hip/hip_runtime.h>

#include "fb_launch.h"
#include "fb_params.h"

namespace {

constexpr int kThreads = 128;  // queries per workgroup
constexpr int kTK = 32;        // keys per LDS tile

template <int C, int RP, bool DENSE>
__global__ __launch_bounds__(kThreads) void fwd_f32_kernel(FwdParams p) {
    constexpr int W = C + RP;
    constexpr int WP = W | 1;          // odd pitch: a thread-per-row walk over the tile is conflict-free
    __shared__ float ks[kTK][WP];
    __shared__ float vs[kTK][C];
    __shared__ float bs[DENSE ? kThreads : 1][kTK + 1];     // dense mode: bias tile of this block's rows

    const int tid = threadIdx.x;
    const int bh = blockIdx.x / p.n_qtiles;
    const int qt = blockIdx.x % p.n_qtiles;
    const int b = bh / p.H, h = bh % p.H;
    const int N = p.N, M = p.M, R = p.R;      // N queries, M keys (M = N unless cross-attention)
    const int i = qt * kThreads + tid;
    const bool valid = i < N;

    const size_t base = (size_t)bh * N * C;
    const size_t kbase = (size_t)bh * M * C;
    const float* qg = (const float*)p.q + base;
    const float* kg = (const float*)p.k + kbase;
    const float* vg = (const float*)p.v + kbase;
    const float* pqg = nullptr;
    const float* pkg = nullptr;
    if (RP > 0) {
        pqg = (const float*)p.phi_q + (size_t)b * p.phi_bstride + (size_t)h * N * R;
        pkg = (const float*)p.phi_k + (size_t)b * p.phik_bstride + (size_t)h * M * R;
    }
    const float* bg = nullptr;
    if (DENSE) bg = (const float*)p.bias + (size_t)b * p.bias_bstride + (size_t)h * N * M;

    float qr[W];
    float o[C];
    // query rows [q*scale | phi_q | 0], 32 at a time through the K tile buffer
    static_assert(kTK == 32 && kThreads % 32 == 0, "row chunks of 32");
    for (int ch = 0; ch < kThreads / 32; ch++) {
        __syncthreads();
        for (int e = tid; e < 32 * W; e += kThreads) {
            const int rr = e / W, c = e % W;
            const int row = qt * kThreads + ch * 32 + rr;
            float x = 0.f;
            if (row < N) {
                if (c < C) x = qg[(size_t)row * C + c] * p.scale;
                else if (c - C < R) x = pqg[(size_t)row * R + (c - C)];
            }
            ks[rr][c] = x;
        }
        __syncthreads();
        if (tid / 32 == ch) {
#pragma unroll
            for (int c = 0; c < W; c++) qr[c] = ks[tid % 32][c];
        }
    }
#pragma unroll
    for (int c = 0; c < C; c++) o[c] = 0.f;

    float m = -INFINITY, l = 0.f;
    const int n_keys = p.causal ? min(M, (qt + 1) * kThreads) : M;

    for (int j0 = 0; j0 < n_keys; j0 += kTK) {
        __syncthreads();
        for (int e = tid; e < kTK * W; e += kThreads) {
            const int jj = e / W, c = e % W;
            const int j = j0 + jj;
            float x = 0.f;
            if (j < M) {
                if (c < C) x = kg[(size_t)j * C + c];
                else if (c - C < R) x = pkg[(size_t)j * R + (c - C)];
            }
            ks[jj][c] = x;
        }
        for (int e = tid; e < kTK * C; e += kThreads) {
            const int jj = e / C, c = e % C;
            const int j = j0 + jj;
            vs[jj][c] = j < M ? vg[(size_t)j * C + c] : 0.f;
        }
        if (DENSE) {
            for (int e = tid; e < kThreads * kTK; e += kThreads) {
                const int rr = e / kTK, jj = e % kTK;
                const int row = qt * kThreads + rr, j = j0 + jj;
                bs[rr][jj] = (row < N && j < M) ? bg[(size_t)row * M + j] : 0.f;
            }
        }
        __syncthreads();

        float s[kTK];
        float mt = -INFINITY;
#pragma unroll
        for (int jj = 0; jj < kTK; jj++) {
            float acc = 0.f;
#pragma unroll
            for (int c = 0; c < W; c++) acc = fmaf(qr[c], ks[jj][c], acc);
            const int j = j0 + jj;
            if (DENSE) acc += bs[tid][jj];
            if (j >= M || (p.causal && j > i)) acc = -INFINITY;
            s[jj] = acc;
            mt = fmaxf(mt, acc);
        }
        const float m_new = fmaxf(m, mt);
        const float alpha = expf(m - m_new);
        l *= alpha;
#pragma unroll
        for (int c = 0; c < C; c++) o[c] *= alpha;
#pragma unroll
        for (int jj = 0; jj < kTK; jj++) {
            const float pj = expf(s[jj] - m_new);
            l += pj;
#pragma unroll
            for (int c = 0; c < C; c++) o[c] = fmaf(pj, vs[jj][c], o[c]);
        }
        m = m_new;
    }

    const float inv = 1.f / l;
    if (valid) p.lse[(size_t)bh * N + i] = m + logf(l);
    // output rows, 32 at a time through the V tile buffer
    for (int ch = 0; ch < kThreads / 32; ch++) {
        __syncthreads();
        if (tid / 32 == ch) {
#pragma unroll
            for (int c = 0; c < C; c++) vs[tid % 32][c] = o[c] * inv;
        }
        __syncthreads();
        for (int e = tid; e < 32 * C; e += kThreads) {
            const int rr = e / C, c = e % C;
            const int row = qt * kThreads + ch * 32 + rr;
            if (row < N) ((float*)p.out)[base + (size_t)row * C + c] = vs[rr][c];
        }
    }
}

template <int C, int RP, bool DENSE>
int launch(const FwdParams& p, hipStream_t stream) {
    FwdParams q = p;
    q.n_qtiles = (p.N + kThreads - 1) / kThreads;
    q.total_tiles = p.B * p.H * q.n_qtiles;
    hipLaunchKernelGGL((fwd_f32_kernel<C, RP, DENSE>), dim3(q.total_tiles), dim3(kThreads), 0, stream, q);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

template <int C>
int dispatch_c(const FwdParams& p, bool dense, hipStream_t stream) {
    if (dense) return launch<C, 0, true>(p, stream);
    if (p.R == 0) return launch<C, 0, false>(p, stream);
    if (p.R <= 8) return launch<C, 8, false>(p, stream);
    if (p.R <= 32) return launch<C, 32, false>(p, stream);
    return launch<C, 64, false>(p, stream);
}

}  // namespace

// Returns 0 on success, 1 on launch failure, -1 when no instantiation fits.
int fb_launch_fwd_f32(const FwdParams& p, int C, bool dense, hipStream_t stream) {
    if (p.R > 64) return -1;
    switch (C) {
        case 16: return dispatch_c<16>(p, dense, stream);
        case 32: return dispatch_c<32>(p, dense, stream);
        case 64: return dispatch_c<64>(p, dense, stream);
        case 128: return dispatch_c<128>(p, dense, stream);
        default: return -1;
    }
}
