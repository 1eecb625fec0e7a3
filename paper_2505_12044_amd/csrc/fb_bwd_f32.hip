// fp32 backward of attention with a factorised additive bias: all arithmetic in fp32 FMA, the
// full-precision companion of fb_fwd_f32.hip (gfx950's fp32 matrix rate equals its fp32 vector
// rate, so there is nothing to gain from MFMA here).
//
// With S = [q*scale | phi_q] . [k | phi_k]^T (FlashBias Eq. 3), P = exp(S - lse) and
// D_i = sum_c dout_ic out_ic, the gradient of the scores is dS = P o (dout V^T - D), and
//   [dq / scale | dphi_q] = dS   [k | phi_k]          (query-side kernel, one pass over the keys)
//   [dk | dphi_k]         = dS^T [q*scale | phi_q]    (key-side kernel, one pass over the queries)
//   dv                    = P^T  dout
// so the factor gradients are the trailing R columns of the contractions that give dq and dk
// (Sec. 3.2 "Speed up training").  Nothing N x N is stored; each kernel recomputes S from the
// operand rows.  Deterministic: every output element is summed by one thread in a fixed order.
//
// Work split: a workgroup of 256 threads owns 64 rows (queries in the first kernel, keys in the
// second), four threads per row, thread t of a row holding the channels c = t (mod 4) of the row's
// operands and accumulators (at most (2 (C + RP) + 2 C) / 4 = 160 registers of state).  The rows
// of the other side pass through LDS in tiles of 32; all threads read the same tile row at the
// same time (a broadcast), and the two dot products of a score are finished with two
// cross-lane additions.  The query-side kernel also writes D (one float per query row) into the
// caller's workspace for the key-side kernel, which runs after it on the same stream.
#include <hip/hip_runtime.h>

#include "fb_launch.h"
#include "fb_params.h"

namespace {

constexpr int kThreads = 256;
constexpr int kRows = kThreads / 4;   // rows per workgroup
constexpr int kTile = 32;             // rows of the other side per LDS tile

__device__ __forceinline__ float quad_sum(float x) {
    x += __shfl_xor(x, 1);
    x += __shfl_xor(x, 2);
    return x;
}

// KEYSIDE = false: rows are queries, tiles are keys; outputs dq, dphi_q, D (and dBias when DENSE).
// KEYSIDE = true:  rows are keys, tiles are queries; outputs dk, dv, dphi_k.
// DENSE: the bias is a materialised [N, M] matrix per head, added to the scores (the training-side
// baseline of Sec. 4.3); its gradient dBias = dS is written by the query-side pass, zero where masked.
template <int C, int RP, bool KEYSIDE, bool DENSE = false>
__global__ __launch_bounds__(kThreads) void bwd_f32_kernel(BwdParams p, float* __restrict__ Dws) {
    constexpr int W = C + RP;
    constexpr int WQ = W / 4, CQ = C / 4;
    static_assert(W % 4 == 0 && C % 4 == 0, "four threads per row");
    __shared__ float ts[kTile][W + 1];       // tile rows [x | phi] of the other side (queries: x = q*scale)
    __shared__ float tv[kTile][C + 1];       // tile rows v (query side) or dout (key side)
    __shared__ float tl[kTile], td[kTile];   // key side: lse and D of the tile's queries
    // dense bias of (this workgroup's rows) x (the tile's rows): [own row][tile row] on the query side,
    // [tile row][own row] on the key side, so that both are filled along the key index (coalesced)
    __shared__ float tb[DENSE ? (KEYSIDE ? kTile : kRows) : 1][DENSE ? (KEYSIDE ? kRows : kTile) + 1 : 1];

    const int tid = threadIdx.x;
    const int t = tid & 3;
    const int bh = blockIdx.x / p.n_tiles;
    const int rt = blockIdx.x % p.n_tiles;
    const int b = bh / p.H, h = bh % p.H;
    const int N = p.N, M = p.M, R = p.R;       // N queries, M keys (M = N unless cross-attention)
    const int NL = KEYSIDE ? M : N;            // rows on this kernel's own side
    const int NO = KEYSIDE ? N : M;            // rows on the streamed side
    const int row = rt * kRows + (tid >> 2);
    const bool valid = row < NL;
    const int rowc = valid ? row : NL - 1;    // clamped: finite values, never stored

    const size_t base = (size_t)bh * N * C;    // query-side tensors
    const size_t kbase = (size_t)bh * M * C;   // key-side tensors
    const float* qg = (const float*)p.q + base;
    const float* kg = (const float*)p.k + kbase;
    const float* vg = (const float*)p.v + kbase;
    const float* og = (const float*)p.out + base;
    const float* dog = (const float*)p.dout + base;
    const float* lseg = p.lse + (size_t)bh * N;
    float* Dg = Dws + (size_t)bh * N;
    const float* bg = nullptr;
    float* dbg = nullptr;
    if (DENSE) {
        bg = (const float*)p.bias + (size_t)b * p.bias_bstride + (size_t)h * N * M;
        dbg = (float*)p.dbias + (size_t)bh * N * M;
    }
    const float* pqg = nullptr;
    const float* pkg = nullptr;
    if (RP > 0) {
        pqg = (const float*)p.phi_q + (size_t)b * p.phi_bstride + (size_t)h * N * R;
        pkg = (const float*)p.phi_k + (size_t)b * p.phik_bstride + (size_t)h * M * R;
    }

    // this thread's channels of its row: a[u] <-> column t + 4u of [x | phi], e[u] <-> channel t + 4u
    float a[WQ], e[CQ];
    float acc_a[WQ], acc_e[KEYSIDE ? CQ : 1];
    float lse_r = 0.f, d_r = 0.f;
#pragma unroll
    for (int u = 0; u < WQ; u++) {
        const int c = t + 4 * u;
        float x = 0.f;
        if (c < C) x = KEYSIDE ? kg[(size_t)rowc * C + c] : qg[(size_t)rowc * C + c] * p.scale;
        else if (c - C < R) x = KEYSIDE ? pkg[(size_t)rowc * R + (c - C)] : pqg[(size_t)rowc * R + (c - C)];
        a[u] = x;
        acc_a[u] = 0.f;
    }
#pragma unroll
    for (int u = 0; u < CQ; u++) {
        const int c = t + 4 * u;
        e[u] = KEYSIDE ? vg[(size_t)rowc * C + c] : dog[(size_t)rowc * C + c];
        if (KEYSIDE) acc_e[u] = 0.f;
    }
    if (!KEYSIDE) {
        float part = 0.f;
#pragma unroll
        for (int u = 0; u < CQ; u++) part = fmaf(e[u], og[(size_t)rowc * C + t + 4 * u], part);
        d_r = quad_sum(part);
        lse_r = lseg[rowc];
        if (valid && t == 0) Dg[row] = d_r;
    }

    // range of the other side this workgroup's rows can see
    int o_begin = 0, o_end = NO;
    if (p.causal) {                                              // (N = M)
        if (KEYSIDE) o_begin = (rt * kRows / kTile) * kTile;      // queries i >= j
        else o_end = min(NO, (rt + 1) * kRows);                  // keys j <= i
    }

    for (int o0 = o_begin; o0 < o_end; o0 += kTile) {
        __syncthreads();
        for (int x = tid; x < kTile * W; x += kThreads) {
            const int rr = x / W, c = x % W;
            const int orow = o0 + rr;
            float val = 0.f;
            if (orow < NO) {
                if (c < C) val = KEYSIDE ? qg[(size_t)orow * C + c] * p.scale : kg[(size_t)orow * C + c];
                else if (c - C < R) val = KEYSIDE ? pqg[(size_t)orow * R + (c - C)] : pkg[(size_t)orow * R + (c - C)];
            }
            ts[rr][c] = val;
        }
        for (int x = tid; x < kTile * C; x += kThreads) {
            const int rr = x / C, c = x % C;
            const int orow = o0 + rr;
            tv[rr][c] = orow < NO ? (KEYSIDE ? dog[(size_t)orow * C + c] : vg[(size_t)orow * C + c]) : 0.f;
        }
        if (KEYSIDE && tid < kTile) {
            const int orow = o0 + tid;
            tl[tid] = orow < NO ? lseg[orow] : 0.f;
            td[tid] = orow < NO ? Dg[orow] : 0.f;
        }
        if (DENSE) {
            if (KEYSIDE) {       // tb[query of the tile][key of this workgroup]
                for (int x = tid; x < kTile * kRows; x += kThreads) {
                    const int rr = x / kRows, cc = x % kRows;
                    const int qi = o0 + rr, kj = rt * kRows + cc;
                    tb[rr][cc] = (qi < N && kj < M) ? bg[(size_t)qi * M + kj] : 0.f;
                }
            } else {             // tb[query of this workgroup][key of the tile]
                for (int x = tid; x < kRows * kTile; x += kThreads) {
                    const int rr = x / kTile, cc = x % kTile;
                    const int qi = rt * kRows + rr, kj = o0 + cc;
                    tb[rr][cc] = (qi < N && kj < M) ? bg[(size_t)qi * M + kj] : 0.f;
                }
            }
        }
        __syncthreads();

#pragma unroll 2
        for (int rr = 0; rr < kTile; rr++) {
            const int orow = o0 + rr;
            float sp = 0.f, dpp = 0.f;
#pragma unroll
            for (int u = 0; u < WQ; u++) sp = fmaf(a[u], ts[rr][t + 4 * u], sp);
#pragma unroll
            for (int u = 0; u < CQ; u++) dpp = fmaf(e[u], tv[rr][t + 4 * u], dpp);
            float s = quad_sum(sp);
            if (DENSE) s += KEYSIDE ? tb[rr][tid >> 2] : tb[tid >> 2][rr];
            const float dp = quad_sum(dpp);     // dout_i . v_j
            // query i and key j of this pair
            const int qi = KEYSIDE ? orow : row;
            const int kj = KEYSIDE ? row : orow;
            const bool live = orow < NO && valid && !(p.causal && kj > qi);
            const float lse_i = KEYSIDE ? tl[rr] : lse_r;
            const float d_i = KEYSIDE ? td[rr] : d_r;
            const float pr = live ? expf(s - lse_i) : 0.f;
            const float ds = pr * (dp - d_i);
            // dBias = dS: the four threads of a row take turns over the tile's keys
            if (DENSE && !KEYSIDE && valid && orow < NO && (rr & 3) == t) dbg[(size_t)row * M + orow] = ds;
#pragma unroll
            for (int u = 0; u < WQ; u++) acc_a[u] = fmaf(ds, ts[rr][t + 4 * u], acc_a[u]);
            if (KEYSIDE) {
#pragma unroll
                for (int u = 0; u < CQ; u++) acc_e[u] = fmaf(pr, tv[rr][t + 4 * u], acc_e[u]);
            }
        }
    }

    if (DENSE && !KEYSIDE && p.causal) {
        // the keys past this workgroup's last query were never visited: their dBias entries are zero
        const int k0 = ((o_end + kTile - 1) / kTile) * kTile;
        const int w = M - k0;
        if (w > 0) {
            for (long long x = tid; x < (long long)kRows * w; x += kThreads) {
                const int rr = (int)(x / w), cc = (int)(x % w);
                const int qi = rt * kRows + rr;
                if (qi < N) dbg[(size_t)qi * M + k0 + cc] = 0.f;
            }
        }
    }
    if (!valid) return;
    float* dxg = (float*)(KEYSIDE ? p.dk : p.dq) + (KEYSIDE ? kbase : base);
    float* dphig = (float*)(KEYSIDE ? p.dphi_k : p.dphi_q);      // [B,H,N or M,R], per batch element; may be NULL
    if (dphig) dphig += (size_t)bh * NL * R;
#pragma unroll
    for (int u = 0; u < WQ; u++) {
        const int c = t + 4 * u;
        // the tile rows carried q*scale (key side) resp. k (query side): dk = dS^T (q*scale), dq = scale dS k
        if (c < C) dxg[(size_t)row * C + c] = KEYSIDE ? acc_a[u] : acc_a[u] * p.scale;
        else if (c - C < R && dphig) dphig[(size_t)row * R + (c - C)] = acc_a[u];
    }
    if (KEYSIDE) {
        float* dvg = (float*)p.dv + kbase;
#pragma unroll
        for (int u = 0; u < CQ; u++) dvg[(size_t)row * C + t + 4 * u] = acc_e[u];
    }
}

template <int C, int RP>
int launch(const BwdParams& pin, hipStream_t stream) {
    BwdParams p = pin;
    float* Dws = (float*)p.workspace;
    p.n_tiles = (p.N + kRows - 1) / kRows;         // query-side pass: tiles of query rows
    p.total_tiles = p.B * p.H * p.n_tiles;
    hipLaunchKernelGGL((bwd_f32_kernel<C, RP, false>), dim3(p.total_tiles), dim3(kThreads), 0, stream, p, Dws);
    if (hipGetLastError() != hipSuccess) return 1;
    p.n_tiles = (p.M + kRows - 1) / kRows;         // key-side pass: tiles of key rows
    p.total_tiles = p.B * p.H * p.n_tiles;
    hipLaunchKernelGGL((bwd_f32_kernel<C, RP, true>), dim3(p.total_tiles), dim3(kThreads), 0, stream, p, Dws);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

template <int C>
int launch_dense(const BwdParams& pin, hipStream_t stream) {
    BwdParams p = pin;
    float* Dws = (float*)p.workspace;
    p.n_tiles = (p.N + kRows - 1) / kRows;
    p.total_tiles = p.B * p.H * p.n_tiles;
    hipLaunchKernelGGL((bwd_f32_kernel<C, 0, false, true>), dim3(p.total_tiles), dim3(kThreads), 0, stream, p, Dws);
    if (hipGetLastError() != hipSuccess) return 1;
    hipLaunchKernelGGL((bwd_f32_kernel<C, 0, true, true>), dim3(p.total_tiles), dim3(kThreads), 0, stream, p, Dws);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

template <int C>
int dispatch_c(const BwdParams& p, hipStream_t stream) {
    if (p.R == 0) return launch<C, 0>(p, stream);
    if (p.R <= 8) return launch<C, 8>(p, stream);
    if (p.R <= 32) return launch<C, 32>(p, stream);
    return launch<C, 64>(p, stream);
}

}  // namespace

// fp32 tensors and fp32 factors (N queries, M keys; causal needs N = M); p.workspace: at least
// 4 B H N bytes (the D row sums).
// Returns 0 on success, 1 on launch failure, -1 when no instantiation fits.
int fb_launch_bwd_f32(const BwdParams& p, int C, hipStream_t stream) {
    if (p.R > 64 || (p.causal && p.N != p.M)) return -1;
    switch (C) {
        case 16: return dispatch_c<16>(p, stream);
        case 32: return dispatch_c<32>(p, stream);
        case 64: return dispatch_c<64>(p, stream);
        case 128: return dispatch_c<128>(p, stream);
        default: return -1;
    }
}

// Dense-bias backward in fp32 (p.bias, p.dbias, p.bias_bstride set; p.R = 0; N = M).
int fb_launch_bwd_dense_f32(const BwdParams& p, int C, hipStream_t stream) {
    if (p.N != p.M) return -1;
    switch (C) {
        case 16: return launch_dense<16>(p, stream);
        case 32: return launch_dense<32>(p, stream);
        case 64: return launch_dense<64>(p, stream);
        case 128: return launch_dense<128>(p, stream);
        default: return -1;
    }
}
