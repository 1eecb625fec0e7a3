// bf16 MFMA backward of attention with a factorised bias, gfx950.
//
// With Aq = [q*scale | phi_q], Ak = [k | phi_k] (FlashBias Eq. 3) and S = Aq Ak^T,
// P = exp(S - lse), the chain rule for L = sum(dO * O) gives
//   dV = P^T dO,  dP = dO V^T,  dS = P o (dP - D),  D_i = sum_c dO_ic O_ic,
//   dAk = dS^T Aq  -> dK = dAk[:, :C],          dphi_k = dAk[:, C:],
//   dAq = dS Ak    -> dQ = scale * dAq[:, :C],  dphi_q = dAq[:, C:].
// The factor gradients are therefore extra columns of the contractions that give dK and
// dQ; no N x N gradient is ever written.
//
// Three kernels, no atomics, deterministic:
//   delta : D = rowsum(dO o O)
//   dkv   : one workgroup per 128 keys (a key is a lane); loops over query tiles staged in
//           LDS; recomputes S and dP, accumulates dV^T and dAk^T in registers
//   dq    : one workgroup per 128 queries (a query is a lane); loops over key tiles staged
//           in LDS; recomputes S and dP, accumulates dAq^T in registers
// Both main kernels use the transposed orientation of the forward kernel: the
// loop-invariant operand sits in registers, score-shaped accumulators feed the next MFMA
// as its B operand without leaving registers, and the transposed A operands come from the
// LDS transpose read.  Recomputing S and dP in both kernels costs 7 contractions instead
// of 5 but needs no atomic accumulation of dQ.
//
// fp32 factors are handled as in the forward (three bf16 limbs, six product columns per
// rank); the gradient of a factor is the sum of the accumulator columns that multiply its
// distinct limbs on the other side.
#include <hip/hip_runtime.h>

#include "fb_device.h"
#include "fb_launch.h"
#include "fb_params.h"

namespace {

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;

// ------------------------------------------------------------------------------------------
// delta
// ------------------------------------------------------------------------------------------
template <int C>
__global__ __launch_bounds__(256) void bwd_delta_kernel(const bf16_t* __restrict__ out,
                                                        const bf16_t* __restrict__ dout,
                                                        float* __restrict__ delta, long long rows) {
    constexpr int LPR = C / 8;   // lanes per row, 16 bytes each
    const long long gid = (long long)blockIdx.x * 256 + threadIdx.x;
    const long long row = gid / LPR;
    const int c8 = (int)(gid % LPR);
    float acc = 0.f;
    if (row < rows) {
        const bf16x8 a = as_bf16x8(*(const u32x4*)(out + row * C + c8 * 8));
        const bf16x8 b = as_bf16x8(*(const u32x4*)(dout + row * C + c8 * 8));
#pragma unroll
        for (int e = 0; e < 8; e++) acc = fmaf((float)a[e], (float)b[e], acc);
    }
#pragma unroll
    for (int off = LPR / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    if (c8 == 0 && row < rows) delta[row] = acc;
}

template <int C, int RP>
struct BwdCfg {
    static constexpr int RP2 = (RP + 31) / 32 * 32;   // factor width padded to whole 32-row MFMA blocks
    static constexpr int KS = (C + RP) / 16;          // k-steps of the score contraction
    static constexpr int W2 = C + RP2;
    static constexpr int MB = W2 / 32;                // 32-column blocks of dAq / dAk
    static constexpr int MBC = C / 32;
    static constexpr int AP = W2 + 8;                 // pitch of the [x | phi] tile
    static constexpr int DP = C + 8;                  // pitch of the plain tile (V or dO)
    static constexpr int T = 64;                      // rows per streamed LDS tile
    static constexpr int XCH = T * C / 8;
    static constexpr int XIT = XCH / kThreads;
    static constexpr int PCH = T * RP2 / 8;
    static constexpr int PIT = (PCH + kThreads - 1) / kThreads;
    static constexpr size_t kTileLds = (size_t)2 * T * (AP + DP) * 2;
    static constexpr size_t kVecLds = (size_t)2 * 2 * T * sizeof(float);   // dkv: lse, D per tile
    static constexpr size_t kEpiLds = (size_t)kWaves * 32 * (RP2 + 1) * sizeof(float);
    static_assert(XCH % kThreads == 0, "tile must split evenly");
};

// Write one wave's factor-gradient columns to LDS scratch and reduce limb columns.
// acc[mb] holds columns mb*32 + 8*g + 4*hf + x (register 4*g + x) for row l32.
template <int C, int RP, bool QSIDE>
FB_DEV void store_dphi(const f32x16* acc_phi /* [RP2/32] */, float* scratch /* wave-private [32][RP2+1] */,
                       void* dst_row /* gradient row of this lane's token or null */, int R,
                       bool f32, int l32, int hf) {
    constexpr int RP2 = BwdCfg<C, RP>::RP2;
#pragma unroll
    for (int mb = 0; mb < RP2 / 32; mb++)
#pragma unroll
        for (int r = 0; r < 16; r++)
            scratch[l32 * (RP2 + 1) + mb * 32 + 8 * (r / 4) + 4 * hf + (r % 4)] = acc_phi[mb][r];
    __syncthreads();
    if (dst_row != nullptr) {
        for (int r = hf; r < R; r += 2) {
            const float* s = scratch + l32 * (RP2 + 1);
            if (f32) {
                // distinct limbs on the other side: query side [a1,a1,a2,a1,a2,a3] -> slots 0,2,5
                // multiply dphi_k; key side [b1,b2,b1,b3,b2,b1] -> slots 0,1,3 multiply dphi_q
                const float val = QSIDE ? (s[6 * r] + s[6 * r + 1] + s[6 * r + 3])
                                        : (s[6 * r] + s[6 * r + 2] + s[6 * r + 5]);
                ((float*)dst_row)[r] = val;
            } else {
                ((bf16_t*)dst_row)[r] = (bf16_t)s[r];
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// dq kernel: lane = query
// ------------------------------------------------------------------------------------------
template <int C, int RP, bool CAUSAL>
__global__ __launch_bounds__(kThreads, 2) void bwd_dq_kernel(BwdParams p) {
    using K = BwdCfg<C, RP>;
    constexpr int BK = K::T, BQ = kWaves * 32;
    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* const kt = (bf16_t*)smem;            // [2][BK][AP]  = [k | phi_k | 0]
    bf16_t* const vt = kt + 2 * BK * K::AP;      // [2][BK][DP]

    const int L = (blockIdx.x & 7) * p.tiles_per_xcd + (blockIdx.x >> 3);
    if (L >= p.total_tiles) return;
    const int bh = L / p.n_tiles;
    int qt = L - bh * p.n_tiles;
    if (CAUSAL) qt = p.n_tiles - 1 - qt;
    const int b = bh / p.H, h = bh - b * p.H;
    const int N = p.N, R = p.R;
    const bool phi_f32 = p.phi_f32 != 0;
    const size_t phi_esz = phi_f32 ? 4 : 2;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hf = lane >> 5;
    const int q0 = qt * BQ;
    const int qi = q0 + wave * 32 + l32;
    const bool qok = qi < N;

    const size_t base = (size_t)bh * N * C;
    const bf16_t* qg = (const bf16_t*)p.q + base;
    const bf16_t* kg = (const bf16_t*)p.k + base;
    const bf16_t* vg = (const bf16_t*)p.v + base;
    const bf16_t* dog = (const bf16_t*)p.dout + base;
    const unsigned char* pqg = nullptr;
    const unsigned char* pkg = nullptr;
    if (RP > 0) {
        const size_t pbase = ((size_t)b * p.phi_bstride + (size_t)h * N * R) * phi_esz;
        pqg = (const unsigned char*)p.phi_q + pbase;
        pkg = (const unsigned char*)p.phi_k + pbase;
    }

    // loop-invariant operands of this lane's query
    bf16x8 qreg[K::KS], doreg[C / 16];
#pragma unroll
    for (int ks = 0; ks < K::KS; ks++) {
        bf16x8 val;
        if (ks < C / 16) {
            u32x4 raw = u32x4{0u, 0u, 0u, 0u};
            if (qok) raw = *(const u32x4*)(qg + (size_t)qi * C + ks * 16 + 8 * hf);
            const bf16x8 x = as_bf16x8(raw);
#pragma unroll
            for (int e = 0; e < 8; e++) val[e] = (bf16_t)((float)x[e] * p.scale);
        } else {
            const int c8 = (ks - C / 16) * 2 + hf;
            if (qok) {
                val = phi_chunk_gather<true>(pqg + (size_t)qi * R * phi_esz, c8, R, phi_f32);
            } else {
#pragma unroll
                for (int e = 0; e < 8; e++) val[e] = (bf16_t)0.f;
            }
        }
        qreg[ks] = val;
    }
#pragma unroll
    for (int cs = 0; cs < C / 16; cs++) {
        u32x4 raw = u32x4{0u, 0u, 0u, 0u};
        if (qok) raw = *(const u32x4*)(dog + (size_t)qi * C + cs * 16 + 8 * hf);
        doreg[cs] = as_bf16x8(raw);
    }
    const float lse2 = qok ? p.lse[(size_t)bh * N + qi] * kLog2e : INFINITY;
    const float dlt = qok ? p.delta[(size_t)bh * N + qi] : 0.f;

    f32x16 dacc[K::MB];
#pragma unroll
    for (int mb = 0; mb < K::MB; mb++)
#pragma unroll
        for (int r = 0; r < 16; r++) dacc[mb][r] = 0.f;

    const int kend = CAUSAL ? min(N, q0 + BQ) : N;
    const int nT = (kend + BK - 1) / BK;

    u32x4 kraw[K::XIT], vraw[K::XIT];
    u32x4 praw[K::PIT > 0 ? K::PIT : 1];

    auto load_tile = [&](int t) {
        const int k0 = t * BK;
#pragma unroll
        for (int it = 0; it < K::XIT; it++) {
            const int e = tid + it * kThreads;
            const int row = e / (C / 8), c8 = e % (C / 8);
            const int j = k0 + row;
            u32x4 a = u32x4{0u, 0u, 0u, 0u}, bb = a;
            if (j < N) {
                a = *(const u32x4*)(kg + (size_t)j * C + c8 * 8);
                bb = *(const u32x4*)(vg + (size_t)j * C + c8 * 8);
            }
            kraw[it] = a;
            vraw[it] = bb;
        }
        if (RP > 0) {
#pragma unroll
            for (int it = 0; it < K::PIT; it++) {
                const int e = tid + it * kThreads;
                if (e < K::PCH) {
                    const int row = e / (K::RP2 / 8), c8 = e % (K::RP2 / 8);
                    const int j = k0 + row;
                    praw[it] = phi_chunk_raw(pkg + (size_t)j * R * phi_esz, c8, R, phi_f32, j < N);
                }
            }
        }
    };
    auto store_tile = [&](int buf) {
        bf16_t* kdst = kt + buf * BK * K::AP;
        bf16_t* vdst = vt + buf * BK * K::DP;
#pragma unroll
        for (int it = 0; it < K::XIT; it++) {
            const int e = tid + it * kThreads;
            const int row = e / (C / 8), c8 = e % (C / 8);
            *(u32x4*)(kdst + row * K::AP + c8 * 8) = kraw[it];
            *(u32x4*)(vdst + row * K::DP + c8 * 8) = vraw[it];
        }
        if (RP > 0) {
#pragma unroll
            for (int it = 0; it < K::PIT; it++) {
                const int e = tid + it * kThreads;
                if (e < K::PCH) {
                    const int row = e / (K::RP2 / 8), c8 = e % (K::RP2 / 8);
                    *(u32x4*)(kdst + row * K::AP + C + c8 * 8) =
                        as_uint4(phi_chunk_finish<false>(praw[it], c8, phi_f32));
                }
            }
        }
    };

    load_tile(0);
    store_tile(0);
    __syncthreads();

    const int i16 = lane & 15, blk = l32 >> 4;
    for (int t = 0; t < nT; t++) {
        const bool more = t + 1 < nT;
        if (more) load_tile(t + 1);
        const bf16_t* ksrc = kt + (t & 1) * BK * K::AP;
        const bf16_t* vsrc = vt + (t & 1) * BK * K::DP;
        const int k0 = t * BK;
#pragma unroll
        for (int kb = 0; kb < BK / 32; kb++) {
            const int kb0 = k0 + kb * 32;
            if (CAUSAL && kb0 > q0 + wave * 32 + 31) continue;
            f32x16 s, dp;
#pragma unroll
            for (int r = 0; r < 16; r++) { s[r] = 0.f; dp[r] = 0.f; }
            const bf16_t* krow = ksrc + (kb * 32 + l32) * K::AP + 8 * hf;
            const bf16_t* vrow = vsrc + (kb * 32 + l32) * K::DP + 8 * hf;
#pragma unroll
            for (int ks = 0; ks < K::KS; ks++)
                s = mfma32(as_bf16x8(*(const u32x4*)(krow + ks * 16)), qreg[ks], s);
#pragma unroll
            for (int cs = 0; cs < C / 16; cs++)
                dp = mfma32(as_bf16x8(*(const u32x4*)(vrow + cs * 16)), doreg[cs], dp);

            bf16x8 dsb[2];
            const bool need_mask = (CAUSAL && kb0 + 31 > q0 + wave * 32) || kb0 + 32 > N;
#pragma unroll
            for (int r = 0; r < 16; r++) {
                float pr = fast_exp2(fmaf(s[r], kLog2e, -lse2));
                if (need_mask) {
                    const int key = kb0 + 8 * (r / 4) + 4 * hf + (r % 4);
                    if (key >= N || (CAUSAL && key > qi)) pr = 0.f;
                }
                dsb[r / 8][r % 8] = (bf16_t)(pr * (dp[r] - dlt));
            }
            // dAq^T[col][query] += Ak^T[col][key] dS^T[key][query]
            const bf16_t* kbase = ksrc + (kb * 32 + 4 * hf + (i16 >> 2)) * K::AP + 16 * blk + 4 * (i16 & 3);
#pragma unroll
            for (int mb = 0; mb < K::MB; mb++) {
#pragma unroll
                for (int kk = 0; kk < 2; kk++) {
                    const bf16_t* ap = kbase + (kk * 16) * K::AP + mb * 32;
                    const bf16x8 a = join_tr(lds_read_tr16(ap), lds_read_tr16(ap + 8 * K::AP));
                    dacc[mb] = mfma32(a, dsb[kk], dacc[mb]);
                }
            }
        }
        if (more) store_tile((t + 1) & 1);
        __syncthreads();
    }

    // dQ = scale * dAq[:, :C]
    if (qok) {
        bf16_t* dqg = (bf16_t*)p.dq + base + (size_t)qi * C;
#pragma unroll
        for (int mb = 0; mb < K::MBC; mb++)
#pragma unroll
            for (int g = 0; g < 4; g++) {
                bf16x4 o4;
#pragma unroll
                for (int x = 0; x < 4; x++) o4[x] = (bf16_t)(dacc[mb][4 * g + x] * p.scale);
                *(u32x2*)(dqg + mb * 32 + 8 * g + 4 * hf) = __builtin_bit_cast(u32x2, o4);
            }
    }
    if (RP > 0) {
        float* scratch = (float*)smem + wave * 32 * (K::RP2 + 1);
        unsigned char* dst = nullptr;
        if (qok) dst = (unsigned char*)p.dphi_q + ((size_t)bh * N + qi) * R * phi_esz;
        store_dphi<C, RP, true>(&dacc[K::MBC], scratch, dst, R, phi_f32, l32, hf);
    }
}

// ------------------------------------------------------------------------------------------
// dkv kernel: lane = key
// ------------------------------------------------------------------------------------------
template <int C, int RP, bool CAUSAL>
__global__ __launch_bounds__(kThreads) void bwd_dkv_kernel(BwdParams p) {
    using K = BwdCfg<C, RP>;
    constexpr int BQ = K::T, BKW = kWaves * 32;
    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* const at = (bf16_t*)smem;             // [2][BQ][AP] = [q*scale | phi_q | 0]
    bf16_t* const dt = at + 2 * BQ * K::AP;       // [2][BQ][DP] = dO
    float* const vec = (float*)(dt + 2 * BQ * K::DP);   // [2][2][BQ]: lse*log2e, D

    const int L = (blockIdx.x & 7) * p.tiles_per_xcd + (blockIdx.x >> 3);
    if (L >= p.total_tiles) return;
    const int bh = L / p.n_tiles;
    const int kt_idx = L - bh * p.n_tiles;        // causal: small key index = most work, first
    const int b = bh / p.H, h = bh - b * p.H;
    const int N = p.N, R = p.R;
    const bool phi_f32 = p.phi_f32 != 0;
    const size_t phi_esz = phi_f32 ? 4 : 2;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hf = lane >> 5;
    const int k0 = kt_idx * BKW;
    const int kw0 = k0 + wave * 32;
    const int ki = kw0 + l32;
    const bool kok = ki < N;

    const size_t base = (size_t)bh * N * C;
    const bf16_t* qg = (const bf16_t*)p.q + base;
    const bf16_t* kg = (const bf16_t*)p.k + base;
    const bf16_t* vg = (const bf16_t*)p.v + base;
    const bf16_t* dog = (const bf16_t*)p.dout + base;
    const float* lseg = p.lse + (size_t)bh * N;
    const float* dltg = p.delta + (size_t)bh * N;
    const unsigned char* pqg = nullptr;
    const unsigned char* pkg = nullptr;
    if (RP > 0) {
        const size_t pbase = ((size_t)b * p.phi_bstride + (size_t)h * N * R) * phi_esz;
        pqg = (const unsigned char*)p.phi_q + pbase;
        pkg = (const unsigned char*)p.phi_k + pbase;
    }

    bf16x8 akreg[K::KS], vreg[C / 16];
#pragma unroll
    for (int ks = 0; ks < K::KS; ks++) {
        bf16x8 val;
        if (ks < C / 16) {
            u32x4 raw = u32x4{0u, 0u, 0u, 0u};
            if (kok) raw = *(const u32x4*)(kg + (size_t)ki * C + ks * 16 + 8 * hf);
            val = as_bf16x8(raw);
        } else {
            const int c8 = (ks - C / 16) * 2 + hf;
            if (kok) {
                val = phi_chunk_gather<false>(pkg + (size_t)ki * R * phi_esz, c8, R, phi_f32);
            } else {
#pragma unroll
                for (int e = 0; e < 8; e++) val[e] = (bf16_t)0.f;
            }
        }
        akreg[ks] = val;
    }
#pragma unroll
    for (int cs = 0; cs < C / 16; cs++) {
        u32x4 raw = u32x4{0u, 0u, 0u, 0u};
        if (kok) raw = *(const u32x4*)(vg + (size_t)ki * C + cs * 16 + 8 * hf);
        vreg[cs] = as_bf16x8(raw);
    }

    f32x16 dvacc[K::MBC], dkacc[K::MB];
#pragma unroll
    for (int r = 0; r < 16; r++) {
#pragma unroll
        for (int mb = 0; mb < K::MBC; mb++) dvacc[mb][r] = 0.f;
#pragma unroll
        for (int mb = 0; mb < K::MB; mb++) dkacc[mb][r] = 0.f;
    }

    const int nQT = (N + BQ - 1) / BQ;
    const int t0 = CAUSAL ? k0 / BQ : 0;

    u32x4 qraw[K::XIT], draw[K::XIT];
    u32x4 praw[K::PIT > 0 ? K::PIT : 1];
    float vecraw = 0.f;

    auto load_tile = [&](int t) {
        const int r0 = t * BQ;
#pragma unroll
        for (int it = 0; it < K::XIT; it++) {
            const int e = tid + it * kThreads;
            const int row = e / (C / 8), c8 = e % (C / 8);
            const int i = r0 + row;
            u32x4 a = u32x4{0u, 0u, 0u, 0u}, bb = a;
            if (i < N) {
                a = *(const u32x4*)(qg + (size_t)i * C + c8 * 8);
                bb = *(const u32x4*)(dog + (size_t)i * C + c8 * 8);
            }
            qraw[it] = a;
            draw[it] = bb;
        }
        if (RP > 0) {
#pragma unroll
            for (int it = 0; it < K::PIT; it++) {
                const int e = tid + it * kThreads;
                if (e < K::PCH) {
                    const int row = e / (K::RP2 / 8), c8 = e % (K::RP2 / 8);
                    const int i = r0 + row;
                    praw[it] = phi_chunk_raw(pqg + (size_t)i * R * phi_esz, c8, R, phi_f32, i < N);
                }
            }
        }
        if (tid < 2 * BQ) {
            const int i = r0 + (tid & (BQ - 1));
            if (tid < BQ) vecraw = i < N ? lseg[i] : INFINITY;   // rows past N get P = 0
            else vecraw = i < N ? dltg[i] : 0.f;
        }
    };
    auto store_tile = [&](int buf) {
        bf16_t* adst = at + buf * BQ * K::AP;
        bf16_t* ddst = dt + buf * BQ * K::DP;
#pragma unroll
        for (int it = 0; it < K::XIT; it++) {
            const int e = tid + it * kThreads;
            const int row = e / (C / 8), c8 = e % (C / 8);
            const bf16x8 x = as_bf16x8(qraw[it]);
            bf16x8 y;
#pragma unroll
            for (int z = 0; z < 8; z++) y[z] = (bf16_t)((float)x[z] * p.scale);
            *(u32x4*)(adst + row * K::AP + c8 * 8) = as_uint4(y);
            *(u32x4*)(ddst + row * K::DP + c8 * 8) = draw[it];
        }
        if (RP > 0) {
#pragma unroll
            for (int it = 0; it < K::PIT; it++) {
                const int e = tid + it * kThreads;
                if (e < K::PCH) {
                    const int row = e / (K::RP2 / 8), c8 = e % (K::RP2 / 8);
                    *(u32x4*)(adst + row * K::AP + C + c8 * 8) =
                        as_uint4(phi_chunk_finish<true>(praw[it], c8, phi_f32));
                }
            }
        }
        if (tid < 2 * BQ) {
            float* d = vec + buf * 2 * BQ + tid;      // [0,BQ): lse*log2e, [BQ,2BQ): D
            *d = tid < BQ ? vecraw * kLog2e : vecraw;
        }
    };

    if (t0 < nQT) {
        load_tile(t0);
        store_tile(t0 & 1);
    }
    __syncthreads();

    const int i16 = lane & 15, blk = l32 >> 4;
    for (int t = t0; t < nQT; t++) {
        const bool more = t + 1 < nQT;
        if (more) load_tile(t + 1);
        const bf16_t* asrc = at + (t & 1) * BQ * K::AP;
        const bf16_t* dsrc = dt + (t & 1) * BQ * K::DP;
        const float* lsrc = vec + (t & 1) * 2 * BQ;
        const float* esrc = lsrc + BQ;
#pragma unroll
        for (int qb = 0; qb < BQ / 32; qb++) {
            const int qb0 = t * BQ + qb * 32;
            if (CAUSAL && qb0 + 31 < kw0) continue;    // every query of the block precedes this wave's keys
            f32x16 s, dp;
#pragma unroll
            for (int r = 0; r < 16; r++) { s[r] = 0.f; dp[r] = 0.f; }
            const bf16_t* arow = asrc + (qb * 32 + l32) * K::AP + 8 * hf;
            const bf16_t* drow = dsrc + (qb * 32 + l32) * K::DP + 8 * hf;
#pragma unroll
            for (int ks = 0; ks < K::KS; ks++)
                s = mfma32(as_bf16x8(*(const u32x4*)(arow + ks * 16)), akreg[ks], s);
#pragma unroll
            for (int cs = 0; cs < C / 16; cs++)
                dp = mfma32(as_bf16x8(*(const u32x4*)(drow + cs * 16)), vreg[cs], dp);

            bf16x8 pb[2], dsb[2];
            const bool need_mask = CAUSAL && qb0 < kw0 + 31;
#pragma unroll
            for (int g = 0; g < 4; g++) {
                const float4 l4 = *(const float4*)(lsrc + qb * 32 + 8 * g + 4 * hf);
                const float4 d4 = *(const float4*)(esrc + qb * 32 + 8 * g + 4 * hf);
                const float lv[4] = {l4.x, l4.y, l4.z, l4.w};
                const float dv[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
                for (int x = 0; x < 4; x++) {
                    const int r = 4 * g + x;
                    float pr = fast_exp2(fmaf(s[r], kLog2e, -lv[x]));
                    if (need_mask) {
                        const int query = qb0 + 8 * g + 4 * hf + x;
                        if (query < ki) pr = 0.f;
                    }
                    pb[r / 8][r % 8] = (bf16_t)pr;
                    dsb[r / 8][r % 8] = (bf16_t)(pr * (dp[r] - dv[x]));
                }
            }
            // dV^T[c][key] += dO^T[c][query] P[query][key];  dAk^T[col][key] += Aq^T[col][query] dS[query][key]
            const int rowoff = qb * 32 + 4 * hf + (i16 >> 2);
            const bf16_t* dbase = dsrc + rowoff * K::DP + 16 * blk + 4 * (i16 & 3);
            const bf16_t* abase = asrc + rowoff * K::AP + 16 * blk + 4 * (i16 & 3);
#pragma unroll
            for (int kk = 0; kk < 2; kk++) {
#pragma unroll
                for (int mb = 0; mb < K::MBC; mb++) {
                    const bf16_t* ap = dbase + (kk * 16) * K::DP + mb * 32;
                    const bf16x8 a = join_tr(lds_read_tr16(ap), lds_read_tr16(ap + 8 * K::DP));
                    dvacc[mb] = mfma32(a, pb[kk], dvacc[mb]);
                }
#pragma unroll
                for (int mb = 0; mb < K::MB; mb++) {
                    const bf16_t* ap = abase + (kk * 16) * K::AP + mb * 32;
                    const bf16x8 a = join_tr(lds_read_tr16(ap), lds_read_tr16(ap + 8 * K::AP));
                    dkacc[mb] = mfma32(a, dsb[kk], dkacc[mb]);
                }
            }
        }
        if (more) store_tile((t + 1) & 1);
        __syncthreads();
    }

    if (kok) {
        bf16_t* dvg = (bf16_t*)p.dv + base + (size_t)ki * C;
        bf16_t* dkg = (bf16_t*)p.dk + base + (size_t)ki * C;
#pragma unroll
        for (int mb = 0; mb < K::MBC; mb++)
#pragma unroll
            for (int g = 0; g < 4; g++) {
                bf16x4 a4, b4;
#pragma unroll
                for (int x = 0; x < 4; x++) {
                    a4[x] = (bf16_t)dvacc[mb][4 * g + x];
                    b4[x] = (bf16_t)dkacc[mb][4 * g + x];
                }
                *(u32x2*)(dvg + mb * 32 + 8 * g + 4 * hf) = __builtin_bit_cast(u32x2, a4);
                *(u32x2*)(dkg + mb * 32 + 8 * g + 4 * hf) = __builtin_bit_cast(u32x2, b4);
            }
    }
    if (RP > 0) {
        float* scratch = (float*)smem + wave * 32 * (K::RP2 + 1);
        unsigned char* dst = nullptr;
        if (kok) dst = (unsigned char*)p.dphi_k + ((size_t)bh * N + ki) * R * phi_esz;
        store_dphi<C, RP, false>(&dkacc[K::MBC], scratch, dst, R, phi_f32, l32, hf);
    }
}

template <typename KernT>
bool set_lds(KernT kern, size_t bytes, bool* done) {
    if (*done) return true;
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) !=
        hipSuccess)
        return false;
    *done = true;
    return true;
}

template <int C, int RP, bool CAUSAL>
int launch(const BwdParams& pin, hipStream_t stream) {
    using K = BwdCfg<C, RP>;
    const size_t lds_dq = K::kTileLds > K::kEpiLds ? K::kTileLds : K::kEpiLds;
    const size_t lds_dkv = K::kTileLds + K::kVecLds;
    auto kdq = bwd_dq_kernel<C, RP, CAUSAL>;
    auto kdkv = bwd_dkv_kernel<C, RP, CAUSAL>;
    static bool done_dq = false, done_dkv = false;
    if (!set_lds(kdq, lds_dq, &done_dq) || !set_lds(kdkv, lds_dkv, &done_dkv)) return 1;

    const long long rows = (long long)pin.B * pin.H * pin.N;
    const long long dthreads = rows * (C / 8);
    hipLaunchKernelGGL((bwd_delta_kernel<C>), dim3((unsigned)((dthreads + 255) / 256)), dim3(256), 0, stream,
                       (const bf16_t*)pin.out, (const bf16_t*)pin.dout, pin.delta, rows);
    if (hipGetLastError() != hipSuccess) return 1;

    BwdParams p = pin;
    p.n_tiles = (p.N + 127) / 128;
    p.total_tiles = p.B * p.H * p.n_tiles;
    p.tiles_per_xcd = (p.total_tiles + 7) / 8;
    hipLaunchKernelGGL(kdkv, dim3(8 * p.tiles_per_xcd), dim3(kThreads), lds_dkv, stream, p);
    if (hipGetLastError() != hipSuccess) return 1;
    hipLaunchKernelGGL(kdq, dim3(8 * p.tiles_per_xcd), dim3(kThreads), lds_dq, stream, p);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

template <int C, int RP>
int dispatch_causal(const BwdParams& p, hipStream_t stream) {
    return p.causal ? launch<C, RP, true>(p, stream) : launch<C, RP, false>(p, stream);
}

template <int C>
int dispatch_rp(const BwdParams& p, int rp, hipStream_t stream) {
    switch (rp) {
        case 0: return dispatch_causal<C, 0>(p, stream);
        case 16: return dispatch_causal<C, 16>(p, stream);
        case 32: return dispatch_causal<C, 32>(p, stream);
        default: return -1;
    }
}

}  // namespace

int fb_launch_bwd_bf16(const BwdParams& p, int C, int rp, hipStream_t stream) {
    switch (C) {
        case 32: return dispatch_rp<32>(p, rp, stream);
        case 64: return dispatch_rp<64>(p, rp, stream);
        case 128: return dispatch_rp<128>(p, rp, stream);
        default: return -1;
    }
}
