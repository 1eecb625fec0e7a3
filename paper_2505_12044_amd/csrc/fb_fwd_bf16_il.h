// bf16 MFMA forward, in-wave interleaved variant: one workgroup of 4 waves (128 query rows of
// one (b, h)), one 32-row query block per wave, ONE wave per SIMD.
//
// Measurements on gfx950 showed that two waves sharing a SIMD overlap their matrix and vector
// work only marginally once each wave's vector work depends on its own MFMA results (a
// dependent MFMA -> VALU -> MFMA stream runs almost as if the waves were serialised), while
// INDEPENDENT MFMA and VALU work inside one wave's instruction stream overlaps almost
// perfectly.  So the overlap is written into the stream itself, one block ahead:
//
//   region 1 :  S_{t+1} = K_{t+1} . Q   (MFMA chain)   interleaved with
//               exp / sum / convert of block t (P_t) and the V_t transpose reads
//   region 2 :  O += V_t P_t            (MFMA chain)   interleaved with
//               the row maxima of S_{t+1}, the K_{t+2} operand reads and the staging of
//               block t+3 (registers -> LDS) / t+5 (global -> registers)
//   barrier
//
// Each MFMA is followed by its share of the vector / LDS work and a scheduling barrier, so
// the order below is the order executed.  Orientation, operand layouts, factor handling,
// masking and the lazy rescale are those of the four-wave kernel in fb_fwd_bf16_impl.h.
// LDS ring of four 32-key blocks: block b is stored in iteration b-3, its K operands are
// read in iteration b-2, its V operands in iteration b; the slot is rewritten in iteration
// b+1, after the barrier that ends iteration b.
#ifndef FB_FWD_BF16_IL_H_
#define FB_FWD_BF16_IL_H_

#include <hip/hip_runtime.h>

#include <type_traits>

#include "fb_device.h"
#include "fb_launch.h"
#include "fb_params.h"

namespace fbil {

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int BK = 32;
constexpr int NBUF = 4;
constexpr int QB = 1;
constexpr float kRescaleTau = 8.0f;
constexpr int LA = 4;        // LDS operand reads run this many MFMAs ahead of their use

template <int C, int RP>
struct Cfg {
    static constexpr int KS = (C + RP) / 16;
    static constexpr int KP = C + RP + 8;
    static constexpr int VP = (C == 32) ? 32 : C + 32;
    static constexpr int BQ = kWaves * QB * 32;
    static constexpr int KCH = BK * C / 8;
    static constexpr int KIT = (KCH + kThreads - 1) / kThreads;
    static constexpr int PCH = BK * RP / 8;
    static constexpr int PIT = (PCH + kThreads - 1) / kThreads;
    static constexpr int KBLK = BK * KP;
    static constexpr int VBLK = BK * VP;
    static constexpr int NV = (C / 32) * 2;           // V operand registers (bf16x8) per block
    static constexpr int N1 = KS * QB;                // MFMAs of region 1
    static constexpr int N2 = NV * QB;                // MFMAs of region 2
    static constexpr size_t kLds = (size_t)NBUF * (KBLK + VBLK) * 2;
};

template <int C, int RP, int PM, bool CAUSAL, bool DENSE>
__global__ __launch_bounds__(kThreads, 2) void fwd_bf16_il_kernel(FwdParams p) {
    using K = Cfg<C, RP>;
    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* const kt = (bf16_t*)smem;                 // [NBUF][BK][KP]
    bf16_t* const vt = kt + NBUF * K::KBLK;           // [NBUF][BK][VP]

    const int L = (blockIdx.x & 7) * p.tiles_per_xcd + (blockIdx.x >> 3);
    if (L >= p.total_tiles) return;
    const int bh = L / p.n_qtiles;
    int qt = L - bh * p.n_qtiles;
    if (CAUSAL) qt = p.n_qtiles - 1 - qt;
    const int b = bh / p.H, h = bh - b * p.H;
    const int N = p.N, R = p.R;
    const bool phi_f32 = PM == 2 && p.phi_f32 != 0;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps everything derived from it scalar
    const int l32 = lane & 31, hf = lane >> 5;
    const int q0 = qt * K::BQ;
    const int qw0 = q0 + wave * (QB * 32);

    const size_t base = (size_t)bh * N * C;
    const bf16_t* qg = (const bf16_t*)p.q + base;
    const bf16_t* kg = (const bf16_t*)p.k + base;
    const bf16_t* vg = (const bf16_t*)p.v + base;
    const size_t phi_esz = phi_f32 ? 4 : 2;
    const unsigned char* pqg = nullptr;
    const unsigned char* pkg = nullptr;
    if (RP > 0) {
        const size_t pbase = ((size_t)b * p.phi_bstride + (size_t)h * N * R) * phi_esz;
        pqg = (const unsigned char*)p.phi_q + pbase;
        pkg = (const unsigned char*)p.phi_k + pbase;
    }
    const bf16_t* bg = nullptr;
    if (DENSE) bg = (const bf16_t*)p.bias + (size_t)b * p.bias_bstride + (size_t)h * N * N;

    // ---- query operand [q*scale | phi_q | 0] (rows past N read row N-1 and are never stored)
    bf16x8 qreg[QB][K::KS];
#pragma unroll
    for (int qb = 0; qb < QB; qb++) {
        const int qc = min(qw0 + qb * 32 + l32, N - 1);
#pragma unroll
        for (int ks = 0; ks < K::KS; ks++) {
            bf16x8 val;
            if (ks < C / 16) {
                const bf16x8 x = as_bf16x8(*(const u32x4*)(qg + (size_t)qc * C + ks * 16 + 8 * hf));
#pragma unroll
                for (int e = 0; e < 8; e++) val[e] = (bf16_t)((float)x[e] * p.scale);
            } else {
                const int c8 = (ks - C / 16) * 2 + hf;
                val = phi_chunk_gather<true>(pqg + (size_t)qc * R * phi_esz, c8, R, phi_f32);
            }
            qreg[qb][ks] = val;
        }
    }

    f32x16 oacc[QB][C / 32];
    float mref[QB], lsum[QB], mx2[QB];
#pragma unroll
    for (int qb = 0; qb < QB; qb++) {
        mref[qb] = -INFINITY;
        lsum[qb] = 0.f;
        mx2[qb] = -INFINITY;
#pragma unroll
        for (int cb = 0; cb < C / 32; cb++)
#pragma unroll
            for (int r = 0; r < 16; r++) oacc[qb][cb][r] = 0.f;
    }

    const int kend = CAUSAL ? min(N, q0 + K::BQ) : N;
    const int nT = (kend + BK - 1) / BK;
    // causal tiles walk the keys from the diagonal back to key 0 (see fb_fwd_bf16_impl.h)
    auto blk_of = [&](int t) { return CAUSAL ? max(nT - 1 - t, 0) : t; };

    // ---- staging: one block in flight in registers ----
    u32x4 kraw[K::KIT], vraw[K::KIT];
    u32x4 praw[K::PIT > 0 ? K::PIT : 1];
    auto load_block = [&](int t) __attribute__((always_inline)) {
        const int k0 = blk_of(t) * BK;
#pragma unroll
        for (int it = 0; it < K::KIT; it++) {
            const int e = tid + it * kThreads;
            if (K::KCH % kThreads == 0 || e < K::KCH) {
                const int row = e / (C / 8), c8 = e % (C / 8);
                const int j = min(k0 + row, N - 1);
                kraw[it] = *(const u32x4*)(kg + (size_t)j * C + c8 * 8);
                vraw[it] = *(const u32x4*)(vg + (size_t)j * C + c8 * 8);
            }
        }
        if (PM != 0) {
#pragma unroll
            for (int it = 0; it < K::PIT; it++) {
                const int e = ((tid + 64 * t) & (kThreads - 1)) + it * kThreads;
                if (K::PCH % kThreads == 0 || e < K::PCH) {
                    const int row = e / (RP / 8), c8 = e % (RP / 8);
                    const int j = min(k0 + row, N - 1);
                    const unsigned char* src = pkg + (size_t)j * R * phi_esz;
                    if (PM == 1) {
                        praw[it] = (c8 * 8 < R) ? *(const u32x4*)(src + c8 * 16) : u32x4{0u, 0u, 0u, 0u};
                    } else {
                        praw[it] = phi_chunk_raw(src, c8, R, phi_f32, true);
                    }
                }
            }
        }
    };
    // t is the block held in (kraw, vraw, praw): the factor-chunk rotation must match its load
    auto store_block = [&](int buf, int t) __attribute__((always_inline)) {
        bf16_t* kdst = kt + buf * K::KBLK;
        bf16_t* vdst = vt + buf * K::VBLK;
#pragma unroll
        for (int it = 0; it < K::KIT; it++) {
            const int e = tid + it * kThreads;
            if (K::KCH % kThreads == 0 || e < K::KCH) {
                const int row = e / (C / 8), c8 = e % (C / 8);
                *(u32x4*)(kdst + row * K::KP + c8 * 8) = kraw[it];
                *(u32x4*)(vdst + row * K::VP + c8 * 8) = vraw[it];
            }
        }
        if (PM != 0) {
#pragma unroll
            for (int it = 0; it < K::PIT; it++) {
                const int e = ((tid + 64 * t) & (kThreads - 1)) + it * kThreads;
                if (K::PCH % kThreads == 0 || e < K::PCH) {
                    const int row = e / (RP / 8), c8 = e % (RP / 8);
                    const u32x4 v = PM == 1 ? praw[it] : as_uint4(phi_chunk_finish<false>(praw[it], c8, phi_f32));
                    *(u32x4*)(kdst + row * K::KP + C + c8 * 8) = v;
                }
            }
        }
    };

    // dense mode: bias values of one block in accumulator order (row qi, keys 8*g+4*hf+0..3)
    u32x2 braw[DENSE ? QB : 1][4];
    const bool bias_fast = DENSE && ((N & 3) == 0);
    auto load_bias = [&](int t) __attribute__((always_inline)) {
        if (!DENSE) return;
        const int k0 = blk_of(t) * BK;
#pragma unroll
        for (int qb = 0; qb < QB; qb++) {
            const int qi = qw0 + qb * 32 + l32;
#pragma unroll
            for (int g = 0; g < 4; g++) {
                const int j = k0 + 8 * g + 4 * hf;
                u32x2 a = u32x2{0u, 0u};
                if (qi < N && j < N && !(CAUSAL && j > qi)) {
                    const bf16_t* src = bg + (size_t)qi * N + j;
                    if (bias_fast) {
                        a = *(const u32x2*)src;
                    } else {
                        bf16x4 tmp;
#pragma unroll
                        for (int x = 0; x < 4; x++) tmp[x] = (j + x < N) ? src[x] : (bf16_t)0.f;
                        a = __builtin_bit_cast(u32x2, tmp);
                    }
                }
                braw[qb][g] = a;
            }
        }
    };
    auto init_s = [&](f32x16 (&s)[QB]) __attribute__((always_inline)) {
#pragma unroll
        for (int qb = 0; qb < QB; qb++) {
            if (DENSE) {
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    const bf16x4 bv = __builtin_bit_cast(bf16x4, braw[qb][g]);
#pragma unroll
                    for (int x = 0; x < 4; x++) s[qb][4 * g + x] = (float)bv[x];
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; r++) s[qb][r] = 0.f;
            }
        }
    };

    const int krow_off = l32 * K::KP + 8 * hf;
    const int i16 = lane & 15, blk = l32 >> 4;
    const int vlane_off = (4 * hf + (i16 >> 2)) * K::VP + 16 * blk + 4 * (i16 & 3);
    bf16x8 ka[K::KS];

    // masks of block t for this lane's rows, and the row maximum (log2 units) of a score block
    auto mask_block = [&](f32x16 (&s)[QB], int kb0) __attribute__((always_inline)) {
#pragma unroll
        for (int qb = 0; qb < QB; qb++) {
            const int qi = qw0 + qb * 32 + l32;
#pragma unroll
            for (int r = 0; r < 16; r++) {
                const int key = kb0 + 8 * (r / 4) + 4 * hf + (r % 4);
                if (key >= N || (CAUSAL && key > qi)) s[qb][r] = -INFINITY;
            }
        }
    };

    // ---- prologue: blocks 0..2 in LDS, blocks 3 and 4 in flight, S_0 and its maxima ready ----
    load_block(0); store_block(0, 0);
    load_block(1); store_block(1, 1);
    load_block(2); store_block(2, 2);
    load_block(3);
    load_bias(0);
    __syncthreads();
    f32x16 sA[QB], sB[QB];
    {
        const bf16_t* kr = kt + 0 * K::KBLK + krow_off;
#pragma unroll
        for (int ks = 0; ks < K::KS; ks++) ka[ks] = as_bf16x8(*(const u32x4*)(kr + ks * 16));
        init_s(sA);
#pragma unroll
        for (int ks = 0; ks < K::KS; ks++)
#pragma unroll
            for (int qb = 0; qb < QB; qb++) sA[qb] = mfma32(ka[ks], qreg[qb][ks], sA[qb]);
        const int kb0 = blk_of(0) * BK;
        if ((kb0 + BK > N) || (CAUSAL && kb0 + BK - 1 > qw0)) mask_block(sA, kb0);
#pragma unroll
        for (int qb = 0; qb < QB; qb++) {
            float m = fmaxf(sA[qb][0], sA[qb][1]);
#pragma unroll
            for (int r = 2; r < 16; r++) m = fmaxf(m, sA[qb][r]);
            mx2[qb] = half_max(m) * kLog2e;
        }
        load_bias(1);
        const bf16_t* kr1 = kt + 1 * K::KBLK + krow_off;
#pragma unroll
        for (int ks = 0; ks < LA && ks < K::KS; ks++) ka[ks] = as_bf16x8(*(const u32x4*)(kr1 + ks * 16));
    }

    // blocks [0, t_plain) (in key order) need no mask for any row of this wave
    int t_plain = N / BK;
    if (CAUSAL) t_plain = min(t_plain, (qw0 + 1) / BK);
    t_plain = min(t_plain, nT);

    int buf = 0;   // t % NBUF
    // One iteration.  scur = S_t (masked, maxima in mx2), snext receives S_{t+1}.
    auto body = [&](int t, f32x16 (&scur)[QB], f32x16 (&snext)[QB]) __attribute__((always_inline)) {
        // wave-uniform: does block t or t+1 need masks / may be invisible?  (Leading blocks in
        // causal reverse order, trailing blocks otherwise.)
        const bool MASKED = CAUSAL ? (t < nT - t_plain) : (t + 1 >= t_plain);
        const int buf1 = (buf + 1) & (NBUF - 1);
        const int buf2 = (buf + 2) & (NBUF - 1);
        const int buf3 = (buf + 3) & (NBUF - 1);
        const int kb0 = blk_of(t) * BK;
        const int kb1 = blk_of(t + 1) * BK;
        // blocks no row of this wave can see (causal): their MFMAs are skipped, P stays 0
        const bool skip_t = MASKED && CAUSAL && kb0 > qw0 + QB * 32 - 1;
        const bool skip_n = MASKED && CAUSAL && kb1 > qw0 + QB * 32 - 1;

        // ---- lazy rescale (rare): raise the reference maximum of rows that outgrew it ----
#pragma unroll
        for (int qb = 0; qb < QB; qb++) {
            if (__builtin_expect(__any(mx2[qb] > mref[qb] + kRescaleTau), 0)) {
                const float mnew = fmaxf(fmaxf(mref[qb], mx2[qb]), -1e30f);
                const float alpha = fast_exp2(mref[qb] - mnew);
                mref[qb] = mnew;
                lsum[qb] *= alpha;
#pragma unroll
                for (int cb = 0; cb < C / 32; cb++)
#pragma unroll
                    for (int r = 0; r < 16; r++) oacc[qb][cb][r] *= alpha;
            }
        }
        float nm[QB], ps[QB][4];
#pragma unroll
        for (int qb = 0; qb < QB; qb++) {
            nm[qb] = mref[qb] == -INFINITY ? 0.f : -mref[qb];
#pragma unroll
            for (int x = 0; x < 4; x++) ps[qb][x] = 0.f;
        }
        init_s(snext);
        __builtin_amdgcn_sched_barrier(0);

        // ================= region 1: S_{t+1} chain | exp/sum/convert of block t | V_t reads ====
        bf16x8 pb[QB][2];
        bf16x8 va[K::NV];
        {
            const bf16_t* vbase = vt + buf * K::VBLK + vlane_off;
            const bf16_t* kr1 = kt + buf1 * K::KBLK + krow_off;
            constexpr int NE = QB * 16;                 // score elements per lane to exponentiate
            constexpr int VPRE = K::NV < LA ? K::NV : LA;   // V operands fetched ahead of region 2
#pragma unroll
            for (int i = 0; i < K::N1; i++) {
                const int ks = i / QB, qb = i % QB;
                if (!skip_n) snext[qb] = mfma32(ka[ks], qreg[qb][ks], snext[qb]);
                // K operand LA steps ahead (the first LA were read during the previous region 2)
                if (qb == QB - 1 && ks + LA < K::KS)
                    ka[ks + LA] = as_bf16x8(*(const u32x4*)(kr1 + (ks + LA) * 16));
                // this step's share of the softmax elements
#pragma unroll
                for (int e = (i * NE) / K::N1; e < ((i + 1) * NE) / K::N1; e++) {
                    const int eq = e / 16, er = e % 16;
                    float pr = fast_exp2(fmaf(scur[eq][er], kLog2e, nm[eq]));
                    // the empty asm pins the computation to this step: without it the
                    // optimiser sinks the whole exponentiation down to its first use
                    asm volatile("" : "+v"(pr));
                    ps[eq][er & 3] += pr;
                    pb[eq][er / 8][er % 8] = (bf16_t)pr;
                }
                // the first VPRE V operands, spread over the second half of the chain
                if (i >= K::N1 / 2) {
                    constexpr int H1 = K::N1 - K::N1 / 2;
                    const int ii = i - K::N1 / 2;
#pragma unroll
                    for (int v = (ii * VPRE) / H1; v < ((ii + 1) * VPRE) / H1; v++) {
                        const bf16_t* vp = vbase + ((v & 1) * 16) * K::VP + (v >> 1) * 32;
                        va[v] = join_tr(lds_read_tr16(vp), lds_read_tr16(vp + 8 * K::VP));
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int qb = 0; qb < QB; qb++) lsum[qb] += (ps[qb][0] + ps[qb][1]) + (ps[qb][2] + ps[qb][3]);
        }

        // ================= region 2: O chain | maxima of S_{t+1} | K_{t+2} reads | staging ======
        store_block(buf3, t + 3);
        load_block(t + 4);
        load_bias(t + 2);
        __builtin_amdgcn_sched_barrier(0);
        {
            const bf16_t* kr = kt + buf2 * K::KBLK + krow_off;
            const bf16_t* vbase = vt + buf * K::VBLK + vlane_off;
            const bool mask_n = MASKED && ((kb1 + BK > N) || (CAUSAL && kb1 + BK - 1 > qw0));
            constexpr int VPRE = K::NV < LA ? K::NV : LA;
            constexpr int KPRE = K::KS < LA ? K::KS : LA;     // K operands of block t+2 fetched here
            float m[QB];
#pragma unroll
            for (int j = 0; j < K::N2; j++) {
                const int v = j / QB, qb = j % QB;
                if (!skip_t) oacc[qb][v >> 1] = mfma32(va[v], pb[qb][v & 1], oacc[qb][v >> 1]);
                // V operand LA steps ahead
                if (qb == QB - 1 && v + VPRE < K::NV) {
                    const int w = v + VPRE;
                    const bf16_t* vp = vbase + ((w & 1) * 16) * K::VP + (w >> 1) * 32;
                    va[w] = join_tr(lds_read_tr16(vp), lds_read_tr16(vp + 8 * K::VP));
                }
                // the first KPRE K operands of block t+2, spread over the second half of the chain
                if (j >= K::N2 / 2) {
                    constexpr int H2k = K::N2 - K::N2 / 2;
                    const int jj = j - K::N2 / 2;
#pragma unroll
                    for (int ks = (jj * KPRE) / H2k; ks < ((jj + 1) * KPRE) / H2k; ks++)
                        ka[ks] = as_bf16x8(*(const u32x4*)(kr + ks * 16));
                }
                // masks and row maxima of S_{t+1}, spread over the second half of the chain
                if (j == K::N2 / 2) {
                    if (mask_n) {
                        asm volatile("" ::: "memory");   // keep this a real (rarely taken) branch
                        mask_block(snext, kb1);
                    }
                }
                if (j >= K::N2 / 2) {
                    constexpr int H2 = K::N2 - K::N2 / 2;
                    const int jj = j - K::N2 / 2;
#pragma unroll
                    for (int e = (jj * 16 * QB) / H2; e < ((jj + 1) * 16 * QB) / H2; e++) {
                        const int eq = e / 16, er = e % 16;
                        m[eq] = er == 0 ? snext[eq][0] : fmaxf(m[eq], snext[eq][er]);
                    }
#pragma unroll
                    for (int qb = 0; qb < QB; qb++) asm volatile("" : "+v"(m[qb]));   // pinned here, see above
                }
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int qb = 0; qb < QB; qb++) mx2[qb] = half_max(m[qb]) * kLog2e;
        }
        __syncthreads();
        buf = buf1;
        (void)kb0;
    };

    for (int t = 0; t < nT; t += 2) {
        body(t, sA, sB);
        if (t + 1 < nT) body(t + 1, sB, sA);
    }

    // ---- epilogue: o = O / l, lse = m + ln l ----
#pragma unroll
    for (int qb = 0; qb < QB; qb++) {
        const int qi = qw0 + qb * 32 + l32;
        const float ltot = half_sum(lsum[qb]);
        const float inv = 1.f / ltot;
        if (qi < N) {
            bf16_t* og = (bf16_t*)p.out + base + (size_t)qi * C;
#pragma unroll
            for (int cb = 0; cb < C / 32; cb++) {
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    bf16x4 o4;
#pragma unroll
                    for (int x = 0; x < 4; x++) o4[x] = (bf16_t)(oacc[qb][cb][4 * g + x] * inv);
                    *(u32x2*)(og + cb * 32 + 8 * g + 4 * hf) = __builtin_bit_cast(u32x2, o4);
                }
            }
            if (hf == 0) p.lse[(size_t)bh * N + qi] = (mref[qb] + __log2f(ltot)) * kLn2;
        }
    }
}

template <int C, int RP, int PM, bool CAUSAL, bool DENSE>
int launch(const FwdParams& pin, hipStream_t stream) {
    using K = Cfg<C, RP>;
    auto kern = fwd_bf16_il_kernel<C, RP, PM, CAUSAL, DENSE>;
    static FbLdsOnce once;
    if (!fb_raise_lds_limit((const void*)kern, K::kLds, once)) return 1;
    FwdParams p = pin;
    p.n_qtiles = (p.N + K::BQ - 1) / K::BQ;
    p.total_tiles = p.B * p.H * p.n_qtiles;
    p.tiles_per_xcd = (p.total_tiles + 7) / 8;
    hipLaunchKernelGGL(kern, dim3(8 * p.tiles_per_xcd), dim3(kThreads), K::kLds, stream, p);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

template <int C, int RP, int PM, bool DENSE>
int dispatch_causal(const FwdParams& p, hipStream_t stream) {
    if (p.causal) return launch<C, RP, PM, true, DENSE>(p, stream);
    return launch<C, RP, PM, false, DENSE>(p, stream);
}

template <int C, int RP>
int dispatch_pm(const FwdParams& p, hipStream_t stream) {
    const bool vec = !p.phi_f32 && (p.R % 8) == 0;
    if (vec) return dispatch_causal<C, RP, 1, false>(p, stream);
    return dispatch_causal<C, RP, 2, false>(p, stream);
}

template <int C>
int dispatch(const FwdParams& p, int rp, bool dense, hipStream_t stream) {
    if (dense) return dispatch_causal<C, 0, 0, true>(p, stream);
    switch (rp) {
        case 0: return dispatch_causal<C, 0, 0, false>(p, stream);
        case 16: return dispatch_pm<C, 16>(p, stream);
        case 32: return dispatch_pm<C, 32>(p, stream);
        default: return -1;
    }
}

}  // namespace fbil

#endif
