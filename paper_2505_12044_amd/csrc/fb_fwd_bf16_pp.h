// bf16 MFMA forward, "ping-pong" variant: one workgroup of 8 waves (256 query rows of one
// (b, h)), two waves per SIMD from the SAME workgroup, split into two groups of four that run
// half an iteration apart.  Every wave alternates
//     VALU phase :  stage a K/V block into LDS, issue its LDS operand reads, softmax(S_t) -> P_t
//     MFMA phase :  O += V_t P_t,   S_{t+1} = K_{t+1} . Q
// with a workgroup barrier between phases; while group 0 is in its MFMA phase group 1 is in
// its VALU phase on the same SIMDs and vice versa, so the matrix pipe and the vector pipe of
// every SIMD are busy at the same time by construction (two independent workgroups per CU
// were observed to fall into lock-step instead and overlap only ~25 % of the time).
//
// Orientation, operand layouts, factor handling and masking are those of the four-wave
// kernel in fb_fwd_bf16_impl.h.  The LDS operand reads of a block are issued inside the MFMA
// phase, right after the chain that consumed the registers they refill, so they overlap the
// wave's own MFMAs and the following softmax instead of lengthening the VALU phase.
// Blocks of 32 keys live in an LDS ring of four.  Numbering the phases so that group 0 runs
// softmax(t) in phase 2t and its MFMA phase t in 2t+1 (group 1: 2t+1 and 2t+2):
//   block b is written in the VALU phases b-3 (phases 2b-6 and 2b-5),
//   its K operands are read in the MFMA phases b-2 (from phase 2b-3 on),
//   its V operands in the MFMA phases b-1 (last: group 1, phase 2b),
// and the slot is rewritten by block b+4 in phases 2b+2 / 2b+3, after a barrier.
#ifndef FB_FWD_BF16_PP_H_
#define FB_FWD_BF16_PP_H_

#include <hip/hip_runtime.h>

#include <type_traits>

#include "fb_device.h"
#include "fb_launch.h"
#include "fb_params.h"


namespace fbpp {

constexpr int kWaves = 8;
constexpr int kThreads = kWaves * 64;
constexpr int BK = 32;
constexpr int NBUF = 4;
constexpr float kSumLimit = 256.0f;   // 2^tau: bound on a lane's partial probability sum per block

template <int C, int RP>
struct Cfg {
    static constexpr int KS = (C + RP) / 16;
    static constexpr int KP = C + RP + 8;
    static constexpr int VP = (C == 32) ? 32 : C + 32;
    static constexpr int BQ = kWaves * 32;
    static constexpr int KCH = BK * C / 8;            // 16-byte chunks of K (or V) per block: <= 512
    static constexpr int KSUB = kThreads / KCH;       // every KSUB-th thread stages one chunk
    static constexpr int PCH = BK * RP / 8;           // factor chunks per block: 64..256
    static constexpr bool PDIV = PCH > 0 && (kThreads % (PCH > 0 ? PCH : 1)) == 0;
    static constexpr int PSUB = PDIV ? kThreads / PCH : 1;
    static constexpr int KBLK = BK * KP;
    static constexpr int VBLK = BK * VP;
    static constexpr size_t kLds = (size_t)NBUF * (KBLK + VBLK) * 2;
    static_assert(kThreads % KCH == 0 && PCH <= kThreads, "staging split");
};

template <int C, int RP, int PM, bool CAUSAL, bool DENSE>
__global__ __launch_bounds__(kThreads, 2) void fwd_bf16_pp_kernel(FwdParams p) {
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
    const int grp = wave >> 2;                        // waves w and w+4 share a SIMD
    const int l32 = lane & 31, hf = lane >> 5;
    const int q0 = qt * K::BQ;
    const int qw0 = q0 + wave * 32;
    const int qi = qw0 + l32;

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

    // ---- query operand [q*scale | phi_q | 0] (rows past N read row N-1 and are never stored); as in the
    // four-wave kernel, with no factors or fp32 factors at C = 64, 128 it is [q | phi_q / scale | 0] and the
    // scale sits in the exponent's multiply-add, so that every forward variant forms the scores the
    // backward recomputes
    const bool rawq = !DENSE && C % 64 == 0 && (PM == 0 || phi_f32);      // wave-uniform
    const float emul = rawq ? p.scale * kLog2e : kLog2e;
    bf16x8 qreg[K::KS];
    {
        const int qc = min(qi, N - 1);
#pragma unroll
        for (int ks = 0; ks < K::KS; ks++) {
            bf16x8 val;
            if (ks < C / 16) {
                const bf16x8 x = as_bf16x8(*(const u32x4*)(qg + (size_t)qc * C + ks * 16 + 8 * hf));
#pragma unroll
                for (int e = 0; e < 8; e++) val[e] = rawq ? x[e] : (bf16_t)((float)x[e] * p.scale);
            } else {
                const int c8 = (ks - C / 16) * 2 + hf;
                val = phi_chunk_gather<true>(pqg + (size_t)qc * R * phi_esz, c8, R, phi_f32, rawq ? p.inv_scale : 1.f);
            }
            qreg[ks] = val;
        }
    }

    f32x16 oacc[C / 32];
#pragma unroll
    for (int cb = 0; cb < C / 32; cb++)
#pragma unroll
        for (int r = 0; r < 16; r++) oacc[cb][r] = 0.f;
    float mref = -INFINITY, lsum = 0.f;
    bool ref_ok = false;   // wave-uniform: every row of the wave has a finite reference maximum

    const int kend = CAUSAL ? min(N, q0 + K::BQ) : N;
    const int nT = (kend + BK - 1) / BK;

    // ---- staging: thread -> at most one K chunk, one V chunk, one factor chunk per block ----
    const bool k_active = (tid % K::KSUB) == 0;
    const int ke = tid / K::KSUB;
    const int krow = ke / (C / 8), kc8 = ke % (C / 8);
    bool p_active = false;
    int prow = 0, pc8 = 0;
    if (PM != 0) {
        const int pe = K::PDIV ? tid / K::PSUB : tid;
        p_active = K::PDIV ? (tid % K::PSUB) == 0 : tid < K::PCH;
        constexpr int kChunksPerRow = RP > 0 ? RP / 8 : 1;
        prow = pe / kChunksPerRow;
        pc8 = pe % kChunksPerRow;
    }
    // two blocks are kept in flight in registers (global latency exceeds one iteration):
    // (kraw, vraw, praw) is the older one, (kraw2, vraw2, praw2) the newer
    u32x4 kraw = u32x4{0u, 0u, 0u, 0u}, vraw = kraw, praw = kraw;
    u32x4 kraw2 = kraw, vraw2 = kraw, praw2 = kraw;
    auto rotate_regs = [&]() {
        kraw = kraw2;
        vraw = vraw2;
        praw = praw2;
    };

    // 32-bit byte offsets inside the head (the entry points reject larger problems); rows past
    // N are clamped to row N-1 by a minimum on the offset
    const unsigned char* kgb = (const unsigned char*)kg;
    const unsigned char* vgb = (const unsigned char*)vg;
    const unsigned grow_off = (unsigned)krow * (unsigned)(C * 2), gcol_off = (unsigned)kc8 * 16u;
    const unsigned kv_last = (unsigned)(N - 1) * (unsigned)(C * 2);
    const unsigned phi_rb = (unsigned)R * (unsigned)phi_esz;
    const unsigned prow_off = (unsigned)prow * phi_rb, phi_last = (unsigned)(N - 1) * phi_rb;
    auto load_block = [&](int t) {
        const int k0 = t * BK;
        if (k_active) {
            const unsigned off = min((unsigned)k0 * (unsigned)(C * 2) + grow_off, kv_last) + gcol_off;
            kraw2 = *(const u32x4*)(kgb + off);
            vraw2 = *(const u32x4*)(vgb + off);
        }
        if (PM != 0) {
            if (p_active) {
                const unsigned char* src = pkg + min((unsigned)k0 * phi_rb + prow_off, phi_last);
                if (PM == 1) {
                    praw2 = (pc8 * 8 < R) ? *(const u32x4*)(src + pc8 * 16) : u32x4{0u, 0u, 0u, 0u};
                } else {
                    praw2 = phi_chunk_raw(src, pc8, R, phi_f32, true);
                }
            }
        }
    };
    auto store_block = [&](int buf) {
        bf16_t* kdst = kt + buf * K::KBLK;
        bf16_t* vdst = vt + buf * K::VBLK;
        if (k_active) {
            *(u32x4*)(kdst + krow * K::KP + kc8 * 8) = kraw;
            *(u32x4*)(vdst + krow * K::VP + kc8 * 8) = vraw;
        }
        if (PM != 0) {
            if (p_active) {
                const u32x4 v = PM == 1 ? praw : as_uint4(phi_chunk_finish<false>(praw, pc8, phi_f32));
                *(u32x4*)(kdst + prow * K::KP + C + pc8 * 8) = v;
            }
        }
    };

    // dense mode: this lane's bias values of one block in accumulator order (row qi, keys
    // 8*g + 4*hf + 0..3); chunks above the diagonal or past the end are not read.
    u32x2 braw[4];
    const bool bias_fast = DENSE && ((N & 3) == 0);
    auto load_bias = [&](int t) {
        if (!DENSE) return;
        const int k0 = t * BK;
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
            braw[g] = a;
        }
    };

    // ---- LDS operand reads ----
    const int krow_off = l32 * K::KP + 8 * hf;
    const int i16 = lane & 15, blk = l32 >> 4;
    const int vlane_off = (4 * hf + (i16 >> 2)) * K::VP + 16 * blk + 4 * (i16 & 3);
    bf16x8 ka[K::KS];
    bf16x8 va[C / 32][2];
    auto read_k = [&](int buf) {
        const bf16_t* kr = kt + buf * K::KBLK + krow_off;
#pragma unroll
        for (int ks = 0; ks < K::KS; ks++) ka[ks] = as_bf16x8(*(const u32x4*)(kr + ks * 16));
    };
    auto read_v = [&](int buf) {
        const bf16_t* vbase = vt + buf * K::VBLK + vlane_off;
#pragma unroll
        for (int cb = 0; cb < C / 32; cb++)
#pragma unroll
            for (int kk = 0; kk < 2; kk++) {
                const bf16_t* vp = vbase + (kk * 16) * K::VP + cb * 32;
                va[cb][kk] = join_tr(lds_read_tr16(vp), lds_read_tr16(vp + 8 * K::VP));
            }
    };

    f32x16 s;
    auto s_chain = [&]() {
        if (DENSE) {
#pragma unroll
            for (int g = 0; g < 4; g++) {
                const bf16x4 bv = __builtin_bit_cast(bf16x4, braw[g]);
#pragma unroll
                for (int x = 0; x < 4; x++) s[4 * g + x] = (float)bv[x];
            }
        } else {
#pragma unroll
            for (int r = 0; r < 16; r++) s[r] = 0.f;
        }
#pragma unroll
        for (int ks = 0; ks < K::KS; ks++) s = mfma32(ka[ks], qreg[ks], s);
    };

    // ---- prologue: blocks 0 and 1 in LDS, block 2 in flight, S_0 computed ----
    load_block(0);
    rotate_regs();
    store_block(0);
    load_block(1);
    rotate_regs();
    store_block(1);
    load_block(2);
    rotate_regs();
    store_block(2);
    load_block(3);
    rotate_regs();
    load_block(4);
    load_bias(0);
    __syncthreads();
    read_k(0);
    s_chain();
    load_bias(1);
    read_v(0);
    read_k(1);
    if (grp == 1) __syncthreads();      // group 1 runs one phase behind group 0

    int buf = 0;                        // t % NBUF
    auto body = [&](int t, auto masked_tag) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        const int kb0 = t * BK;
        const int buf1 = (buf + 1) & (NBUF - 1);
        const int buf2 = (buf + 2) & (NBUF - 1);
        const int buf3 = (buf + 3) & (NBUF - 1);

        // ================= VALU phase =================
        store_block(buf3);              // block t+3 (loaded two iterations ago)
        rotate_regs();
        load_block(t + 5);
        __builtin_amdgcn_sched_barrier(0);

        if (MASKED) {
#pragma unroll
            for (int r = 0; r < 16; r++) {
                const int key = kb0 + 8 * (r / 4) + 4 * hf + (r % 4);
                if (key >= N || (CAUSAL && key > qi)) s[r] = -INFINITY;
            }
        }
        bf16x8 pb[2];
        // P = exp2(S log2e - mref), packed to bf16, and this lane's partial row sum
        auto exps = [&](float nm) __attribute__((always_inline)) {
            float ps[4] = {0.f, 0.f, 0.f, 0.f};   // independent partial sums: short dependency chains
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                const bf16x2 pr2 = {(bf16_t)fast_exp2(fmaf(s[r], emul, nm)),
                                    (bf16_t)fast_exp2(fmaf(s[r + 1], emul, nm))};
                ps[(r >> 1) & 3] = pair_sum(pr2, ps[(r >> 1) & 3]);
                pb[r / 8][r % 8] = pr2[0];
                pb[r / 8][r % 8 + 1] = pr2[1];
            }
            return (ps[0] + ps[1]) + (ps[2] + ps[3]);
        };
        // Fast path without the row maximum (see fb_fwd_bf16_impl.h): the partial row sum bounds
        // every probability; inf and NaN fail the test as well.
        float psum = 0.f;
        bool done = false;
        if (ref_ok) {
            psum = exps(-mref);
            done = !__any(!(psum < kSumLimit));
        }
        if (!done) {
            asm volatile("" ::: "memory");   // keep this a real (rarely taken) branch
            const float mx = half_max(max16(s)) * emul;
            if (__any(mx > mref)) {
                const float mnew = fmaxf(fmaxf(mref, mx), -1e30f);
                const float alpha = fast_exp2(mref - mnew);
                mref = mnew;
                lsum *= alpha;
#pragma unroll
                for (int cb = 0; cb < C / 32; cb++)
#pragma unroll
                    for (int r = 0; r < 16; r++) oacc[cb][r] *= alpha;
            }
            psum = exps(mref == -INFINITY ? 0.f : -mref);
            if (!ref_ok) ref_ok = !__any(mref == -INFINITY);
        }
        lsum += psum;
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();

        // ================= MFMA phase =================
        // a block no row of this wave can see contributes P = 0: its chains are skipped
        const bool skip_t = MASKED && CAUSAL && kb0 > qw0 + 31;
        const bool skip_n = MASKED && CAUSAL && kb0 + BK > qw0 + 31;
        // Each MFMA is followed by the LDS read that refills the operand registers it has
        // just consumed (V of block t+1, then K of block t+2), so the reads are spread over
        // the chain instead of stalling the wave in one burst.
        __builtin_amdgcn_s_setprio(2);
        {
            const bf16_t* vbase = vt + buf1 * K::VBLK + vlane_off;
#pragma unroll
            for (int cb = 0; cb < C / 32; cb++)
#pragma unroll
                for (int kk = 0; kk < 2; kk++) {
                    if (!skip_t) oacc[cb] = mfma32(va[cb][kk], pb[kk], oacc[cb]);
                    const bf16_t* vp = vbase + (kk * 16) * K::VP + cb * 32;
                    va[cb][kk] = join_tr(lds_read_tr16(vp), lds_read_tr16(vp + 8 * K::VP));
                    __builtin_amdgcn_sched_barrier(0);
                }
        }
        {
            if (DENSE) {
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    const bf16x4 bv = __builtin_bit_cast(bf16x4, braw[g]);
#pragma unroll
                    for (int x = 0; x < 4; x++) s[4 * g + x] = (float)bv[x];
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; r++) s[r] = 0.f;
            }
            const bf16_t* kr = kt + buf2 * K::KBLK + krow_off;
#pragma unroll
            for (int ks = 0; ks < K::KS; ks++) {
                if (!skip_n) s = mfma32(ka[ks], qreg[ks], s);
                ka[ks] = as_bf16x8(*(const u32x4*)(kr + ks * 16));
                __builtin_amdgcn_sched_barrier(0);
            }
            load_bias(t + 2);
        }
        __builtin_amdgcn_s_setprio(0);
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        buf = buf1;
    };

    int t_plain = N / BK;
    if (CAUSAL) t_plain = min(t_plain, (qw0 + 1) / BK);
    t_plain = min(t_plain, nT);
    int t = 0;
    for (; t < t_plain; t++) body(t, std::false_type{});
    for (; t < nT; t++) body(t, std::true_type{});
    if (grp == 0) __syncthreads();      // balance group 1's extra barrier

    // ---- epilogue: o = O / l, lse = m + ln l ----
    const float ltot = half_sum(lsum);
    const float inv = 1.f / ltot;
    if (qi < N) {
        bf16_t* og = (bf16_t*)p.out + base + (size_t)qi * C;
#pragma unroll
        for (int cb = 0; cb < C / 32; cb++) {
#pragma unroll
            for (int g = 0; g < 4; g++) {
                bf16x4 o4;
#pragma unroll
                for (int x = 0; x < 4; x++) o4[x] = (bf16_t)(oacc[cb][4 * g + x] * inv);
                *(u32x2*)(og + cb * 32 + 8 * g + 4 * hf) = __builtin_bit_cast(u32x2, o4);
            }
        }
        if (hf == 0) p.lse[(size_t)bh * N + qi] = (mref + __log2f(ltot)) * kLn2;
    }
}

template <int C, int RP, int PM, bool CAUSAL, bool DENSE>
int launch(const FwdParams& pin, hipStream_t stream) {
    using K = Cfg<C, RP>;
    auto kern = fwd_bf16_pp_kernel<C, RP, PM, CAUSAL, DENSE>;
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
        case 48: return dispatch_pm<C, 48>(p, stream);
        case 64: return dispatch_pm<C, 64>(p, stream);
        default: return -1;
    }
}

}  // namespace fbpp

#endif
