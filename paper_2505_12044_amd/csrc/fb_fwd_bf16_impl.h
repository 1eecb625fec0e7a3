// bf16 MFMA forward for attention with an additive bias, gfx950.
//
//   low-rank mode: scores = [q*scale | phi_q | 0] . [k | phi_k | 0]   (FlashBias Eq. 3)
//   dense mode   : scores = (q*scale) . k + bias block read from HBM  (the baseline of
//                  Example 3.9)
//
// Work split.  One workgroup = 4 waves = BQ = 128*QB query rows of one (b, h); it walks the
// key/value sequence in blocks of 32 keys.  Each wave owns 32*QB query rows.
//
// Orientation.  Every contraction is computed transposed so that a query is a LANE and the
// keys (or output channels) of a 32-wide block sit in that lane's accumulator registers:
//   S^T[key][query]   = sum_c  Kt[key][c]   * Qreg[query][c]      (A = K block from LDS)
//   O^T[chan][query] += sum_key V^T[chan][key] * P^T[key][query]   (A = V via LDS transpose read)
// The query operand is loop-invariant and stays in registers; the softmax row maximum and
// sum are per-lane reductions over registers plus ONE exchange with the lane 32 away; the
// exponentiated scores are already in the B-operand layout of the second MFMA, so P never
// touches LDS; and rescaling O by a per-query factor is a per-lane multiply.
//
// Pipeline (per wave, one 32-key block per iteration t, LDS ring of three blocks):
//   S  = MFMA chain over K operands of block t          (read from LDS during iteration t-1)
//   regs -> LDS: block t+2   |  global -> regs: block t+3
//   issue LDS transpose reads of V block t              (latency hidden by the softmax)
//   softmax(S) -> P
//   issue LDS reads of K operands of block t+1          (latency hidden by the next chain)
//   O += MFMA chain over V operands and P
//   barrier
// so neither MFMA chain waits on an LDS round trip, and with two workgroups per CU (two
// waves per SIMD, <= 256 registers each) one wave's softmax overlaps the other's MFMAs.
#ifndef FB_FWD_BF16_IMPL_H_
#define FB_FWD_BF16_IMPL_H_

#include <hip/hip_runtime.h>

#include <type_traits>

#include "fb_device.h"
#include "fb_fwd_bf16_dma.h"
#include "fb_fwd_bf16_pp.h"
#include "fb_launch.h"
#include "fb_params.h"

namespace {

constexpr int kPrioMfma = 2;   // wave priority while an MFMA chain is being issued
constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int BK = 32;       // keys per block
constexpr int NBUF = 3;      // LDS ring depth
// The running reference maximum of a row is only raised when a lane's partial sum of the
// block's probabilities reaches 2^tau; until then every probability is below 2^tau, which
// fp32 sums and bf16 P (same exponent range) hold without loss.  The final o = O / l is
// unaffected by the choice of reference.
constexpr float kSumLimit = 256.0f;   // 2^tau, tau = 8

// A piece of NB = 16, 8 or 4 bytes between global memory / LDS and the low words of a u32x4.
template <int NB>
FB_DEV void ld_piece(u32x4& r, const unsigned char* src) {
    if constexpr (NB == 16) {
        r = *(const u32x4*)src;
    } else if constexpr (NB == 8) {
        const u32x2 t = *(const u32x2*)src;
        r.x = t.x; r.y = t.y;
    } else {
        r.x = *(const unsigned*)src;
    }
}
template <int NB>
FB_DEV void st_piece(unsigned char* dst, const u32x4& r) {
    if constexpr (NB == 16) *(u32x4*)dst = r;
    else if constexpr (NB == 8) *(u32x2*)dst = u32x2{r.x, r.y};
    else *(unsigned*)dst = r.x;
}

template <int C, int RP, int QB>
struct Cfg {
    static constexpr int KS = (C + RP) / 16;          // MFMA k-steps of the score contraction
    static constexpr int KP = C + RP + 8;             // K-block row pitch (elements): 16 B pad
    static constexpr int VP = (C == 32) ? 32 : C + 32;  // V-block row pitch: odd multiple of 64 B
    static constexpr int BQ = kWaves * QB * 32;
    static constexpr int KCH = BK * C / 8;            // 16-byte chunks of the K (or V) part of a block
    static constexpr int KIT = (KCH + kThreads - 1) / kThreads;   // per-thread chunks
    static constexpr int PCH = BK * RP / 8;           // chunks of the factor part
    static constexpr int PIT = (PCH + kThreads - 1) / kThreads;
    // whole-chunk factor copies (bf16 factors, R % 8 == 0): pieces sized so that every thread has one
    static constexpr int PPB = RP == 0 ? 16 : ((RP % 64) == 0 ? 16 : ((RP % 32) == 0 ? 8 : 4));
    static constexpr int PPIT = RP == 0 ? 1 : BK * RP * 2 / (PPB * kThreads);
    static constexpr int FIT = (BK * (RP / 6) + kThreads - 1) / kThreads > 0
                                   ? (BK * (RP / 6) + kThreads - 1) / kThreads : 1;   // fp32 (row, rank) items per thread
    static constexpr int KBLK = BK * KP;              // elements per K block buffer
    static constexpr int VBLK = BK * VP;
    static constexpr size_t kLds = (size_t)NBUF * (KBLK + VBLK) * 2;
    static constexpr size_t kBiasLds = (size_t)kWaves * QB * 32 * (BK + 4) * 2;   // dense mode only
    static_assert((C % 32) == 0 && (RP % 16) == 0, "shape granularity");
};

// PM (factor mode): 3 = fp32 factors, one thread per (key, rank) item: three limbs -> six
// product columns; otherwise:
// 0 = no factors, 1 = bf16 factors with R % 8 == 0 (whole 16-byte chunks are
// copied), 2 = general (bf16 factors of any R gathered element-wise, fp32 factors split into
// limbs).
// 4 = ALiBi factors generated in the kernel from the head's slope m (App. D, "decomposition
// in JIT"): phi_q(i) = [-m (i - q0), m], phi_k(j) = [1, j - q0] as fp32 items (R = 2), where q0
// is the tile's first query row.  The product is -m (i - j) for every tile origin; measuring
// positions from q0 keeps the operands small near the diagonal, where the bias matters, so
// the result does not degrade with N.  No factor memory is read.
// One tile: the 128 * QB query rows [qt * BQ, (qt + 1) * BQ) of head bh against all keys they see.
// CG: channels per head in global memory.  CG < C (head dimension 16 run on the C = 32 tiles)
// zero-fills channels CG..C-1 of q, k and v on the way in and never stores them.
template <int C, int RP, int QB, int PM, bool CAUSAL, bool DENSE, int CG = C>
FB_DEV void fwd_tile(const FwdParams& p, unsigned char* smem, const int bh, const int qt, const bool asc = false) {
    using K = Cfg<C, RP, QB>;
    bf16_t* const kt = (bf16_t*)smem;                 // [NBUF][BK][KP]
    bf16_t* const vt = kt + NBUF * K::KBLK;           // [NBUF][BK][VP]
    const int b = bh / p.H, h = bh - b * p.H;
    const int N = p.N, M = p.M, R = PM == 4 ? 2 : p.R;   // N queries, M keys
    const bool phi_f32 = PM == 3 || PM == 4;
    const bool ITEMS = PM == 3 || PM == 4;     // key-side factors handled as (key, rank) items
    // fp32 factors are split into limbs here anyway, so the query operand can carry the log2 e
    // of the exponential (q * scale * log2 e, phi_q * log2 e) and the score accumulator can start
    // at minus the row's reference maximum: the softmax then needs no multiply-add per score.
    // bf16 factors are copied as they are (a rescaled copy would round them again), so those
    // modes keep the multiply-add.  The start value takes 16 registers per query block: used on
    // the 32-channel tiles, where the vector ALU is the bound (-7 % on the C = 16 point-cloud
    // shape) and the registers are free.  At C = 128 it gains 1-2 % at most, and it rounds
    // q * scale * log2 e where the backward rounds q * scale: scores that differ by one bf16
    // rounding between the passes leave the rows of dS summing to ~1e-3 D instead of zero, which
    // factor gradients of absolute positions (ALiBi) multiply by up to N.  Not used there.
    // (The same fold for bf16 factors - phi_q * log2 e carried as two bf16 limbs, the factor k-steps
    // issued twice against the same K operand registers - was measured and lost: the extra MFMA per
    // block costs more than the sixteen multiply-adds it saves, 0.0695 against 0.0668 ms on the
    // Pairformer shape.)
    constexpr bool FOLD = !DENSE && (PM == 3 || PM == 4) && C == 32;
    // RAWQ (head dimensions 64 and 128; no factors, fp32 factors or factors made in the kernel): the
    // query operand is q itself, not bf16(q scale).  q k^T scale + phi_q phi_k^T = scale (q k^T +
    // (phi_q / scale) phi_k^T): the factor columns carry 1/scale (applied in fp32, before the limb
    // split) and the scale goes into the exponent's multiply-add.  One rounding less on the scores,
    // and the backward, which recomputes exactly these scores, can read q in place as well.
    constexpr bool RAWQ = !DENSE && !FOLD && C % 64 == 0 && CG == C && (PM == 0 || PM == 3 || PM == 4);
    const float qmul = FOLD ? kLog2e : (RAWQ ? p.inv_scale : 1.f);       // factor of the query-side factor columns
    const float emul = RAWQ ? p.scale * kLog2e : kLog2e;                 // scores to exponents of two
    const float slope = PM == 4 ? p.slopes[h] * qmul : 0.f;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps everything derived from it scalar

    const int l32 = lane & 31, hf = lane >> 5;
    const int q0 = qt * K::BQ;
    const int qw0 = q0 + wave * (QB * 32);

    const size_t base = (size_t)bh * N * CG;
    const size_t kbase = (size_t)bh * M * CG;
    const bf16_t* qg = (const bf16_t*)p.q + base;
    const bf16_t* kg = (const bf16_t*)p.k + kbase;
    const bf16_t* vg = (const bf16_t*)p.v + kbase;
    const size_t phi_esz = phi_f32 ? 4 : 2;
    const unsigned char* pqg = nullptr;
    const unsigned char* pkg = nullptr;
    if (RP > 0) {
        pqg = (const unsigned char*)p.phi_q + ((size_t)b * p.phi_bstride + (size_t)h * N * R) * phi_esz;
        pkg = (const unsigned char*)p.phi_k + ((size_t)b * p.phik_bstride + (size_t)h * M * R) * phi_esz;
    }
    const bf16_t* bg = nullptr;
    if (DENSE) bg = (const bf16_t*)p.bias + (size_t)b * p.bias_bstride + (size_t)h * N * M;

    bf16x8 qreg[QB][K::KS];     // query operand, filled in the prologue below

    f32x16 oacc[QB][C / 32];
    float mref[QB], lsum[QB];
    bool ref_ok[QB];      // wave-uniform: every row of the wave has a finite reference maximum
    f32x16 sinit[QB];   // FOLD: minus the reference maximum, the score chain's start value
#pragma unroll
    for (int qb = 0; qb < QB; qb++) {
        if (FOLD) {
#pragma unroll
            for (int r = 0; r < 16; r++) sinit[qb][r] = 0.f;
        }
        mref[qb] = -INFINITY;
        lsum[qb] = 0.f;
        ref_ok[qb] = false;
#pragma unroll
        for (int cb = 0; cb < C / 32; cb++)
#pragma unroll
            for (int r = 0; r < 16; r++) oacc[qb][cb][r] = 0.f;
    }

    const int kend = CAUSAL ? min(M, q0 + K::BQ) : M;
    const int nT = (kend + BK - 1) / BK;
    // Causal tiles start at their diagonal blocks: with a recency bias such as ALiBi the row
    // maximum is then met at once and the accumulator is never rescaled again (walking up to
    // the diagonal it would be rescaled in nearly every block).  The other blocks follow either
    // downwards to key 0 or (asc) upwards from key 0.  The first tile of a workgroup's pair
    // goes up and the second down: the workgroups of one head, launched together, then read
    // the same key block at the same time in both phases (the tile n-1-u reaches block t after
    // 4 QB + t steps whatever u is, and every second tile reaches block 0 after the same total
    // number of steps), so a K/V block is fetched into the XCD's L2 once instead of once per
    // straggling workgroup.
    const int nd = CAUSAL ? nT - q0 / BK : 0;      // blocks on the tile's diagonal (taken first, downwards)
    auto blk_of = [&](int t) {
        if (!CAUSAL) return t;
        if (asc && t >= nd) return min(t - nd, nT - 1);
        return max(nT - 1 - t, 0);
    };

    // ---- block staging: global -> registers -> LDS.  Rows past M are clamped to row M-1; the
    // keys they stand for are masked to -inf before the softmax, so their values never count.
    // The K and V rows of a block are copied in pieces of KPB bytes, sized so that every thread
    // holds at least one piece (16 bytes for C >= 64, 8 for C = 32, 4 for 16-channel rows): no
    // thread is idle, so the staging code carries no exec-mask branches.
    constexpr int KBYTES = BK * CG * 2;
    constexpr int KPB = KBYTES / kThreads >= 16 ? 16 : KBYTES / kThreads;
    constexpr int KITP = KBYTES / (KPB * kThreads);
    static_assert(KPB == 16 || KPB == 8 || KPB == 4, "piece size");
    // Whole-chunk factor copies (PM == 1) in per-thread pieces as well, where 16-byte chunks would leave
    // threads idle and cost exec-mask branches (C <= 64: -4 % on the Pairformer shape); at C = 128 the
    // 16-byte chunk copy measured 8 % faster on the long-sequence shape and is kept.
    constexpr bool PPIECES = PM == 1 && C <= 64;
    // fp32 factor items.  When a block has fewer items than the workgroup has threads (small R), one
    // wave takes all of a block's items (64 per pass) and the waves take turns block by block: the
    // other three skip the item code behind a scalar branch instead of running it with a quarter
    // of their lanes (-1.4 % per launch at R = 2, C = 128).
    constexpr bool DUTY = (PM == 3 || PM == 4) && BK * (RP / 6) < kThreads;
    constexpr int FITN = DUTY ? (BK * (RP / 6) + 63) / 64 : K::FIT;
    constexpr int PRW = PPIECES ? K::PPIT : (K::PIT > 0 ? K::PIT : 1);
    struct Stage {                       // one block in flight between global memory and LDS
        u32x4 kraw[KITP], vraw[KITP];
        u32x4 praw[PRW];
        float fraw[FITN];                // fp32 factors: one (key row, rank) item
    };
    auto init_stage = [&](Stage& g) {    // chunks and items a thread never loads stay zero
#pragma unroll
        for (int it = 0; it < KITP; it++) {
            g.kraw[it] = u32x4{0u, 0u, 0u, 0u};
            g.vraw[it] = u32x4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int it = 0; it < PRW; it++) g.praw[it] = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int it = 0; it < FITN; it++) g.fraw[it] = 0.f;
    };
    Stage st;
    init_stage(st);
    // fp32 factors: item e = (key row, rank r) of a block, spread evenly over the four waves (or all
    // in the wave on duty)
    int fitem_row[FITN], fitem_r[FITN];
    bool fitem_ok[FITN];
    const float* pkf = (const float*)pkg;
    if (ITEMS) {
#pragma unroll
        for (int it = 0; it < FITN; it++) {
            const int e = DUTY ? lane + 64 * it : lane * kWaves + wave + it * kThreads;
            fitem_ok[it] = e < BK * R;
            fitem_row[it] = fitem_ok[it] ? e / R : 0;
            fitem_r[it] = fitem_ok[it] ? e - fitem_row[it] * R : 0;
        }
        // the columns past 6R of every ring slot stay zero for the whole kernel
        for (int e = tid; e < NBUF * BK * (RP / 2); e += kThreads) {
            const int row = e / (RP / 2), c2 = e % (RP / 2);
            *(unsigned*)(kt + (size_t)row * K::KP + C + 2 * c2) = 0u;   // rows of all slots are contiguous
        }
        __syncthreads();   // before any thread writes item columns into the same rows
    }

    // This thread's chunks of a block: byte offset of the chunk's row inside the block and of the
    // chunk inside the row (rows of CG elements); chunks of the channels past CG are never
    // loaded and stay zero.  All offsets inside one head fit 32 bits (the entry points reject
    // larger problems).  A row past M is clamped to row M-1 by a minimum on the byte offset,
    // so one code path serves whole and partial blocks without a multiply.
    unsigned grow[KITP], gcol[KITP], klds[KITP], vlds[KITP];
#pragma unroll
    for (int it = 0; it < KITP; it++) {
        const int byte = (tid + it * kThreads) * KPB;
        const int row = byte / (CG * 2), colb = byte % (CG * 2);
        grow[it] = (unsigned)(row * CG * 2);
        gcol[it] = (unsigned)colb;
        klds[it] = (unsigned)(row * K::KP * 2 + colb);     // byte offsets inside a ring slot
        vlds[it] = (unsigned)(row * K::VP * 2 + colb);
    }
    if (CG < C) {
        // channels the caller's rows do not have: zero in every ring slot, once (no piece ever lands there)
        constexpr int ZW = (C - CG) / 2;      // dwords per row
        for (int e = tid; e < NBUF * BK * ZW; e += kThreads) {
            const int row = e / ZW, c2 = e % ZW;
            *(unsigned*)(kt + (size_t)row * K::KP + CG + 2 * c2) = 0u;
            *(unsigned*)(vt + (size_t)row * K::VP + CG + 2 * c2) = 0u;
        }
    }
    // whole-chunk factor pieces (PM == 1): LDS byte offset, memory row offset and column byte of each
    unsigned prow[PRW], pcolb[PRW], plds[PRW];
    bool pvalid[PRW];
    if (PPIECES) {
#pragma unroll
        for (int it = 0; it < PRW; it++) {
            const int byte = (tid + it * kThreads) * K::PPB;
            const int row = byte / (RP * 2 > 0 ? RP * 2 : 1), colb = byte % (RP * 2 > 0 ? RP * 2 : 1);
            pvalid[it] = colb < R * 2;                              // a piece lies wholly inside or outside the R columns
            prow[it] = (unsigned)row;
            pcolb[it] = pvalid[it] ? (unsigned)colb : 0u;          // outside: read column 0 (valid memory), store zero
            plds[it] = (unsigned)(row * K::KP * 2 + (C * 2) + colb);
        }
    }
    const unsigned char* kgb = (const unsigned char*)kg;
    const unsigned char* vgb = (const unsigned char*)vg;
    const unsigned kv_last = (unsigned)(M - 1) * (unsigned)(CG * 2);       // byte offset of the last row
    const unsigned phi_rb = (unsigned)R * (unsigned)phi_esz;                // bytes per factor row
    const unsigned phi_last = (unsigned)(M - 1) * phi_rb;
    unsigned fitem_off[FITN], fitem_col[FITN];
    if (PM == 3) {
#pragma unroll
        for (int it = 0; it < FITN; it++) {
            fitem_off[it] = (unsigned)fitem_row[it] * phi_rb;
            fitem_col[it] = (unsigned)fitem_r[it] * 4u;
        }
    }

    auto load_block = [&](int t, Stage& g) {
        const int k0 = blk_of(t) * BK;
        const unsigned boff = (unsigned)k0 * (unsigned)(CG * 2);
        const unsigned pboff = (unsigned)k0 * phi_rb;
#pragma unroll
        for (int it = 0; it < KITP; it++) {
            const unsigned off = min(boff + grow[it], kv_last) + gcol[it];
            ld_piece<KPB>(g.kraw[it], kgb + off);
            ld_piece<KPB>(g.vraw[it], vgb + off);
        }
        const bool on_duty = !DUTY || (t & (kWaves - 1)) == wave;     // wave-uniform
        if (PM == 3) {
            if (on_duty) {
#pragma unroll
                for (int it = 0; it < FITN; it++)
                    if (fitem_ok[it])
                        g.fraw[it] = *(const float*)(pkg + (min(pboff + fitem_off[it], phi_last) + fitem_col[it]));
            }
        } else if (PM == 4) {
            if (on_duty) {
#pragma unroll
                for (int it = 0; it < FITN; it++)
                    g.fraw[it] = fitem_r[it] == 0 ? 1.f : (float)(k0 + fitem_row[it] - q0);
            }
        } else if (PPIECES) {
#pragma unroll
            for (int it = 0; it < PRW; it++) {
                const unsigned char* src = pkg + min(pboff + __umul24(prow[it], phi_rb), phi_last) + pcolb[it];
                ld_piece<K::PPB>(g.praw[it], src);
            }
        } else if (PM != 0) {
#pragma unroll
            for (int it = 0; it < K::PIT; it++) {
                // general mode: rotate the factor chunks over the waves from block to block so
                // the conversion work is shared (whole-chunk copies need no conversion)
                const int e = ((tid + (PM == 2 ? 64 * t : 0)) & (kThreads - 1)) + it * kThreads;
                if (K::PCH % kThreads == 0 || e < K::PCH) {
                    const int row = e / (RP / 8), c8 = e % (RP / 8);
                    const unsigned char* src = pkg + min(pboff + __umul24((unsigned)row, phi_rb), phi_last);
                    if (PM == 1) {
                        g.praw[it] = (c8 * 8 < R) ? *(const u32x4*)(src + c8 * 16) : u32x4{0u, 0u, 0u, 0u};
                    } else {
                        g.praw[it] = phi_chunk_raw(src, c8, R, phi_f32, true);
                    }
                }
            }
        }
    };

    // t is the block whose registers are being stored (the rotation must match load_block)
    auto store_block = [&](int buf, int t, const Stage& g) {
        bf16_t* kdst = kt + buf * K::KBLK;
        bf16_t* vdst = vt + buf * K::VBLK;
        // One wait for every load in flight (they were issued a whole iteration ago) instead of the
        // wait per store the compiler would place: -9 % on the Pairformer shape, -3 % on the point-cloud
        // shape, neutral at C = 128.
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0); expcnt and lgkmcnt unconstrained
#pragma unroll
        for (int it = 0; it < KITP; it++) {
            st_piece<KPB>((unsigned char*)kdst + klds[it], g.kraw[it]);
            st_piece<KPB>((unsigned char*)vdst + vlds[it], g.vraw[it]);
        }
        if (ITEMS) {
            if (!DUTY || (t & (kWaves - 1)) == wave) {      // same block, same wave as in load_block
#pragma unroll
                for (int it = 0; it < FITN; it++)
                    if (fitem_ok[it]) phi_item_store_k(kdst + fitem_row[it] * K::KP + C + 6 * fitem_r[it], g.fraw[it]);
            }
        } else if (PPIECES) {
#pragma unroll
            for (int it = 0; it < PRW; it++) {
                u32x4 v = g.praw[it];
                if (!pvalid[it]) v = u32x4{0u, 0u, 0u, 0u};      // a select, not a branch
                st_piece<K::PPB>((unsigned char*)kdst + plds[it], v);
            }
        } else if (PM != 0) {
#pragma unroll
            for (int it = 0; it < K::PIT; it++) {
                const int e = ((tid + (PM == 2 ? 64 * t : 0)) & (kThreads - 1)) + it * kThreads;
                if (K::PCH % kThreads == 0 || e < K::PCH) {
                    const int row = e / (RP / 8), c8 = e % (RP / 8);
                    const u32x4 v = PM == 1 ? g.praw[it] : as_uint4(phi_chunk_finish<false>(g.praw[it], c8, phi_f32));
                    *(u32x4*)(kdst + row * K::KP + C + c8 * 8) = v;
                }
            }
        }
    };

    // dense mode: each wave streams the [32*QB rows] x [32 keys] bias block of its own rows
    // with coalesced 16-byte loads (four lanes per 64-byte row segment), one block ahead, into
    // registers, parks it in a wave-private LDS tile and reads it back in accumulator order
    // (row = lane % 32, keys 8*g + 4*hf + 0..3) as the initial value of the S chain.  Chunks
    // wholly above the diagonal or past the end are never read.
    constexpr int BP = BK + 4;                       // bias tile row pitch (elements): 72 bytes
    bf16_t* const bt = vt + NBUF * K::VBLK + wave * (QB * 32 * BP);
    u32x4 braw[DENSE ? QB : 1][2];
    const bool bias_fast = DENSE && ((M & 7) == 0);
    auto load_bias = [&](int t) {
        if (!DENSE) return;
        const int k0 = blk_of(t) * BK;
#pragma unroll
        for (int qb = 0; qb < QB; qb++) {
#pragma unroll
            for (int i = 0; i < 2; i++) {
                const int e = lane + 64 * i;
                const int row = e >> 2, c = e & 3;
                const int qi = qw0 + qb * 32 + row;
                const int j = k0 + 8 * c;
                u32x4 a = u32x4{0u, 0u, 0u, 0u};
                if (qi < N && j < M && !(CAUSAL && j > qi)) {
                    const bf16_t* src = bg + (size_t)qi * M + j;
                    if (bias_fast) {
                        a = *(const u32x4*)src;
                    } else {
                        bf16x8 tmp;
#pragma unroll
                        for (int x = 0; x < 8; x++) tmp[x] = (j + x < M) ? src[x] : (bf16_t)0.f;
                        a = as_uint4(tmp);
                    }
                }
                braw[qb][i] = a;
            }
        }
    };
    auto stage_bias = [&]() {
        if (!DENSE) return;
#pragma unroll
        for (int qb = 0; qb < QB; qb++) {
#pragma unroll
            for (int i = 0; i < 2; i++) {
                const int e = lane + 64 * i;
                const int row = e >> 2, c = e & 3;
                u32x2* d = (u32x2*)(bt + (qb * 32 + row) * BP + 8 * c);   // 8-byte aligned
                d[0] = u32x2{braw[qb][i].x, braw[qb][i].y};
                d[1] = u32x2{braw[qb][i].z, braw[qb][i].w};
            }
        }
    };

    // ---- LDS operand reads ----
    const int krow_off = l32 * K::KP + 8 * hf;
    // lane -> (row group, column group) of the LDS transpose read: the 16-lane group
    // blk = l32 / 16 covers channels 16*blk..+15, lane i = lane % 16 supplies row i/4, columns
    // 4*(i%4)..+3; the half hf selects keys 4*hf..4*hf+3 (+8 for the high part), matching the
    // keys of accumulator registers 0..3 / 4..7 of each 16-key group.
    const int i16 = lane & 15, blk = l32 >> 4;
    const int vlane_off = (4 * hf + (i16 >> 2)) * K::VP + 16 * blk + 4 * (i16 & 3);

    // k-steps over channels the caller's rows do not have (CG < C) are all zero on both sides
    auto kstep_live = [](int ks) constexpr { return !(ks < C / 16 && ks * 16 >= CG); };
    bf16x8 ka[K::KS];
    auto read_k = [&](int buf) {
        const bf16_t* krow = kt + buf * K::KBLK + krow_off;
#pragma unroll
        for (int ks = 0; ks < K::KS; ks++)
            if (kstep_live(ks)) ka[ks] = as_bf16x8(*(const u32x4*)(krow + ks * 16));
    };

    // ---- prologue: blocks 0 and 1 into LDS, block 2 in flight, K operands of block 0 ----
    // Blocks 0 and 1 and the query rows are requested together, so the tile's set-up costs one
    // global round trip instead of three.
    {
        Stage st1;
        init_stage(st1);
        load_block(0, st);
        load_block(1, st1);
        // ---- query operand [q*scale | phi_q | 0] in registers (B-operand layout).  Rows past N
        // read row N-1 (finite values) and are never stored.
        const float qscale = FOLD ? p.scale * kLog2e : p.scale;
#pragma unroll
        for (int qb = 0; qb < QB; qb++) {
            const int qi = min(qw0 + qb * 32 + l32, N - 1);
#pragma unroll
            for (int ks = 0; ks < K::KS; ks++) {
                bf16x8 val;
                if (ks < C / 16) {
                    if (ks * 16 < CG) {
                        const bf16x8 x = as_bf16x8(*(const u32x4*)(qg + (size_t)qi * CG + ks * 16 + 8 * hf));
#pragma unroll
                        for (int e = 0; e < 8; e++) val[e] = RAWQ ? x[e] : (bf16_t)((float)x[e] * qscale);
                    } else {
#pragma unroll
                        for (int e = 0; e < 8; e++) val[e] = (bf16_t)0.f;
                    }
                } else {
                    const int c8 = (ks - C / 16) * 2 + hf;
                    if (PM == 4) val = phi_chunk_from_pair(c8, -slope * (float)(qi - q0), slope);
                    else val = phi_chunk_gather<true>(pqg + (size_t)qi * R * phi_esz, c8, R, phi_f32, qmul);
                }
                qreg[qb][ks] = val;
            }
        }
        store_block(0, 0, st);
        store_block(1, 1, st1);
    }
    load_block(2, st);
    load_bias(0);
    stage_bias();
    load_bias(1);
    __syncthreads();
    read_k(0);

    int buf = 0;                 // t % NBUF
    // One block.  MASKED instances apply the causal / sequence-end masks and may skip the
    // MFMA chains of a block no row of this wave can see; interior blocks carry none of that.
    // slot_tag: the ring slot of block t when it is known at compile time (the steady-state loop is
    // unrolled by the ring depth, which turns every LDS address of a block into lane offset +
    // immediate), else -1 and the running `buf` is used.
    auto body = [&](int t, auto masked_tag, auto slot_tag) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        constexpr int SB = decltype(slot_tag)::value;
        const int kb0 = blk_of(t) * BK;
        const int cbuf = SB >= 0 ? SB : buf;                                              // t % NBUF
        const int buf1 = SB >= 0 ? (SB + 1) % NBUF : (buf == NBUF - 1 ? 0 : buf + 1);     // (t+1) % NBUF
        const int buf2 = SB >= 0 ? (SB + 2) % NBUF : (buf1 == NBUF - 1 ? 0 : buf1 + 1);   // (t+2) % NBUF
        // wave-uniform: is this block wholly invisible to this wave (causal), or does it need masks?
        const bool skip = MASKED && CAUSAL && kb0 > qw0 + QB * 32 - 1;

        // ---- S^T = Kt . Qreg ----
        f32x16 s[QB];
#pragma unroll
        for (int qb = 0; qb < QB; qb++) {
            if (DENSE) {
                const bf16_t* brow = bt + (qb * 32 + l32) * BP + 4 * hf;
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    const bf16x4 bv = __builtin_bit_cast(bf16x4, *(const u32x2*)(brow + 8 * g));
#pragma unroll
                    for (int x = 0; x < 4; x++) s[qb][4 * g + x] = (float)bv[x];
                }
            } else if (FOLD) {
                s[qb] = sinit[qb];
            } else {
#pragma unroll
                for (int r = 0; r < 16; r++) s[qb][r] = 0.f;
            }
        }
        // The V operand reads of this block are spread over the S chain (one transpose-read
        // pair per MFMA) so they neither stall the wave in a burst nor wait for the softmax.
        bf16x8 va[C / 32][2];
        {
            const bf16_t* vbase = vt + cbuf * K::VBLK + vlane_off;
            constexpr int NV = (C / 32) * 2;
            __builtin_amdgcn_s_setprio(kPrioMfma);
#pragma unroll
            for (int ks = 0; ks < K::KS; ks++) {
                if (!skip) {
#pragma unroll
                    for (int qb = 0; qb < QB; qb++)
                        if (kstep_live(ks)) s[qb] = mfma32(ka[ks], qreg[qb][ks], s[qb]);
                }
                // distribute the NV reads over the KS steps
#pragma unroll
                for (int i = (ks * NV) / K::KS; i < ((ks + 1) * NV) / K::KS; i++) {
                    const bf16_t* vp = vbase + ((i & 1) * 16) * K::VP + (i >> 1) * 32;
                    va[i >> 1][i & 1] = join_tr(lds_read_tr16(vp), lds_read_tr16(vp + 8 * K::VP));
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            __builtin_amdgcn_s_setprio(0);
        }

        // K operands of the next block right behind the score chain: they land during the softmax, so
        // the wait for all LDS traffic that precedes the barrier finds them done (issued between the
        // MFMAs of the value contraction they completed only at the barrier: +2-3 % per launch)
        read_k(buf1);
        __builtin_amdgcn_sched_barrier(0);
        // ---- staging: block t+2 registers -> LDS, block t+3 global -> registers ----
        store_block(buf2, t + 2, st);
        load_block(t + 3, st);
        stage_bias();                   // block t+1 (loaded one iteration ago) -> wave-private LDS
        load_bias(t + 2);
        __builtin_amdgcn_sched_barrier(0);

        // ---- online softmax: a row lives in this lane and the one 32 away ----
        bf16x8 pb[QB][2];
#pragma unroll
        for (int qb = 0; qb < QB; qb++) {
            if (MASKED) {
                const int qi = qw0 + qb * 32 + l32;
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    const int key = kb0 + 8 * (r / 4) + 4 * hf + (r % 4);
                    if (key >= M || (CAUSAL && key > qi)) s[qb][r] = -INFINITY;
                }
            }
            // P = exp2(S log2e - mref), packed to bf16, and this lane's partial row sum (FOLD: the
            // scores arrive as S log2e - mref)
            auto exps = [&](float nm) __attribute__((always_inline)) {
                float ps[4] = {0.f, 0.f, 0.f, 0.f};   // independent partial sums: short dependency chains
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    const bf16x2 pr2 = {(bf16_t)fast_exp2(FOLD ? s[qb][r] : fmaf(s[qb][r], emul, nm)),
                                        (bf16_t)fast_exp2(FOLD ? s[qb][r + 1] : fmaf(s[qb][r + 1], emul, nm))};
                    ps[(r >> 1) & 3] = pair_sum(pr2, ps[(r >> 1) & 3]);
                    pb[qb][r / 8][r % 8] = pr2[0];
                    pb[qb][r / 8][r % 8 + 1] = pr2[1];
                }
                return (ps[0] + ps[1]) + (ps[2] + ps[3]);
            };
            // Fast path: once every row of the wave has a finite reference maximum, the block's row
            // maximum is not computed at all.  Any reference is exact as long as nothing overflows,
            // and the partial row sum (needed anyway) bounds every probability from above: if it
            // stays below 2^tau in every lane, so did each of them.  inf and NaN fail the test too.
            float psum = 0.f;
            bool done = false;
            if (ref_ok[qb]) {
                psum = exps(-mref[qb]);
                done = !__any(!(psum < kSumLimit));
            }
            if (!done) {
                // first visible blocks of a tile, or the scores outgrew the reference: take the true
                // row maximum, rescale what has been accumulated, and redo the exponentials
                asm volatile("" ::: "memory");   // keep this a real (rarely taken) branch
                // FOLD: what the scores already carry (0 while the row has no reference)
                const float emb = mref[qb] == -INFINITY ? 0.f : mref[qb];
                const float mx = FOLD ? half_max(max16(s[qb])) + emb : half_max(max16(s[qb])) * emul;
                if (__any(mx > mref[qb])) {
                    const float mnew = fmaxf(fmaxf(mref[qb], mx), -1e30f);
                    const float alpha = fast_exp2(mref[qb] - mnew);
                    mref[qb] = mnew;
                    lsum[qb] *= alpha;
#pragma unroll
                    for (int cb = 0; cb < C / 32; cb++)
#pragma unroll
                        for (int r = 0; r < 16; r++) oacc[qb][cb][r] *= alpha;
                }
                // a row that has not met a visible key yet (causal, reverse order) keeps p = 0
                const float emb2 = mref[qb] == -INFINITY ? 0.f : mref[qb];
                if (FOLD) {
#pragma unroll
                    for (int r = 0; r < 16; r++) {
                        s[qb][r] += emb - emb2;     // masked scores stay -inf
                        sinit[qb][r] = -emb2;
                    }
                }
                psum = exps(-emb2);
                if (!ref_ok[qb]) ref_ok[qb] = !__any(mref[qb] == -INFINITY);
            }
            lsum[qb] += psum;
        }
        __builtin_amdgcn_sched_barrier(0);

        // ---- O^T += V^T . P^T ----
        {
            constexpr int NM = (C / 32) * 2;
            __builtin_amdgcn_s_setprio(kPrioMfma);
#pragma unroll
            for (int i = 0; i < NM; i++) {
                if (!skip) {
#pragma unroll
                    for (int qb = 0; qb < QB; qb++)
                        oacc[qb][i >> 1] = mfma32(va[i >> 1][i & 1], pb[qb][i & 1], oacc[qb][i >> 1]);
                }
            }
            __builtin_amdgcn_s_setprio(0);
        }
        __syncthreads();
        if (SB < 0) buf = buf1;
    };
    using Dyn = std::integral_constant<int, -1>;
    // blocks [t, t_end) without masks: single steps until the ring is at slot 0, then whole turns of
    // the ring with compile-time slots, then the remainder
    auto plain_run = [&](int t, int t_end) {
        for (; t < t_end && buf != 0; t++) body(t, std::false_type{}, Dyn{});
        for (; t + NBUF <= t_end; t += NBUF) {
            body(t, std::false_type{}, std::integral_constant<int, 0>{});
            body(t + 1, std::false_type{}, std::integral_constant<int, 1>{});
            body(t + 2, std::false_type{}, std::integral_constant<int, 2>{});
        }
        for (; t < t_end; t++) body(t, std::false_type{}, Dyn{});
    };
    static_assert(NBUF == 3, "plain_run unrolls three slots");

    // leading blocks that need no mask for any row of this wave, then the rest
    int t_plain = M / BK;
    if (CAUSAL) t_plain = min(t_plain, (qw0 + 1) / BK);
    t_plain = min(t_plain, nT);
    if (CAUSAL) {   // reverse order: the masked blocks (diagonal, sequence end) come first
        int t = 0;
        for (; t < nT - t_plain; t++) body(t, std::true_type{}, Dyn{});
        plain_run(t, nT);
    } else {
        plain_run(0, t_plain);
        for (int t = t_plain; t < nT; t++) body(t, std::true_type{}, Dyn{});
    }

    // ---- epilogue: o = O / l, lse = m + ln l ----
#pragma unroll
    for (int qb = 0; qb < QB; qb++) {
        const int qi = qw0 + qb * 32 + l32;
        const float ltot = half_sum(lsum[qb]);
        const float inv = 1.f / ltot;
        if (qi < N) {
            bf16_t* og = (bf16_t*)p.out + base + (size_t)qi * CG;
#pragma unroll
            for (int cb = 0; cb < C / 32; cb++) {
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    if (cb * 32 + 8 * g >= CG) continue;
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

// Work units.  Non-causal: one tile per workgroup.  Causal: the tile qt sees 4 * QB * (qt + 1)
// key blocks, so a workgroup takes the pair (n - 1 - u, u): every workgroup then walks the
// same number of key blocks and the launch has no long tail of heavy tiles (with single
// tiles per workgroup the heaviest tile alone lasts almost half of the whole launch at
// N = 4096).  Units are numbered so that each XCD gets a contiguous run (workgroup w lands
// on XCD w % 8): the workgroups sharing one head's K/V also share one L2.
template <int C, int RP, int QB, int PM, bool CAUSAL, bool DENSE, int CG = C>
__global__ __launch_bounds__(kThreads, 2) void fwd_bf16_kernel(FwdParams p) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int L = (blockIdx.x & 7) * p.tiles_per_xcd + (blockIdx.x >> 3);
    if (L >= p.total_tiles) return;
    int bh, u;
    if (DENSE && p.bias_bstride == 0) {
        // bias shared over the batch: the B workgroups that read the same bias tile are
        // neighbours in the launch order, so the tile is fetched from HBM once per XCD
        const int rest = L / p.B;
        const int bb = L - rest * p.B;
        const int hh = rest / p.n_units;
        u = rest - hh * p.n_units;
        bh = bb * p.H + hh;
    } else {
        bh = L / p.n_units;
        u = L - bh * p.n_units;
    }
    if (CAUSAL) {
        const int heavy = p.n_qtiles - 1 - u;
        fwd_tile<C, RP, QB, PM, CAUSAL, DENSE, CG>(p, smem, bh, heavy, p.causal_up != 0);
        if (u != heavy) {
            __syncthreads();   // the LDS ring is reused: every wave must have left the first tile
            fwd_tile<C, RP, QB, PM, CAUSAL, DENSE, CG>(p, smem, bh, u);
        }
    } else {
        fwd_tile<C, RP, QB, PM, CAUSAL, DENSE, CG>(p, smem, bh, u);
    }
}

template <int C, int RP, int QB, int PM, bool CAUSAL, bool DENSE, int CG = C>
int launch(const FwdParams& pin, hipStream_t stream) {
    using K = Cfg<C, RP, QB>;
    auto kern = fwd_bf16_kernel<C, RP, QB, PM, CAUSAL, DENSE, CG>;
    static FbLdsOnce once;
    constexpr size_t lds_bytes = K::kLds + (DENSE ? K::kBiasLds : 0);
    if (!fb_raise_lds_limit((const void*)kern, lds_bytes, once)) return 1;
    FwdParams p = pin;
    p.n_qtiles = (p.N + K::BQ - 1) / K::BQ;
    p.n_units = CAUSAL ? (p.n_qtiles + 1) / 2 : p.n_qtiles;
    p.total_tiles = p.B * p.H * p.n_units;
    p.tiles_per_xcd = (p.total_tiles + 7) / 8;
    hipLaunchKernelGGL(kern, dim3(8 * p.tiles_per_xcd), dim3(kThreads), lds_bytes, stream, p);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

template <int C, int RP, int QB, int PM, bool DENSE, int CG = C>
int dispatch_causal(const FwdParams& p, hipStream_t stream) {
    if (p.causal) return launch<C, RP, QB, PM, true, DENSE, CG>(p, stream);
    return launch<C, RP, QB, PM, false, DENSE, CG>(p, stream);
}

template <int C, int RP, int PM, bool DENSE, int CG = C>
int dispatch_qb(const FwdParams& p, int qb, hipStream_t stream) {
    if constexpr (C <= 64) {
        if (qb == 2) return dispatch_causal<C, RP, 2, PM, DENSE, CG>(p, stream);
    }
    return dispatch_causal<C, RP, 1, PM, DENSE, CG>(p, stream);
}

template <int C, int RP, int CG = C>
int dispatch_pm(const FwdParams& p, int qb, hipStream_t stream) {
    if (p.phi_f32) return dispatch_qb<C, RP, 3, false, CG>(p, qb, stream);
    if ((p.R % 8) == 0) return dispatch_qb<C, RP, 1, false, CG>(p, qb, stream);
    return dispatch_qb<C, RP, 2, false, CG>(p, qb, stream);
}

// rp: padded factor width (multiple of 16, <= 64); qb: 32-row query blocks per wave of the
// four-wave kernel (1 or 2; 2 exists for C <= 64 only and falls back to 1 otherwise), 8 for the
// eight-wave ping-pong kernel, 16 for the direct-to-LDS kernel.
// Returns 0 on success, 1 on launch failure, -1 when no instantiation fits.
template <int C>
int fwd_bf16_dispatch(const FwdParams& p, int rp, bool dense, int qb, hipStream_t stream) {
    if (qb == 8) return fbpp::dispatch<C>(p, rp, dense, stream);
    if (qb == 16) {
        const int rc = fbdma::dispatch<C>(p, rp, dense, stream);
        if (rc >= 0) return rc;
        qb = 1;   // shapes the direct-to-LDS kernel does not take
    }
    if (dense) return dispatch_qb<C, 0, 0, true>(p, qb, stream);
    switch (rp) {
        case 0: return dispatch_qb<C, 0, 0, false>(p, qb, stream);
        case 16: return dispatch_pm<C, 16>(p, qb, stream);
        case 32: return dispatch_pm<C, 32>(p, qb, stream);
        case 48: return dispatch_pm<C, 48>(p, qb, stream);
        case 64: return dispatch_pm<C, 64>(p, qb, stream);
        default: break;
    }
    // wider factor blocks: the C (R - 1) extra channels of the multiplicative form (App. I), always
    // whole 16-byte chunks of bf16 columns; one query block per wave (the operand registers of two
    // would not fit two waves per SIMD)
    if constexpr (C <= 64) {
        if (p.phi_f32 || (p.R % 8) != 0) return -1;
        if (rp == 96) return dispatch_causal<C, 96, 1, 1, false>(p, stream);
        if (rp == 128) return dispatch_causal<C, 128, 1, 1, false>(p, stream);
    }
    return -1;
}

}  // namespace

#endif
