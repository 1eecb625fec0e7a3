// bf16 MFMA backward of attention with a factorised bias, gfx950.
//
// With Aq = [q*scale | phi_q], Ak = [k | phi_k] (FlashBias Eq. 3) and S = Aq Ak^T,
// P = exp(S - lse), the chain rule for L = sum(dO * O) gives
//   dV = P^T dO,  dP = dO V^T,  dS = P o (dP - D),  D_i = sum_c dO_ic O_ic,
//   dAk = dS^T Aq  -> dK = dAk[:, :C],          dphi_k = dAk[:, C:],
//   dAq = dS Ak    -> dQ = scale * dAq[:, :C],  dphi_q = dAq[:, C:].
// The factor gradients are extra columns of the contractions that give dK and dQ; no N x N
// gradient is ever written.  No atomics; results are deterministic.
//
// Kernels:
//   pre   : writes the concatenated operands Aq = [q*scale | phi_q | 0], Ak = [k | phi_k | 0]
//           (bf16, width W = C + 32 or C + 64 when R > 0; fp32 factors as three bf16 limbs, six product
//           columns per rank as in the forward) into the workspace -- or, for C = 64, 128, only their
//           factor columns, the channel columns being read from k (and from q, where the scores are
//           formed from q itself) in place
//   main<DKV = false> : a lane owns a query; streams 32-key blocks;   accumulates dAq^T; runs first and
//                       leaves (lse * log2 e, D) per query row for the other
//   main<DKV = true>  : a lane owns a key;   streams 32-query blocks; accumulates dV^T, dAk^T
// Both main kernels recompute S and dP (7 contractions instead of 5, but no atomic dQ).  They
// use the transposed orientation of the forward: the lane-side operands stay in registers,
// score-shaped accumulators feed the next MFMA as its B operand without leaving registers,
// and the transposed A operands come from the LDS transpose read.
//
// Streaming.  Because the operand rows exist in memory, a streamed block is a pure
// copy, done with direct-to-LDS loads (global_load_lds_dwordx4 from inline assembly, see
// fb_fwd_bf16_dma.h for why) into a ring of four block slots; nothing passes through
// registers.  One barrier per iteration, in the middle:
//     S, dP chains of block i | exp / dS | wait, barrier | issue block i+3 |
//     output chains of block i, first operand reads of block i+1
// A direct load writes 64 consecutive 16-byte pieces, so a 32-row tile of width W is kept as
// W/64 panels [32][64] (and one [32][32] panel if W % 64), each unpadded with an XOR chunk
// swizzle that makes both the row reads and the transpose reads bank-conflict free.
#include <hip/hip_runtime.h>

#include <type_traits>

#include <cmath>
#include "fb_device.h"
#include "fb_launch.h"
#include "fb_params.h"

namespace {

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int BT = 32;       // streamed rows per block
constexpr int NSLOT = 4;       // ring slots of the dq kernel
constexpr int NSLOT_DKV = 5;   // ring slots of the dkv kernel (a block is used in two iterations)

FB_DEV int swz64(int r) { return (((r >> 1) & 1) << 2) | ((r >> 2) & 3); }
FB_DEV int swz32(int r) { return (r >> 2) & 3; }

// s_waitcnt with only vmcnt constrained
template <int N>
FB_DEV void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}
FB_DEV void wait_vmcnt_n(int n) {   // n is wave-uniform; larger values wait for 12 (stricter, still correct)
    switch (n) {
        case 0: wait_vmcnt<0>(); break;
        case 1: wait_vmcnt<1>(); break;
        case 2: wait_vmcnt<2>(); break;
        case 3: wait_vmcnt<3>(); break;
        case 4: wait_vmcnt<4>(); break;
        case 5: wait_vmcnt<5>(); break;
        case 6: wait_vmcnt<6>(); break;
        case 7: wait_vmcnt<7>(); break;
        case 8: wait_vmcnt<8>(); break;
        case 9: wait_vmcnt<9>(); break;
        case 10: wait_vmcnt<10>(); break;
        case 11: wait_vmcnt<11>(); break;
        default: wait_vmcnt<12>(); break;
    }
}

// lane l reads sbase + voff (bytes); its 16 bytes land at LDS byte address lds_addr + 16 * l
FB_DEV void dma16(const void* sbase, unsigned voff, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(voff), "s"(sbase), "s"(lds_addr) : "memory", "m0");
}

// 32-row tile of W bf16 columns stored as panels (see the header comment)
template <int W>
struct Tile {
    static constexpr int NP64 = W / 64;
    static constexpr bool HAS32 = (W % 64) != 0;
    static constexpr int BYTES = W * 64;
    static constexpr int NDMA = NP64 * 4 + (HAS32 ? 2 : 0);   // direct loads per tile
    // direct load d of the tile: row and 16-byte source chunk fetched by `lane`, LDS offset of the load
    FB_DEV static void dma_map(int d, int lane, int& row, int& chunk, int& dst) {
        if (d < NP64 * 4) {
            row = (d & 3) * 8 + (lane >> 3);
            chunk = (d >> 2) * 8 + ((lane & 7) ^ swz64(row));
            dst = (d >> 2) * 4096 + (d & 3) * 1024;
        } else {
            const int e = d - NP64 * 4;
            row = e * 16 + (lane >> 2);
            chunk = NP64 * 8 + ((lane & 3) ^ swz32(row));
            dst = NP64 * 4096 + e * 1024;
        }
    }
};

template <int C, int RP>
struct Cfg {
    static constexpr int RP2 = (RP + 31) / 32 * 32;    // factor columns kept in the workspace rows (0, 32 or 64)
    static constexpr int W = C + RP2;
    static constexpr int KS = (C + RP) / 16;           // k-steps of the score contraction
    static constexpr int CS = C / 16;                  // k-steps of the dP contraction
    static constexpr int MB = W / 32;                  // 32-column blocks of dAq / dAk
    static constexpr int MBC = C / 32;
    using T1 = Tile<W>;
    using T2 = Tile<C>;
    static constexpr int kVecBytes = 1024;             // (lse2, D) of 32 rows in the first 256 bytes
    static constexpr size_t kEpiLds = (size_t)kWaves * 32 * (RP2 + 1) * sizeof(float);
};

// ------------------------------------------------------------------------------------------
// prep / vec
// ------------------------------------------------------------------------------------------
// One side per launch: QSIDE writes Aq = [q*scale | phi_q | 0] for the B*H*N query rows,
// otherwise Ak = [k | phi_k | 0] for the B*H*M key rows.
// A workgroup covers kPrepRows<C, RP> whole rows (one thread per 16-byte piece; the few threads past
// the last whole row idle), so a thread's row and piece come from its index by a division by a
// constant, and the head and position of the row from one block-uniform division plus a wrap.
//
// SPLIT: the main kernels read the C channel columns straight from the caller's q or k rows, and
// only the factor columns are written, as rows of RP2 columns (key side: a plain saving, the k
// columns were a copy; query side: the scale moves out of the q columns, see fmul).
template <int C, int RP, bool SPLIT>
constexpr int kPrepRows = 256 / ((SPLIT ? Cfg<C, RP>::RP2 : Cfg<C, RP>::W) / 8);

// fmul: factor of the factor columns (1, or 1/scale on the query side of a launch whose q columns
// carry no scale: q k^T scale + phi_q phi_k^T = scale (q k^T + (phi_q / scale) phi_k^T); applied to fp32
// factors before the limb split, as the forward does, and to bf16 factors only as a power of two).
template <int C, int RP, bool QSIDE, bool SPLIT>
FB_DEV void bwd_prep_block(const BwdParams& p, bf16_t* __restrict__ dst, const unsigned block, const float fmul) {
    using K = Cfg<C, RP>;
    static_assert(!SPLIT || (RP > 0 && C % 64 == 0), "split rows: whole 64-column panels of channels, and factor columns to write");
    constexpr int CPR = (SPLIT ? K::RP2 : K::W) / 8;
    constexpr int RPB = kPrepRows<C, RP, SPLIT>;
    constexpr int DW = SPLIT ? K::RP2 : K::W;                 // columns of a destination row
    constexpr int C0 = SPLIT ? C / 8 : 0;                     // first piece of a destination row
    const unsigned len = (unsigned)(QSIDE ? p.N : p.M);
    const unsigned dr = threadIdx.x / CPR;
    const int c = (int)(threadIdx.x - dr * CPR) + C0;
    const long long row0 = (long long)block * RPB;            // block-uniform
    const long long row = row0 + dr;                          // (b*H + h)*len + i
    const long long rows = (long long)p.B * p.H * len;
    if (dr >= (unsigned)RPB || row >= rows) return;
    bf16x8 a;
    if (c < C / 8) {
        bf16x8 x;
        if (c * 8 < p.Cg) {
            x = as_bf16x8(*(const u32x4*)((const bf16_t*)(QSIDE ? p.q : p.k) + row * p.Cg + c * 8));
        } else {      // channels the caller's rows do not have
#pragma unroll
            for (int e = 0; e < 8; e++) x[e] = (bf16_t)0.f;
        }
        if (QSIDE) {
#pragma unroll
            for (int e = 0; e < 8; e++) a[e] = (bf16_t)((float)x[e] * p.scale);
        } else {
            a = x;
        }
    } else {
        const bool f32 = p.phi_f32 != 0;
        const size_t esz = f32 ? 4 : 2;
        // rows < 2^31: the block's first row splits into head and position once, the thread's row wraps
        const unsigned bh0 = (unsigned)((unsigned long long)row0 / len);
        unsigned bb = bh0 / (unsigned)p.H;
        unsigned h = bh0 - bb * (unsigned)p.H;
        unsigned i = (unsigned)((unsigned long long)row0 - (unsigned long long)bh0 * len) + dr;
        while (i >= len) {
            i -= len;
            if (++h == (unsigned)p.H) { h = 0; ++bb; }
        }
        const int pc = c - C / 8;
        if (p.slopes != nullptr) {
            // ALiBi factors of Example 3.4 from the head's slope and the row's position (App. D)
            const float m = p.slopes[h];
            float pair[2];
            pair[0] = QSIDE ? -m * (float)i : 1.f;
            pair[1] = QSIDE ? m : (float)i;
            a = phi_chunk_switch<QSIDE>(pair, pc, 2, true, fmul);
        } else {
            const size_t off = ((size_t)bb * (QSIDE ? p.phi_bstride : p.phik_bstride) + ((size_t)h * len + i) * p.R) * esz;
            const unsigned char* src = (const unsigned char*)(QSIDE ? p.phi_q : p.phi_k) + off;
            if (!f32 && (p.R & 7) == 0) {
                // bf16 factors in whole 16-byte pieces: a copy (rows and the batch stride are then multiples of 16 bytes)
                u32x4 raw = u32x4{0u, 0u, 0u, 0u};
                if (pc * 8 < p.R) raw = *(const u32x4*)(src + pc * 16);
                a = as_bf16x8(raw);
            } else {
                a = phi_chunk_switch<QSIDE>(src, pc, p.R, f32, fmul);
            }
            if (!f32 && fmul != 1.f) {      // a power of two: exact
#pragma unroll
                for (int e = 0; e < 8; e++) a[e] = (bf16_t)((float)a[e] * fmul);
            }
        }
    }
    *(u32x4*)(dst + row * DW + (c - C0) * 8) = as_uint4(a);
}

// The whole pre-pass in one launch: the first nb_q workgroups write the query-side rows, the rest the
// key-side rows.  SQ, SK: that side is written in the split form (factor columns only).
template <int C, int RP, bool SQ = false, bool SK = false>
__global__ __launch_bounds__(256) void bwd_pre_kernel(BwdParams p, bf16_t* __restrict__ aq, bf16_t* __restrict__ ak,
                                                      unsigned nb_q, float qmul) {
    const unsigned blk = blockIdx.x;
    if (blk < nb_q) {
        bwd_prep_block<C, RP, true, SQ>(p, aq, blk, qmul);
    } else {
        bwd_prep_block<C, RP, false, SK>(p, ak, blk - nb_q, 1.f);
    }
}

// Head dimension 16: rows of 16 channels widened to 32 with zeros (the main kernels stream
// v and dO tiles of 32 channels).  One thread per 16-byte piece of the destination.
__global__ __launch_bounds__(256) void bwd_pad16_kernel(const bf16_t* __restrict__ src, bf16_t* __restrict__ dst,
                                                        long long rows) {
    const long long gid = (long long)blockIdx.x * 256 + threadIdx.x;
    const long long row = gid >> 2;
    const int c = (int)(gid & 3);
    if (row >= rows) return;
    u32x4 x = u32x4{0u, 0u, 0u, 0u};
    if (c < 2) x = *(const u32x4*)(src + row * 16 + c * 8);
    *(u32x4*)(dst + row * 32 + c * 8) = x;
}

// Write one wave's factor-gradient columns to LDS scratch and reduce limb columns.
// acc[mb] holds columns mb*32 + 8*g + 4*hf + x (register 4*g + x) for row l32.
// raw: the R columns are written as float without any limb summing (gradients of bf16 columns
// kept in fp32 for a later reduction).
template <int RP2, bool QSIDE>
FB_DEV void store_dphi(const f32x16* acc_phi /* [RP2/32] */, float* scratch /* wave-private [32][RP2+1] */,
                       void* dst_row /* gradient row of this lane's token or null */, int R,
                       bool f32, bool raw, int l32, int hf, float* dslope = nullptr, float pos = 0.f) {
#pragma unroll
    for (int mb = 0; mb < RP2 / 32; mb++)
#pragma unroll
        for (int r = 0; r < 16; r++)
            scratch[l32 * (RP2 + 1) + mb * 32 + 8 * (r / 4) + 4 * hf + (r % 4)] = acc_phi[mb][r];
    __syncthreads();
    if (QSIDE && dslope != nullptr && hf == 0) {
        // ALiBi factors phi_q(i) = [-m i, m] against phi_k(j) = [1, j] (fp32 limb columns): the chain rule
        // onto the slope is dphi_q[i,1] - i dphi_q[i,0] = sum_j dS_ij (j - i).  Both terms come from the same
        // bf16 dS values through fp32 accumulators, so whatever the rows of dS fail to sum to (the error of
        // D = rowsum(dO o O)) cancels here instead of being multiplied by the position.
        const float* s = scratch + l32 * (RP2 + 1);
        const float g0 = s[0] + s[1] + s[3], g1 = s[6] + s[7] + s[9];
        *dslope = g1 - pos * g0;
    }
    if (dst_row != nullptr) {
        for (int r = hf; r < R; r += 2) {
            const float* s = scratch + l32 * (RP2 + 1);
            if (raw) {
                ((float*)dst_row)[r] = s[r];
            } else if (f32) {
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
// main kernel.  "lane side" = the 128 rows owned by the workgroup (keys when DKV, else
// queries); "streamed side" = the other index, walked in blocks of 32 rows.
//   T1 tile: rows of the streamed operand of S (Aq when DKV, else Ak), width W
//   T2 tile: rows of the streamed operand of dP (dO when DKV, else V), width C
// ------------------------------------------------------------------------------------------
// Operand rows [channels | factor columns] of one side.  Whole rows in the workspace: main = the rows,
// phi = main + C, both pitches W.  Split: main = the caller's q or k rows (pitch C), phi = rows of the
// RP2 factor columns in the workspace.
struct OperandRows {
    const bf16_t* main; int main_pitch;
    const bf16_t* phi;  int phi_pitch;
};
struct MainArgs {
    OperandRows aq;       // B*H*N rows
    OperandRows ak;       // B*H*M rows
    const float2* vec;    // [B*H*N]  (lse * log2 e, D): written by the dq kernel, read by the dkv kernel
    float2* vec_w;        // the same rows, for the dq kernel
    float exp_mul;        // S exp_mul - lse2 is the exponent of P to base two: log2 e, times the scale where the q columns carry none
    float dkv_mul;        // factor of d[K | phi_k] (the scale, where the q columns carry none)
};

// DENSE (RP = 0 only): the bias is a dense [N][M] matrix instead of factors.  Every wave also
// copies the 32 x 32 bias tile of (its lane rows) x (the streamed block) into the slot, two
// direct loads per block; the S chain starts from those values; the dq kernel writes
// dS = dBias from its packed operand registers.
template <int C, int RP, bool CAUSAL, bool DKV, bool DENSE>
FB_DEV void bwd_tile(const BwdParams& p, const MainArgs& a, unsigned char* smem, const int bh, const int tile) {
    static_assert(!DENSE || RP == 0, "dense bias and factors are exclusive");
    using K = Cfg<C, RP>;
    using T1 = typename K::T1;
    using T2 = typename K::T2;
    constexpr int kBiasTile = 32 * 32 * 2;     // one wave's tile: 32 rows of 64 bytes
    constexpr int kOffT2 = T1::BYTES, kOffVec = T1::BYTES + T2::BYTES;
    constexpr int kOffBias = kOffVec + (DKV ? K::kVecBytes : 0);
    constexpr int kSlotBytes = kOffBias + (DENSE ? kWaves * kBiasTile : 0);
    constexpr int ND = T1::NDMA + T2::NDMA + (DKV ? 1 : 0);       // direct loads per block
    constexpr int NDW = (ND + kWaves - 1) / kWaves;               // ... per wave, at most
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;

    // NL rows on the lane side (keys when DKV, else queries), NS rows on the streamed side
    const int NL = DKV ? p.M : p.N, NS = DKV ? p.N : p.M, R = p.R;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, hf = lane >> 5;
    const int r0 = tile * 128;            // first lane-side row of the workgroup
    const int rw0 = r0 + wave * 32;       // ... of this wave
    const int ri = rw0 + l32;             // this lane's row
    const int rc = min(ri, NL - 1);       // rows past the end compute on the last row and are not stored

    const size_t lbase = (size_t)bh * NL, sbase_rows = (size_t)bh * NS;
    const OperandRows& L1 = DKV ? a.ak : a.aq;                                      // lane-side operand of S
    const OperandRows& S1 = DKV ? a.aq : a.ak;                                      // streamed operand of S
    const bf16_t* l1m = L1.main + lbase * L1.main_pitch;
    const bf16_t* l1p = L1.phi + lbase * L1.phi_pitch;
    const bf16_t* l2g = (const bf16_t*)(DKV ? p.v : p.dout) + lbase * C;            // lane-side operand of dP
    const bf16_t* t1m = S1.main + sbase_rows * S1.main_pitch;
    const bf16_t* t1p = S1.phi + sbase_rows * S1.phi_pitch;
    const float emul = a.exp_mul;
    const bf16_t* t2g = (const bf16_t*)(DKV ? p.dout : p.v) + sbase_rows * C;
    const float2* vecg = a.vec + (size_t)bh * p.N;                                  // per query row

    // ---- lane-side operands, loop invariant ----
    bf16x8 l1reg[K::KS], l2reg[K::CS];
#pragma unroll
    for (int ks = 0; ks < K::KS; ks++)
        l1reg[ks] = as_bf16x8(*(const u32x4*)(ks * 16 < C ? l1m + (size_t)rc * L1.main_pitch + ks * 16 + 8 * hf
                                                          : l1p + (size_t)rc * L1.phi_pitch + (ks * 16 - C) + 8 * hf));
#pragma unroll
    for (int cs = 0; cs < K::CS; cs++)
        l2reg[cs] = as_bf16x8(*(const u32x4*)(l2g + (size_t)rc * C + cs * 16 + 8 * hf));
    float my_lse2 = 0.f, my_d = 0.f;    // dq kernel: this lane's row (formed below, behind the first block loads)

    f32x16 acc1[K::MB];                 // dAk^T or dAq^T
    f32x16 acc2[DKV ? K::MBC : 1];      // dV^T
#pragma unroll
    for (int r = 0; r < 16; r++) {
#pragma unroll
        for (int mb = 0; mb < K::MB; mb++) acc1[mb][r] = 0.f;
#pragma unroll
        for (int mb = 0; mb < (DKV ? K::MBC : 1); mb++) acc2[mb][r] = 0.f;
    }

    // ---- streamed block range ----
    const int nblk_all = (NS + BT - 1) / BT;
    int b_begin = 0, b_end = nblk_all;
    if (CAUSAL) {
        if (DKV) b_begin = r0 / BT;                            // queries before the first key see nothing
        else b_end = min(nblk_all, (min(NS, r0 + 128) + BT - 1) / BT);
    }
    const int nIt = b_end - b_begin;
    auto blk_of = [&](int i) __attribute__((always_inline)) { return min(b_begin + i, nblk_all - 1); };

    // ---- this wave's share of a block's direct loads: load d = wave + 4*j, j < NDW ----
    // Every wave issues NDW loads per block so that the vmcnt waits are compile-time constants and
    // the issue code carries no per-load guards: where ND is not a multiple of four the surplus
    // slots repeat load ND-1 (same source, same destination, same bytes as the wave that owns it).
    // wave-uniform per load: running source pointer of the block being issued, bytes per block,
    // LDS offset inside a slot, row-offset limit for the sequence's last (partial) block;
    // per lane: byte offset of its source row (a chunk of two rows for the vec rows) and of its
    // 16 bytes inside the row
    unsigned dma_rowoff[NDW], dma_col[NDW], dma_taillim[NDW];
    const unsigned char* dma_ptr[NDW];
    int dma_bstride[NDW], dma_dst[NDW];
    const int tail_left = NS - (nblk_all - 1) * BT - 1;      // last valid row of the sequence's last block
    int dma_blk = blk_of(0);                                 // block the running pointers stand at
#pragma unroll
    for (int j = 0; j < NDW; j++) {
        const int d = min(wave + kWaves * j, ND - 1);
        const unsigned char* dma_src_j;
        int dma_pitch_j, dma_lshift_j;
        int row = 0, chunk = 0, dst = 0;
        if (d < T1::NDMA) {
            T1::dma_map(d, lane, row, chunk, dst);
            // a panel of 64 (or the last 32) columns comes from one array: the channel rows, or the factor
            // rows when it starts at or behind column C (split rows have C % 64 == 0, so no panel mixes)
            const int panel = d < T1::NP64 * 4 ? (d >> 2) : T1::NP64;
            const bool fpart = panel * 64 >= C;
            const int pitch_el = fpart ? S1.phi_pitch : S1.main_pitch;
            dma_src_j = (const unsigned char*)(fpart ? t1p : t1m);
            dma_bstride[j] = BT * pitch_el * 2; dma_pitch_j = pitch_el * 2; dma_lshift_j = 0;
            dma_col[j] = (unsigned)(fpart ? chunk - C / 8 : chunk) * 16u;
            dma_dst[j] = dst;
        } else if (d < T1::NDMA + T2::NDMA) {
            T2::dma_map(d - T1::NDMA, lane, row, chunk, dst);
            dma_src_j = (const unsigned char*)t2g;
            dma_bstride[j] = BT * C * 2; dma_pitch_j = C * 2; dma_lshift_j = 0;
            dma_col[j] = (unsigned)chunk * 16u;
            dma_dst[j] = kOffT2 + dst;
        } else {
            // vec: 32 rows x 8 bytes = 16 chunks of two rows; the other lanes repeat chunk 15
            row = min(lane, 15);
            dma_src_j = (const unsigned char*)vecg;
            dma_bstride[j] = BT * 8; dma_pitch_j = 16; dma_lshift_j = 1;
            dma_col[j] = 0u;
            dma_dst[j] = kOffVec;
        }
        dma_dst[j] = __builtin_amdgcn_readfirstlane(dma_dst[j]);     // wave-uniform by construction: keep it scalar
        dma_rowoff[j] = (unsigned)(row * dma_pitch_j);
        dma_taillim[j] = (unsigned)__builtin_amdgcn_readfirstlane((tail_left >> dma_lshift_j) * dma_pitch_j);
        dma_ptr[j] = dma_src_j + (size_t)dma_blk * dma_bstride[j];
    }
    // Blocks are issued in ascending order of i (the clamp in blk_of makes the index stall at the
    // last block), so the source pointers advance by at most one block per call.
    auto issue_block = [&](int i, int slot) __attribute__((always_inline)) {
        const int blk = blk_of(i);
        const bool adv = blk != dma_blk;       // wave-uniform; false once the index is clamped (and on the first call)
        dma_blk = blk;
        const bool tail = blk == nblk_all - 1; // rows past the sequence end repeat the last valid row
        const unsigned sbase = lds0 + slot * kSlotBytes;
#pragma unroll
        for (int j = 0; j < NDW; j++) {
            dma_ptr[j] += adv ? dma_bstride[j] : 0;
            const unsigned voff = min(dma_rowoff[j], tail ? dma_taillim[j] : ~0u) + dma_col[j];
            dma16(dma_ptr[j], voff, sbase + dma_dst[j]);
        }
    };
    // ---- dense bias tile of this wave: rows = queries, columns = keys, 64-byte rows; lane l of
    // load i covers tile row 16*i + l/4; chunk position l%4 holds 8-key chunk (l%4) ^ ((row>>2)&3)
    const int b_ = bh / p.H, h_ = bh - b_ * p.H;
    const unsigned char* bias_src = nullptr;   // wave-uniform base of this wave's tiles
    size_t bias_bstep = 0;                     // bytes per streamed block
    int bias_var[2], bias_pitch = 0, bias_lshift = 0;
    unsigned bias_fix[2];
    if (DENSE) {
        const bf16_t* bg = (const bf16_t*)p.bias + (size_t)b_ * p.bias_bstride + (size_t)h_ * p.N * p.M;
        const int Mk = p.M;
#pragma unroll
        for (int i = 0; i < 2; i++) {
            const int trow = 16 * i + (lane >> 2);
            const int c = (lane & 3) ^ ((trow >> 2) & 3);
            if (!DKV) {
                // lane side = queries: fixed row per lane; the key chunk is clamped at the sequence end
                const int rbase = min(rw0, NL - 1);
                bias_fix[i] = (unsigned)(min(rw0 + trow, NL - 1) - rbase) * (unsigned)(Mk * 2);
                bias_var[i] = c;
                bias_src = (const unsigned char*)(bg + (size_t)rbase * Mk);
            } else {
                // lane side = keys: fixed 8-key chunk per lane; the query row is clamped at the end
                const int kb = min(rw0, Mk - 8);
                bias_fix[i] = (unsigned)(min(rw0 + 8 * c, Mk - 8) - kb) * 2u;
                bias_var[i] = trow;
                bias_src = (const unsigned char*)(bg + kb);
            }
        }
        bias_pitch = DKV ? Mk * 2 : 16;
        bias_lshift = DKV ? 0 : 3;
        bias_bstep = DKV ? (size_t)BT * Mk * 2 : (size_t)BT * 2;
    }
    auto issue_bias = [&](int i, int slot) __attribute__((always_inline)) {
        if (!DENSE) return;
        const int blk = blk_of(i);
        const int left = NS - blk * BT - 1;
        const unsigned dst = lds0 + slot * kSlotBytes + kOffBias + wave * kBiasTile;
#pragma unroll
        for (int x = 0; x < 2; x++) {
            const unsigned voff = (unsigned)(min(bias_var[x], left >> bias_lshift) * bias_pitch) + bias_fix[x];
            dma16(bias_src + (size_t)blk * bias_bstep, voff, dst + x * 1024);
        }
    };
    // all but the newest block's loads (plus `stores` global stores issued since) may remain
    auto wait_prev_loads = [&](int stores) __attribute__((always_inline)) {
        constexpr int NLD = NDW + (DENSE ? 2 : 0);
        if (stores == 0) wait_vmcnt<NLD>();
        else wait_vmcnt_n(NLD + stores);
    };
    // per-lane offsets of the bias values of this lane's accumulator registers inside a tile:
    // group g <-> registers 4g..4g+3
    int boff[4];
#pragma unroll
    for (int g = 0; g < 4; g++) {
        if (!DKV) {
            boff[g] = l32 * 64 + ((g ^ ((l32 >> 2) & 3)) << 4) + hf * 8;             // row = query l32, keys 8g+4hf..
        } else {
            const int trow = 8 * g + 4 * hf + ((lane & 15) >> 2);                       // transpose read
            const int chunk = 2 * (l32 >> 4) + (((lane & 15) & 3) >> 1);
            boff[g] = trow * 64 + ((chunk ^ ((trow >> 2) & 3)) << 4) + (lane & 1) * 8;
        }
    }
    auto bias_init = [&](f32x16& s, int slot_off) __attribute__((always_inline)) {
        const unsigned char* tp = smem + (slot_off + kOffBias + wave * kBiasTile);
#pragma unroll
        for (int g = 0; g < 4; g++) {
            bf16x4 bv;
            if (!DKV) bv = __builtin_bit_cast(bf16x4, *(const u32x2*)(tp + boff[g]));
            else bv = __builtin_bit_cast(bf16x4, lds_read_tr16((const bf16_t*)(tp + boff[g])));
#pragma unroll
            for (int x = 0; x < 4; x++) s[4 * g + x] = (float)bv[x];
        }
    };

    // ---- per-lane LDS read offsets (bytes inside a panel) ----
    int rb64[4], rb32[2];                 // row operand, k-step j of a panel: 16 bytes at row l32
#pragma unroll
    for (int j = 0; j < 4; j++) rb64[j] = l32 * 128 + (((2 * j + hf) ^ swz64(l32)) << 4);
#pragma unroll
    for (int j = 0; j < 2; j++) rb32[j] = l32 * 64 + (((2 * j + hf) ^ swz32(l32)) << 4);
    const int i16 = lane & 15, blk16 = l32 >> 4;
    int tr64[2][2], tr32[2];              // transpose reads: 32-column block m of a panel, half hi
#pragma unroll
    for (int hi = 0; hi < 2; hi++) {
        const int row = 8 * hi + 4 * hf + (i16 >> 2);
#pragma unroll
        for (int m = 0; m < 2; m++)
            tr64[m][hi] = row * 128 + (((m * 4 + 2 * blk16 + ((i16 & 3) >> 1)) ^ swz64(row)) << 4) + (i16 & 1) * 8;
        tr32[hi] = row * 64 + (((2 * blk16 + ((i16 & 3) >> 1)) ^ swz32(row)) << 4) + (i16 & 1) * 8;
    }
    // The same offsets with a slot's byte offset added, built once per block instead of once per
    // read (the slot is a run-time value, the rest of a read's address is an immediate).
    constexpr bool ANY64 = T1::NP64 > 0 || T2::NP64 > 0;
    constexpr bool ANY32 = T1::HAS32 || T2::HAS32;
    struct RowBase { int b64[4]; int b32[2]; };
    struct TrBase { int t64[2][2]; int t32[2]; };
    auto mk_row = [&](int off) __attribute__((always_inline)) {
        RowBase r;
#pragma unroll
        for (int j = 0; j < 4; j++) r.b64[j] = ANY64 ? rb64[j] + off : 0;
#pragma unroll
        for (int j = 0; j < 2; j++) r.b32[j] = ANY32 ? rb32[j] + off : 0;
        return r;
    };
    auto mk_tr = [&](int off) __attribute__((always_inline)) {
        TrBase t;
#pragma unroll
        for (int hi = 0; hi < 2; hi++) {
#pragma unroll
            for (int m = 0; m < 2; m++) t.t64[m][hi] = ANY64 ? tr64[m][hi] + off : 0;
            t.t32[hi] = ANY32 ? tr32[hi] + off : 0;
        }
        return t;
    };
    // operand n of a block, in consumption order:
    //   [0, KS)            S   k-step n          row read of T1
    //   [KS, KS+CS)        dP  k-step n-KS       row read of T2
    //   then NO1 = 2*MB    output 1, (mb, kk)    transpose read of T1
    //   then NO2 = 2*MBC   output 2 (DKV only)   transpose read of T2   (LAZY_DS: output 2 before output 1)
    constexpr int NO1 = 2 * K::MB, NO2 = DKV ? 2 * K::MBC : 0;
    constexpr int NA = K::KS + K::CS;          // operands of the first half
    // dkv kernel, one wave per SIMD: a wave hides about five vector instructions under each MFMA.
    // With eight or more dV MFMAs (C = 128) the dS arithmetic of a block (sub, mul, convert: 40
    // instructions) fits under them, which leaves only the exponentials under the S / dP chains;
    // smaller head dimensions have too few dV MFMAs and keep everything under the first half.
    constexpr bool LAZY_DS = DKV && NO2 >= 8;
    constexpr int NOPS = NA + NO1 + NO2;
    // LDS operand reads run LA MFMAs ahead of their use; the first half never reads past its own block
    // (measured: look-ahead 2..4 for dq and 5..12 for dkv all run within 1 %)
    constexpr int LA_WANT = DKV ? 6 : 3;
    constexpr int LA_CAP = (NO1 + NO2) < NA ? (NO1 + NO2) : NA;
    constexpr int LA = LA_CAP < LA_WANT ? LA_CAP : LA_WANT;
    bf16x8 opr[LA + 1];
    auto row_read = [&](const RowBase& rb, int toff, int np64, int ks) __attribute__((always_inline)) {
        if (ks < np64 * 4) return as_bf16x8(*(const u32x4*)(smem + rb.b64[ks & 3] + (toff + (ks >> 2) * 4096)));
        return as_bf16x8(*(const u32x4*)(smem + rb.b32[ks - np64 * 4] + (toff + np64 * 4096)));
    };
    auto tr_read = [&](const TrBase& tb, int toff, int np64, int mb, int kk) __attribute__((always_inline)) {
        if (mb < np64 * 2) {
            const int imm = toff + (mb >> 1) * 4096 + kk * 2048;
            return join_tr(lds_read_tr16((const bf16_t*)(smem + tb.t64[mb & 1][0] + imm)),
                           lds_read_tr16((const bf16_t*)(smem + tb.t64[mb & 1][1] + imm)));
        }
        const int imm = toff + np64 * 4096 + kk * 1024;
        return join_tr(lds_read_tr16((const bf16_t*)(smem + tb.t32[0] + imm)),
                       lds_read_tr16((const bf16_t*)(smem + tb.t32[1] + imm)));
    };
    // operand n of a block whose slot offset is folded into rb (row reads) / tb (transpose reads);
    // callers keep a rolling window opr[n % (LA + 1)]
    auto read_op = [&](const RowBase& rb, const TrBase& tb, int n) __attribute__((always_inline)) {
        if (n < K::KS) return row_read(rb, 0, T1::NP64, n);
        if (n < NA) return row_read(rb, kOffT2, T2::NP64, n - K::KS);
        if (LAZY_DS) {
            // the P-side output (dV) first: its operand is complete when the first half ends, while dS
            // is still being formed under these MFMAs
            if (n < NA + NO2) return tr_read(tb, kOffT2, T2::NP64, (n - NA) >> 1, (n - NA) & 1);
            return tr_read(tb, 0, T1::NP64, (n - NA - NO2) >> 1, (n - NA - NO2) & 1);
        }
        if (n < NA + NO1) return tr_read(tb, 0, T1::NP64, (n - NA) >> 1, (n - NA) & 1);
        return tr_read(tb, kOffT2, T2::NP64, (n - NA - NO1) >> 1, (n - NA - NO1) & 1);
    };

    // Head dimension 16 on the 32-channel operand rows: channels 16..31 are zero on both sides, so the
    // second k-step of the S chain and of the dP chain contribute nothing (the operand is still read,
    // which keeps the rolling window's positions).
    const bool narrow = C == 32 && p.Cg == 16;          // wave-uniform
    auto dead_step = [&](int n) __attribute__((always_inline)) {
        return C == 32 && narrow && (n == 1 || n == K::KS + 1);
    };

    // P and dS of one accumulator element r (streamed row sb0 + 8*(r/4) + 4*hf + (r%4), lane row ri)
    auto elem = [&](int r, const f32x16& s, const f32x16& dp, float lvx, float dvx, bool need_mask, int sb0,
                    bf16x8 (&pb)[2], bf16x8 (&dsb)[2]) __attribute__((always_inline)) {
        float pr = fast_exp2(fmaf(s[r], emul, -lvx));
        float ds = pr * (dp[r] - dvx);
        if (need_mask) {
            const int srow = sb0 + 8 * (r / 4) + 4 * hf + (r % 4);
            const bool dead = srow >= NS || (CAUSAL && (DKV ? (srow < ri) : (srow > ri)));
            if (dead) { pr = 0.f; ds = 0.f; }   // also discards the filler rows past N
        }
        if (DKV) pb[r / 8][r % 8] = (bf16_t)pr;
        dsb[r / 8][r % 8] = (bf16_t)ds;
    };

    if constexpr (DKV) {
        // One wave per SIMD (the accumulators alone take 144 registers), so the overlap of
        // matrix and vector work is written into the instruction stream: while the S and dP
        // chains of block i+1 run, the exponentials and dS of block i are computed, one
        // accumulator element per MFMA.  Iteration i:
        //     S, dP chains of block i+1  ||  P, dS of block i
        //     wait, barrier, issue block i+4
        //     output chains of block i, first operand reads of block i+2, (lse2, D) of block i+1
        // (LAZY_DS: only P under the first chains, dS under the dV chains, then the dK chains)
        // Ring of five slots: blocks i (transpose reads), i+1 (row reads), i+2 (prefetch),
        // i+3 (landing), i+4 (being issued).
        static_assert(NSLOT_DKV == 5, "slot arithmetic below assumes five slots");
        // SV: the S and dP tiles are produced by hand-placed MFMA forms with VGPR results (the
        // vector ALU reads them next); the compiler's own choice at one wave per SIMD is an AGPR
        // result and a v_accvgpr_read per element, 32 per block (-4 % per backward on the headline
        // shape together with the copy-free swap of the tile pairs below).  Not with a dense bias,
        // whose tile is the chain's start value.
        // Only where the kernel leaves the register allocator room (operand rows of at most 144
        // columns): in the wider instantiations every VGPR is taken, the allocator parks values in
        // spare AGPRs around the statements it cannot see into, and a copy of a tile placed right
        // behind an inner link of a chain would read it too early (seen as a wrong dK at C = 128,
        // R = 9 fp32 factors; those instantiations keep the compiler's forms).
        constexpr bool SV = !DENSE && C + RP <= 144;
        // one link of the S (n < KS) or dP chain of a block into the VGPR tiles st / dt
        auto chain_link = [&](int n, f32x16& st, f32x16& dt, bf16x8 o) __attribute__((always_inline)) {
            constexpr int CS = NA - K::KS;
            // the last live link of each chain (head dimension 16: the second link of each chain is dead)
            const bool last_s = n == K::KS - 1, last_d = n == NA - 1;
            if (n < K::KS) {
                if (n == 0) mfma32_vdst_first(st, o, l1reg[n]);
                else if (last_s) mfma32_vdst_last(st, o, l1reg[n]);
                else mfma32_vdst(st, o, l1reg[n]);
            } else {
                if (n == K::KS) mfma32_vdst_first(dt, o, l2reg[n - K::KS]);
                else if (last_d) mfma32_vdst_last(dt, o, l2reg[n - K::KS]);
                else mfma32_vdst(dt, o, l2reg[n - K::KS]);
            }
            (void)CS;
        };
        static_assert(K::KS >= 2 && NA - K::KS >= 2, "a first and a last link per chain");
        issue_block(0, 0); issue_bias(0, 0);
        issue_block(1, 1); issue_bias(1, 1);
        issue_block(2, 2); issue_bias(2, 2);
        issue_block(3, 3); issue_bias(3, 3);
        wait_vmcnt<0>();
        __syncthreads();
        f32x16 sA, dA, sB, dB;
        {
            const RowBase r0 = mk_row(0);
            const TrBase t0 = mk_tr(0);
#pragma unroll
            for (int r = 0; r < 16; r++) { sA[r] = 0.f; dA[r] = 0.f; }
            if (DENSE) bias_init(sA, 0);
#pragma unroll
            for (int n = 0; n < NA; n++) {
                const bf16x8 o = read_op(r0, t0, n);
                // (SV: a chain's last link carries its wait states, so it is issued even when it adds zeros)
                if (dead_step(n) && !(SV && (n == NA - 1 || n == K::KS - 1))) continue;
                if (SV) {
                    chain_link(n, sA, dA, o);
                } else {
                    if (n < K::KS) sA = mfma32(o, l1reg[n], sA);
                    else dA = mfma32(o, l2reg[n - K::KS], dA);
                }
            }
        }
        RowBase rb1 = mk_row(kSlotBytes);     // rows of block i+1
#pragma unroll
        for (int n = 0; n < LA; n++) opr[n] = read_op(rb1, TrBase{}, n);
        // (lse2, D) of the 16 streamed rows this lane's accumulator registers belong to, one block ahead
        float vq[4][4], vd[4][4];
        const int vlane = kOffVec + 32 * hf;
        auto read_vec = [&](int off) __attribute__((always_inline)) {
            const unsigned char* vp = smem + (vlane + off);
#pragma unroll
            for (int g = 0; g < 4; g++) {
                const float4 x0 = *(const float4*)(vp + 64 * g);
                const float4 x1 = *(const float4*)(vp + 64 * g + 16);
                vq[g][0] = x0.x; vd[g][0] = x0.y; vq[g][1] = x0.z; vd[g][1] = x0.w;
                vq[g][2] = x1.x; vd[g][2] = x1.y; vq[g][3] = x1.z; vd[g][3] = x1.w;
            }
        };
        read_vec(0);
        int sl = 0;   // slot of block i
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        auto body = [&](int i, const f32x16& sc, const f32x16& dc, f32x16& sn, f32x16& dn)
                        __attribute__((always_inline)) {
            const int sl1 = sl + 1 >= NSLOT_DKV ? sl + 1 - NSLOT_DKV : sl + 1;
            const int sl2 = sl + 2 >= NSLOT_DKV ? sl + 2 - NSLOT_DKV : sl + 2;
            const int sl4 = sl == 0 ? NSLOT_DKV - 1 : sl - 1;
            const TrBase tb0 = mk_tr(sl * kSlotBytes);          // transpose reads of block i
            const RowBase rb2 = mk_row(sl2 * kSlotBytes);       // rows of block i+2
            const int sb0 = blk_of(i) * BT;
            const bool need_mask = (sb0 + BT > NS) || (CAUSAL && sb0 < rw0 + 31);
            bf16x8 pb[2], dsb[2];
            float prf[16];                                      // P of block i in fp32, until dS is formed
            f32x16 sinit = zero;
            if (DENSE) bias_init(sinit, sl1 * kSlotBytes);      // S of block i+1 starts from its bias tile
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int n = 0; n < NA; n++) {
                opr[(n + LA) % (LA + 1)] = read_op(rb1, tb0, n + LA);   // past NA: output operands of block i
                if (!dead_step(n) || (SV && (n == NA - 1 || n == K::KS - 1))) {
                    if (SV) {
                        chain_link(n, sn, dn, opr[n % (LA + 1)]);
                    } else {
                        if (n < K::KS) sn = mfma32(opr[n % (LA + 1)], l1reg[n], n == 0 ? sinit : sn);
                        else dn = mfma32(opr[n % (LA + 1)], l2reg[n - K::KS], n == K::KS ? zero : dn);
                    }
                }
#pragma unroll
                for (int e = (n * 16) / NA; e < ((n + 1) * 16) / NA; e++) {
                    if (LAZY_DS) {
                        prf[e] = fast_exp2(fmaf(sc[e], emul, -vq[e >> 2][e & 3]));
                        pb[e / 8][e % 8] = (bf16_t)prf[e];
                    } else {
                        elem(e, sc, dc, vq[e >> 2][e & 3], vd[e >> 2][e & 3], false, sb0, pb, dsb);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if (need_mask) {
                // rare (diagonal blocks, sequence end): zero the dead elements afterwards, behind a real
                // branch, so the common path carries no compares and selects.  NaNs from filler rows
                // past N are discarded here as well.  LAZY_DS: with P zeroed, dS = P (dP - D) formed
                // later is zero too; the (lse, D) pair of a filler row past the sequence end is whatever
                // follows in memory, so its D is replaced to keep 0 * (dP - D) at 0.
                asm volatile("" ::: "memory");
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    const int srow = sb0 + 8 * (r / 4) + 4 * hf + (r % 4);
                    if (srow >= NS || (CAUSAL && srow < ri)) {
                        pb[r / 8][r % 8] = (bf16_t)0.f;
                        if (LAZY_DS) prf[r] = 0.f;
                        else dsb[r / 8][r % 8] = (bf16_t)0.f;
                    }
                    if (LAZY_DS && srow >= NS) vd[r >> 2][r & 3] = 0.f;
                }
            }
            // block i+2 has landed; everyone has left block i-1
            wait_prev_loads(0);
            __syncthreads();
            issue_block(i + 4, sl4);
            issue_bias(i + 4, sl4);
            bf16x8 nxt[LA];
#pragma unroll
            for (int n = NA; n < NOPS; n++) {
                if (n + LA < NOPS) opr[(n + LA) % (LA + 1)] = read_op(rb1, tb0, n + LA);
                else nxt[n + LA - NOPS] = read_op(rb2, tb0, n + LA - NOPS);   // row operands of block i+2
                const int m = n - NA;
                if (!LAZY_DS) {
                    if (m < NO1) acc1[m >> 1] = mfma32(opr[n % (LA + 1)], dsb[m & 1], acc1[m >> 1]);
                    else acc2[(m - NO1) >> 1] = mfma32(opr[n % (LA + 1)], pb[(m - NO1) & 1], acc2[(m - NO1) >> 1]);
                } else if (m < NO2) {
                    acc2[m >> 1] = mfma32(opr[n % (LA + 1)], pb[m & 1], acc2[m >> 1]);
                    // dS of block i under the dV MFMAs, 16 / NO2 elements per MFMA
#pragma unroll
                    for (int e = (m * 16) / NO2; e < ((m + 1) * 16) / NO2; e++)
                        dsb[e / 8][e % 8] = (bf16_t)(prf[e] * (dc[e] - vd[e >> 2][e & 3]));
                    __builtin_amdgcn_sched_barrier(0);
                } else {
                    acc1[(m - NO2) >> 1] = mfma32(opr[n % (LA + 1)], dsb[(m - NO2) & 1], acc1[(m - NO2) >> 1]);
                }
            }
#pragma unroll
            for (int n = 0; n < LA; n++) opr[n] = nxt[n];
            read_vec(sl1 * kSlotBytes);
            rb1 = rb2;
            sl = sl1;
        };
        int i = 0;
        if (SV) {      // two steps at a time: the two pairs of score tiles swap roles without copies
            for (; i + 2 <= nIt; i += 2) {
                body(i, sA, dA, sB, dB);
                body(i + 1, sB, dB, sA, dA);
            }
        }
        // (with compiler-placed MFMA results, unrolling by two makes the register allocator shuffle all
        // accumulators between VGPRs and AGPRs; the 32 copies are cheaper there)
        for (; i < nIt; i++) {
            body(i, sA, dA, sB, dB);
            sA = sB;
            dA = dB;
        }
    } else {
        // Two waves per SIMD: the other workgroup's wave fills the gaps.  Iteration i:
        //     S, dP chains of block i | P, dS | wait, barrier | issue block i+3 |
        //     output chains of block i, first operand reads of block i+1
        issue_block(0, 0); issue_bias(0, 0);
        issue_block(1, 1); issue_bias(1, 1);
        issue_block(2, 2); issue_bias(2, 2);
        // This kernel owns every query row once and already holds the row's dO: it forms
        // D = rowsum(dO o O) and lse log2 e itself and leaves the pair for the dkv kernel, which is
        // launched behind it (no separate pass over out and dO).  Placed here so that the row loads
        // are in flight together with the first blocks.
        {
            const bf16_t* og = (const bf16_t*)p.out + (lbase + rc) * p.Cg;
            float dsum = 0.f;
#pragma unroll
            for (int cs = 0; cs < K::CS; cs++) {
                if (cs * 16 < p.Cg) {      // (head dimension 16: the widened dO rows hold zeros there, out has no such channels)
                    const bf16x8 o8 = as_bf16x8(*(const u32x4*)(og + cs * 16 + 8 * hf));
#pragma unroll
                    for (int e = 0; e < 8; e++) dsum = fmaf((float)o8[e], (float)l2reg[cs][e], dsum);
                }
            }
            dsum += __shfl_xor(dsum, 32);
            my_d = dsum;
            my_lse2 = p.lse[lbase + rc] * kLog2e;
            if (hf == 0 && ri < NL) a.vec_w[lbase + ri] = make_float2(my_lse2, my_d);
        }
        wait_vmcnt<0>();
        __syncthreads();
        RowBase rb0 = mk_row(0);
        bf16_t* dbg = nullptr;      // dBias rows of this (b, h)
        if (DENSE) dbg = (bf16_t*)p.dbias + (size_t)bh * p.N * p.M;
#pragma unroll
        for (int n = 0; n < LA; n++) opr[n] = read_op(rb0, TrBase{}, n);

        for (int i = 0; i < nIt; i++) {
            const int slot = i & (NSLOT - 1);
            const TrBase tb0 = mk_tr(slot * kSlotBytes);
            const RowBase rbn = mk_row(((i + 1) & (NSLOT - 1)) * kSlotBytes);
            const int sb0 = blk_of(i) * BT;      // first streamed row of the block

            // ---------------- first half: S and dP chains ----------------
            f32x16 s, dp;
#pragma unroll
            for (int r = 0; r < 16; r++) { s[r] = 0.f; dp[r] = 0.f; }
            if (DENSE) bias_init(s, slot * kSlotBytes);
#pragma unroll
            for (int n = 0; n < NA; n++) {
                opr[(n + LA) % (LA + 1)] = read_op(rb0, tb0, n + LA);   // n + LA < NOPS: the output operands follow
                if (dead_step(n)) continue;
                if (n < K::KS) s = mfma32(opr[n % (LA + 1)], l1reg[n], s);
                else dp = mfma32(opr[n % (LA + 1)], l2reg[n - K::KS], dp);
            }
            // ---------------- P and dS in accumulator layout ----------------
            bf16x8 pb[2], dsb[2];
#pragma unroll
            for (int r = 0; r < 16; r++) elem(r, s, dp, my_lse2, my_d, false, sb0, pb, dsb);
            if ((sb0 + BT > NS) || (CAUSAL && sb0 + BT - 1 > rw0)) {
                // rare (diagonal blocks, sequence end): zero the dead elements behind a real branch
                asm volatile("" ::: "memory");
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    const int srow = sb0 + 8 * (r / 4) + 4 * hf + (r % 4);
                    if (srow >= NS || (CAUSAL && srow > ri)) dsb[r / 8][r % 8] = (bf16_t)0.f;
                }
            }
            // ---------------- dBias = dS, straight from the packed operand registers ----------------
            int nstores = 0;
            if (DENSE) {
                const int Mk = p.M;
                if (ri < NL) {
                    bf16_t* drow = dbg + (size_t)ri * Mk + sb0 + 4 * hf;
#pragma unroll
                    for (int g = 0; g < 4; g++) {
                        if (sb0 + 8 * g + 4 * hf < Mk) {
                            const u32x4 w = as_uint4(dsb[g >> 1]);
                            *(u32x2*)(drow + 8 * g) = (g & 1) ? u32x2{w.z, w.w} : u32x2{w.x, w.y};
                        }
                    }
                }
                // the wait below may count the stores only when every one of them is certain to issue
                if (rw0 + 31 < NL && sb0 + BT <= Mk) nstores = 4;
            }
            // ---------------- block i+1 has landed; everyone has left block i-1 ----------------
            wait_prev_loads(nstores);
            __syncthreads();
            issue_block(i + 3, (i + 3) & (NSLOT - 1));
            issue_bias(i + 3, (i + 3) & (NSLOT - 1));

            // ---------------- second half: output chains ----------------
            bf16x8 nxt[LA];      // first operands of block i+1 (the window restarts at 0 with every block)
#pragma unroll
            for (int n = NA; n < NOPS; n++) {
                if (n + LA < NOPS) opr[(n + LA) % (LA + 1)] = read_op(rb0, tb0, n + LA);
                else nxt[n + LA - NOPS] = read_op(rbn, tb0, n + LA - NOPS);
                const int m = n - NA;
                acc1[m >> 1] = mfma32(opr[n % (LA + 1)], dsb[m & 1], acc1[m >> 1]);
            }
#pragma unroll
            for (int n = 0; n < LA; n++) opr[n] = nxt[n];
            rb0 = rbn;
        }
        if (DENSE && CAUSAL && ri < NL) {
            // key blocks above the diagonal are never visited: their dBias is zero
            for (int blk = b_end; blk < nblk_all; blk++) {
                bf16_t* drow = dbg + (size_t)ri * p.M + blk * BT + 4 * hf;
#pragma unroll
                for (int g = 0; g < 4; g++)
                    if (blk * BT + 8 * g + 4 * hf < p.M) *(u32x2*)(drow + 8 * g) = u32x2{0u, 0u};
            }
        }
    }
    wait_vmcnt<0>();     // no direct load may outlive this tile's use of the ring
    __syncthreads();

    // ---- epilogue ----
    if (DKV && a.dkv_mul != 1.f) {      // wave-uniform: the q columns carried no scale
#pragma unroll
        for (int mb = 0; mb < K::MB; mb++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc1[mb][r] *= a.dkv_mul;
    }
    const bool rok = ri < NL;
    const int Cg = p.Cg;      // channels of the caller's gradient rows (< C: the rest is not stored)
    const size_t base = (size_t)bh * NL * Cg;
    const bool g32 = p.grad_f32 != 0;      // wave-uniform
    if (rok) {
        if (DKV) {
            bf16_t* dvg = (bf16_t*)p.dv + base + (size_t)ri * Cg;
            bf16_t* dkg = (bf16_t*)p.dk + base + (size_t)ri * Cg;
            float* dkf = (float*)p.dk + base + (size_t)ri * Cg;
#pragma unroll
            for (int mb = 0; mb < K::MBC; mb++)
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    if (mb * 32 + 8 * g >= Cg) continue;
                    bf16x4 a4, b4;
                    f32x4 bf;
#pragma unroll
                    for (int x = 0; x < 4; x++) {
                        a4[x] = (bf16_t)acc2[mb][4 * g + x];
                        b4[x] = (bf16_t)acc1[mb][4 * g + x];
                        bf[x] = acc1[mb][4 * g + x];
                    }
                    *(u32x2*)(dvg + mb * 32 + 8 * g + 4 * hf) = __builtin_bit_cast(u32x2, a4);
                    if (g32) *(f32x4*)(dkf + mb * 32 + 8 * g + 4 * hf) = bf;
                    else *(u32x2*)(dkg + mb * 32 + 8 * g + 4 * hf) = __builtin_bit_cast(u32x2, b4);
                }
        } else {
            bf16_t* dqg = (bf16_t*)p.dq + base + (size_t)ri * Cg;
            float* dqf = (float*)p.dq + base + (size_t)ri * Cg;
#pragma unroll
            for (int mb = 0; mb < K::MBC; mb++)
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    if (mb * 32 + 8 * g >= Cg) continue;
                    bf16x4 o4;
                    f32x4 of;
#pragma unroll
                    for (int x = 0; x < 4; x++) {
                        of[x] = acc1[mb][4 * g + x] * p.scale;
                        o4[x] = (bf16_t)of[x];
                    }
                    if (g32) *(f32x4*)(dqf + mb * 32 + 8 * g + 4 * hf) = of;
                    else *(u32x2*)(dqg + mb * 32 + 8 * g + 4 * hf) = __builtin_bit_cast(u32x2, o4);
                }
        }
    }
    if (RP > 0) {
        const bool f32 = p.phi_f32 != 0;
        const size_t esz = (f32 || g32) ? 4 : 2;
        float* scratch = (float*)smem + wave * 32 * (K::RP2 + 1);
        unsigned char* dst = nullptr;
        unsigned char* const dphi = (unsigned char*)(DKV ? p.dphi_k : p.dphi_q);     // NULL: factor gradients not wanted
        if (rok && dphi != nullptr) dst = dphi + ((size_t)bh * NL + ri) * R * esz;
        // the key-side limb order applies to the key's own gradient and vice versa
        float* dsl = nullptr;
        if (!DKV && rok && p.slopes != nullptr && p.dslope != nullptr) dsl = p.dslope + (size_t)bh * NL + ri;
        store_dphi<K::RP2, !DKV>(&acc1[K::MBC], scratch, dst, R, f32, g32, l32, hf, dsl, (float)ri);
    }
}

// Work units: one 128-row tile per workgroup, or when causal the tile pair (n-1-u, u), whose
// streamed ranges add up to the same length for every u (no tail of heavy tiles).
template <int C, int RP, bool CAUSAL, bool DKV, bool DENSE = false>
__global__ __launch_bounds__(kThreads, (DKV || DENSE || C + RP > 160) ? 1 : 2) void bwd_main_kernel(BwdParams p, MainArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int L = (blockIdx.x & 7) * p.tiles_per_xcd + (blockIdx.x >> 3);
    if (L >= p.total_tiles) return;
    const int n_units = CAUSAL ? (p.n_tiles + 1) / 2 : p.n_tiles;   // p.n_tiles: 128-row tiles of the lane side
    const int bh = L / n_units;
    const int u = L - bh * n_units;
    if (CAUSAL) {
        const int other = p.n_tiles - 1 - u;
        // heavier tile first: high query tiles for dq, low key tiles for dkv
        bwd_tile<C, RP, CAUSAL, DKV, DENSE>(p, a, smem, bh, DKV ? u : other);
        if (u != other) {
            __syncthreads();   // the epilogue's LDS scratch is reused as ring memory
            bwd_tile<C, RP, CAUSAL, DKV, DENSE>(p, a, smem, bh, DKV ? other : u);
        }
    } else {
        bwd_tile<C, RP, CAUSAL, DKV, DENSE>(p, a, smem, bh, u);
    }
}

// Pre-pass and the two main kernels.  DENSE: the bias is a dense matrix streamed tile by tile
// (RP = 0) and the dq kernel also writes dBias.
template <int C, int RP, bool CAUSAL, bool DENSE = false>
int launch(const BwdParams& pin, hipStream_t stream) {
    using K = Cfg<C, RP>;
    constexpr size_t slot = K::T1::BYTES + K::T2::BYTES + (DENSE ? (size_t)kWaves * 32 * 32 * 2 : 0);
    constexpr size_t ring_dq = (size_t)NSLOT * slot;
    constexpr size_t ring_dkv = (size_t)NSLOT_DKV * (slot + K::kVecBytes);
    constexpr size_t lds_dq = ring_dq > K::kEpiLds ? ring_dq : K::kEpiLds;
    constexpr size_t lds_dkv = ring_dkv > K::kEpiLds ? ring_dkv : K::kEpiLds;
    auto kdq = bwd_main_kernel<C, RP, CAUSAL, false, DENSE>;
    auto kdkv = bwd_main_kernel<C, RP, CAUSAL, true, DENSE>;
    static FbLdsOnce once_dq, once_dkv;
    if (!fb_raise_lds_limit((const void*)kdq, lds_dq, once_dq) || !fb_raise_lds_limit((const void*)kdkv, lds_dkv, once_dkv))
        return 1;

    const long long rows = (long long)pin.B * pin.H * pin.N;      // query rows
    const long long rowsk = (long long)pin.B * pin.H * pin.M;     // key rows
    // Split rows (C a multiple of 64, caller's rows of C channels): the k columns of the key-side rows were
    // a copy, so the kernels read k itself.  On the query side the q columns carry the scale; it can move
    // onto the factor columns (as 1/scale) and into the exponent and the dK epilogue, so that q is read in
    // place too -- where the forward formed its scores that way as well (lse and D belong to the forward's
    // scores, and the recomputed ones must be those): no factors, fp32 factors (scaled before the limb
    // split) and ALiBi factors made in the kernels; and wherever bf16(q scale) = q scale, i.e. for a scale
    // that is a power of two (head dimension 64 at the default scale with bf16 factors, and the
    // multiplicative form, whose prepared rows carry their scale already).  Never with a dense bias, which
    // enters the chain unscaled.
    constexpr bool kCanSplit = C % 64 == 0;
    int mant_exp = 0;
    const bool pow2 = std::frexp(pin.scale, &mant_exp) == 0.5f;
    const bool split_k = kCanSplit && pin.Cg == C;
    const bool split_q = split_k && !DENSE && (pow2 || RP == 0 || pin.phi_f32 != 0 || pin.slopes != nullptr);
    // workspace: vec [rows] float2 | Aq [rows][W or RP2] bf16 | Ak [rowsk][W or RP2] bf16  (each a multiple of 16 bytes)
    unsigned char* ws = (unsigned char*)pin.workspace;
    MainArgs a;
    a.vec = (const float2*)ws;
    a.vec_w = (float2*)ws;
    bf16_t* aq = (bf16_t*)(ws + (((size_t)rows * 8 + 15) & ~(size_t)15));
    bf16_t* ak = aq + (size_t)rows * (split_q ? K::RP2 : K::W);
    a.aq = split_q ? OperandRows{(const bf16_t*)pin.q, C, aq, K::RP2} : OperandRows{aq, K::W, aq + C, K::W};
    a.ak = split_k ? OperandRows{(const bf16_t*)pin.k, C, ak, K::RP2} : OperandRows{ak, K::W, ak + C, K::W};
    a.exp_mul = split_q ? kLog2e * pin.scale : kLog2e;
    a.dkv_mul = split_q ? pin.scale : 1.f;
    const float qmul = split_q ? 1.f / pin.scale : 1.f;

    BwdParams p = pin;
    bool narrow = false;
    if constexpr (C == 32) {
        if (pin.Cg == 16) {
            // widened copies of v and dO behind the operand rows; out and dO keep their 16-channel rows
            // for the row sums
            narrow = true;
            constexpr int RPB = kPrepRows<C, RP, false>;
            const unsigned nb_q = (unsigned)((rows + RPB - 1) / RPB);
            const unsigned nb_k = (unsigned)((rowsk + RPB - 1) / RPB);
            bf16_t* vpad = ak + (size_t)rowsk * K::W;
            bf16_t* dpad = vpad + (size_t)rowsk * 32;
            hipLaunchKernelGGL(bwd_pad16_kernel, dim3((unsigned)((rowsk * 4 + 255) / 256)), dim3(256), 0, stream,
                               (const bf16_t*)pin.v, vpad, rowsk);
            hipLaunchKernelGGL(bwd_pad16_kernel, dim3((unsigned)((rows * 4 + 255) / 256)), dim3(256), 0, stream,
                               (const bf16_t*)pin.dout, dpad, rows);
            hipLaunchKernelGGL((bwd_pre_kernel<C, RP>), dim3(nb_q + nb_k), dim3(256), 0, stream, pin, aq, ak, nb_q, 1.f);
            if (hipGetLastError() != hipSuccess) return 1;
            p.v = vpad;
            p.dout = dpad;
        }
    }
    if (!narrow) {
        if (pin.Cg != C) return -1;
        auto blocks = [](long long r, int rows_per_block) { return (unsigned)((r + rows_per_block - 1) / rows_per_block); };
        if constexpr (kCanSplit && RP > 0) {
            constexpr int RS = kPrepRows<C, RP, true>, RW = kPrepRows<C, RP, false>;
            if (split_q) {
                const unsigned nb_q = blocks(rows, RS), nb_k = blocks(rowsk, RS);
                if (nb_q + nb_k) hipLaunchKernelGGL((bwd_pre_kernel<C, RP, true, true>), dim3(nb_q + nb_k), dim3(256), 0, stream, pin, aq, ak, nb_q, qmul);
            } else if (split_k) {
                const unsigned nb_q = blocks(rows, RW), nb_k = blocks(rowsk, RS);
                if (nb_q + nb_k) hipLaunchKernelGGL((bwd_pre_kernel<C, RP, false, true>), dim3(nb_q + nb_k), dim3(256), 0, stream, pin, aq, ak, nb_q, 1.f);
            } else {
                const unsigned nb_q = blocks(rows, RW), nb_k = blocks(rowsk, RW);
                if (nb_q + nb_k) hipLaunchKernelGGL((bwd_pre_kernel<C, RP>), dim3(nb_q + nb_k), dim3(256), 0, stream, pin, aq, ak, nb_q, 1.f);
            }
        } else {
            // no factor columns to write for a split side (RP = 0): its workgroups are simply not launched
            constexpr int RW = kPrepRows<C, RP, false>;
            const unsigned nb_q = split_q ? 0u : blocks(rows, RW);
            const unsigned nb_k = split_k ? 0u : blocks(rowsk, RW);
            if (nb_q + nb_k) hipLaunchKernelGGL((bwd_pre_kernel<C, RP>), dim3(nb_q + nb_k), dim3(256), 0, stream, pin, aq, ak, nb_q, 1.f);
        }
        if (hipGetLastError() != hipSuccess) return 1;
    }

    auto set_tiles = [](BwdParams& p, int lane_rows) {
        p.n_tiles = (lane_rows + 127) / 128;
        const int n_units = CAUSAL ? (p.n_tiles + 1) / 2 : p.n_tiles;
        p.total_tiles = p.B * p.H * n_units;
        p.tiles_per_xcd = (p.total_tiles + 7) / 8;
    };
    // dq first: it also leaves (lse log2 e, D) of every query row for the dkv kernel
    set_tiles(p, p.N);
    hipLaunchKernelGGL(kdq, dim3(8 * p.tiles_per_xcd), dim3(kThreads), lds_dq, stream, p, a);
    if (hipGetLastError() != hipSuccess) return 1;
    set_tiles(p, p.M);
    hipLaunchKernelGGL(kdkv, dim3(8 * p.tiles_per_xcd), dim3(kThreads), lds_dkv, stream, p, a);
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
        case 48: return dispatch_causal<C, 48>(p, stream);
        case 64: return dispatch_causal<C, 64>(p, stream);
        default: break;
    }
    // wider rows: the C (R - 1) extra channels of the multiplicative form (bf16 columns)
    if constexpr (C <= 64) {
        if (p.phi_f32) return -1;
        if (rp == 96) return dispatch_causal<C, 96>(p, stream);
        if (rp == 128) return dispatch_causal<C, 128>(p, stream);
    }
    return -1;
}

}  // namespace

size_t fb_bwd_workspace_bytes(long long rows_q, long long rows_k, int C, int R) {
    // R alone does not say whether the factors are fp32 (6 R columns): size for the widest rows.
    // Head dimension 16 runs on 32-channel operand rows and adds widened copies of v and dO.
    const int w = (C == 16 ? 32 : C) + (R > 64 ? 128 : (R > 0 ? 64 : 0)) + (C == 16 ? 32 : 0);
    return (((size_t)rows_q * 8 + 15) & ~(size_t)15) + (size_t)(rows_q + rows_k) * w * 2;
}

int fb_launch_bwd_dense_bf16(const BwdParams& p, int C, hipStream_t stream) {
    switch (C) {
        case 16: return p.causal ? launch<32, 0, true, true>(p, stream) : launch<32, 0, false, true>(p, stream);   // p.Cg = 16
        case 32: return p.causal ? launch<32, 0, true, true>(p, stream) : launch<32, 0, false, true>(p, stream);
        case 64: return p.causal ? launch<64, 0, true, true>(p, stream) : launch<64, 0, false, true>(p, stream);
        case 128: return p.causal ? launch<128, 0, true, true>(p, stream) : launch<128, 0, false, true>(p, stream);
        default: return -1;
    }
}

int fb_launch_bwd_bf16(const BwdParams& p, int C, int rp, hipStream_t stream) {
    switch (C) {
        case 16: return dispatch_rp<32>(p, rp, stream);      // p.Cg = 16
        case 32: return dispatch_rp<32>(p, rp, stream);
        case 64: return dispatch_rp<64>(p, rp, stream);
        case 128: return dispatch_rp<128>(p, rp, stream);
        default: return -1;
    }
}
