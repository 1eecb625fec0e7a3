// bf16 MFMA forward, direct-to-LDS variant with the matrix / vector overlap written into one
// wave's instruction stream.
//
// One workgroup = 4 waves = 128 query rows, one 32-row query block per wave.  Each iteration
// has two regions, every MFMA followed by its share of the vector / LDS work and a scheduling
// barrier, so the order in the source is the order executed:
//   region 1 :  S_{t+1} = K_{t+1} . Q   (MFMA chain)  interleaved with exp / sum / convert of
//               block t (P_t) and the V_t transpose reads
//   region 2 :  O += V_t P_t            (MFMA chain)  interleaved with the row maxima of
//               S_{t+1} and the K_{t+2} operand reads
//   barrier
// Orientation, operand layouts, factor handling, masking and the lazy rescale are those of the
// four-wave kernel in fb_fwd_bf16_impl.h.  Nothing on the key side passes through registers on
// its way from HBM: every wave issues 128-bit global loads that write LDS directly
// (global_load_lds_dwordx4), several blocks ahead, so there are neither staging registers nor
// LDS stores, and a tile's set-up is short.
//
// The direct loads are issued from inline assembly.  The compiler therefore does not know
// that LDS is written asynchronously (with the builtin it makes every later LDS transpose read
// wait for vmcnt(0), which serialises the pipeline); the kernel does the vmcnt bookkeeping
// itself: there are no register-destination global loads inside the main loop, each wave
// knows how many direct loads it issues per iteration, and before the barrier that ends an
// iteration it waits until only that many remain outstanding.  M0 (the LDS base of a direct
// load) is written inside the asm block; nothing else in this kernel uses M0.
//
// LDS layout.  A direct load writes 64 consecutive 16-byte slots (lane l -> slot l), so the
// K and V tiles are unpadded row-major [32 keys][C]; bank conflicts are avoided by choosing
// WHICH 16-byte chunk of a row each lane fetches: chunk c of row r is stored at chunk position
// c ^ swz(r), with swz chosen per head dimension so that both access patterns are
// conflict-free: the K operand reads (16 consecutive rows, same chunk) and the V transpose
// reads (4 consecutive rows x 4 consecutive chunks).  The factor rows of a block are one
// contiguous span of phi_k; it is copied raw into a small ring and converted (zero padding,
// or the three-limb split of fp32 factors) into the padded operand layout by an
// LDS -> registers -> LDS pass two iterations before its first use.  Dense bias tiles
// (baseline mode) are copied per wave, 32 query rows x 32 keys.
//
// Rings (block b = the b-th key block in the order this tile walks them):
//   K_b        4 slots  issued in iteration b-4, read in iterations b-2 (first operands) and b-1
//   V_b        3 slots  issued in iteration b-2, read in iteration b
//   raw phi_b  3 slots  issued in iteration b-5, converted in iteration b-3 into
//   phi ops_b  4 slots  read with K_b
//   bias_b     3 slots  issued in iteration b-3, read at the start of iteration b-1
// At the end of iteration t everything issued before iteration t has landed (vmcnt wait) and
// is published by the barrier; a slot is refilled only after the barrier that follows its
// last reader.
#ifndef FB_FWD_BF16_DMA_H_
#define FB_FWD_BF16_DMA_H_

#include <hip/hip_runtime.h>

#include "fb_device.h"
#include "fb_launch.h"
#include "fb_params.h"

namespace fbdma {

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int BK = 32;
constexpr int NKB = 4;       // K / factor operand ring slots
constexpr int NVB = 3;       // V ring slots
constexpr int NRB = 3;       // raw factor ring slots
constexpr int NBB = 3;       // bias ring slots
constexpr int LA = 4;        // LDS operand reads run this many MFMAs ahead of their use
constexpr float kRescaleTau = 8.0f;

// chunk-position swizzle of row r (see the header comment)
template <int C>
FB_DEV int swz(int r) {
    if (C == 128) return ((r & 3) << 2) | ((r >> 2) & 3);
    if (C == 64) return (((r >> 1) & 1) << 2) | ((r >> 2) & 3);
    return (r >> 2) & 3;
}

template <int C, int RP, bool DENSE>
struct Cfg {
    static constexpr int KSC = C / 16;                // k-steps over the channels
    static constexpr int KS = (C + RP) / 16;          // ... plus the factor columns
    static constexpr int CPR = C / 8;                 // 16-byte chunks per row
    static constexpr int RPD = 64 / CPR;              // rows written by one direct load
    static constexpr int NDMA = CPR / 4;              // K/V direct loads per wave per iteration
    static constexpr int PP = RP + 8;                 // factor operand row pitch (elements)
    static constexpr int KBLK = BK * C;               // elements per K or V slot
    static constexpr int PBLK = BK * PP;              // elements per factor operand slot
    static constexpr int RAWB = (RP / 16) * 1024;     // bytes per raw factor slot (>= 32 * R * esz)
    static constexpr int BIASB = 32 * BK * 2;         // bytes per wave per bias slot
    static constexpr int NV = (C / 32) * 2;
    static constexpr int BQ = kWaves * 32;
    static constexpr int kOffV = NKB * KBLK * 2;
    static constexpr int kOffP = kOffV + NVB * KBLK * 2;
    static constexpr int kOffRaw = kOffP + (RP > 0 ? NKB * PBLK * 2 : 0);
    static constexpr int kOffBias = kOffRaw + (RP > 0 ? NRB * RAWB : 0);
    static constexpr int kLds = kOffBias + (DENSE ? NBB * kWaves * BIASB : 0);
};

// s_waitcnt with only vmcnt constrained
// (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt_hi[15:14])
template <int N>
FB_DEV void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// One 16-byte-per-lane direct load: lane l reads sbase + voff (bytes) and its 16 bytes land
// at LDS byte address lds_addr + 16 * l.  sbase and lds_addr are wave-uniform.
FB_DEV void dma16(const void* sbase, unsigned voff, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(voff), "s"(sbase), "s"(lds_addr) : "memory", "m0");
}

// PM: 0 none, 1 bf16 factors with R % 8 == 0, 2 other bf16 factors, 3 fp32 factors (limb items)
template <int C, int RP, int PM, bool CAUSAL, bool DENSE>
__global__ __launch_bounds__(kThreads, 2) void fwd_bf16_dma_kernel(FwdParams p) {
    using K = Cfg<C, RP, DENSE>;
    extern __shared__ __align__(16) unsigned char smem[];
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
    const bf16_t* const kt = (const bf16_t*)smem;                       // [NKB][BK][C]   swizzled
    const bf16_t* const vt = (const bf16_t*)(smem + K::kOffV);          // [NVB][BK][C]   swizzled
    bf16_t* const pt = (bf16_t*)(smem + K::kOffP);                      // [NKB][BK][PP]  factor operands
    const unsigned char* const rawp = smem + K::kOffRaw;                // [NRB][RAWB]    raw factor rows

    const int L = (blockIdx.x & 7) * p.tiles_per_xcd + (blockIdx.x >> 3);
    if (L >= p.total_tiles) return;
    int bh, qt;
    if (DENSE && p.bias_bstride == 0) {   // shared bias: batch-minor order (see fb_fwd_bf16_impl.h)
        const int rest = L / p.B;
        const int bb = L - rest * p.B;
        const int hh = rest / p.n_qtiles;
        qt = rest - hh * p.n_qtiles;
        bh = bb * p.H + hh;
    } else {
        bh = L / p.n_qtiles;
        qt = L - bh * p.n_qtiles;
    }
    if (CAUSAL) qt = p.n_qtiles - 1 - qt;
    const int b = bh / p.H, h = bh - b * p.H;
    const int N = p.N, R = p.R;
    constexpr bool phi_f32 = PM == 3;
    constexpr int phi_esz = phi_f32 ? 4 : 2;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, hf = lane >> 5;
    const int q0 = qt * K::BQ;
    const int qw0 = q0 + wave * 32;
    const int qi = qw0 + l32;

    const size_t base = (size_t)bh * N * C;
    const bf16_t* qg = (const bf16_t*)p.q + base;
    const bf16_t* kg = (const bf16_t*)p.k + base;
    const bf16_t* vg = (const bf16_t*)p.v + base;
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
    // scale sits in the exponent's multiply-add
    constexpr bool RAWQ = !DENSE && C % 64 == 0 && (PM == 0 || PM == 3);
    const float emul = RAWQ ? p.scale * kLog2e : kLog2e;
    bf16x8 qreg[K::KS];
    {
        const int qc = min(qi, N - 1);
#pragma unroll
        for (int ks = 0; ks < K::KS; ks++) {
            bf16x8 val;
            if (ks < K::KSC) {
                const bf16x8 x = as_bf16x8(*(const u32x4*)(qg + (size_t)qc * C + ks * 16 + 8 * hf));
#pragma unroll
                for (int e = 0; e < 8; e++) val[e] = RAWQ ? x[e] : (bf16_t)((float)x[e] * p.scale);
            } else {
                const int c8 = (ks - K::KSC) * 2 + hf;
                val = phi_chunk_gather<true>(pqg + (size_t)qc * R * phi_esz, c8, R, phi_f32, RAWQ ? p.inv_scale : 1.f);
            }
            qreg[ks] = val;
        }
    }

    f32x16 oacc[C / 32];
#pragma unroll
    for (int cb = 0; cb < C / 32; cb++)
#pragma unroll
        for (int r = 0; r < 16; r++) oacc[cb][r] = 0.f;
    float mref = -INFINITY, lsum = 0.f, mx2 = -INFINITY;

    const int kend = CAUSAL ? min(N, q0 + K::BQ) : N;
    const int nT = (kend + BK - 1) / BK;
    const int nTall = (N + BK - 1) / BK;
    // causal tiles walk the keys from the diagonal back to key 0 (see fb_fwd_bf16_impl.h); walk
    // positions past the end (the prefetch overruns by up to five) re-load a valid block
    auto blk_of = [&](int t) __attribute__((always_inline)) {
        return CAUSAL ? max(nT - 1 - t, 0) : min(t, nTall - 1);
    };
    // blocks [0, t_plain) (in key order) need no mask for any row of this wave
    int t_plain = N / BK;
    if (CAUSAL) t_plain = min(t_plain, (qw0 + 1) / BK);
    t_plain = min(t_plain, nT);

    // ---- direct loads: this wave's share of one K block and one V block ----
    // load d (0..CPR-1): d < CPR/2 -> K rows [d*RPD, +RPD), else V rows [(d-CPR/2)*RPD, +RPD);
    // lane l -> row l / CPR of that group, chunk position l % CPR holds global chunk position ^ swz(row)
    int dma_row[K::NDMA];
    unsigned dma_goff[K::NDMA];      // byte offset of this lane's chunk inside its row
#pragma unroll
    for (int i = 0; i < K::NDMA; i++) {
        const int sub = (wave + kWaves * i) % (K::CPR / 2);
        dma_row[i] = sub * K::RPD + lane / K::CPR;
        dma_goff[i] = (unsigned)(((lane % K::CPR) ^ swz<C>(dma_row[i])) * 16);
    }
    auto issue_kv = [&](int tk, int sk, int tv, int sv) __attribute__((always_inline)) {
        const int k0k = blk_of(tk) * BK, k0v = blk_of(tv) * BK;
#pragma unroll
        for (int i = 0; i < K::NDMA; i++) {
            const int d = wave + kWaves * i;                       // wave-uniform
            const bool isk = d < K::CPR / 2;
            const int sub = d % (K::CPR / 2);
            const int k0 = isk ? k0k : k0v;
            const unsigned voff = (unsigned)(min(dma_row[i], N - 1 - k0) * (C * 2)) + dma_goff[i];
            const bf16_t* src = (isk ? kg : vg) + (size_t)k0 * C;
            const unsigned dst = lds0 + (isk ? sk * (K::KBLK * 2) : K::kOffV + sv * (K::KBLK * 2)) + sub * 1024;
            dma16(src, voff, dst);
        }
    };

    // ---- factor rows: raw copy (wave w issues the w-th 1 KB piece of the block's span) ----
    const int phi_blk_bytes = BK * R * phi_esz;                       // span of a full block
    const int phi_all_bytes = N * R * phi_esz;                        // multiple of 16 (checked by the host)
    const int nphi_w = (RP > 0 && wave * 1024 < phi_blk_bytes) ? 1 : 0;   // direct loads per iteration, this wave
    auto issue_phi = [&](int t, int slot) __attribute__((always_inline)) {
        if (RP == 0 || !nphi_w) return;
        const int boff = blk_of(t) * phi_blk_bytes;
        const int last = (min(phi_all_bytes - boff, phi_blk_bytes) >> 4) - 1;   // last valid chunk
        const unsigned voff = (unsigned)(min(wave * 64 + lane, last) << 4);
        dma16(pkg + boff, voff, lds0 + K::kOffRaw + slot * K::RAWB + wave * 1024);
    };
    // raw slot -> operand slot: pad to RP columns (zeros stay from the initial fill) or split limbs
    auto convert_phi = [&](int rslot, int pslot) __attribute__((always_inline)) {
        if (RP == 0) return;
        const unsigned char* src = rawp + rslot * K::RAWB;
        bf16_t* dst = pt + pslot * K::PBLK;
        if (PM == 3) {
            constexpr int IT = (BK * (RP / 6) + kThreads - 1) / kThreads;
#pragma unroll
            for (int it = 0; it < IT; it++) {
                const int e = tid + it * kThreads;
                if (e < BK * R) {
                    const int row = e / R, r = e - row * R;
                    phi_item_store_k(dst + row * K::PP + 6 * r, ((const float*)src)[e]);
                }
            }
        } else if (PM == 1) {
            constexpr int IT = (BK * RP / 8 + kThreads - 1) / kThreads;
            const int cpr = R >> 3;
#pragma unroll
            for (int it = 0; it < IT; it++) {
                const int e = tid + it * kThreads;
                if (e < BK * cpr) {
                    const int row = e / cpr, c8 = e - row * cpr;
                    *(u32x4*)(dst + row * K::PP + c8 * 8) = ((const u32x4*)src)[e];
                }
            }
        } else if (PM == 2) {
            constexpr int IT = (BK * RP + kThreads - 1) / kThreads;
#pragma unroll
            for (int it = 0; it < IT; it++) {
                const int e = tid + it * kThreads;
                if (e < BK * R) {
                    const int row = e / R, r = e - row * R;
                    dst[row * K::PP + r] = ((const bf16_t*)src)[e];
                }
            }
        }
    };

    // ---- dense mode: per-wave bias tile [32 query rows][32 keys], two direct loads per block.
    // lane l of load i covers row 16*i + l/4; chunk position l%4 holds key chunk (l%4) ^ ((row>>2)&3)
    unsigned bias_voff[2];
    if (DENSE) {
#pragma unroll
        for (int i = 0; i < 2; i++) {
            const int row = 16 * i + (lane >> 2);
            const int c = (lane & 3) ^ ((row >> 2) & 3);
            bias_voff[i] = (unsigned)(min(qw0 + row, N - 1) - min(qw0, N - 1)) * (unsigned)(N * 2) + c * 16;
        }
    }
    auto issue_bias = [&](int t, int slot) __attribute__((always_inline)) {
        if (!DENSE) return;
        const bf16_t* src = bg + (size_t)min(qw0, N - 1) * N + blk_of(t) * BK;   // N % 32 == 0 here
#pragma unroll
        for (int i = 0; i < 2; i++)
            dma16(src, bias_voff[i], lds0 + K::kOffBias + (slot * kWaves + wave) * K::BIASB + i * 1024);
    };
    auto init_s = [&](f32x16& s, int slot) __attribute__((always_inline)) {
        if (DENSE) {
            // accumulator register 4*g + x <-> key 8*g + 4*hf + x of row l32
            const unsigned char* brow = smem + K::kOffBias + (slot * kWaves + wave) * K::BIASB + l32 * 64 + hf * 8;
#pragma unroll
            for (int g = 0; g < 4; g++) {
                const bf16x4 bv = __builtin_bit_cast(bf16x4, *(const u32x2*)(brow + ((g ^ ((l32 >> 2) & 3)) << 4)));
#pragma unroll
                for (int x = 0; x < 4; x++) s[4 * g + x] = (float)bv[x];
            }
        } else {
#pragma unroll
            for (int r = 0; r < 16; r++) s[r] = 0.f;
        }
    };

    // ---- per-lane LDS read offsets (elements) ----
    // K operand ks (channels): row l32, chunk 2*ks + hf at position (2*ks + hf) ^ swz(l32)
    int koff[K::KSC];
#pragma unroll
    for (int ks = 0; ks < K::KSC; ks++) koff[ks] = l32 * C + (((2 * ks + hf) ^ swz<C>(l32)) * 8);
    const int poff = l32 * K::PP + 8 * hf;           // factor operand ks: + (ks - KSC) * 16
    // V transpose read of channel block cb, part hi (keys +8): rows 4*hf + i16/4 (+ 8*hi), 16-lane
    // group blk covers channels 16*blk..+15, lane supplies columns 4*(i16%4)..+3
    const int i16 = lane & 15, blk = l32 >> 4;
    int voff[C / 32][2];
#pragma unroll
    for (int cb = 0; cb < C / 32; cb++)
#pragma unroll
        for (int hi = 0; hi < 2; hi++) {
            const int row = 8 * hi + 4 * hf + (i16 >> 2);
            const int chunk = cb * 4 + 2 * blk + ((i16 & 3) >> 1);
            voff[cb][hi] = row * C + ((chunk ^ swz<C>(row)) * 8) + (i16 & 1) * 4;
        }
    bf16x8 ka[K::KS];
    bf16x8 va[K::NV];
    auto read_k = [&](int slot, int ks) __attribute__((always_inline)) {
        if (ks < K::KSC) ka[ks] = as_bf16x8(*(const u32x4*)(kt + slot * K::KBLK + koff[ks]));
        else ka[ks] = as_bf16x8(*(const u32x4*)(pt + slot * K::PBLK + poff + (ks - K::KSC) * 16));
    };
    auto read_v = [&](int slot, int v) __attribute__((always_inline)) {
        // v = 2*cb + kk: keys kk*16.. of the block (swz ignores row bit 4)
        const bf16_t* vb = vt + slot * K::KBLK + (v & 1) * 16 * C;
        va[v] = join_tr(lds_read_tr16(vb + voff[v >> 1][0]), lds_read_tr16(vb + voff[v >> 1][1]));
    };
    auto mask_block = [&](f32x16& s, int kb0) __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < 16; r++) {
            const int key = kb0 + 8 * (r / 4) + 4 * hf + (r % 4);
            if (key >= N || (CAUSAL && key > qi)) s[r] = -INFINITY;
        }
    };

    // ---- prologue ----
    if (RP > 0) {   // operand columns the conversion never writes stay zero for the whole kernel
        for (int e = tid; e < NKB * K::PBLK / 2; e += kThreads) ((unsigned*)pt)[e] = 0u;
    }
    issue_kv(0, 0, 0, 0);
    issue_kv(1, 1, 1, 1);
    issue_kv(2, 2, 2, 2);       // V_2 is loaded again by iteration 0 (harmless, keeps the issue uniform)
    issue_kv(3, 3, 2, 2);
    issue_phi(0, 0); issue_phi(1, 1); issue_phi(2, 2);
    issue_bias(0, 0); issue_bias(1, 1); issue_bias(2, 2);
    wait_vmcnt<0>();
    __syncthreads();
    convert_phi(0, 0); convert_phi(1, 1); convert_phi(2, 2);
    __syncthreads();
    issue_phi(3, 0); issue_phi(4, 1);
    f32x16 sA, sB;
    {
#pragma unroll
        for (int ks = 0; ks < K::KS; ks++) read_k(0, ks);
        init_s(sA, 0);
#pragma unroll
        for (int ks = 0; ks < K::KS; ks++) sA = mfma32(ka[ks], qreg[ks], sA);
        const int kb0 = blk_of(0) * BK;
        if ((kb0 + BK > N) || (CAUSAL && kb0 + BK - 1 > qw0)) mask_block(sA, kb0);
        mx2 = half_max(max16(sA)) * emul;
#pragma unroll
        for (int ks = 0; ks < LA && ks < K::KS; ks++) read_k(1, ks);
    }
    wait_vmcnt<0>();
    __syncthreads();   // iteration 0 refills the slot of K_0: every wave must be done reading it

    int kslot = 0, vslot = 0;   // slots of block t in the 4-rings and the 3-rings
    auto body = [&](int t, f32x16& scur, f32x16& snext) __attribute__((always_inline)) {
        const bool MASKED = CAUSAL ? (t < nT - t_plain) : (t + 1 >= t_plain);
        const int kslot1 = (kslot + 1) & (NKB - 1), kslot2 = (kslot + 2) & (NKB - 1),
                  kslot3 = (kslot + 3) & (NKB - 1);
        const int vslot1 = vslot == 2 ? 0 : vslot + 1;     // (t + 1) % 3
        const int vslot2 = vslot == 0 ? 2 : vslot - 1;     // (t + 2) % 3
        const int kb1 = blk_of(t + 1) * BK;
        const bool skip_t = MASKED && CAUSAL && blk_of(t) * BK > qw0 + 31;
        const bool skip_n = MASKED && CAUSAL && kb1 > qw0 + 31;

        // ---- this iteration's direct loads.  K_{t+4} goes into the slot of K_t (all its operands
        // were read by the end of iteration t-1), V_{t+2} into the slot of V_{t-1}, the raw
        // factors of block t+5 into the slot of block t+2 (converted in iteration t-1), the bias
        // of block t+3 into the slot of block t (read at the start of iteration t-1).
        issue_kv(t + 4, kslot, t + 2, vslot2);
        issue_phi(t + 5, vslot2);
        issue_bias(t + 3, vslot);
        convert_phi(vslot, kslot3);     // factors of block t+3: raw slot (t+3) % 3 == t % 3
        __builtin_amdgcn_sched_barrier(0);

        // ---- lazy rescale (rare) ----
        if (__builtin_expect(__any(mx2 > mref + kRescaleTau), 0)) {
            const float mnew = fmaxf(fmaxf(mref, mx2), -1e30f);
            const float alpha = fast_exp2(mref - mnew);
            mref = mnew;
            lsum *= alpha;
#pragma unroll
            for (int cb = 0; cb < C / 32; cb++)
#pragma unroll
                for (int r = 0; r < 16; r++) oacc[cb][r] *= alpha;
        }
        const float nm = mref == -INFINITY ? 0.f : -mref;
        float ps[4] = {0.f, 0.f, 0.f, 0.f};
        init_s(snext, vslot1);
        __builtin_amdgcn_sched_barrier(0);

        // ================= region 1: S_{t+1} chain | exp of block t | first V_t operands =========
        bf16x8 pb[2];
        constexpr int VPRE = K::NV < LA ? K::NV : LA;
#pragma unroll
        for (int i = 0; i < K::KS; i++) {
            if (!skip_n) snext = mfma32(ka[i], qreg[i], snext);
            if (i + LA < K::KS) read_k(kslot1, i + LA);
#pragma unroll
            for (int e = (i * 16) / K::KS; e < ((i + 1) * 16) / K::KS; e++) {
                float pr = fast_exp2(fmaf(scur[e], emul, nm));
                // the empty asm pins the computation to this step: without it the optimiser
                // sinks the whole exponentiation down to its first use
                asm volatile("" : "+v"(pr));
                ps[e & 3] += pr;
                pb[e / 8][e % 8] = (bf16_t)pr;
            }
            if (i >= K::KS / 2) {
                constexpr int H1 = K::KS - K::KS / 2;
                const int ii = i - K::KS / 2;
#pragma unroll
                for (int v = (ii * VPRE) / H1; v < ((ii + 1) * VPRE) / H1; v++) read_v(vslot, v);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        lsum += (ps[0] + ps[1]) + (ps[2] + ps[3]);

        // ================= region 2: O chain | maxima of S_{t+1} | first K_{t+2} operands ==========
        {
            const bool mask_n = MASKED && ((kb1 + BK > N) || (CAUSAL && kb1 + BK - 1 > qw0));
            constexpr int KPRE = K::KS < LA ? K::KS : LA;
            float m = -INFINITY;
#pragma unroll
            for (int j = 0; j < K::NV; j++) {
                if (!skip_t) oacc[j >> 1] = mfma32(va[j], pb[j & 1], oacc[j >> 1]);
                if (j + VPRE < K::NV) read_v(vslot, j + VPRE);
                if (j >= K::NV / 2) {
                    constexpr int H2 = K::NV - K::NV / 2;
                    const int jj = j - K::NV / 2;
#pragma unroll
                    for (int ks = (jj * KPRE) / H2; ks < ((jj + 1) * KPRE) / H2; ks++) read_k(kslot2, ks);
                    if (jj == 0 && mask_n) {
                        asm volatile("" ::: "memory");   // keep this a real (rarely taken) branch
                        mask_block(snext, kb1);
                    }
#pragma unroll
                    for (int e = (jj * 16) / H2; e < ((jj + 1) * 16) / H2; e++) m = e == 0 ? snext[0] : fmaxf(m, snext[e]);
                    asm volatile("" : "+v"(m));
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            mx2 = half_max(m) * emul;
        }
        // everything issued before this iteration must have landed before the barrier: only this
        // iteration's own direct loads (NDMA for K/V, two for a bias tile, one for factors) may remain
        if (nphi_w) wait_vmcnt<K::NDMA + (DENSE ? 2 : 0) + 1>();
        else wait_vmcnt<K::NDMA + (DENSE ? 2 : 0)>();
        __syncthreads();
        kslot = kslot1;
        vslot = vslot1;
    };

    for (int t = 0; t < nT; t += 2) {
        body(t, sA, sB);
        if (t + 1 < nT) body(t + 1, sB, sA);
    }
    wait_vmcnt<0>();   // no direct load may outlive the workgroup's LDS allocation

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
    using K = Cfg<C, RP, DENSE>;
    auto kern = fwd_bf16_dma_kernel<C, RP, PM, CAUSAL, DENSE>;
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
    if (p.phi_f32) return dispatch_causal<C, RP, 3, false>(p, stream);
    if ((p.R % 8) == 0) return dispatch_causal<C, RP, 1, false>(p, stream);
    return dispatch_causal<C, RP, 2, false>(p, stream);
}

// The direct loads move whole 16-byte pieces: every (b, h) factor matrix must start on a
// 16-byte boundary (N * R * element size a multiple of 16); a dense bias needs whole key
// blocks (N % 32 == 0).
inline bool supported(const FwdParams& p, bool dense) {
    if (dense) return (p.N % BK) == 0;
    if (p.R == 0) return true;
    const long long esz = p.phi_f32 ? 4 : 2;
    return ((long long)p.N * p.R * esz) % 16 == 0 && ((long long)p.phi_bstride * esz) % 16 == 0;
}

// Returns 0 on success, 1 on launch failure, -1 when no instantiation fits.
template <int C>
int dispatch(const FwdParams& p, int rp, bool dense, hipStream_t stream) {
    if (!supported(p, dense)) return -1;
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

}  // namespace fbdma

#endif
