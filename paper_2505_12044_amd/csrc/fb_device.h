// Device-side building blocks for the gfx950 (CDNA4, wave64) bf16 kernels: vector types,
// MFMA wrappers with their operand layouts, cross-half lane exchange, the LDS transpose
// read, and the bf16 limb split used for fp32 bias factors.
#ifndef FB_DEVICE_H_
#define FB_DEVICE_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

#define FB_DEV __device__ __forceinline__

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// ---- MFMA 32x32x16 bf16, fp32 accumulate -------------------------------------------------
// D[32x32] += A[32x16] * B[16x32].  Lane l (0..63), hf = l / 32:
//   A operand: row l % 32, the eight k-slots 8*hf .. 8*hf+7
//   B operand: column l % 32, the same eight k-slots
//   D / C: column l % 32, rows 8*(r/4) + 4*hf + (r%4) for accumulator register r = 0..15.
// Only "same k-slot on both operands" matters for correctness, so a kernel may assign any
// eight of its contraction indices to a lane's slots as long as A and B agree.
FB_DEV f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// The same instruction with the result pinned to ordinary registers.  A kernel that runs one wave
// per SIMD owns 512 registers, 256 of them accumulation registers (AGPRs) that only MFMAs and
// v_accvgpr moves can touch; the compiler then gives every MFMA an AGPR result, also the score
// tiles the vector ALU reads next (one v_accvgpr_read per element).  These forms keep such tiles in
// VGPRs while the builtin form keeps the long-lived output accumulators in AGPRs.
// The compiler does not know what the statements are, so it places none of the wait states an MFMA
// result needs before another kind of instruction may read or overwrite it (11 after an 8-pass
// MFMA).  Inside a chain the next link is the next such statement; the last link of a chain is
// issued with the _last form, which carries the wait states itself, so that whatever the compiler
// puts behind it (a copy, a spill, a reuse of the registers of a result nobody reads) is safe.
FB_DEV void mfma32_vdst_first(f32x16& d, bf16x8 a, bf16x8 b) {    // d = a . b
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(d) : "v"(a), "v"(b));
}
FB_DEV void mfma32_vdst(f32x16& d, bf16x8 a, bf16x8 b) {          // d += a . b
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d) : "v"(a), "v"(b));
}
FB_DEV void mfma32_vdst_last(f32x16& d, bf16x8 a, bf16x8 b) {     // d += a . b, then the result's wait states
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0\n\ts_nop 7\n\ts_nop 2" : "+v"(d) : "v"(a), "v"(b));
}

FB_DEV bf16x8 as_bf16x8(u32x4 u) { return __builtin_bit_cast(bf16x8, u); }
FB_DEV u32x4 as_uint4(bf16x8 v) { return __builtin_bit_cast(u32x4, v); }

// Exchange across the two 32-lane halves (v_permlane32_swap): given registers (a, b) the
// instruction returns ({a.lo, b.lo}, {a.hi, b.hi}) where .lo/.hi are the values held by lanes
// 0..31 / 32..63.  Feeding the same value twice yields both halves' values in every lane.
// The second operand goes through an empty asm so the compiler cannot see that the two
// inputs are equal (it would otherwise treat the two results as equal as well).
struct HalfPair { float lo, hi; };
FB_DEV HalfPair half_pair(float x) {
    const unsigned u = __builtin_bit_cast(unsigned, x);
    unsigned w = u;
    asm volatile("" : "+v"(w));
    auto r = __builtin_amdgcn_permlane32_swap(u, w, false, false);
    HalfPair p;
    p.lo = __builtin_bit_cast(float, (unsigned)r[0]);
    p.hi = __builtin_bit_cast(float, (unsigned)r[1]);
    return p;
}
FB_DEV float half_max(float x) { const HalfPair p = half_pair(x); return fmaxf(p.lo, p.hi); }
FB_DEV float half_sum(float x) { const HalfPair p = half_pair(x); return p.lo + p.hi; }

// ---- LDS transpose read (ds_read_b64_tr_b16) ----------------------------------------------
// Within each group of 16 lanes, lane i passes the address of four consecutive 16-bit
// elements; read as a 4 x 16 matrix M[e][j] whose row e, columns 4*(i%4)..4*(i%4)+3 come
// from lane i = 4*e + j/4, lane j receives column j: {M[0][j], M[1][j], M[2][j], M[3][j]}.
// With a row-major [row][col] tile and lane i pointing at &tile[r0 + i/4][c0 + 4*(i%4)],
// lane j therefore receives tile[r0..r0+3][c0 + j]: four rows of one column.
FB_DEV s16x4 lds_read_tr16(const bf16_t* p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) s16x4*)(p));
}
FB_DEV bf16x8 join_tr(s16x4 lo, s16x4 hi) {
    s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

FB_DEV float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// acc + a.x + a.y for a packed bf16 pair (v_dot2c_f32_bf16 against {1, 1}): the softmax row sum
// taken over the bf16-rounded probabilities, i.e. over exactly the values the second MFMA
// multiplies with V, at one instruction per two elements.
FB_DEV float pair_sum(bf16x2 a, float acc) {
    const bf16x2 ones = {(bf16_t)1.0f, (bf16_t)1.0f};
    return __builtin_amdgcn_fdot2_f32_bf16(a, ones, acc, false);
}

// Maximum of the 16 accumulator registers as a shallow tree (three-input maxima, depth 3)
// rather than a 15-deep dependent chain.
FB_DEV float max3f(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }
FB_DEV float max16(const f32x16& s) {
    const float a = max3f(s[0], s[1], s[2]), b = max3f(s[3], s[4], s[5]), c = max3f(s[6], s[7], s[8]);
    const float d = max3f(s[9], s[10], s[11]), e = max3f(s[12], s[13], s[14]);
    return max3f(max3f(a, b, c), max3f(d, e, s[15]), a);
}

// ---- bf16 limbs of an fp32 value ----------------------------------------------------------
// x = x1 + x2 + x3 (+ ~2^-24 |x|) with each limb a bf16 value.  For a product a*b the six
// column pairs (a1,b1) (a1,b2) (a2,b1) (a1,b3) (a2,b2) (a3,b1) recover it to ~2^-24.
FB_DEV bf16_t bf16_limb(float x, int n) {
    bf16_t l = (bf16_t)x;
    if (n == 0) return l;
    x -= (float)l;
    l = (bf16_t)x;
    if (n == 1) return l;
    x -= (float)l;
    return (bf16_t)x;
}
// limb index used in product column `slot` (0..5) on the query side and on the key side
FB_DEV int q_limb_of_slot(int slot) { return (0x210100 >> (4 * slot)) & 0xF; }  // 0,0,1,0,1,2
FB_DEV int k_limb_of_slot(int slot) { return (0x012010 >> (4 * slot)) & 0xF; }  // 0,1,0,2,1,0

// Key-side product columns of one fp32 factor value: [b1, b2, b1, b3, b2, b1] (12 bytes at a
// 4-byte aligned LDS address).
FB_DEV void phi_item_store_k(bf16_t* dst, float x) {
    const bf16_t l1 = (bf16_t)x;
    const float r1 = x - (float)l1;
    const bf16_t l2 = (bf16_t)r1;
    const bf16_t l3 = (bf16_t)(r1 - (float)l2);
    bf16x2 a = {l1, l2}, b = {l1, l3}, c = {l2, l1};
    unsigned* d = (unsigned*)dst;
    d[0] = __builtin_bit_cast(unsigned, a);
    d[1] = __builtin_bit_cast(unsigned, b);
    d[2] = __builtin_bit_cast(unsigned, c);
}

// Eight consecutive columns [8*c8, 8*c8+8) of a factor row widened to the padded layout.
//   bf16 factors: column j holds phi[j] for j < R, else 0.
//   fp32 factors: column j holds limb (slot j % 6) of phi[j / 6] for j / 6 < R, else 0.
// `mul` scales an fp32 factor before it is split.
template <bool QSIDE>
FB_DEV bf16x8 phi_chunk_gather(const void* row, int c8, int R, bool f32, float mul = 1.f) {
    bf16x8 out;
#pragma unroll
    for (int e = 0; e < 8; e++) {
        const int j = c8 * 8 + e;
        bf16_t val = (bf16_t)0.f;
        if (!f32) {
            if (j < R) val = ((const bf16_t*)row)[j];
        } else {
            const int r = j / 6, slot = j - 6 * r;
            if (r < R) {
                const float x = ((const float*)row)[r] * mul;
                val = bf16_limb(x, QSIDE ? q_limb_of_slot(slot) : k_limb_of_slot(slot));
            }
        }
        out[e] = val;
    }
    return out;
}

// Two-step variant for the key side, so the global loads of the next tile can stay in
// flight during compute: phi_chunk_raw issues the loads, phi_chunk_finish converts.
FB_DEV u32x4 phi_chunk_raw(const void* row, int c8, int R, bool f32, bool row_valid) {
    u32x4 raw = u32x4{0u, 0u, 0u, 0u};
    if (!row_valid) return raw;
    if (!f32) {
        if ((R & 7) == 0) {
            if (c8 * 8 < R) raw = *(const u32x4*)((const bf16_t*)row + c8 * 8);
        } else {
            raw = as_uint4(phi_chunk_gather<false>(row, c8, R, false));
        }
    } else {
        const int r0 = (c8 * 8) / 6;
        const float* f = (const float*)row;
        if (r0 < R) raw.x = __builtin_bit_cast(unsigned, f[r0]);
        if (r0 + 1 < R) raw.y = __builtin_bit_cast(unsigned, f[r0 + 1]);
        if (r0 + 2 < R) raw.z = __builtin_bit_cast(unsigned, f[r0 + 2]);
    }
    return raw;
}
template <bool QSIDE = false>
FB_DEV bf16x8 phi_chunk_finish(u32x4 raw, int c8, bool f32) {
    if (!f32) return as_bf16x8(raw);
    bf16x8 out;
    const int r0 = (c8 * 8) / 6;
#pragma unroll
    for (int e = 0; e < 8; e++) {
        const int j = c8 * 8 + e;
        const int r = j / 6, slot = j - 6 * r;
        const int d = r - r0;
        const unsigned u = d == 0 ? raw.x : (d == 1 ? raw.y : raw.z);
        out[e] = bf16_limb(__builtin_bit_cast(float, u),
                           QSIDE ? q_limb_of_slot(slot) : k_limb_of_slot(slot));
    }
    return out;
}

// Query-side columns [8*c8, 8*c8+8) of the padded limb layout for two fp32 factor values
// (x0, x1) computed in the kernel instead of read from memory: column j holds limb
// (slot j % 6) of x_{j / 6} for j < 12, else 0.
FB_DEV bf16x8 phi_chunk_from_pair(int c8, float x0, float x1) {
    bf16x8 out;
#pragma unroll
    for (int e = 0; e < 8; e++) {
        const int j = c8 * 8 + e;
        const int r = j / 6, slot = j - 6 * r;
        out[e] = r < 2 ? bf16_limb(r == 0 ? x0 : x1, q_limb_of_slot(slot)) : (bf16_t)0.f;
    }
    return out;
}

// phi_chunk_gather with the chunk index known at compile time: the rank and limb slot of each
// of the eight columns are constants, so an fp32 chunk costs at most three loads and three
// limb splits instead of eight of each.
template <bool QSIDE, int C8>
FB_DEV bf16x8 phi_chunk_static(const void* row, int R, bool f32, float mul = 1.f) {
    bf16x8 out;
    if (!f32) {
#pragma unroll
        for (int e = 0; e < 8; e++) out[e] = (C8 * 8 + e < R) ? ((const bf16_t*)row)[C8 * 8 + e] : (bf16_t)0.f;
        return out;
    }
    constexpr int r0 = (C8 * 8) / 6;
    bf16_t limb[3][3];
#pragma unroll
    for (int d = 0; d < 3; d++) {
        const float x = (r0 + d < R && r0 + d <= (C8 * 8 + 7) / 6) ? ((const float*)row)[r0 + d] * mul : 0.f;
        const bf16_t l1 = (bf16_t)x;
        const float e1 = x - (float)l1;
        const bf16_t l2 = (bf16_t)e1;
        limb[d][0] = l1;
        limb[d][1] = l2;
        limb[d][2] = (bf16_t)(e1 - (float)l2);
    }
#pragma unroll
    for (int e = 0; e < 8; e++) {
        constexpr int dummy = 0; (void)dummy;
        const int j = C8 * 8 + e;
        const int r = j / 6, slot = j - 6 * r;
        out[e] = limb[r - r0][QSIDE ? q_limb_of_slot(slot) : k_limb_of_slot(slot)];
    }
    return out;
}
template <bool QSIDE>
FB_DEV bf16x8 phi_chunk_switch(const void* row, int c8, int R, bool f32, float mul = 1.f) {   // mul: fp32 factors only
    if (!f32) return phi_chunk_gather<QSIDE>(row, c8, R, false);   // any chunk index (rows wider than 64 columns)
    switch (c8) {
        case 0: return phi_chunk_static<QSIDE, 0>(row, R, f32, mul);
        case 1: return phi_chunk_static<QSIDE, 1>(row, R, f32, mul);
        case 2: return phi_chunk_static<QSIDE, 2>(row, R, f32, mul);
        case 3: return phi_chunk_static<QSIDE, 3>(row, R, f32, mul);
        case 4: return phi_chunk_static<QSIDE, 4>(row, R, f32, mul);
        case 5: return phi_chunk_static<QSIDE, 5>(row, R, f32, mul);
        case 6: return phi_chunk_static<QSIDE, 6>(row, R, f32, mul);
        default: return phi_chunk_static<QSIDE, 7>(row, R, f32, mul);
    }
}

#endif
