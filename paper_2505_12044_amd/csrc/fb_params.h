// Host/device-shared parameter blocks for the attention kernels (plain data only).
#ifndef FB_PARAMS_H_
#define FB_PARAMS_H_

#include <stddef.h>
#include <stdint.h>

struct FwdParams {
    const void* q;        // [B,H,N,C]
    const void* k;
    const void* v;
    const void* phi_q;    // [Bp,H,N,R] or null
    const void* phi_k;
    const float* slopes;  // [H] per-head ALiBi slopes (in-kernel factor generation only)
    const void* bias;     // [Bb,H,N,N] or null (dense-bias mode)
    void* out;            // [B,H,N,C]
    float* lse;           // [B,H,N]
    int B, H, N, R;       // N = number of queries
    int M;                // number of keys (= N except for cross-attention, four-wave bf16 kernel only)
    int causal;
    int phi_f32;          // factors stored as float (else bf16)
    long long phi_bstride;   // elements between batch items of phi_q (0 when shared over batch)
    long long phik_bstride;  // ... of phi_k
    long long bias_bstride;  // elements between batch items of bias (0 when shared)
    float scale;
    float inv_scale;      // 1 / scale, formed on the host (the backward forms the same value there)
    int causal_up;        // causal pairs: the first tile walks its off-diagonal blocks upwards from key 0
    int n_qtiles;         // query tiles per (b,h)
    int n_units;          // work units (workgroups) per (b,h): tiles, or tile pairs when causal
    int total_tiles;      // B*H*n_units
    int tiles_per_xcd;    // ceil(total_tiles / 8)
};

struct BwdParams {
    const void* q; const void* k; const void* v;
    const void* phi_q; const void* phi_k;
    const void* out; const float* lse; const void* dout;
    void* dq; void* dk; void* dv; void* dphi_q; void* dphi_k;
    const float* slopes;  // [H] ALiBi slopes: factors phi_q(i) = [-m i, m], phi_k(j) = [1, j] are generated in the
                          // pre-pass instead of read (phi_q, phi_k, dphi_q, dphi_k NULL, R = 2, phi_f32 = 1); else NULL
    float* dslope;        // [B,H,N] or NULL (with slopes only): per-row gradient of the head's slope, sum_j dS_ij (j - i)
    const void* bias;     // [Bb,H,N,M] dense-bias backward only
    void* dbias;          // [B,H,N,M]
    long long bias_bstride;  // elements between batch items of bias (0 when shared)
    void* workspace;      // device scratch: (lse2, D) rows and the concatenated operand rows
    int B, H, N, R;       // N = number of queries
    int M;                // number of keys (= N except for cross-attention)
    int Cg;               // channels per head in caller memory (16 runs on the C = 32 kernels), else C
    int causal;
    int phi_f32;
    int grad_f32;         // dq, dk, dphi_q, dphi_k are written as float (multiplicative bias: the fold kernel
                          // sums them, so they must not be rounded to bf16 first); dv stays bf16
    long long phi_bstride;   // elements between batch items of phi_q (0 when shared over batch)
    long long phik_bstride;  // ... of phi_k
    float scale;
    int n_tiles;          // tiles per (b,h) along the kernel's outer dimension
    int total_tiles;
    int tiles_per_xcd;
};

#endif
