/*
 * flashbias.h — C-ABI of the MI355X (gfx950) low-rank-bias attention library.
 *
 * The operation is exact softmax attention with an additive bias (FlashBias,
 * arxiv 2505.12044, Sec. 2.1, Eq. 1):
 *
 *     o = softmax(q k^T * scale + b [+ causal mask]) v,     scale = 1/sqrt(C) by default,
 *
 * where the bias is supplied as low-rank factors b = phi_q phi_k^T (Sec. 3.2, Eq. 2) and
 * is folded into the score contraction as [q*scale | phi_q] [k | phi_k]^T (Eq. 3), so the
 * N x N bias never exists in device memory.  fb_dense_bias_attn_fwd is the baseline the
 * paper compares against (fused attention that streams a materialised bias tile by tile,
 * Example 3.9).
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller: contiguous, row-major,
 *     16-byte aligned.  The library never allocates, frees or keeps them.
 *   - Layouts: q, k, v, out, dout, dq, dk, dv: [B, H, N, C];  lse: [B, H, N] float;
 *     phi_q, phi_k: [Bp, H, N, R] with Bp = 1 when phi_batch_broadcast != 0, else Bp = B;
 *     bias: [Bb, H, N, N] with Bb = 1 when bias_batch_broadcast != 0, else Bb = B.
 *   - Queries and keys have the same length N (self-attention); with causal != 0 key j is
 *     visible to query i iff j <= i (0-based).  N may be any positive value (ragged tails
 *     are handled inside the kernels).
 *   - dtype is the storage type of q, k, v, out (and dout, dq, dk, dv, bias); phi_dtype is
 *     the storage type of phi_q, phi_k (and dphi_q, dphi_k).  With dtype = FB_BF16 all
 *     contractions run as bf16 MFMA with fp32 accumulation; fp32 factors are then split
 *     into three bf16 limbs inside the kernel (six product columns per rank), which keeps
 *     ~24 bits of each factor (needed e.g. for ALiBi positions up to N).  With
 *     dtype = FB_F32 everything is fp32 FMA and phi_dtype must be FB_F32.
 *   - Supported: C in {16, 32, 64, 128}; 0 <= R, with the
 *     padded factor width (R for bf16 factors, 6R for fp32 factors in a bf16 run, rounded up
 *     to 16) at most 64; fp32 forward: R <= 64.  R = 0 (phi pointers may be NULL) is plain
 *     attention.  C = 16 (the PDE-solver head dimension of Sec. 4.3) runs on the 32-channel
 *     bf16 tiles with the missing channels zero-filled inside the kernels.
 *   - scale <= 0 selects 1/sqrt(C).
 *   - stream is a hipStream_t passed as void*; NULL is the default stream.  Calls only
 *     enqueue work: they never synchronise and never block on the device.
 *   - Return value: FB_OK or an fb_status for errors detectable on the host (bad argument,
 *     unsupported shape, misalignment, workspace too small, launch failure).  Outputs are
 *     fully overwritten on success and untouched on error.  Thread-safe; the only process-wide
 *     state is the atomic variant selection of fb_tune_set (a test hook) and the static scratch
 *     of fb_lowrank_attn_bwd_noalloc.
 *   - Size limits (FB_ERR_SHAPE beyond them): B H N < 2^31 rows; N C < 2^30 and N R < 2^30
 *     elements inside one head.  Offsets above the head level are 64-bit, so tensors may exceed
 *     2^31 elements.
 */
#ifndef FLASHBIAS_H_
#define FLASHBIAS_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FB_OK = 0,
    FB_ERR_NULL = 1,         /* a required pointer is NULL                          */
    FB_ERR_SHAPE = 2,        /* B, H, N <= 0, R < 0, or sizes overflow the indexing */
    FB_ERR_UNSUPPORTED = 3,  /* C / R / dtype combination has no kernel             */
    FB_ERR_ALIGN = 4,        /* a pointer is not 16-byte aligned                    */
    FB_ERR_WORKSPACE = 5,    /* workspace NULL or smaller than the size query says  */
    FB_ERR_LAUNCH = 6,       /* the HIP runtime rejected a launch                   */
    FB_ERR_TOO_LARGE = 7     /* problem needs more scratch than the allocation-free entry point owns */
} fb_status;

typedef enum { FB_F32 = 0, FB_BF16 = 1 } fb_dtype;

/* Library version: major * 10000 + minor * 100 + patch. */
int fb_version(void);

/* Static, NUL-terminated description of a status code. */
const char* fb_status_string(int status);

/*
 * Test hook: selects among kernel variants that compute the same result (the parity tests
 * run every variant; benchmarks compare them).  Results never depend on it beyond rounding
 * order.  The state is process-wide and atomic: each entry point reads a knob once, on the
 * host, when it is called, so a call enqueued (or captured into a graph) keeps the variant it
 * was issued with.  Returns FB_OK, FB_ERR_NULL, FB_ERR_SHAPE (value out of range) or
 * FB_ERR_UNSUPPORTED (unknown name).
 *   "fwd_qb"      bf16 forward kernel variant; 0 restores the automatic choice.
 *                 1, 2 = four-wave kernel with that many 32-row query blocks per wave
 *                 8    = eight-wave ping-pong kernel
 *                 16   = direct-to-LDS kernel (falls back to 1 for shapes it does not take)
 *   "fwd_causal_up" 1 (default): of the two query tiles a workgroup of the causal four-wave
 *                 kernel takes, the first walks its off-diagonal key blocks upwards from key 0
 *                 and the second downwards, so the workgroups of a head read the same block at
 *                 the same time (fewer L2 misses); 0: both walk downwards from the diagonal.
 */
int fb_tune_set(const char* name, int value);

/*
 * Forward with factorised bias (Eq. 3; tiled evaluation as in the proof of Corollary 3.7).
 *   out [B,H,N,C] dtype, lse [B,H,N] float: natural-log log-sum-exp of each score row
 *   (scaled, biased, masked), which the backward consumes.
 */
int fb_lowrank_attn_fwd(const void* q, const void* k, const void* v,
                        const void* phi_q, const void* phi_k,
                        void* out, float* lse,
                        int B, int H, int N, int C, int R, int causal,
                        fb_dtype dtype, fb_dtype phi_dtype, int phi_batch_broadcast,
                        float scale, void* stream);

/*
 * Cross-attention form of fb_lowrank_attn_fwd (Eq. 1 with N queries and M keys): q, out
 * [B,H,N,C], k, v [B,H,M,C], phi_q [Bp,H,N,R], phi_k [Bp,H,M,R], lse [B,H,N].  No causal mask
 * (its alignment is undefined for N != M).  dtype FB_BF16 or FB_F32 (fp32 factors), as for
 * fb_lowrank_attn_fwd.
 */
int fb_lowrank_xattn_fwd(const void* q, const void* k, const void* v,
                         const void* phi_q, const void* phi_k, void* out, float* lse,
                         int B, int H, int N, int M, int C, int R,
                         fb_dtype dtype, fb_dtype phi_dtype, int phi_batch_broadcast,
                         float scale, void* stream);

/*
 * Forward with the ALiBi bias b_ij = -m_h (i - j) (0-based positions, every (i, j); the
 * causal mask is separate) generated inside the kernel from the per-head slopes: the rank-2
 * factors of Example 3.4 are computed from tile indices, so no factor tensor is read
 * (App. D, "decomposition in JIT").  Positions are measured from the tile's first query row
 * and carried as fp32 (three bf16 limbs), so the bias is exact to fp32 rounding at any N.
 *   slopes [H] float, device memory, 4-byte aligned.  Needs dtype = FB_BF16 and N <= 2^24.
 * Same result as fb_lowrank_attn_fwd with phi_q(i) = [-m_h i, m_h], phi_k(j) = [1, j] in fp32.
 */
int fb_alibi_attn_fwd(const void* q, const void* k, const void* v, const float* slopes,
                      void* out, float* lse, int B, int H, int N, int C, int causal,
                      fb_dtype dtype, float scale, void* stream);

/*
 * Forward with a dense bias streamed from device memory (the baseline of Example 3.9:
 * HBM traffic Theta(N M C^2 / S + N M)).  bias has the storage type `dtype`.
 */
int fb_dense_bias_attn_fwd(const void* q, const void* k, const void* v, const void* bias,
                           void* out, float* lse,
                           int B, int H, int N, int C, int causal,
                           fb_dtype dtype, int bias_batch_broadcast,
                           float scale, void* stream);

/*
 * Forward with a MULTIPLICATIVE low-rank bias (App. I):
 *   out = softmax((q k^T * scale) o (phi_q phi_k^T)) v,   o = element-wise product,
 * evaluated as plain attention over the reweighted repeats q' = [q o phi_q,1 | ... | q o phi_q,R],
 * k' = [k o phi_k,1 | ... | k o phi_k,R] (C R channels, scale of the original C), so the N x N
 * bias is never formed.  A pre-pass writes q' * scale and k' (bf16) into the workspace; the
 * additive-bias forward kernels then run with the first C channels as q / k and the other
 * C (R - 1) as extra columns of the same contraction.
 *   phi_q, phi_k [Bp,H,N,R], R >= 1, 4-byte aligned; needs dtype = FB_BF16 and C (R - 1) <= 128
 *   for C <= 64 (C = 64: R <= 3; C = 32: R <= 5; C = 16: R <= 9); C = 128 takes R = 1 only (its
 *   score operand already fills the registers two waves per SIMD leave).  Corollary I.2 puts
 *   the useful range at small R in any case.
 *   workspace: device scratch of at least fb_lowrank_mulbias_attn_fwd_workspace_bytes(...)
 *   = 4 B H N C R bytes, 16-byte aligned, owned by the caller, contents ignored on entry,
 *   reusable once the call's work on `stream` has finished.
 * lse is the log-sum-exp of the scaled, bias-multiplied, masked score row.
 */
size_t fb_lowrank_mulbias_attn_fwd_workspace_bytes(int B, int H, int N, int C, int R, fb_dtype dtype);

int fb_lowrank_mulbias_attn_fwd(const void* q, const void* k, const void* v,
                                const void* phi_q, const void* phi_k, void* out, float* lse,
                                int B, int H, int N, int C, int R, int causal,
                                fb_dtype dtype, fb_dtype phi_dtype, int phi_batch_broadcast,
                                float scale, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Backward of fb_alibi_attn_fwd: dq, dk, dv [B,H,N,C] for an upstream gradient dout, with the
 * ALiBi factors generated in the pre-pass from the slopes and the absolute positions (App. D:
 * the paper's in-kernel variant is timed for training as well as inference).  Positions are exact
 * fp32 integers: N <= 2^24.  Needs dtype = FB_BF16; workspace as for fb_lowrank_attn_bwd with R = 2.
 *   dslope_rows [B,H,N] float, 4-byte aligned, or NULL (slopes that are constants of the model):
 *   row i receives sum_j dS_ij (j - i), the contribution of query i to dL/dm_h for the bias
 *   -m_h (i - j) (Example 3.4); a caller that trains the slopes sums it over i and the batch.  It is
 *   formed from the two factor-gradient columns inside the kernel, where the part of them that
 *   grows with the position cancels exactly, so it stays accurate at any N (the raw factor
 *   gradients of absolute positions do not: see fb_lowrank_attn_bwd with such factors).
 */
size_t fb_alibi_attn_bwd_workspace_bytes(int B, int H, int N, int C, fb_dtype dtype);

int fb_alibi_attn_bwd(const void* q, const void* k, const void* v, const float* slopes,
                      const void* out, const float* lse, const void* dout,
                      void* dq, void* dk, void* dv, float* dslope_rows,
                      int B, int H, int N, int C, int causal, fb_dtype dtype, float scale,
                      void* workspace, size_t workspace_bytes, void* stream);

/*
 * Backward of fb_lowrank_mulbias_attn_fwd (chain rule on App. I's reformulation; the appendix
 * itself stops at the forward): dq, dk, dv [B,H,N,C] dtype and dphi_q, dphi_k [B,H,N,R]
 * phi_dtype, always per batch element.  The pre-pass of the forward is repeated, the
 * additive-bias backward kernels give the gradients of the reweighted repeats q', k', and a
 * fold kernel applies dq = scale sum_r phi_q,r dq'_r, dphi_q,r = scale sum_c q_c dq'_r,c (and
 * the same without the scale on the key side).  Same limits as the forward.
 *   workspace: fb_lowrank_mulbias_attn_bwd_workspace_bytes(...) bytes (the repeats in bf16, their
 *   gradients in fp32 — dq and dphi are sums over them and are rounded once, at the end — and
 *   the additive backward's scratch), 16-byte aligned, caller-owned.
 */
size_t fb_lowrank_mulbias_attn_bwd_workspace_bytes(int B, int H, int N, int C, int R, fb_dtype dtype);

int fb_lowrank_mulbias_attn_bwd(const void* q, const void* k, const void* v,
                                const void* phi_q, const void* phi_k,
                                const void* out, const float* lse, const void* dout,
                                void* dq, void* dk, void* dv, void* dphi_q, void* dphi_k,
                                int B, int H, int N, int C, int R, int causal,
                                fb_dtype dtype, fb_dtype phi_dtype, int phi_batch_broadcast,
                                float scale, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Backward of fb_lowrank_attn_fwd for an upstream gradient dout (loss L = sum(dout * out)):
 * dq, dk, dv [B,H,N,C] dtype; dphi_q, dphi_k [B,H,N,R] phi_dtype, always per batch element
 * (a caller whose factors are shared over the batch sums them over B); either may be NULL when
 * that gradient is not wanted (fixed biases).  The factor
 * gradients are the trailing R columns of the same contractions that give dq and dk
 * (Sec. 3.2 "Speed up training"; Sec. 4.1 "Implementation choices").
 * `out` and `lse` are the forward's results.  dtype = FB_BF16, or FB_F32 (all tensors and the
 * factors float, N keys = N queries: the full-precision path, fp32 FMA arithmetic, which uses only
 * the first 4 B H N bytes of the workspace, for D).
 * workspace: device scratch of at least fb_lowrank_attn_bwd_workspace_bytes(...) bytes,
 * 16-byte aligned, owned by the caller; its contents on entry are ignored and it may be
 * reused as soon as the call's work on `stream` has finished.  It receives, per (b, h, i):
 * (lse * log2 e, D_i = sum_c dout * out) and the concatenated bf16 operand rows
 * [q*scale | phi_q | 0] and [k | phi_k | 0] that the two main kernels stream
 * (8 + 4 * (C + 64) bytes per row when R > 0, 8 + 4 * C otherwise; C = 16 counts as 32 and
 * adds 32-channel copies of v and dout, 128 more bytes per row).
 * Results are deterministic (no floating-point atomics).
 */
size_t fb_lowrank_attn_bwd_workspace_bytes(int B, int H, int N, int C, int R, fb_dtype dtype);

int fb_lowrank_attn_bwd(const void* q, const void* k, const void* v,
                        const void* phi_q, const void* phi_k,
                        const void* out, const float* lse, const void* dout,
                        void* dq, void* dk, void* dv, void* dphi_q, void* dphi_k,
                        int B, int H, int N, int C, int R, int causal,
                        fb_dtype dtype, fb_dtype phi_dtype, int phi_batch_broadcast,
                        float scale, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Allocation-free variant of fb_lowrank_attn_bwd, for callers that cannot allocate device
 * memory or carry a workspace: code under HIP graph capture, tight serving / training loops,
 * harnesses that forbid hipMalloc.  Same arguments without the workspace, same kernels, same
 * (bit-identical) results; the scratch that fb_lowrank_attn_bwd takes from the caller lives in
 * a static device array of FB_STATIC_SCRATCH_BYTES inside the library, one copy per GPU, held
 * from library load until the process ends.  The call allocates and frees nothing.
 *   Limit: fb_lowrank_attn_bwd_workspace_bytes(B, H, N, C, R, dtype) <= FB_STATIC_SCRATCH_BYTES
 *   (e.g. B H N <= 86480 rows at C = 128 with factors); larger problems return
 *   FB_ERR_TOO_LARGE and launch nothing.
 *   Every call on a GPU uses that GPU's one array: calls that overlap on the same GPU (two
 *   streams, two threads) race on it and must be serialised by the caller.  Nothing in the
 *   array has to start at zero (the pre-pass rewrites every byte the main kernels read), so
 *   calls of different sizes may follow each other freely.
 */
#define FB_STATIC_SCRATCH_BYTES ((size_t)64 << 20)

int fb_lowrank_attn_bwd_noalloc(const void* q, const void* k, const void* v,
                                const void* phi_q, const void* phi_k,
                                const void* out, const float* lse, const void* dout,
                                void* dq, void* dk, void* dv, void* dphi_q, void* dphi_k,
                                int B, int H, int N, int C, int R, int causal,
                                fb_dtype dtype, fb_dtype phi_dtype, int phi_batch_broadcast,
                                float scale, void* stream);

/*
 * Backward of fb_dense_bias_attn_fwd, the training-side baseline: besides dq, dk, dv it has
 * to write the dense gradient dbias [B,H,N,N] (= dL/dS, storage type `dtype`, always per batch
 * element), the N x N object that the factorised form never materialises (Sec. 4.3).  Entries
 * above the diagonal are zero when causal.
 * dtype FB_BF16 (needs N % 8 == 0) or FB_F32 (the fp32 FMA path).  Workspace as for
 * fb_lowrank_attn_bwd with R = 0.
 */
size_t fb_dense_bias_attn_bwd_workspace_bytes(int B, int H, int N, int C, fb_dtype dtype);

int fb_dense_bias_attn_bwd(const void* q, const void* k, const void* v, const void* bias,
                           const void* out, const float* lse, const void* dout,
                           void* dq, void* dk, void* dv, void* dbias,
                           int B, int H, int N, int C, int causal,
                           fb_dtype dtype, int bias_batch_broadcast, float scale,
                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * Cross-attention form of fb_lowrank_attn_bwd: q, out, dout, dq [B,H,N,C]; k, v, dk, dv
 * [B,H,M,C]; phi_q, dphi_q [.,H,N,R]; phi_k, dphi_k [.,H,M,R]; lse [B,H,N].  No causal mask.
 * dtype FB_BF16 or FB_F32.  Workspace as for fb_lowrank_attn_bwd, sized by the query below.
 */
size_t fb_lowrank_xattn_bwd_workspace_bytes(int B, int H, int N, int M, int C, int R, fb_dtype dtype);

int fb_lowrank_xattn_bwd(const void* q, const void* k, const void* v,
                         const void* phi_q, const void* phi_k,
                         const void* out, const float* lse, const void* dout,
                         void* dq, void* dk, void* dv, void* dphi_q, void* dphi_k,
                         int B, int H, int N, int M, int C, int R,
                         fb_dtype dtype, fb_dtype phi_dtype, int phi_batch_broadcast,
                         float scale, void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FLASHBIAS_H_ */
