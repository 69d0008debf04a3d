/*
 * pop_ops.h -- single steps of the POP prefill path, exported so that each kernel can be checked
 * against the same step of a reference implementation and timed on its own.  Same conventions as
 * pop.h: DEVICE pointers are caller-owned, 16-byte aligned; work is enqueued on `stream`.
 */
#ifndef POP_OPS_H_
#define POP_OPS_H_

#include "pop.h"

#ifdef __cplusplus
extern "C" {
#endif

/* LN(.) of Sec. 2.1 as RMSNorm: out[r,:] = bf16(x[r,:] * rsqrt(mean(x[r,:]^2) + eps) * gamma).
 * x DEVICE fp32 [rows, d], gamma DEVICE fp32 [d], out DEVICE bf16 [rows, d]; d % 8 == 0, d <= 8192. */
pop_status pop_op_rmsnorm(const float* x, const float* gamma, void* out, int32_t rows, int32_t d, float eps,
                          pop_stream stream);

/* Projection of Sec. 2.1 (Attn / FFN blocks): C = A[M,K] * W[N,K]^T, bf16 inputs, fp32 accumulation.
 *   epilogue 0: out bf16 [M, ldc] = C          1: out fp32 [M, ldc] += C (residual update)
 *            2: W is [2N, K] (gate rows, then up rows); out bf16 [M, ldc] = act(gate) * up
 *            3: out fp32 [M, ldc] = C
 * Requirements: K, lda, ldw multiples of 8; ldc multiple of 4; operands below 2 GiB each.
 * Errors: POP_EINVAL / POP_EALIGN / POP_ESHAPE on a violated requirement, POP_EHIP. */
pop_status pop_op_gemm(const void* A, int64_t lda, const void* W, int64_t ldw, void* out, int64_t ldc,
                       int32_t M, int32_t N, int32_t K, int32_t epilogue, int32_t act, pop_stream stream);

/* The same projection (Sec. 2.1, Attn / FFN blocks; the short prompts of Sec. 4.3, where a projection is
 * weight streaming) with scratch memory that allows a deterministic split of K (few rows, long K: the
 * projections of short prompts are weight streaming, and more work-groups stream faster).  The library
 * decides whether and how far to split; parts are added in a fixed order, so results do not depend on
 * timing.  epilogue 0, 1 or 3.  dev_scratch DEVICE, 16-byte aligned, scratch_bytes >= 32 M N allows the
 * deepest split (8 parts of fp32 [M, N]); less only limits it. */
pop_status pop_op_gemm_splitk(const void* A, int64_t lda, const void* W, int64_t ldw, void* out, int64_t ldc,
                              int32_t M, int32_t N, int32_t K, int32_t epilogue, void* dev_scratch,
                              size_t scratch_bytes, pop_stream stream);

/* pop_op_gemm_splitk for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the scratch is a fixed array of POP_STATIC_SCRATCH_BYTES
 * in the library's device image, one copy per GPU, held until the process ends.  Same kernels, same split,
 * same bits as pop_op_gemm_splitk with a scratch buffer of that size.  The call allocates nothing.
 * Limit: 32 M N <= POP_STATIC_SCRATCH_BYTES (M N <= 524288, e.g. 64 rows x 8192 columns); POP_ENOSPACE beyond,
 * before anything is enqueued.  All calls on one GPU share that GPU's array: calls that overlap in time on one
 * GPU (different streams, different threads) race and must be serialised by the caller.  The array keeps the
 * last call's partial products; every call overwrites what it reads, so nothing needs clearing.
 * Other errors as pop_op_gemm_splitk; POP_EHIP if the array's address cannot be obtained. */
#define POP_STATIC_SCRATCH_BYTES (16u << 20)
size_t pop_static_scratch_bytes(void);
pop_status pop_op_gemm_splitk_static(const void* A, int64_t lda, const void* W, int64_t ldw, void* out, int64_t ldc,
                                     int32_t M, int32_t N, int32_t K, int32_t epilogue, pop_stream stream);

/* Same contraction for M <= 64 rows with the bandwidth-bound kernel of the boundary token
 * (Sec. 3.3, "Boundary Handling"): epilogue 0: out fp32 = C, 1: out fp32 += C, 2: GLU -> bf16.
 * Operands are dense (lda = ldw = K). */
pop_status pop_op_gemv(const void* x, const void* W, void* out, int64_t ldo, int32_t M, int32_t N, int32_t K,
                       int32_t epilogue, int32_t act, pop_stream stream);

/* The normalisation of Sec. 2.1 (the LN of the layer equations; RMSNorm here) fused into the same kernel:
 * the rows of x are DEVICE fp32 [M, K], normalised as pop_op_rmsnorm does (same bits) and rounded to bf16
 * before the contraction.  gamma DEVICE fp32 [K].  M <= 4, K <= 8192 and 2 M K + 16 M <= 49152 (the
 * normalised rows are held in LDS); POP_ESHAPE otherwise. */
pop_status pop_op_gemv_norm(const void* x, const void* gamma, float eps, const void* W, void* out, int64_t ldo,
                            int32_t M, int32_t N, int32_t K, int32_t epilogue, int32_t act, pop_stream stream);

/* RoPE on q and k followed by causal GQA attention (Sec. 2.1: K/V generation and Attn) over packed
 * sequences.  qkv DEVICE bf16 [T, (Hq + 2 Hkv) * hd], rows q | k | v, q and k are rotated IN PLACE;
 * out DEVICE bf16 [T, Hq * hd].  host_cu_seqlens HOST [n_seqs + 1].  window 0 = global.
 * workspace: at least pop_op_rope_attention_workspace(...) bytes. */
size_t pop_op_rope_attention_workspace(int32_t T, int32_t n_seqs, int32_t n_kv_heads, int32_t head_dim);
pop_status pop_op_rope_attention(void* qkv, const int32_t* host_cu_seqlens, int32_t n_seqs, int32_t n_q_heads,
                                 int32_t n_kv_heads, int32_t head_dim, float rope_theta, int32_t window,
                                 void* out, void* workspace, size_t workspace_bytes, pop_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* POP_OPS_H_ */
