/*
 * stage2bw_kernels.h -- C ABI of the single kernels the 2BW stage is made of, for parity tests
 * and stand-alone roofline measurements.  Every pointer is a DEVICE pointer owned by the caller
 * unless its name ends in _host; `stream` is a hipStream_t (NULL = null stream).  Calls only
 * enqueue.  Return value: 0, or a negative STAGE_ERR_* code from stage2bw.h (INVALID_ARG when a
 * shape or alignment the kernel assumes does not hold; nothing is launched then).
 * Not thread-safe: first calls set up process-wide state without locks.
 *
 * dtype: 0 = fp32, 1 = bf16 (2-byte elements, fp32 accumulation and statistics).
 * All row strides and contiguous extents must be multiples of 8 elements; base pointers 16-byte
 * aligned.
 *
 * The operations are the steps of one transformer block's forward and reverse-mode gradient
 * (the stage of Section 3.1 is a stack of such blocks; Section 5 names the models):
 * projections with fused bias / residual / GELU, masked softmax attention, LayerNorm, the
 * in-place coalescing of weight gradients (Section 3.1) and the Adam form of the delayed
 * update W(t+1) = W(t) - nu * step(grad f(W(t-1))) (Section 3.1, Semantics).
 */
#ifndef STAGE2BW_KERNELS_H
#define STAGE2BW_KERNELS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * C[M,N] = epilogue(sum_k A(m,k) B(k,n)),  A(m,k) = trans_a ? A[k*lda+m] : A[m*lda+k],
 * B(k,n) = trans_b ? B[n*ldb+k] : B[k*ldb+n].
 * epilogue 0: C = acc (+ bias[n]) (+ aux[m,n])            (forward projection, residual)
 *          1: u = acc + bias[n]; C = u; aux_out = GELU(u)  (FC1)
 *          2: C = acc * GELU'(aux[m,n])                     (data gradient through GELU)
 *          3: C fp32: C = (accumulate ? C : 0) + acc        (weight gradient, coalesced in place)
 * bf16 supports the pairs the stage issues: (trans_a,trans_b,epilogue) in
 * {(0,0,0),(0,0,1),(0,0,2),(0,1,0),(0,1,2),(1,0,3)}; fp32 supports all.  bf16: A and B each smaller than
 * 2 GiB (rows * ld * 2 bytes), INVALID_ARG otherwise.
 */
int k2bw_gemm(int dtype, int trans_a, int trans_b, int epilogue, int M, int N, int K, const void* A,
              int lda, const void* B, int ldb, void* C, int ldc, const void* bias, const void* aux,
              void* aux_out, int accumulate, void* stream);

/* The coalesced weight gradient of n_seg microbatches in one product (bf16; Section 3.1's sum over the
 * microbatches of a batch, taken inside the reduction): C[M,N] (fp32) = (accumulate ? C : 0) +
 * sum over s < n_seg of X_s^T dY_s, X_s: [T, M] (ld = lda) at A0 + a_idx[s] * a_stride_bytes,
 * dY_s: [T, N] (ld = ldb) at B0 + b_idx[s] * b_stride_bytes.  n_seg 1..8, indices 0..15 (host arrays of
 * n_seg bytes), strides multiples of 256 bytes, T a multiple of 64; INVALID_ARG otherwise. */
int k2bw_gemm_wgrad_segmented(int M, int N, int T, int n_seg, const void* A0, int lda,
                              int64_t a_stride_bytes, const uint8_t* a_idx_host, const void* B0, int ldb,
                              int64_t b_stride_bytes, const uint8_t* b_idx_host, float* C, int ldc,
                              int accumulate, void* stream);

/* The FC2 data gradient with the GELU derivative and the FC1 bias gradient in one pass (bf16):
 * du[M,N] = (dy[M,K] w[N,K]^T) * GELU'(u[M,N]);  dbias[N] (fp32) = (accumulate ? dbias : 0) +
 * sum over rows of du, summed from the fp32 values before du is rounded to bf16.
 * workspace: k2bw_gemm_dgrad_gelu_bias_workspace(M, N) floats. */
int64_t k2bw_gemm_dgrad_gelu_bias_workspace(int M, int N);
int k2bw_gemm_dgrad_gelu_bias(int M, int N, int K, const void* dy, int lda, const void* w, int ldb,
                              void* du, int ldc, const void* u, float* dbias, int accumulate,
                              float* workspace, void* stream);

/* y = gain*(x-mean)*rstd + shift per row of length h (biased variance, eps under the root);
 * mean, rstd: fp32 [rows]. */
int k2bw_layernorm_fwd(int dtype, int rows, int h, float eps, const void* x, const void* gain,
                       const void* shift, void* y, float* mean, float* rstd, void* stream);

/* Floats of workspace k2bw_layernorm_bwd needs for row length h. */
int64_t k2bw_layernorm_bwd_workspace(int h);
/* dx = (dres ? dres : 0) + LN'(dy); dgain_dshift: fp32 [2h] = (sum_r dy*xhat | sum_r dy);
 * dx_colsum: fp32 [h] = sum_r dx (the bias gradient of the projection whose output gradient dx
 * is), may be NULL.  Both are overwritten or added to according to accumulate. */
int k2bw_layernorm_bwd(int dtype, int rows, int h, const void* dy, const void* x, const float* mean,
                       const float* rstd, const void* gain, const void* dres, void* dx,
                       float* dgain_dshift, float* dx_colsum, int accumulate, float* workspace,
                       void* stream);

/* Floats of workspace k2bw_bias_grad needs for n columns. */
int64_t k2bw_bias_grad_workspace(int n);
/* out[n] (fp32) = (accumulate ? out : 0) + sum over rows of y[rows, n]. */
int k2bw_bias_grad(int dtype, int rows, int n, const void* y, float* out, int accumulate,
                   float* workspace, void* stream);

/* k2bw_bias_grad for callers that cannot allocate device memory or carry a workspace (code under
 * HIP graph capture, serving loops, harnesses that forbid hipMalloc): same kernels, same result bit
 * for bit, with the partial rows in a device array that is part of the library image (64 x 32768
 * floats = 8 MiB on every GPU the library is loaded on, held until the process ends).  Calls no
 * hipMalloc / hipFree or other allocating routine.  n above k2bw_bias_grad_static_max_cols()
 * (32768): INVALID_ARG, nothing launched.  The first call on a device looks the array's address up
 * once (hipGetSymbolAddress; HIP error -> STAGE_ERR_HIP).  All calls on one GPU share the array:
 * calls on different streams of one GPU that may overlap race on it; calls on one stream are
 * ordered and need no clearing in between (every partial row read is rewritten by the same call). */
int k2bw_bias_grad_static_max_cols(void);
int k2bw_bias_grad_static(int dtype, int rows, int n, const void* y, float* out, int accumulate,
                          void* stream);

/* qkv: [b*s, 3h] with columns Q|K|V, each head-major, h = a*dh; o: [b*s, h]; lse: fp32 [b,a,s].
 * mask_mode 0 none, 1 causal (key j <= query i), 2 key padding (key j < seqlens[n]; a length
 * outside [1, s] is read as the nearest end of that range, so no row is empty and no key past the
 * sequence is touched). */
int k2bw_attention_fwd(int dtype, int b, int s, int a, int dh, int mask_mode, const int32_t* seqlens,
                       const void* qkv, void* o, float* lse, void* stream);
/* dqkv: [b*s, 3h]; delta: fp32 scratch [b,a,s].  dbias_qkv (bf16 with head size 32, 64, 80 or 128
 * only; may be NULL): fp32 [3h] = (accumulate ? dbias_qkv : 0) + column sums of dqkv, taken from
 * the fp32 values inside the kernels; workspace: k2bw_attention_bwd_workspace(b, s, a, dh) floats,
 * needed iff dbias_qkv is given. */
int64_t k2bw_attention_bwd_workspace(int b, int s, int a, int dh);
int k2bw_attention_bwd(int dtype, int b, int s, int a, int dh, int mask_mode, const int32_t* seqlens,
                       const void* qkv, const void* o, const float* lse, const void* d_o, void* dqkv,
                       float* delta, float* dbias_qkv, int accumulate, float* workspace, void* stream);

/* One Adam step over n parameters (n multiple of 4) from the coalesced sum G, g = G/m_micro:
 * moments updated in place; w_next = w_cur - lr*mhat/(sqrt(vhat)+eps) with bias correction for
 * step `step` (>= 1).  w_next may equal w_cur.  w_next_bf16 (may be NULL) also receives the new
 * weights rounded to bf16. */
int k2bw_adam(int64_t n, const float* w_cur, float* w_next, void* w_next_bf16, float* m, float* v,
              const float* G, float lr, float beta1, float beta2, float eps, int m_micro, int64_t step,
              void* stream);

/* Tuning aid: force the bf16 GEMM's kernel variant (0 = built-in choice).  Register-staged:
 * 2: 128x128 tile / 4 waves, 3: 256x256 / 8 waves, 6: 128x128 with two K groups of 4 waves.
 * Direct-to-LDS loads through a ring of four LDS stages: 22: 128x128 / 8 waves, K tiles of 64;
 * 23: 256x256 / 8 waves, K tiles of 32 (K not a multiple of the K tile: 6 and 3 instead).
 * Other ids: INVALID_ARG.  Process-wide. */
int k2bw_tune_gemm_tile(int id);

/* dy = (y - target) * scale, element-wise over n elements (n a multiple of 8 in bf16, of 4 in
 * fp32): the gradient of scale/2 * sum (y - target)^2, which a multi-stage run puts behind its
 * last stage in place of the seeded boundary gradient. */
int k2bw_squared_error_grad(int dtype, int64_t n, const void* y, const void* target, float scale,
                            void* dy, void* stream);

/* SGD with momentum as Section 3.1 prints it: g = G/m_micro, m <- beta m + (1-beta) g,
 * w_next = w_cur - lr m (fp32; w_next may equal w_cur), and, if w_next_bf16 is not NULL, its bf16
 * rounding.  n: multiple of 4. */
int k2bw_momentum(int64_t n, const float* w_cur, float* w_next, void* w_next_bf16, float* m,
                  const float* G, float lr, float beta, int m_micro, void* stream);

/* Plain 16-byte copy (bytes multiple of 16): the reference kernel for scaling HBM counters. */
int k2bw_copy(const void* in, void* out, int64_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* STAGE2BW_KERNELS_H */
