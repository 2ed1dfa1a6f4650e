// Host-side launchers of the gfx950 kernels.  Every launcher validates the shapes its kernel
// assumes and returns hipErrorInvalidValue instead of launching when they do not hold.
#pragma once
#include "common.hpp"

namespace k2bw {

enum Dtype : int { kF32 = 0, kBF16 = 1 };

// ---------------------------------------------------------------------------- GEMM
// C[M,N] = epilogue( sum_k A(m,k) * B(k,n) )
//   A(m,k) = trans_a ? A[k*lda + m] : A[m*lda + k]
//   B(k,n) = trans_b ? B[n*ldb + k] : B[k*ldb + n]
// dtype is the element type of A, B (and of C, aux, aux_out unless the epilogue says fp32).
// Leading dimensions and the contiguous extents must be multiples of 8 elements.
enum Epilogue : int {
  kEpiStore = 0,     // C = acc (+ bias[n]) (+ residual[m,n])
  kEpiGelu = 1,      // u = acc + bias[n]; C = u; aux_out = GELU(u)
  kEpiGeluGrad = 2,  // C = acc * GELU'(aux[m,n])
  kEpiAccum = 3      // C is fp32: C = (accumulate ? C : 0) + acc   (weight-gradient coalescing)
};

constexpr int kGemmMaxSegments = 8;   // pieces of a segmented reduction range (see GemmDesc::n_seg)
struct GemmDesc {
  const void* A = nullptr;
  const void* B = nullptr;
  void* C = nullptr;
  int M = 0, N = 0, K = 0;
  int lda = 0, ldb = 0, ldc = 0;
  bool trans_a = false, trans_b = false;
  int epilogue = kEpiStore;
  const void* bias = nullptr;      // [N], element type = dtype, or null
  const void* aux = nullptr;       // residual (kEpiStore) or pre-activation u (kEpiGeluGrad), ld = ldc
  void* aux_out = nullptr;         // GELU(u) (kEpiGelu), ld = ldc
  bool accumulate = false;         // kEpiAccum
  // kEpiGeluGrad, bf16 only: if set, fp32 [ceil(M/32)][N] receives the column sums of every
  // 32-row strip of the result (before rounding to bf16): the bias gradient of the projection
  // whose output gradient C is, reduced afterwards with colsum_finalize
  float* colsum_partial = nullptr;
  // bf16 only, optional: `prefetch_bytes` bytes at `prefetch` that a later launch on the stream reads
  // (the stage passes the next GEMM's weights); this launch touches their cache lines on its way in,
  // so that they come from the memory-side cache and not from HBM when they are needed.  Never written.
  const void* prefetch = nullptr;
  int64_t prefetch_bytes = 0;
  // bf16, kEpiAccum form only: the reduction range made of n_seg pieces of K / n_seg rows each that lie
  // in different buffers (the operands of several microbatches' weight-gradient products, summed by
  // one product of reduction length n_seg * T).  Piece s of A starts at A + a_seg_idx[s] * a_seg_stride
  // bytes, piece s of B at B + b_seg_idx[s] * b_seg_stride bytes: buffers carved at a constant
  // stride from one allocation, indices 0..15, strides multiples of 256 bytes.  n_seg = 1: plain.
  int n_seg = 1;
  uint8_t a_seg_idx[kGemmMaxSegments] = {}, b_seg_idx[kGemmMaxSegments] = {};
  int64_t a_seg_stride = 0, b_seg_stride = 0;
  int dtype = kF32;
};
hipError_t gemm(const GemmDesc& d, hipStream_t stream);
// 1..4 independent GEMMs of the same form, epilogue and dtype; bf16 runs them in one launch.
constexpr int kGemmMaxGroup = 24;   // GEMMs of one form and epilogue that may share a launch
hipError_t gemm_grouped(const GemmDesc* d, int count, hipStream_t stream);
// CUs of the current device (a launch of T tiles takes ceil(T / CUs) rounds of one tile per CU).
int gemm_compute_units();
// Name (with template arguments, as a kernel trace prints it) of the kernel such a call runs.
void gemm_kernel_name(const GemmDesc* d, int count, char* out, size_t cap);

// ---------------------------------------------------------------------------- LayerNorm
// y = gain * (x - mean) * rstd + shift over rows of length h; saves mean, rstd (fp32 per row).
// gain, shift: element type = dtype (the weight version buffers hold every parameter in it).
hipError_t layernorm_fwd(const void* x, const void* gain, const void* shift, void* y,
                         float* mean, float* rstd, int rows, int h, float eps, int dtype,
                         hipStream_t stream);
// dx = dres + rstd * (dxhat - mean(dxhat) - xhat * mean(dxhat * xhat)), dxhat = dy * gain;
// dres may be null.  Column sums go to partial[parts][3h] (fp32: sum_r dy*xhat | sum_r dy | sum_r dx);
// *parts_out receives the number of partial rows written.  partial must hold
// 3 * ln_bwd_max_parts() * h floats.
int ln_bwd_max_parts();
hipError_t layernorm_bwd(const void* dy, const void* x, const float* mean, const float* rstd,
                         const void* gain, const void* dres, void* dx, float* partial,
                         int* parts_out, int rows, int h, int dtype, hipStream_t stream);

// ---------------------------------------------------------------------------- column sums
// partial[parts][n] = per-slab column sums of y[rows, n] (ld = ldy); parts <= colsum_max_parts().
int colsum_max_parts();
hipError_t colsum_partial(const void* y, int rows, int n, int ldy, float* partial, int* parts_out,
                          int dtype, hipStream_t stream);
// out[n] = (accumulate ? out[n] : 0) + sum_p partial[p][n]
hipError_t colsum_finalize(const float* partial, int parts, int n, float* out, bool accumulate,
                           hipStream_t stream);

// Grouped forms: column sums of up to 4 matrices [rows, n_i] in one launch into
// partial[parts][sum n_i] (segment i starts at column sum_{j<i} n_j), and the final reduction
// of up to kFinalizeMaxItems (partial, out) pairs in one launch (n and ld multiples of 4, pointers 16-byte aligned).
struct ColsumItem { const void* y; int n; int ld; };
hipError_t colsum_partial_grouped(const ColsumItem* items, int count, int rows, float* partial, int* parts_out,
                                  int* total_cols_out, int dtype, hipStream_t stream);
struct FinalizeItem { const float* partial; int parts; int ld; int n; float* out; };
constexpr int kFinalizeMaxItems = 64;   // segments per launch (the launch's arguments stay under 4 KB)
hipError_t colsum_finalize_grouped(const FinalizeItem* items, int count, bool accumulate, hipStream_t stream);

// ---------------------------------------------------------------------------- attention
// qkv: [b*s, 3h] rows = tokens, columns Q|K|V each head-major (head size dh = h/a).
// o: [b*s, h]; lse: [b, a, s] fp32 (log-sum-exp of the scaled, masked scores).
// mask_mode 0 none, 1 causal, 2 key padding with seqlens[b] (device int32).
struct AttnDesc {
  int b = 0, s = 0, a = 0, dh = 0;
  int mask_mode = 0;
  const int32_t* seqlens = nullptr;
  int dtype = kF32;
  // backward, bf16 only: if set, fp32 [attention_colsum_rows(b, s)][3h] receives per-workgroup column
  // sums of dQ | dK | dV (before rounding to bf16): the bias gradient of the QKV projection,
  // reduced afterwards with colsum_finalize
  float* colsum_partial = nullptr;
};
int attention_colsum_rows(int b, int s);
bool attention_mfma_supported(const AttnDesc& d);   // bf16 with head size 32, 64, 80 or 128
hipError_t attention_fwd(const AttnDesc& d, const void* qkv, void* o, float* lse,
                         hipStream_t stream);
// dqkv: [b*s, 3h]; delta: scratch [b, a, s] fp32 (rowsum(dO*O)).
hipError_t attention_bwd(const AttnDesc& d, const void* qkv, const void* o, const float* lse,
                         const void* d_o, void* dqkv, float* delta, hipStream_t stream);

// ---------------------------------------------------------------------------- optimizer
// One Adam step on n parameters with the coalesced gradient sum G (g = G * inv_m):
//   m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2;
//   w_next = w_cur - lr * (m * c1) / (sqrt(v * c2) + eps),  c1 = 1/(1-b1^t), c2 = 1/(1-b2^t).
// fp32 mode: w_cur, w_next are the two version buffers (fp32), w_next_lp = null.
// bf16 mode: w_cur == w_next == master (fp32, in place), w_next_lp = bf16 buffer to write.
struct AdamDesc {
  const float* w_cur = nullptr;
  float* w_next = nullptr;
  bf16_t* w_next_lp = nullptr;
  float* m = nullptr;
  float* v = nullptr;
  const float* G = nullptr;
  int64_t n = 0;
  float lr = 0, beta1 = 0, beta2 = 0, eps = 0, inv_m = 1, c1 = 1, c2 = 1;
  float omb1 = 0, omb2 = 0;        // 1 - beta, rounded once from double
};
hipError_t adam_step(const AdamDesc& d, hipStream_t stream);
// SGD with momentum (Section 3.1's printed form); uses w_*, m, G, n, lr, beta1, inv_m of the descriptor.
hipError_t momentum_step(const AdamDesc& d, hipStream_t stream);

// ---------------------------------------------------------------------------- conversions / copies
// dy = (y - target) * scale over n elements (n a multiple of 8 in bf16, 4 in fp32)
hipError_t squared_error_grad(const void* y, const void* target, void* dy, float scale, int64_t n, int dtype,
                              hipStream_t stream);
hipError_t convert_f32_to_bf16(const float* in, bf16_t* out, int64_t n, hipStream_t stream);
hipError_t convert_bf16_to_f32(const bf16_t* in, float* out, int64_t n, hipStream_t stream);
hipError_t copy_bytes(const void* in, void* out, int64_t bytes, hipStream_t stream);
// dst[c][r] = src[r][c] for bf16 matrices src [rows][cols] (rows, cols multiples of 8), any number of them;
// kTransposeMaxItems per launch.
struct TransposeItem { const void* src; void* dst; int rows, cols; };
constexpr int kTransposeMaxItems = 32;
hipError_t transpose_bf16_grouped(const TransposeItem* items, int count, hipStream_t stream);

}  // namespace k2bw
