// C ABI over the single kernels (see include/stage2bw_kernels.h): argument marshalling only.
#include <cmath>

#include "../../include/stage2bw.h"
#include "../../include/stage2bw_kernels.h"
#include "kernels.hpp"

using namespace k2bw;

namespace {
int rc_of(hipError_t e) {
  if (e == hipSuccess) return STAGE_OK;
  if (e == hipErrorInvalidValue) return STAGE_ERR_INVALID_ARG;
  if (e == hipErrorOutOfMemory) return STAGE_ERR_OOM;
  return STAGE_ERR_HIP;
}
bool dtype_ok(int d) { return d == kF32 || d == kBF16; }

// Partial rows for k2bw_bias_grad_static: device memory that exists from library load to process end
// on every GPU that loads the library, so the call never allocates.
constexpr int kStaticParts = 64;            // == colsum_max_parts()
constexpr int kStaticMaxCols = 32768;
constexpr int kStaticMaxDevices = 64;
static __device__ __align__(256) float scratch[kStaticParts * kStaticMaxCols];
float* scratch_ptr[kStaticMaxDevices] = {};  // per device: the address of that device's copy of `scratch`
}  // namespace

extern "C" {

int k2bw_gemm(int dtype, int trans_a, int trans_b, int epilogue, int M, int N, int K, const void* A, int lda,
              const void* B, int ldb, void* C, int ldc, const void* bias, const void* aux, void* aux_out,
              int accumulate, void* stream) {
  if (!dtype_ok(dtype)) return STAGE_ERR_INVALID_ARG;
  GemmDesc d;
  d.dtype = dtype; d.trans_a = trans_a != 0; d.trans_b = trans_b != 0; d.epilogue = epilogue;
  d.M = M; d.N = N; d.K = K; d.A = A; d.lda = lda; d.B = B; d.ldb = ldb; d.C = C; d.ldc = ldc;
  d.bias = bias; d.aux = aux; d.aux_out = aux_out; d.accumulate = accumulate != 0;
  return rc_of(gemm(d, static_cast<hipStream_t>(stream)));
}

int k2bw_gemm_wgrad_segmented(int M, int N, int T, int n_seg, const void* A0, int lda, int64_t a_stride_bytes,
                              const uint8_t* a_idx_host, const void* B0, int ldb, int64_t b_stride_bytes,
                              const uint8_t* b_idx_host, float* C, int ldc, int accumulate, void* stream) {
  if (n_seg < 1 || n_seg > kGemmMaxSegments || T <= 0 || !a_idx_host || !b_idx_host) return STAGE_ERR_INVALID_ARG;
  GemmDesc d;
  d.dtype = kBF16; d.trans_a = true; d.epilogue = kEpiAccum;
  d.M = M; d.N = N; d.K = n_seg * T; d.A = A0; d.lda = lda; d.B = B0; d.ldb = ldb; d.C = C; d.ldc = ldc;
  d.accumulate = accumulate != 0;
  d.n_seg = n_seg; d.a_seg_stride = a_stride_bytes; d.b_seg_stride = b_stride_bytes;
  for (int s = 0; s < n_seg; ++s) { d.a_seg_idx[s] = a_idx_host[s]; d.b_seg_idx[s] = b_idx_host[s]; }
  if (n_seg == 1) {   // a plain product on the one piece
    d.A = static_cast<const char*>(A0) + a_stride_bytes * a_idx_host[0];
    d.B = static_cast<const char*>(B0) + b_stride_bytes * b_idx_host[0];
  }
  return rc_of(gemm(d, static_cast<hipStream_t>(stream)));
}

int64_t k2bw_gemm_dgrad_gelu_bias_workspace(int M, int N) {
  if (M <= 0 || N <= 0) return STAGE_ERR_INVALID_ARG;
  return (int64_t)((M + 31) / 32) * N;
}

int k2bw_gemm_dgrad_gelu_bias(int M, int N, int K, const void* dy, int lda, const void* w, int ldb, void* du, int ldc,
                              const void* u, float* dbias, int accumulate, float* workspace, void* stream) {
  if (!dbias || !workspace) return STAGE_ERR_INVALID_ARG;
  GemmDesc d;
  d.dtype = kBF16; d.trans_b = true; d.epilogue = kEpiGeluGrad;
  d.M = M; d.N = N; d.K = K; d.A = dy; d.lda = lda; d.B = w; d.ldb = ldb; d.C = du; d.ldc = ldc; d.aux = u;
  d.colsum_partial = workspace;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = gemm(d, s);
  if (e != hipSuccess) return rc_of(e);
  return rc_of(colsum_finalize(workspace, (M + 31) / 32, N, dbias, accumulate != 0, s));
}

int k2bw_layernorm_fwd(int dtype, int rows, int h, float eps, const void* x, const void* gain, const void* shift,
                       void* y, float* mean, float* rstd, void* stream) {
  if (!dtype_ok(dtype)) return STAGE_ERR_INVALID_ARG;
  return rc_of(layernorm_fwd(x, gain, shift, y, mean, rstd, rows, h, eps, dtype, static_cast<hipStream_t>(stream)));
}

int64_t k2bw_layernorm_bwd_workspace(int h) {
  if (h <= 0) return STAGE_ERR_INVALID_ARG;
  return (int64_t)ln_bwd_max_parts() * 3 * h;
}

int k2bw_layernorm_bwd(int dtype, int rows, int h, const void* dy, const void* x, const float* mean,
                       const float* rstd, const void* gain, const void* dres, void* dx, float* dgain_dshift,
                       float* dx_colsum, int accumulate, float* workspace, void* stream) {
  if (!dtype_ok(dtype) || !dgain_dshift || !workspace) return STAGE_ERR_INVALID_ARG;
  int parts = 0;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = layernorm_bwd(dy, x, mean, rstd, gain, dres, dx, workspace, &parts, rows, h, dtype, s);
  if (e != hipSuccess) return rc_of(e);
  FinalizeItem fin[2] = {{workspace, parts, 3 * h, 2 * h, dgain_dshift}, {workspace + 2 * h, parts, 3 * h, h, dx_colsum}};
  return rc_of(colsum_finalize_grouped(fin, dx_colsum ? 2 : 1, accumulate != 0, s));
}

int64_t k2bw_bias_grad_workspace(int n) {
  if (n <= 0) return STAGE_ERR_INVALID_ARG;
  return (int64_t)colsum_max_parts() * n;
}

int k2bw_bias_grad(int dtype, int rows, int n, const void* y, float* out, int accumulate, float* workspace,
                   void* stream) {
  if (!dtype_ok(dtype) || !out || !workspace) return STAGE_ERR_INVALID_ARG;
  int parts = 0;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = colsum_partial(y, rows, n, n, workspace, &parts, dtype, s);
  if (e != hipSuccess) return rc_of(e);
  return rc_of(colsum_finalize(workspace, parts, n, out, accumulate != 0, s));
}

int k2bw_bias_grad_static_max_cols(void) { return kStaticMaxCols; }

int k2bw_bias_grad_static(int dtype, int rows, int n, const void* y, float* out, int accumulate, void* stream) {
  if (!dtype_ok(dtype) || !out || n <= 0 || n > kStaticMaxCols || colsum_max_parts() > kStaticParts)
    return STAGE_ERR_INVALID_ARG;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return STAGE_ERR_HIP;
  if (dev < 0 || dev >= kStaticMaxDevices) return STAGE_ERR_INVALID_ARG;
  if (!scratch_ptr[dev]) {
    // The array's name is only a host-side handle; its address on the current device has to be asked for.
    float* p = nullptr;
    if (hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch)) != hipSuccess || !p)
      return STAGE_ERR_HIP;
    scratch_ptr[dev] = p;
  }
  float* partial = scratch_ptr[dev];
  int parts = 0;
  hipStream_t s = static_cast<hipStream_t>(stream);
  // Every partial row the second kernel reads is written in full by the first: nothing needs clearing.
  hipError_t e = colsum_partial(y, rows, n, n, partial, &parts, dtype, s);
  if (e != hipSuccess) return rc_of(e);
  return rc_of(colsum_finalize(partial, parts, n, out, accumulate != 0, s));
}

int k2bw_attention_fwd(int dtype, int b, int s, int a, int dh, int mask_mode, const int32_t* seqlens,
                       const void* qkv, void* o, float* lse, void* stream) {
  AttnDesc d;
  d.b = b; d.s = s; d.a = a; d.dh = dh; d.mask_mode = mask_mode; d.seqlens = seqlens; d.dtype = dtype;
  return rc_of(attention_fwd(d, qkv, o, lse, static_cast<hipStream_t>(stream)));
}

int k2bw_attention_bwd(int dtype, int b, int s, int a, int dh, int mask_mode, const int32_t* seqlens,
                       const void* qkv, const void* o, const float* lse, const void* d_o, void* dqkv, float* delta,
                       float* dbias_qkv, int accumulate, float* workspace, void* stream) {
  AttnDesc d;
  d.b = b; d.s = s; d.a = a; d.dh = dh; d.mask_mode = mask_mode; d.seqlens = seqlens; d.dtype = dtype;
  if (dbias_qkv && (!workspace || !attention_mfma_supported(d))) return STAGE_ERR_INVALID_ARG;
  d.colsum_partial = dbias_qkv ? workspace : nullptr;
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipError_t e = attention_bwd(d, qkv, o, lse, d_o, dqkv, delta, st);
  if (e != hipSuccess || !dbias_qkv) return rc_of(e);
  return rc_of(colsum_finalize(workspace, attention_colsum_rows(b, s), 3 * a * dh, dbias_qkv, accumulate != 0, st));
}

int64_t k2bw_attention_bwd_workspace(int b, int s, int a, int dh) {
  if (b <= 0 || s <= 0 || a <= 0 || dh <= 0) return STAGE_ERR_INVALID_ARG;
  return (int64_t)attention_colsum_rows(b, s) * 3 * a * dh;
}

int k2bw_adam(int64_t n, const float* w_cur, float* w_next, void* w_next_bf16, float* m, float* v, const float* G,
              float lr, float beta1, float beta2, float eps, int m_micro, int64_t step, void* stream) {
  if (m_micro < 1 || step < 1 || !(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f))
    return STAGE_ERR_INVALID_ARG;
  AdamDesc d;
  d.n = n; d.w_cur = w_cur; d.w_next = w_next; d.w_next_lp = static_cast<bf16_t*>(w_next_bf16);
  d.m = m; d.v = v; d.G = G; d.lr = lr; d.beta1 = beta1; d.beta2 = beta2; d.eps = eps;
  d.inv_m = 1.0f / (float)m_micro;
  d.c1 = (float)(1.0 / (1.0 - std::pow((double)beta1, (double)step)));
  d.c2 = (float)(1.0 / (1.0 - std::pow((double)beta2, (double)step)));
  return rc_of(adam_step(d, static_cast<hipStream_t>(stream)));
}

int k2bw_momentum(int64_t n, const float* w_cur, float* w_next, void* w_next_bf16, float* m, const float* G, float lr,
                  float beta, int m_micro, void* stream) {
  if (m_micro < 1 || !(beta >= 0.f && beta < 1.f)) return STAGE_ERR_INVALID_ARG;
  AdamDesc d;
  d.n = n; d.w_cur = w_cur; d.w_next = w_next; d.w_next_lp = static_cast<bf16_t*>(w_next_bf16);
  d.m = m; d.G = G; d.lr = lr; d.beta1 = beta; d.inv_m = 1.0f / (float)m_micro;
  return rc_of(momentum_step(d, static_cast<hipStream_t>(stream)));
}

int k2bw_squared_error_grad(int dtype, int64_t n, const void* y, const void* target, float scale, void* dy, void* stream) {
  if (!dtype_ok(dtype)) return STAGE_ERR_INVALID_ARG;
  return rc_of(squared_error_grad(y, target, dy, scale, n, dtype, static_cast<hipStream_t>(stream)));
}

int k2bw_copy(const void* in, void* out, int64_t bytes, void* stream) {
  return rc_of(copy_bytes(in, out, bytes, static_cast<hipStream_t>(stream)));
}

}  // extern "C"

namespace k2bw { void gemm_bf16_set_tile(int id); }
extern "C" int k2bw_tune_gemm_tile(int id) {
  if (id != 0 && id != 2 && id != 3 && id != 6 && id != 22 && id != 23) return STAGE_ERR_INVALID_ARG;
  k2bw::gemm_bf16_set_tile(id);
  return STAGE_OK;
}
