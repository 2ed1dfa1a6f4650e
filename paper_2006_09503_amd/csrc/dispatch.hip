// Shape validation and routing of GEMM and attention calls to the kernel families.
#include <cstdio>

#include "kernels.hpp"

namespace k2bw {

hipError_t gemm_f32(const GemmDesc& d, hipStream_t stream);
hipError_t gemm_bf16(const GemmDesc& d, hipStream_t stream);
hipError_t gemm_bf16_grouped(const GemmDesc* d, int count, hipStream_t stream);
void gemm_bf16_kernel_name(const GemmDesc* d, int count, char* out, size_t cap);
hipError_t attention_fwd_simple(const AttnDesc& d, const void* qkv, void* o, float* lse, hipStream_t st);
hipError_t attention_bwd_simple(const AttnDesc& d, const void* qkv, const void* o, const float* lse,
                                const void* d_o, void* dqkv, float* delta, hipStream_t st);
hipError_t attention_fwd_mfma(const AttnDesc& d, const void* qkv, void* o, float* lse, hipStream_t st);
hipError_t attention_bwd_mfma(const AttnDesc& d, const void* qkv, const void* o, const float* lse,
                              const void* d_o, void* dqkv, float* delta, hipStream_t st);

namespace {
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
}

namespace {
hipError_t check_gemm(const GemmDesc& d) {
  if (!d.A || !d.B || !d.C || d.M <= 0 || d.N <= 0 || d.K <= 0) return hipErrorInvalidValue;
  // extents of the stored matrices along their contiguous dimension
  const int a_cols = d.trans_a ? d.M : d.K;
  const int b_cols = d.trans_b ? d.K : d.N;
  if (d.lda < a_cols || d.ldb < b_cols || d.ldc < d.N) return hipErrorInvalidValue;
  if (d.epilogue == kEpiGelu && (!d.bias || !d.aux_out)) return hipErrorInvalidValue;
  if (d.epilogue == kEpiGeluGrad && !d.aux) return hipErrorInvalidValue;
  if (d.epilogue < kEpiStore || d.epilogue > kEpiAccum) return hipErrorInvalidValue;
  if (d.colsum_partial && (d.dtype != kBF16 || d.epilogue != kEpiGeluGrad || !aligned16(d.colsum_partial)))
    return hipErrorInvalidValue;
  if (d.dtype == kF32) return hipSuccess;
  if (d.dtype != kBF16) return hipErrorInvalidValue;
  // 16-byte vector accesses along the contiguous dimensions
  if (a_cols % 8 || b_cols % 8 || d.lda % 8 || d.ldb % 8 || !aligned16(d.A) || !aligned16(d.B))
    return hipErrorInvalidValue;
  return hipSuccess;
}
}  // namespace

hipError_t gemm(const GemmDesc& d, hipStream_t stream) {
  hipError_t e = check_gemm(d);
  if (e != hipSuccess) return e;
  return d.dtype == kF32 ? gemm_f32(d, stream) : gemm_bf16(d, stream);
}

void gemm_kernel_name(const GemmDesc* d, int count, char* out, size_t cap) {
  if (d[0].dtype == kBF16) gemm_bf16_kernel_name(d, count, out, cap);
  else snprintf(out, cap, "gemm_f32_kernel<%s, %s, %d>", d[0].trans_a ? "true" : "false", d[0].trans_b ? "true" : "false", d[0].epilogue);
}

hipError_t gemm_grouped(const GemmDesc* d, int count, hipStream_t stream) {
  if (!d || count < 1 || count > kGemmMaxGroup) return hipErrorInvalidValue;
  for (int g = 0; g < count; ++g) {
    hipError_t e = check_gemm(d[g]);
    if (e != hipSuccess) return e;
    if (d[g].dtype != d[0].dtype) return hipErrorInvalidValue;
  }
  if (d[0].dtype == kBF16) return gemm_bf16_grouped(d, count, stream);
  for (int g = 0; g < count; ++g) {
    hipError_t e = gemm_f32(d[g], stream);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

namespace {
hipError_t check_attn(const AttnDesc& d) {
  if (d.b <= 0 || d.s <= 0 || d.a <= 0 || d.dh <= 0 || d.dh % 8 || d.dh > 128) return hipErrorInvalidValue;
  if (d.mask_mode < 0 || d.mask_mode > 2) return hipErrorInvalidValue;
  if (d.mask_mode == 2 && !d.seqlens) return hipErrorInvalidValue;
  if (d.dtype != kF32 && d.dtype != kBF16) return hipErrorInvalidValue;
  return hipSuccess;
}
}  // namespace

hipError_t attention_fwd(const AttnDesc& d, const void* qkv, void* o, float* lse, hipStream_t stream) {
  hipError_t e = check_attn(d);
  if (e != hipSuccess) return e;
  if (!qkv || !o || !lse || !aligned16(qkv) || !aligned16(o)) return hipErrorInvalidValue;
  if (attention_mfma_supported(d)) return attention_fwd_mfma(d, qkv, o, lse, stream);
  return attention_fwd_simple(d, qkv, o, lse, stream);
}

hipError_t attention_bwd(const AttnDesc& d, const void* qkv, const void* o, const float* lse, const void* d_o,
                         void* dqkv, float* delta, hipStream_t stream) {
  hipError_t e = check_attn(d);
  if (e != hipSuccess) return e;
  if (!qkv || !o || !lse || !d_o || !dqkv || !delta) return hipErrorInvalidValue;
  if (!aligned16(qkv) || !aligned16(o) || !aligned16(d_o) || !aligned16(dqkv)) return hipErrorInvalidValue;
  if (attention_mfma_supported(d)) return attention_bwd_mfma(d, qkv, o, lse, d_o, dqkv, delta, stream);
  if (d.colsum_partial) return hipErrorInvalidValue;   // only the MFMA kernels produce the column sums
  return attention_bwd_simple(d, qkv, o, lse, d_o, dqkv, delta, stream);
}

}  // namespace k2bw
