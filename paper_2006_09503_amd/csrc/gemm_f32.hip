// fp32 GEMM for the fp32 (parity) mode of the stage: LDS-tiled, plain FMA, fp32 throughout.
// 64x64 output tile per 256-thread workgroup, 4x4 outputs per thread, K step 16.
// Any M, N, K; every access is guarded.  The fp32 mode exists to show parity with the fp64
// oracle at 1e-4; throughput is carried by the bf16 MFMA kernel.
#include "kernels.hpp"

namespace k2bw {
namespace {

constexpr int TM = 64, TN = 64, TK = 16;

struct F32Params {
  const float* A; const float* B; float* C;
  int M, N, K, lda, ldb, ldc;
  const float* bias; const float* aux; float* aux_out;
  int accumulate;
};

template <bool TA, bool TB, int EPI>
__global__ __launch_bounds__(256) void gemm_f32_kernel(F32Params p) {
  __shared__ float As[TK][TM + 4];
  __shared__ float Bs[TK][TN + 4];
  const int tid = threadIdx.x;
  const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
  const int tx = tid % 16, ty = tid / 16;  // thread owns rows ty*4.., cols tx*4..
  float acc[4][4] = {};

  for (int k0 = 0; k0 < p.K; k0 += TK) {
    // 64x16 elements of A and of B, 4 per thread each
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = tid + i * 256;
      int mm, kk;
      if (TA) { mm = e % TM; kk = e / TM; } else { kk = e % TK; mm = e / TK; }
      const int gm = m0 + mm, gk = k0 + kk;
      float v = 0.f;
      if (gm < p.M && gk < p.K) v = TA ? p.A[(int64_t)gk * p.lda + gm] : p.A[(int64_t)gm * p.lda + gk];
      As[kk][mm] = v;
      int nn, kb;
      if (TB) { kb = e % TK; nn = e / TK; } else { nn = e % TN; kb = e / TN; }
      const int gn = n0 + nn, gkb = k0 + kb;
      float w = 0.f;
      if (gn < p.N && gkb < p.K) w = TB ? p.B[(int64_t)gn * p.ldb + gkb] : p.B[(int64_t)gkb * p.ldb + gn];
      Bs[kb][nn] = w;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < TK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }

#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int gm = m0 + ty * 4 + i;
    if (gm >= p.M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int gn = n0 + tx * 4 + j;
      if (gn >= p.N) continue;
      const int64_t idx = (int64_t)gm * p.ldc + gn;
      float v = acc[i][j];
      if (EPI == kEpiStore) {
        if (p.bias) v += p.bias[gn];
        if (p.aux) v += p.aux[idx];
        p.C[idx] = v;
      } else if (EPI == kEpiGelu) {
        v += p.bias[gn];
        p.C[idx] = v;
        p.aux_out[idx] = gelu_f(v);
      } else if (EPI == kEpiGeluGrad) {
        p.C[idx] = v * gelu_grad_f(p.aux[idx]);
      } else {
        p.C[idx] = p.accumulate ? p.C[idx] + v : v;
      }
    }
  }
}

template <bool TA, bool TB>
hipError_t launch_epi(const F32Params& p, int epi, dim3 grid, hipStream_t s) {
  switch (epi) {
    case kEpiStore: hipLaunchKernelGGL((gemm_f32_kernel<TA, TB, kEpiStore>), grid, dim3(256), 0, s, p); break;
    case kEpiGelu: hipLaunchKernelGGL((gemm_f32_kernel<TA, TB, kEpiGelu>), grid, dim3(256), 0, s, p); break;
    case kEpiGeluGrad: hipLaunchKernelGGL((gemm_f32_kernel<TA, TB, kEpiGeluGrad>), grid, dim3(256), 0, s, p); break;
    case kEpiAccum: hipLaunchKernelGGL((gemm_f32_kernel<TA, TB, kEpiAccum>), grid, dim3(256), 0, s, p); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace

hipError_t gemm_f32(const GemmDesc& d, hipStream_t stream) {
  F32Params p{static_cast<const float*>(d.A), static_cast<const float*>(d.B), static_cast<float*>(d.C),
              d.M, d.N, d.K, d.lda, d.ldb, d.ldc, static_cast<const float*>(d.bias), static_cast<const float*>(d.aux),
              static_cast<float*>(d.aux_out), d.accumulate ? 1 : 0};
  dim3 grid(ceil_div(d.N, TN), ceil_div(d.M, TM));
  if (d.trans_a) return d.trans_b ? launch_epi<true, true>(p, d.epilogue, grid, stream)
                                  : launch_epi<true, false>(p, d.epilogue, grid, stream);
  return d.trans_b ? launch_epi<false, true>(p, d.epilogue, grid, stream)
                   : launch_epi<false, false>(p, d.epilogue, grid, stream);
}

}  // namespace k2bw
