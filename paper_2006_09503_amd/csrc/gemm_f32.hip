// fp32 GEMM on the gfx950 matrix cores for the fp32 mode of the stage: v_mfma_f32_32x32x2_f32, fp32
// operands and accumulation throughout (fp32 MFMA peak of the part: 157.3 TFLOP/s).
//
// A 256-thread workgroup (2 x 2 waves) computes a 128 x 128 tile of C in K steps of 16 through two LDS
// stages; a wave owns 64 x 64 (2 x 2 MFMA blocks, 64 accumulator registers).  Both operand tiles sit in
// LDS k-major, [16 k][128 rows + 32 pad] floats: an MFMA fragment is then one 4-byte read per lane of 32
// consecutive rows at k (lanes 0..31) and at k+1 (lanes 32..63), and the pad of 32 puts the two halves
// on disjoint banks.  Global loads are 16-byte vectors along whichever index is contiguous in HBM (the
// tile of step kt+1 is in flight in registers while step kt runs its MFMAs); one barrier per K step.
// Any M, N, K: what lies outside the matrices is loaded as zero and never stored; operands whose leading
// dimension or base address do not allow 16-byte loads take guarded 4-byte loads instead.
//
// Lane layout of v_mfma_f32_32x32x2_f32: lane l supplies element (l % 32, l / 32) of the first operand
// (32 x 2) and (l / 32, l % 32) of the second (2 x 32); it receives column l % 32 of D, rows
// 8*(r/4) + 4*(l/32) + (r % 4) for accumulator register r.  As in the bf16 kernels the B tile is fed as the
// first operand and the A tile as the second, so a lane owns one row m of C and four consecutive columns
// per register quad: the epilogue's accesses are 16-byte vectors.
#include "kernels.hpp"

namespace k2bw {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BN = 128, BK = 16, LDT = 128 + 32;   // LDT: floats per k row of a staged tile
constexpr int kThreads = 256;

struct F32Params {
  const float* A; const float* B; float* C;
  int M, N, K, lda, ldb, ldc;
  const float* bias; const float* aux; float* aux_out;
  int accumulate;
  int vec_a, vec_b, vec_c;   // 16-byte accesses allowed on A, on B, on C / aux / aux_out / bias
};

// One operand's 128 x 16 tile on its way from HBM to LDS.  ROW_CONTIG: element (row, k) at X[k*ld + row],
// else at X[row*ld + k].  Two 16-byte pieces per thread.
template <bool ROW_CONTIG>
struct TileMover {
  float4 v[2];
  __device__ __forceinline__ void load(const float* __restrict__ X, int ld, int row0, int rows, int k0, int K, bool vec,
                                       int tid) {
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      int r, k;
      if (ROW_CONTIG) { k = tid / 32 + 8 * it; r = (tid % 32) * 4; }
      else { r = tid / 4 + 64 * it; k = (tid % 4) * 4; }
      const int gr = row0 + r, gk = k0 + k;
      float e[4] = {0.f, 0.f, 0.f, 0.f};
      if (ROW_CONTIG) {
        if (gk < K) {
          const float* p = X + (int64_t)gk * ld + gr;
          if (vec && gr + 3 < rows) {
            const float4 q = *reinterpret_cast<const float4*>(p);
            e[0] = q.x; e[1] = q.y; e[2] = q.z; e[3] = q.w;
          } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) if (gr + i < rows) e[i] = p[i];
          }
        }
      } else {
        if (gr < rows) {
          const float* p = X + (int64_t)gr * ld + gk;
          if (vec && gk + 3 < K) {
            const float4 q = *reinterpret_cast<const float4*>(p);
            e[0] = q.x; e[1] = q.y; e[2] = q.z; e[3] = q.w;
          } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) if (gk + i < K) e[i] = p[i];
          }
        }
      }
      v[it] = make_float4(e[0], e[1], e[2], e[3]);
    }
  }
  __device__ __forceinline__ void store(float* __restrict__ tile, int tid) const {
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      if (ROW_CONTIG) {
        const int k = tid / 32 + 8 * it, r = (tid % 32) * 4;
        *reinterpret_cast<float4*>(tile + k * LDT + r) = v[it];
      } else {
        const int r = tid / 4 + 64 * it, k = (tid % 4) * 4;
        tile[(k + 0) * LDT + r] = v[it].x; tile[(k + 1) * LDT + r] = v[it].y;
        tile[(k + 2) * LDT + r] = v[it].z; tile[(k + 3) * LDT + r] = v[it].w;
      }
    }
  }
};

template <bool TA, bool TB, int EPI>
__global__ __launch_bounds__(kThreads) void gemm_f32_mfma_kernel(F32Params p) {
  __shared__ __attribute__((aligned(16))) float sA[2][BK * LDT];
  __shared__ __attribute__((aligned(16))) float sB[2][BK * LDT];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;

  f32x16 acc[2][2];
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

  TileMover<TA> mv_a;     // A(m,k): m contiguous iff trans_a
  TileMover<!TB> mv_b;    // B(k,n): n contiguous iff not trans_b
  const int nk = (p.K + BK - 1) / BK;
  mv_a.load(p.A, p.lda, m0, p.M, 0, p.K, p.vec_a != 0, tid);
  mv_b.load(p.B, p.ldb, n0, p.N, 0, p.K, p.vec_b != 0, tid);
  mv_a.store(sA[0], tid);
  mv_b.store(sB[0], tid);
  __syncthreads();

  const int half = lane >> 5, l32 = lane & 31;
  for (int kt = 0; kt < nk; ++kt) {
    const float* a_t = sA[kt & 1];
    const float* b_t = sB[kt & 1];
    if (kt + 1 < nk) {   // uniform: the next tile travels in registers while this one is multiplied
      mv_a.load(p.A, p.lda, m0, p.M, (kt + 1) * BK, p.K, p.vec_a != 0, tid);
      mv_b.load(p.B, p.ldb, n0, p.N, (kt + 1) * BK, p.K, p.vec_b != 0, tid);
    }
#pragma unroll
    for (int kk = 0; kk < BK; kk += 2) {
      float af[2], bf[2];
#pragma unroll
      for (int mi = 0; mi < 2; ++mi) af[mi] = a_t[(kk + half) * LDT + wm * 64 + mi * 32 + l32];
#pragma unroll
      for (int ni = 0; ni < 2; ++ni) bf[ni] = b_t[(kk + half) * LDT + wn * 64 + ni * 32 + l32];
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(bf[ni], af[mi], acc[mi][ni], 0, 0, 0);
    }
    if (kt + 1 < nk) {
      mv_a.store(sA[(kt + 1) & 1], tid);
      mv_b.store(sB[(kt + 1) & 1], tid);
    }
    __syncthreads();
  }

  // Epilogue: lane owns row m and, per register quad g, columns n .. n+3.
#pragma unroll
  for (int mi = 0; mi < 2; ++mi) {
    const int gm = m0 + wm * 64 + mi * 32 + l32;
    if (gm >= p.M) continue;
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int gn = n0 + wn * 64 + ni * 32 + 8 * g + 4 * half;
        if (gn >= p.N) continue;
        const int64_t idx = (int64_t)gm * p.ldc + gn;
        float v[4] = {acc[mi][ni][4 * g], acc[mi][ni][4 * g + 1], acc[mi][ni][4 * g + 2], acc[mi][ni][4 * g + 3]};
        const bool whole = p.vec_c && gn + 3 < p.N;
        auto rd4 = [&](const float* src, float (&o)[4]) {
          if (whole) { const float4 q = *reinterpret_cast<const float4*>(src); o[0] = q.x; o[1] = q.y; o[2] = q.z; o[3] = q.w; }
          else {
#pragma unroll
            for (int i = 0; i < 4; ++i) o[i] = gn + i < p.N ? src[i] : 0.f;
          }
        };
        auto wr4 = [&](float* dst, const float (&o)[4]) {
          if (whole) *reinterpret_cast<float4*>(dst) = make_float4(o[0], o[1], o[2], o[3]);
          else {
#pragma unroll
            for (int i = 0; i < 4; ++i) if (gn + i < p.N) dst[i] = o[i];
          }
        };
        if (EPI == kEpiStore) {
          if (p.bias) { float b[4]; rd4(p.bias + gn, b);
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] += b[i]; }
          if (p.aux) { float r[4]; rd4(p.aux + idx, r);
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] += r[i]; }
          wr4(p.C + idx, v);
        } else if (EPI == kEpiGelu) {
          float b[4]; rd4(p.bias + gn, b);
#pragma unroll
          for (int i = 0; i < 4; ++i) v[i] += b[i];
          wr4(p.C + idx, v);
#pragma unroll
          for (int i = 0; i < 4; ++i) v[i] = gelu_f(v[i]);
          wr4(p.aux_out + idx, v);
        } else if (EPI == kEpiGeluGrad) {
          float u[4]; rd4(p.aux + idx, u);
#pragma unroll
          for (int i = 0; i < 4; ++i) v[i] *= gelu_grad_f(u[i]);
          wr4(p.C + idx, v);
        } else {
          if (p.accumulate) { float c[4]; rd4(p.C + idx, c);
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = c[i] + v[i]; }
          wr4(p.C + idx, v);
        }
      }
  }
}

template <bool TA, bool TB>
hipError_t launch_epi(const F32Params& p, int epi, dim3 grid, hipStream_t s) {
  switch (epi) {
    case kEpiStore: hipLaunchKernelGGL((gemm_f32_mfma_kernel<TA, TB, kEpiStore>), grid, dim3(kThreads), 0, s, p); break;
    case kEpiGelu: hipLaunchKernelGGL((gemm_f32_mfma_kernel<TA, TB, kEpiGelu>), grid, dim3(kThreads), 0, s, p); break;
    case kEpiGeluGrad: hipLaunchKernelGGL((gemm_f32_mfma_kernel<TA, TB, kEpiGeluGrad>), grid, dim3(kThreads), 0, s, p); break;
    case kEpiAccum: hipLaunchKernelGGL((gemm_f32_mfma_kernel<TA, TB, kEpiAccum>), grid, dim3(kThreads), 0, s, p); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

bool vec16(const void* ptr, int ld) { return (reinterpret_cast<uintptr_t>(ptr) & 15) == 0 && ld % 4 == 0; }

}  // namespace

hipError_t gemm_f32(const GemmDesc& d, hipStream_t stream) {
  F32Params p{static_cast<const float*>(d.A), static_cast<const float*>(d.B), static_cast<float*>(d.C),
              d.M, d.N, d.K, d.lda, d.ldb, d.ldc, static_cast<const float*>(d.bias), static_cast<const float*>(d.aux),
              static_cast<float*>(d.aux_out), d.accumulate ? 1 : 0, 0, 0, 0};
  p.vec_a = vec16(d.A, d.lda);
  p.vec_b = vec16(d.B, d.ldb);
  p.vec_c = vec16(d.C, d.ldc) && (!d.aux || vec16(d.aux, d.ldc)) && (!d.aux_out || vec16(d.aux_out, d.ldc)) &&
            (!d.bias || vec16(d.bias, 4));
  dim3 grid(ceil_div(d.N, BN), ceil_div(d.M, BM));
  if (d.trans_a) return d.trans_b ? launch_epi<true, true>(p, d.epilogue, grid, stream)
                                  : launch_epi<true, false>(p, d.epilogue, grid, stream);
  return d.trans_b ? launch_epi<false, true>(p, d.epilogue, grid, stream)
                   : launch_epi<false, false>(p, d.epilogue, grid, stream);
}

}  // namespace k2bw
