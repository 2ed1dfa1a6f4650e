// bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulation.
//
// One workgroup computes a BM x BN tile of C in K steps of 64.  Both operand tiles are staged
// in LDS in one common form -- [row][64 k] bf16, 128-byte rows, 16-byte chunks XOR-swizzled by
// row -- whatever the operand's layout in HBM:
//   * K contiguous in HBM (activations as A, W read for the data gradient): 16-byte global
//     loads go to LDS as they are;
//   * K strided in HBM (W[K,N] read for the forward, both operands of the weight gradient):
//     each thread loads a 4(k) x 8(row) patch with four 16-byte loads along the contiguous
//     dimension, transposes it in registers and writes eight 8-byte pieces.
// so the MFMA loop is the same for the forward (NN), data-gradient (NT) and weight-gradient
// (TN) forms.  Two LDS stages; the global loads of step k+1 are in flight while step k runs
// on the matrix cores.  Each wave owns a WM x WN sub-tile = (WM/32) x (WN/32) accumulators of
// 32x32 (16 fp32 registers per lane each).
//
// Lane layout of v_mfma_f32_32x32x16_bf16: lane l supplies row (l % 32) of A and column
// (l % 32) of B, k = 8*(l/32) .. +7; it receives column (l % 32) of D, rows
// 8*(r/4) + 4*(l/32) + (r % 4) for accumulator register r.
#include "kernels.hpp"

namespace k2bw {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BK = 64;

struct BfParams {
  const bf16_t* A; const bf16_t* B; void* C;
  int M, N, K, lda, ldb, ldc;
  const bf16_t* bias; const bf16_t* aux; bf16_t* aux_out;
  int accumulate;
  int tiles_m, tiles_n;
};

// chunk swizzle: conflict-free for 8 or 16 consecutive rows reading the same logical chunk
__device__ __forceinline__ int swz(int row) { return (row + (row >> 3)) & 7; }

// Operand with K contiguous in HBM: tile rows = R, 8 chunks of 8 bf16 per row.
template <int R, int NT>
struct DirectLoader {
  static constexpr int kIters = R * 8 / NT;
  static_assert(R * 8 % NT == 0, "tile/threads mismatch");
  uint4 regs[kIters];
  // base: element (row0, k = 0); rows_valid: rows of the tile inside the matrix
  __device__ __forceinline__ void load(const bf16_t* base, int ld, int rows_valid, int k0, int K, int tid) {
#pragma unroll
    for (int i = 0; i < kIters; ++i) {
      const int idx = tid + i * NT;
      const int row = idx >> 3, c = idx & 7;
      const int k = k0 + c * 8;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (row < rows_valid && k < K) v = *reinterpret_cast<const uint4*>(base + (int64_t)row * ld + k);
      regs[i] = v;
    }
  }
  __device__ __forceinline__ void store(uint4* tile, int tid) const {
#pragma unroll
    for (int i = 0; i < kIters; ++i) {
      const int idx = tid + i * NT;
      const int row = idx >> 3, c = idx & 7;
      tile[row * 8 + (c ^ swz(row))] = regs[i];
    }
  }
};

__device__ __forceinline__ uint32_t word(const uint4& v, int i) {
  return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w;
}

// Operand with the row index contiguous in HBM (element (row, k) at base[k*ld + row]).
template <int R, int NT>
struct TransposingLoader {
  static constexpr int kUnits = (BK / 4) * (R / 8);  // 4(k) x 8(row) patches per tile
  static constexpr int kIters = kUnits / NT;
  static_assert(kUnits % NT == 0, "tile/threads mismatch");
  uint4 regs[kIters][4];
  __device__ __forceinline__ void load(const bf16_t* base, int ld, int rows_valid, int k0, int K, int tid) {
#pragma unroll
    for (int i = 0; i < kIters; ++i) {
      const int u = tid + i * NT;
      const int rc = u % (R / 8), kq = u / (R / 8);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int k = k0 + kq * 4 + j;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (rc * 8 < rows_valid && k < K) v = *reinterpret_cast<const uint4*>(base + (int64_t)k * ld + rc * 8);
        regs[i][j] = v;
      }
    }
  }
  __device__ __forceinline__ void store(uint4* tile, int tid) const {
    uint2* t2 = reinterpret_cast<uint2*>(tile);
#pragma unroll
    for (int i = 0; i < kIters; ++i) {
      const int u = tid + i * NT;
      const int rc = u % (R / 8), kq = u / (R / 8);
#pragma unroll
      for (int ii = 0; ii < 8; ++ii) {
        const int wd = ii >> 1;
        const uint32_t w0 = word(regs[i][0], wd), w1 = word(regs[i][1], wd);
        const uint32_t w2 = word(regs[i][2], wd), w3 = word(regs[i][3], wd);
        uint2 o;
        if (ii & 1) {
          o.x = (w0 >> 16) | (w1 & 0xffff0000u);
          o.y = (w2 >> 16) | (w3 & 0xffff0000u);
        } else {
          o.x = (w0 & 0xffffu) | (w1 << 16);
          o.y = (w2 & 0xffffu) | (w3 << 16);
        }
        const int row = rc * 8 + ii;
        t2[(row * 8 + ((kq >> 1) ^ swz(row))) * 2 + (kq & 1)] = o;
      }
    }
  }
};

template <int R, int NT, bool K_CONTIGUOUS>
struct LoaderSel { using type = DirectLoader<R, NT>; };
template <int R, int NT>
struct LoaderSel<R, NT, false> { using type = TransposingLoader<R, NT>; };

template <int BM, int BN, int WM, int WN, bool TA, bool TB, int EPI>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64) void gemm_bf16_kernel(BfParams p) {
  constexpr int NT = (BM / WM) * (BN / WN) * 64;
  constexpr int MI = WM / 32, NI = WN / 32;
  constexpr int WAVES_N = BN / WN;
  extern __shared__ uint4 smem[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;

  // Workgroup -> tile: consecutive workgroup ids land on different XCDs (round-robin over 8),
  // so give each XCD a contiguous run of tiles: they share A rows / B columns in that XCD's L2.
  const int n_tiles = p.tiles_m * p.tiles_n;
  int wg = blockIdx.x;
  {
    const int per_xcd = n_tiles / 8;
    if (wg < per_xcd * 8) wg = (wg % 8) * per_xcd + wg / 8;
  }
  const int bm = wg / p.tiles_n, bn = wg % p.tiles_n;
  const int m0 = bm * BM, n0 = bn * BN;

  const bf16_t* a_base = TA ? p.A + m0 : p.A + (int64_t)m0 * p.lda;
  const bf16_t* b_base = TB ? p.B + (int64_t)n0 * p.ldb : p.B + n0;
  const int a_rows = p.M - m0, b_rows = p.N - n0;

  typename LoaderSel<BM, NT, !TA>::type ld_a;
  typename LoaderSel<BN, NT, TB>::type ld_b;

  constexpr int kStage = (BM + BN) * 8;  // uint4 per stage
  f32x16 acc[MI][NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

  const int nk = (p.K + BK - 1) / BK;
  ld_a.load(a_base, p.lda, a_rows, 0, p.K, tid);
  ld_b.load(b_base, p.ldb, b_rows, 0, p.K, tid);
  ld_a.store(smem, tid);
  ld_b.store(smem + BM * 8, tid);
  __syncthreads();

  const int a_row0 = wm * WM + (lane & 31);
  const int b_row0 = wn * WN + (lane & 31);
  const int khalf = lane >> 5;

  for (int kt = 0; kt < nk; ++kt) {
    const uint4* sA = smem + (kt & 1) * kStage;
    const uint4* sB = sA + BM * 8;
    const bool more = kt + 1 < nk;
    if (more) {
      ld_a.load(a_base, p.lda, a_rows, (kt + 1) * BK, p.K, tid);
      ld_b.load(b_base, p.ldb, b_rows, (kt + 1) * BK, p.K, tid);
    }
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 af[MI], bfr[NI];
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) {
        const int row = a_row0 + mi * 32;
        af[mi] = __builtin_bit_cast(bf16x8, sA[row * 8 + ((ks * 2 + khalf) ^ swz(row))]);
      }
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) {
        const int row = b_row0 + ni * 32;
        bfr[ni] = __builtin_bit_cast(bf16x8, sB[row * 8 + ((ks * 2 + khalf) ^ swz(row))]);
      }
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mi], bfr[ni], acc[mi][ni], 0, 0, 0);
    }
    if (more) {
      uint4* dA = smem + ((kt + 1) & 1) * kStage;
      ld_a.store(dA, tid);
      ld_b.store(dA + BM * 8, tid);
    }
    __syncthreads();
  }

  // epilogue: lane holds column (lane % 32), rows 8*(r/4) + 4*(lane/32) + r%4 of each 32x32 block
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
      const int col = n0 + wn * WN + ni * 32 + (lane & 31);
      if (col >= p.N) continue;
      float bias = 0.f;
      if (EPI == kEpiStore || EPI == kEpiGelu) bias = p.bias ? bf16_to_f32(p.bias[col]) : 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm * WM + mi * 32 + 8 * (r >> 2) + 4 * khalf + (r & 3);
        if (row >= p.M) continue;
        const int64_t idx = (int64_t)row * p.ldc + col;
        float v = acc[mi][ni][r];
        if (EPI == kEpiStore) {
          v += bias;
          if (p.aux) v += bf16_to_f32(p.aux[idx]);
          static_cast<bf16_t*>(p.C)[idx] = f32_to_bf16(v);
        } else if (EPI == kEpiGelu) {
          v += bias;
          static_cast<bf16_t*>(p.C)[idx] = f32_to_bf16(v);
          p.aux_out[idx] = f32_to_bf16(gelu_f(v));
        } else if (EPI == kEpiGeluGrad) {
          static_cast<bf16_t*>(p.C)[idx] = f32_to_bf16(v * gelu_grad_f(bf16_to_f32(p.aux[idx])));
        } else {
          float* c = static_cast<float*>(p.C) + idx;
          *c = p.accumulate ? *c + v : v;
        }
      }
    }
  }
}

template <int BM, int BN, int WM, int WN, bool TA, bool TB, int EPI>
hipError_t launch(BfParams p, hipStream_t s) {
  constexpr int NT = (BM / WM) * (BN / WN) * 64;
  constexpr size_t lds = 2 * (BM + BN) * 8 * sizeof(uint4);
  auto kern = gemm_bf16_kernel<BM, BN, WM, WN, TA, TB, EPI>;
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    configured = true;
  }
  p.tiles_m = ceil_div(p.M, BM);
  p.tiles_n = ceil_div(p.N, BN);
  hipLaunchKernelGGL(kern, dim3(p.tiles_m * p.tiles_n), dim3(NT), lds, s, p);
  return hipGetLastError();
}

template <bool TA, bool TB, int EPI>
hipError_t pick_tile(const BfParams& p, hipStream_t s) {
  // 256x256 tiles when they still give every CU work; otherwise 128x128.
  const int64_t big = (int64_t)ceil_div(p.M, 256) * ceil_div(p.N, 256);
  if (big >= 192) return launch<256, 256, 128, 128, TA, TB, EPI>(p, s);
  return launch<128, 128, 64, 64, TA, TB, EPI>(p, s);
}

}  // namespace

hipError_t gemm_bf16(const GemmDesc& d, hipStream_t stream) {
  BfParams p{static_cast<const bf16_t*>(d.A), static_cast<const bf16_t*>(d.B), d.C,
             d.M, d.N, d.K, d.lda, d.ldb, d.ldc, static_cast<const bf16_t*>(d.bias), static_cast<const bf16_t*>(d.aux),
             static_cast<bf16_t*>(d.aux_out), d.accumulate ? 1 : 0, 0, 0};
  if (!d.trans_a && !d.trans_b) {
    if (d.epilogue == kEpiStore) return pick_tile<false, false, kEpiStore>(p, stream);
    if (d.epilogue == kEpiGelu) return pick_tile<false, false, kEpiGelu>(p, stream);
  } else if (!d.trans_a && d.trans_b) {
    if (d.epilogue == kEpiStore) return pick_tile<false, true, kEpiStore>(p, stream);
    if (d.epilogue == kEpiGeluGrad) return pick_tile<false, true, kEpiGeluGrad>(p, stream);
  } else if (d.trans_a && !d.trans_b) {
    if (d.epilogue == kEpiAccum) return pick_tile<true, false, kEpiAccum>(p, stream);
  }
  return hipErrorInvalidValue;  // form/epilogue pair the stage never issues
}

}  // namespace k2bw
