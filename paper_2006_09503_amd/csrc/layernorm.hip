// LayerNorm forward / backward and column-sum kernels (HBM-bound).
//
// A row of length h is handled by R threads (R = 64: one wavefront, 128 or 256: two or four
// wavefronts of the 256-thread workgroup), each owning CPT chunks of 8 consecutive elements,
// chunk index = sub + c*R, so that the R threads' 16-byte accesses are contiguous.  The row
// stays in registers between the statistics and the normalisation: one read, one write.
// Statistics are fp32: mean first, then the centred sum of squares (biased variance).
#include "kernels.hpp"

namespace k2bw {
namespace {

constexpr int kWg = 256;

struct ColsumGroup {
  const void* y[4];
  int n[4], ld[4], block0[4], col0[4];
  int count, rows, rows_per_part, total_cols;
  float* partial;
};
struct FinalizeGroup {
  const float* partial[kFinalizeMaxItems];
  float* out[kFinalizeMaxItems];
  int parts[kFinalizeMaxItems], n[kFinalizeMaxItems], ld[kFinalizeMaxItems], block0[kFinalizeMaxItems];
  int count, accumulate;
};

// sum over the R threads that share a row; R == 64 needs no LDS
template <int R>
__device__ __forceinline__ float group_sum(float v, float* red, int tid) {
  v = wave_sum(v);
  if (R == 64) return v;
  constexpr int W = R / 64;           // waves per row
  const int wave = tid >> 6;
  __syncthreads();                    // red may still be read from the previous call
  if ((tid & 63) == 0) red[wave] = v;
  __syncthreads();
  float s = 0.f;
  const int first = (wave / W) * W;
#pragma unroll
  for (int i = 0; i < W; ++i) s += red[first + i];
  return s;
}

template <typename T, int R, int CPT>
__global__ __launch_bounds__(kWg) void ln_fwd_kernel(const T* __restrict__ x, const T* __restrict__ gain,
                                                      const T* __restrict__ shift, T* __restrict__ y,
                                                      float* __restrict__ mean_out, float* __restrict__ rstd_out,
                                                      int rows, int h, float eps) {
  constexpr int ROWS = kWg / R;
  __shared__ float red[4];
  const int tid = threadIdx.x;
  const int sub = tid % R;
  const int row = blockIdx.x * ROWS + tid / R;
  const bool row_ok = row < rows;
  float v[CPT][8];
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < CPT; ++c) {
    const int col = (sub + c * R) * 8;
    if (row_ok && col < h) {
      load8(x + (int64_t)row * h + col, v[c]);
#pragma unroll
      for (int i = 0; i < 8; ++i) s += v[c][i];
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) v[c][i] = 0.f;
    }
  }
  const float mean = group_sum<R>(s, red, tid) / (float)h;
  float q = 0.f;
#pragma unroll
  for (int c = 0; c < CPT; ++c) {
    const int col = (sub + c * R) * 8;
    if (col < h) {
#pragma unroll
      for (int i = 0; i < 8; ++i) { const float d = v[c][i] - mean; q += d * d; }
    }
  }
  const float var = group_sum<R>(q, red, tid) / (float)h;
  const float rstd = 1.0f / sqrtf(var + eps);
  if (!row_ok) return;
#pragma unroll
  for (int c = 0; c < CPT; ++c) {
    const int col = (sub + c * R) * 8;
    if (col < h) {
      float g[8], b[8], o[8];
      load8(gain + col, g);
      load8(shift + col, b);
#pragma unroll
      for (int i = 0; i < 8; ++i) o[i] = g[i] * ((v[c][i] - mean) * rstd) + b[i];
      store8(y + (int64_t)row * h + col, o);
    }
  }
  if (sub == 0) { mean_out[row] = mean; rstd_out[row] = rstd; }
}

// Backward.  Workgroups stride over row groups and keep per-column sums of dy*xhat, dy and of the
// result dx in registers; each workgroup writes one row of partial[parts][3h] (dy*xhat | dy | dx).
// The third block is the bias gradient of the projection that produced this kernel's residual
// operand (its output gradient is exactly dx), so no separate pass over dx is needed for it.
template <typename T, int R, int CPT>
__global__ __launch_bounds__(kWg) void ln_bwd_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                      const float* __restrict__ mean_in, const float* __restrict__ rstd_in,
                                                      const T* __restrict__ gain, const T* __restrict__ dres,
                                                      T* __restrict__ dx, float* __restrict__ partial, int rows, int h) {
  constexpr int ROWS = kWg / R;
  __shared__ float red[4];
  __shared__ float comb[(ROWS > 1) ? (ROWS - 1) * R * CPT * 8 : 1];
  const int tid = threadIdx.x;
  const int sub = tid % R, rsub = tid / R;
  float gsum[CPT][8], bsum[CPT][8], osum[CPT][8], gn[CPT][8];
#pragma unroll
  for (int c = 0; c < CPT; ++c) {
    const int col = (sub + c * R) * 8;
    if (col < h) load8(gain + col, gn[c]);
#pragma unroll
    for (int i = 0; i < 8; ++i) { gsum[c][i] = 0.f; bsum[c][i] = 0.f; osum[c][i] = 0.f; if (col >= h) gn[c][i] = 0.f; }
  }
  // Two row groups per trip, all loads of both issued before any arithmetic: the kernel is bound
  // by memory latency, not bandwidth, at the sizes a stage gives it.
  constexpr int U = CPT <= 2 ? 2 : 1;   // (longer rows already keep enough loads in flight, and registers are short)
  const int n_groups = (rows + ROWS - 1) / ROWS;
  for (int grp0 = blockIdx.x; grp0 < n_groups; grp0 += U * gridDim.x) {
    int row[U];
    bool row_ok[U];
    float mean[U], rstd[U];
    float xh[U][CPT][8], dxh[U][CPT][8], res[U][CPT][8];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int grp = grp0 + u * gridDim.x;
      row[u] = grp * ROWS + rsub;
      row_ok[u] = grp < n_groups && row[u] < rows;
      mean[u] = row_ok[u] ? mean_in[row[u]] : 0.f;
      rstd[u] = row_ok[u] ? rstd_in[row[u]] : 0.f;
#pragma unroll
      for (int c = 0; c < CPT; ++c) {
        const int col = (sub + c * R) * 8;
        if (row_ok[u] && col < h) {
          load8(x + (int64_t)row[u] * h + col, xh[u][c]);
          load8(dy + (int64_t)row[u] * h + col, dxh[u][c]);
          if (dres) load8(dres + (int64_t)row[u] * h + col, res[u][c]);
        } else {
#pragma unroll
          for (int i = 0; i < 8; ++i) { xh[u][c][i] = 0.f; dxh[u][c][i] = 0.f; }
        }
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float s1 = 0.f, s2 = 0.f;
#pragma unroll
      for (int c = 0; c < CPT; ++c) {
        const int col = (sub + c * R) * 8;
        if (row_ok[u] && col < h) {
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const float dv = dxh[u][c][i];
            xh[u][c][i] = (xh[u][c][i] - mean[u]) * rstd[u];
            dxh[u][c][i] = dv * gn[c][i];
            s1 += dxh[u][c][i];
            s2 += dxh[u][c][i] * xh[u][c][i];
            gsum[c][i] += dv * xh[u][c][i];
            bsum[c][i] += dv;
          }
        }
      }
      const float c1 = group_sum<R>(s1, red, tid) / (float)h;
      const float c2 = group_sum<R>(s2, red, tid) / (float)h;
      if (row_ok[u]) {
#pragma unroll
        for (int c = 0; c < CPT; ++c) {
          const int col = (sub + c * R) * 8;
          if (col < h) {
            float o[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) o[i] = rstd[u] * (dxh[u][c][i] - c1 - xh[u][c][i] * c2);
            if (dres) {
#pragma unroll
              for (int i = 0; i < 8; ++i) o[i] += res[u][c][i];
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) osum[c][i] += o[i];
            store8(dx + (int64_t)row[u] * h + col, o);
          }
        }
      }
    }
  }
  // combine the ROWS sub-rows of this workgroup, then one partial row per workgroup
#pragma unroll
  for (int which = 0; which < 3; ++which) {
    if (ROWS > 1) {
      __syncthreads();
      if (rsub > 0) {
#pragma unroll
        for (int c = 0; c < CPT; ++c)
#pragma unroll
          for (int i = 0; i < 8; ++i)
            comb[(((rsub - 1) * CPT + c) * 8 + i) * R + sub] = which == 0 ? gsum[c][i] : which == 1 ? bsum[c][i] : osum[c][i];
      }
      __syncthreads();
    }
    if (rsub == 0) {
#pragma unroll
      for (int c = 0; c < CPT; ++c) {
        const int col = (sub + c * R) * 8;
        if (col < h) {
          float o[8];
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            o[i] = which == 0 ? gsum[c][i] : which == 1 ? bsum[c][i] : osum[c][i];
            for (int rr = 1; rr < ROWS; ++rr) o[i] += comb[(((rr - 1) * CPT + c) * 8 + i) * R + sub];
          }
          store8(partial + (int64_t)blockIdx.x * 3 * h + which * h + col, o);
        }
      }
    }
  }
}

// Backward for long rows (h >= 2048).  With 256 threads the per-column sums of a row of 8192 take 96
// registers per thread next to the row itself, one wave per SIMD fits, and a CU has too few loads in
// flight to keep HBM busy.  Here a workgroup has 1024 threads, R = 256, 512 or 1024 of them share a row
// with one or two 16-byte chunks each, so the sums are 24 or 48 registers and sixteen waves stay resident
// per CU.  A workgroup is alone on its CU, so nothing else hides its trips to HBM: the U rows per thread
// of the next step are requested (and held as loaded, 16 bytes per chunk) before the arithmetic of the
// current step starts, and the row sums of all U rows share one barrier (the exchange buffer alternates
// between steps, so a wave that runs ahead cannot overwrite sums that a slower one still reads).
// Same partial-row layout as the kernel above; the grid is one workgroup per CU at most.
constexpr int kWgWide = 1024;

template <typename T> struct Raw8;
template <> struct Raw8<bf16_t> { uint4 a; };
template <> struct Raw8<float> { float4 a, b; };
__device__ __forceinline__ void load_raw(const bf16_t* p, Raw8<bf16_t>& r) { r.a = *reinterpret_cast<const uint4*>(p); }
__device__ __forceinline__ void load_raw(const float* p, Raw8<float>& r) {
  r.a = *reinterpret_cast<const float4*>(p);
  r.b = *reinterpret_cast<const float4*>(p + 4);
}
__device__ __forceinline__ void unpack_raw(const Raw8<bf16_t>& r, float (&v)[8]) {
  v[0] = __uint_as_float(r.a.x << 16); v[1] = __uint_as_float(r.a.x & 0xffff0000u);
  v[2] = __uint_as_float(r.a.y << 16); v[3] = __uint_as_float(r.a.y & 0xffff0000u);
  v[4] = __uint_as_float(r.a.z << 16); v[5] = __uint_as_float(r.a.z & 0xffff0000u);
  v[6] = __uint_as_float(r.a.w << 16); v[7] = __uint_as_float(r.a.w & 0xffff0000u);
}
__device__ __forceinline__ void unpack_raw(const Raw8<float>& r, float (&v)[8]) {
  v[0] = r.a.x; v[1] = r.a.y; v[2] = r.a.z; v[3] = r.a.w;
  v[4] = r.b.x; v[5] = r.b.y; v[6] = r.b.z; v[7] = r.b.w;
}

template <typename T, int R, int CPT, int U>
__global__ __launch_bounds__(kWgWide) void ln_bwd_wide_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                              const float* __restrict__ mean_in,
                                                              const float* __restrict__ rstd_in, const T* __restrict__ gain,
                                                              const T* __restrict__ dres, T* __restrict__ dx,
                                                              float* __restrict__ partial, int rows, int h) {
  constexpr int ROWS = kWgWide / R;
  constexpr int W = R / 64;   // waves per row
  // Requesting a step ahead costs 12 registers per chunk next to the 24 of the column sums; the budget of a
  // 1024-thread workgroup is 128, so it is done for 2-byte elements with one chunk per thread; with one chunk
  // per thread the sums of the results live in LDS (one 16-byte slot per thread and column quad, touched by
  // its owner only).
  constexpr bool kAhead = sizeof(T) == 2 && CPT == 1;
  constexpr bool kLdsSums = CPT == 1;
  __shared__ float red[2][2 * U][16];
  __shared__ float4 osum_lds[kLdsSums ? 2 * kWgWide : 1];
  __shared__ float comb[(ROWS > 1) ? (ROWS - 1) * R * CPT * 8 : 1];
  const int tid = threadIdx.x;
  const int sub = tid % R, rsub = tid / R;
  const int wave = tid >> 6, first_wave = (wave / W) * W;
  float gsum[CPT][8], bsum[CPT][8], osum[CPT][8], gn[CPT][8];
#pragma unroll
  for (int c = 0; c < CPT; ++c) {
    const int col = (sub + c * R) * 8;
    if (col < h) load8(gain + col, gn[c]);
#pragma unroll
    for (int i = 0; i < 8; ++i) { gsum[c][i] = 0.f; bsum[c][i] = 0.f; osum[c][i] = 0.f; if (col >= h) gn[c][i] = 0.f; }
  }
  const int n_groups = (rows + ROWS - 1) / ROWS;
  const int stride = U * gridDim.x;
  // the rows of the step after the one being worked on, as loaded
  Raw8<T> nx[U][CPT], ndy[U][CPT], nres[U][CPT];
  float nmean[U], nrstd[U];
  auto fetch = [&](int grp0) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int grp = grp0 + u * gridDim.x;
      const int row = grp * ROWS + rsub;
      const bool ok = grp < n_groups && row < rows;
      nmean[u] = ok ? mean_in[row] : 0.f;
      nrstd[u] = ok ? rstd_in[row] : 0.f;
#pragma unroll
      for (int c = 0; c < CPT; ++c) {
        const int col = (sub + c * R) * 8;
        if (ok && col < h) {
          load_raw(x + (int64_t)row * h + col, nx[u][c]);
          load_raw(dy + (int64_t)row * h + col, ndy[u][c]);
          if (dres) load_raw(dres + (int64_t)row * h + col, nres[u][c]);
          else nres[u][c] = Raw8<T>{};
        } else {
          nx[u][c] = Raw8<T>{}; ndy[u][c] = Raw8<T>{}; nres[u][c] = Raw8<T>{};
        }
      }
    }
  };
  if (kLdsSums) {
    osum_lds[tid] = make_float4(0.f, 0.f, 0.f, 0.f);
    osum_lds[kWgWide + tid] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
  if (kAhead && (int)blockIdx.x < n_groups) fetch(blockIdx.x);
  int parity = 0;
  for (int grp0 = blockIdx.x; grp0 < n_groups; grp0 += stride) {
    if (!kAhead) fetch(grp0);
    int row[U];
    bool row_ok[U];
    float mean[U], rstd[U];
    float xh[U][CPT][8], dxh[U][CPT][8];
    Raw8<T> res[U][CPT];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int grp = grp0 + u * gridDim.x;
      row[u] = grp * ROWS + rsub;
      row_ok[u] = grp < n_groups && row[u] < rows;
      mean[u] = nmean[u];
      rstd[u] = nrstd[u];
#pragma unroll
      for (int c = 0; c < CPT; ++c) {
        const int col = (sub + c * R) * 8;
        if (row_ok[u] && col < h) {
          unpack_raw(nx[u][c], xh[u][c]);
          unpack_raw(ndy[u][c], dxh[u][c]);
          res[u][c] = nres[u][c];
        } else {
#pragma unroll
          for (int i = 0; i < 8; ++i) { xh[u][c][i] = 0.f; dxh[u][c][i] = 0.f; }
        }
      }
    }
    if (kAhead && grp0 + stride < n_groups) fetch(grp0 + stride);
    float s1[U], s2[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      s1[u] = 0.f; s2[u] = 0.f;
#pragma unroll
      for (int c = 0; c < CPT; ++c) {
        const int col = (sub + c * R) * 8;
        if (row_ok[u] && col < h) {
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const float dv = dxh[u][c][i];
            xh[u][c][i] = (xh[u][c][i] - mean[u]) * rstd[u];
            dxh[u][c][i] = dv * gn[c][i];
            s1[u] += dxh[u][c][i];
            s2[u] += dxh[u][c][i] * xh[u][c][i];
            gsum[c][i] += dv * xh[u][c][i];
            bsum[c][i] += dv;
          }
        }
      }
      s1[u] = wave_sum(s1[u]);
      s2[u] = wave_sum(s2[u]);
    }
    if ((tid & 63) == 0) {
#pragma unroll
      for (int u = 0; u < U; ++u) { red[parity][2 * u][wave] = s1[u]; red[parity][2 * u + 1][wave] = s2[u]; }
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float a = 0.f, b = 0.f;
#pragma unroll
      for (int i = 0; i < W; ++i) { a += red[parity][2 * u][first_wave + i]; b += red[parity][2 * u + 1][first_wave + i]; }
      const float c1 = a / (float)h, c2 = b / (float)h;
      if (row_ok[u]) {
#pragma unroll
        for (int c = 0; c < CPT; ++c) {
          const int col = (sub + c * R) * 8;
          if (col < h) {
            float o[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) o[i] = rstd[u] * (dxh[u][c][i] - c1 - xh[u][c][i] * c2);
            if (dres) {
              float rv[8];
              unpack_raw(res[u][c], rv);
#pragma unroll
              for (int i = 0; i < 8; ++i) o[i] += rv[i];
            }
            if (kLdsSums) {
              float4 lo = osum_lds[tid], hi = osum_lds[kWgWide + tid];
              lo.x += o[0]; lo.y += o[1]; lo.z += o[2]; lo.w += o[3];
              hi.x += o[4]; hi.y += o[5]; hi.z += o[6]; hi.w += o[7];
              osum_lds[tid] = lo; osum_lds[kWgWide + tid] = hi;
            } else {
#pragma unroll
              for (int i = 0; i < 8; ++i) osum[c][i] += o[i];
            }
            store8(dx + (int64_t)row[u] * h + col, o);
          }
        }
      }
    }
    parity ^= 1;
  }
  if (kLdsSums) {
    const float4 lo = osum_lds[tid], hi = osum_lds[kWgWide + tid];
    osum[0][0] = lo.x; osum[0][1] = lo.y; osum[0][2] = lo.z; osum[0][3] = lo.w;
    osum[0][4] = hi.x; osum[0][5] = hi.y; osum[0][6] = hi.z; osum[0][7] = hi.w;
  }
  // combine the ROWS sub-rows of this workgroup, then one partial row per workgroup
#pragma unroll
  for (int which = 0; which < 3; ++which) {
    if (ROWS > 1) {
      __syncthreads();
      if (rsub > 0) {
#pragma unroll
        for (int c = 0; c < CPT; ++c)
#pragma unroll
          for (int i = 0; i < 8; ++i)
            comb[(((rsub - 1) * CPT + c) * 8 + i) * R + sub] = which == 0 ? gsum[c][i] : which == 1 ? bsum[c][i] : osum[c][i];
      }
      __syncthreads();
    }
    if (rsub == 0) {
#pragma unroll
      for (int c = 0; c < CPT; ++c) {
        const int col = (sub + c * R) * 8;
        if (col < h) {
          float o[8];
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            o[i] = which == 0 ? gsum[c][i] : which == 1 ? bsum[c][i] : osum[c][i];
            for (int rr = 1; rr < ROWS; ++rr) o[i] += comb[(((rr - 1) * CPT + c) * 8 + i) * R + sub];
          }
          store8(partial + (int64_t)blockIdx.x * 3 * h + which * h + col, o);
        }
      }
    }
  }
}

template <typename T>
__global__ __launch_bounds__(kWg) void colsum_partial_kernel(const T* __restrict__ y, int rows, int n, int ld,
                                                              float* __restrict__ partial, int rows_per_part) {
  __shared__ float comb[7][8][32];
  const int tid = threadIdx.x;
  const int cc = tid % 32, rl = tid / 32;      // column chunk, row lane
  const int col = (blockIdx.x * 32 + cc) * 8;
  const int r0 = blockIdx.y * rows_per_part;
  const int r1 = min(rows, r0 + rows_per_part);
  float s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (col < n) {
    for (int r = r0 + rl; r < r1; r += 8) {
      float v[8];
      load8(y + (int64_t)r * ld + col, v);
#pragma unroll
      for (int i = 0; i < 8; ++i) s[i] += v[i];
    }
  }
  if (rl > 0) {
#pragma unroll
    for (int i = 0; i < 8; ++i) comb[rl - 1][i][cc] = s[i];
  }
  __syncthreads();
  if (rl == 0 && col < n) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int rr = 0; rr < 7; ++rr) s[i] += comb[rr][i][cc];
    store8(partial + (int64_t)blockIdx.y * n + col, s);
  }
}

// 16 columns x 16 part-lanes per workgroup: 64-byte segments per part row, 8 loads in flight per
// thread, then an LDS tree over the part-lanes.
__global__ __launch_bounds__(kWg) void colsum_finalize_kernel(const float* __restrict__ partial, int parts, int n,
                                                               int ld, float* __restrict__ out, int accumulate) {
  __shared__ float red[16][17];
  const int c = threadIdx.x & 15, pl = threadIdx.x >> 4;
  const int col = blockIdx.x * 16 + c;
  float s = 0.f;
  if (col < n) {
    int p = pl;
    for (; p + 7 * 16 < parts; p += 8 * 16) {
      float v[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = partial[(int64_t)(p + i * 16) * ld + col];
#pragma unroll
      for (int i = 0; i < 8; ++i) s += v[i];
    }
    for (; p < parts; p += 16) s += partial[(int64_t)p * ld + col];
  }
  red[pl][c] = s;
  __syncthreads();
  if (pl == 0 && col < n) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) t += red[i][c];
    out[col] = accumulate ? out[col] + t : t;
  }
}

// Column sums of up to 4 matrices with the same row count in one launch: blockIdx.x walks the
// 256-column blocks of all segments, blockIdx.y the row slabs.  partial is [parts][total_cols]:
// segment s owns columns [col0_s, col0_s + n_s).
template <typename T>
__global__ __launch_bounds__(kWg) void colsum_partial_grouped_kernel(ColsumGroup g) {
  __shared__ float comb[7][8][32];
  int sidx = 0;
#pragma unroll
  for (int q = 1; q < 4; ++q)
    if (q < g.count && (int)blockIdx.x >= g.block0[q]) sidx = q;
  const T* y = static_cast<const T*>(g.y[sidx]);
  const int n = g.n[sidx], ld = g.ld[sidx];
  const int tid = threadIdx.x;
  const int cc = tid % 32, rl = tid / 32;
  const int col = ((blockIdx.x - g.block0[sidx]) * 32 + cc) * 8;
  const int r0 = blockIdx.y * g.rows_per_part;
  const int r1 = min(g.rows, r0 + g.rows_per_part);
  float s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (col < n) {
    for (int r = r0 + rl; r < r1; r += 8) {
      float v[8];
      load8(y + (int64_t)r * ld + col, v);
#pragma unroll
      for (int i = 0; i < 8; ++i) s[i] += v[i];
    }
  }
  if (rl > 0) {
#pragma unroll
    for (int i = 0; i < 8; ++i) comb[rl - 1][i][cc] = s[i];
  }
  __syncthreads();
  if (rl == 0 && col < n) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int rr = 0; rr < 7; ++rr) s[i] += comb[rr][i][cc];
    store8(g.partial + (int64_t)blockIdx.y * g.total_cols + g.col0[sidx] + col, s);
  }
}

// out_s[n_s] (+)= sum over parts_s rows of partial_s, for up to kFinalizeMaxItems segments in one launch.
// A workgroup owns 64 columns: 16 threads x 16 bytes cover 256 contiguous bytes of a row (whole cache lines; with
// one float per thread a workgroup used half of every line it touched), 16 such groups walk the rows.
__global__ __launch_bounds__(kWg) void colsum_finalize_grouped_kernel(FinalizeGroup g) {
  __shared__ float4 red[16][17];
  int sidx = 0;
  for (int q = 1; q < g.count; ++q)
    if ((int)blockIdx.x >= g.block0[q]) sidx = q;
  const float* partial = g.partial[sidx];
  const int parts = g.parts[sidx], n = g.n[sidx], ld = g.ld[sidx];
  const int c = threadIdx.x & 15, pl = threadIdx.x >> 4;
  const int col = ((blockIdx.x - g.block0[sidx]) * 16 + c) * 4;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  if (col < n) {
    int p = pl;
    for (; p + 7 * 16 < parts; p += 8 * 16) {
      float4 v[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = *reinterpret_cast<const float4*>(partial + (int64_t)(p + i * 16) * ld + col);
#pragma unroll
      for (int i = 0; i < 8; ++i) { s.x += v[i].x; s.y += v[i].y; s.z += v[i].z; s.w += v[i].w; }
    }
    for (; p < parts; p += 16) {
      const float4 v = *reinterpret_cast<const float4*>(partial + (int64_t)p * ld + col);
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
  }
  red[pl][c] = s;
  __syncthreads();
  if (pl == 0 && col < n) {
    float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int i = 0; i < 16; ++i) { const float4 v = red[i][c]; t.x += v.x; t.y += v.y; t.z += v.z; t.w += v.w; }
    float4* out = reinterpret_cast<float4*>(g.out[sidx] + col);
    if (g.accumulate) { const float4 o = *out; t.x += o.x; t.y += o.y; t.z += o.z; t.w += o.w; }
    *out = t;
  }
}

// R, CPT for a row length: the fewest threads per row that keep CPT <= 4, else up to 8.
struct RowShape { int R, CPT; };
RowShape row_shape(int h) {
  const int chunks = h / 8;
  for (int R : {64, 128, 256}) {
    const int cpt = (chunks + R - 1) / R;
    if (cpt <= 4) return {R, cpt};
  }
  return {256, (chunks + 255) / 256};
}

#define LN_DISPATCH(KERNEL_CALL)                                             \
  switch (rs.R * 16 + rs.CPT) {                                              \
    case 64 * 16 + 1: KERNEL_CALL(64, 1); break;                             \
    case 64 * 16 + 2: KERNEL_CALL(64, 2); break;                             \
    case 64 * 16 + 3: KERNEL_CALL(64, 3); break;                             \
    case 64 * 16 + 4: KERNEL_CALL(64, 4); break;                             \
    case 128 * 16 + 3: KERNEL_CALL(128, 3); break;                           \
    case 128 * 16 + 4: KERNEL_CALL(128, 4); break;                           \
    case 256 * 16 + 3: KERNEL_CALL(256, 3); break;                           \
    case 256 * 16 + 4: KERNEL_CALL(256, 4); break;                           \
    case 256 * 16 + 5: KERNEL_CALL(256, 5); break;                           \
    case 256 * 16 + 6: KERNEL_CALL(256, 6); break;                           \
    case 256 * 16 + 7: KERNEL_CALL(256, 7); break;                           \
    case 256 * 16 + 8: KERNEL_CALL(256, 8); break;                           \
    default: return hipErrorInvalidValue;                                    \
  }

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

}  // namespace

hipError_t layernorm_fwd(const void* x, const void* gain, const void* shift, void* y, float* mean,
                         float* rstd, int rows, int h, float eps, int dtype, hipStream_t stream) {
  if (rows <= 0 || h <= 0 || h % 8 || h > 16384 || !x || !y || !gain || !shift || !mean || !rstd)
    return hipErrorInvalidValue;
  if (!aligned16(x) || !aligned16(y) || !aligned16(gain) || !aligned16(shift)) return hipErrorInvalidValue;
  const RowShape rs = row_shape(h);
  const int grid = ceil_div(rows, kWg / rs.R);
#define CALL_FWD(R_, C_)                                                                                  \
  if (dtype == kBF16)                                                                                     \
    hipLaunchKernelGGL((ln_fwd_kernel<bf16_t, R_, C_>), dim3(grid), dim3(kWg), 0, stream,                 \
                       static_cast<const bf16_t*>(x), static_cast<const bf16_t*>(gain),                   \
                       static_cast<const bf16_t*>(shift), static_cast<bf16_t*>(y), mean, rstd,            \
                       rows, h, eps);                                                                     \
  else                                                                                                    \
    hipLaunchKernelGGL((ln_fwd_kernel<float, R_, C_>), dim3(grid), dim3(kWg), 0, stream,                  \
                       static_cast<const float*>(x), static_cast<const float*>(gain),                     \
                       static_cast<const float*>(shift), static_cast<float*>(y), mean, rstd,              \
                       rows, h, eps)
  LN_DISPATCH(CALL_FWD)
#undef CALL_FWD
  return hipGetLastError();
}

int ln_bwd_max_parts() { return 512; }

hipError_t layernorm_bwd(const void* dy, const void* x, const float* mean, const float* rstd,
                         const void* gain, const void* dres, void* dx, float* partial, int* parts_out,
                         int rows, int h, int dtype, hipStream_t stream) {
  if (rows <= 0 || h <= 0 || h % 8 || h > 16384 || !dy || !x || !mean || !rstd || !gain || !dx || !partial ||
      !parts_out)
    return hipErrorInvalidValue;
  if (!aligned16(dy) || !aligned16(x) || !aligned16(dx) || !aligned16(gain) || !aligned16(partial) ||
      (dres && !aligned16(dres)))
    return hipErrorInvalidValue;
  if (h >= 2048) {
    // long rows: 1024-thread workgroups, at most one per CU (256 partial rows)
    const int chunks = h / 8;
    const int R = chunks <= 256 ? 256 : chunks <= 512 ? 512 : 1024;
    const int cpt = ceil_div(chunks, R);   // 1, or 2 above h = 8192 (h <= 16384)
    const int groups = ceil_div(rows, kWgWide / R);
    const int grid = groups < 256 ? groups : 256;
#define CALL_WIDE(R_, C_, U_)                                                                                \
  if (dtype == kBF16)                                                                                        \
    hipLaunchKernelGGL((ln_bwd_wide_kernel<bf16_t, R_, C_, U_>), dim3(grid), dim3(kWgWide), 0, stream,       \
                       static_cast<const bf16_t*>(dy), static_cast<const bf16_t*>(x), mean, rstd,            \
                       static_cast<const bf16_t*>(gain),                                                     \
                       static_cast<const bf16_t*>(dres), static_cast<bf16_t*>(dx), partial, rows, h);        \
  else                                                                                                       \
    hipLaunchKernelGGL((ln_bwd_wide_kernel<float, R_, C_, U_>), dim3(grid), dim3(kWgWide), 0, stream,        \
                       static_cast<const float*>(dy), static_cast<const float*>(x), mean, rstd,              \
                       static_cast<const float*>(gain),                                                      \
                       static_cast<const float*>(dres), static_cast<float*>(dx), partial, rows, h)
    if (cpt == 1 && R == 256) { CALL_WIDE(256, 1, 2); }
    else if (cpt == 1 && R == 512) { CALL_WIDE(512, 1, 2); }
    else if (cpt == 1) { CALL_WIDE(1024, 1, 2); }
    else if (cpt == 2) { CALL_WIDE(1024, 2, 1); }
    else return hipErrorInvalidValue;
#undef CALL_WIDE
    *parts_out = grid;
    return hipGetLastError();
  }
  const RowShape rs = row_shape(h);
  const int groups = ceil_div(rows, kWg / rs.R);
  const int grid = groups < ln_bwd_max_parts() ? groups : ln_bwd_max_parts();
#define CALL_BWD(R_, C_)                                                                                    \
  if (dtype == kBF16)                                                                                       \
    hipLaunchKernelGGL((ln_bwd_kernel<bf16_t, R_, C_>), dim3(grid), dim3(kWg), 0, stream,                   \
                       static_cast<const bf16_t*>(dy), static_cast<const bf16_t*>(x), mean, rstd,           \
                       static_cast<const bf16_t*>(gain),                                                    \
                       static_cast<const bf16_t*>(dres), static_cast<bf16_t*>(dx), partial, rows, h);       \
  else                                                                                                      \
    hipLaunchKernelGGL((ln_bwd_kernel<float, R_, C_>), dim3(grid), dim3(kWg), 0, stream,                    \
                       static_cast<const float*>(dy), static_cast<const float*>(x), mean, rstd,             \
                       static_cast<const float*>(gain),                                                     \
                       static_cast<const float*>(dres), static_cast<float*>(dx), partial, rows, h)
  LN_DISPATCH(CALL_BWD)
#undef CALL_BWD
  *parts_out = grid;
  return hipGetLastError();
}

int colsum_max_parts() { return 64; }

hipError_t colsum_partial(const void* y, int rows, int n, int ldy, float* partial, int* parts_out, int dtype,
                          hipStream_t stream) {
  if (rows <= 0 || n <= 0 || n % 8 || ldy % 8 || ldy < n || !y || !partial || !parts_out) return hipErrorInvalidValue;
  if (!aligned16(y) || !aligned16(partial)) return hipErrorInvalidValue;
  int parts = ceil_div(rows, 64);
  if (parts > colsum_max_parts()) parts = colsum_max_parts();
  const int rows_per_part = ceil_div(rows, parts);
  parts = ceil_div(rows, rows_per_part);
  dim3 grid(ceil_div(n, 256), parts);
  if (dtype == kBF16)
    hipLaunchKernelGGL((colsum_partial_kernel<bf16_t>), grid, dim3(kWg), 0, stream, static_cast<const bf16_t*>(y),
                       rows, n, ldy, partial, rows_per_part);
  else
    hipLaunchKernelGGL((colsum_partial_kernel<float>), grid, dim3(kWg), 0, stream, static_cast<const float*>(y),
                       rows, n, ldy, partial, rows_per_part);
  *parts_out = parts;
  return hipGetLastError();
}

hipError_t colsum_finalize(const float* partial, int parts, int n, float* out, bool accumulate,
                           hipStream_t stream) {
  if (parts <= 0 || n <= 0 || !partial || !out) return hipErrorInvalidValue;
  hipLaunchKernelGGL(colsum_finalize_kernel, dim3(ceil_div(n, 16)), dim3(kWg), 0, stream, partial, parts, n, n, out,
                     accumulate ? 1 : 0);
  return hipGetLastError();
}

hipError_t colsum_partial_grouped(const ColsumItem* items, int count, int rows, float* partial, int* parts_out,
                                  int* total_cols_out, int dtype, hipStream_t stream) {
  if (!items || count < 1 || count > 4 || rows <= 0 || !partial || !parts_out || !total_cols_out || !aligned16(partial))
    return hipErrorInvalidValue;
  ColsumGroup g{};
  g.count = count;
  int blocks = 0, cols = 0;
  for (int i = 0; i < count; ++i) {
    const ColsumItem& it = items[i];
    if (!it.y || it.n <= 0 || it.n % 8 || it.ld % 8 || it.ld < it.n || !aligned16(it.y)) return hipErrorInvalidValue;
    g.y[i] = it.y; g.n[i] = it.n; g.ld[i] = it.ld; g.block0[i] = blocks; g.col0[i] = cols;
    blocks += ceil_div(it.n, 256);
    cols += it.n;
  }
  int parts = ceil_div(rows, 64);
  if (parts > colsum_max_parts()) parts = colsum_max_parts();
  g.rows = rows;
  g.rows_per_part = ceil_div(rows, parts);
  parts = ceil_div(rows, g.rows_per_part);
  g.total_cols = cols;
  g.partial = partial;
  dim3 grid(blocks, parts);
  if (dtype == kBF16)
    hipLaunchKernelGGL((colsum_partial_grouped_kernel<bf16_t>), grid, dim3(kWg), 0, stream, g);
  else
    hipLaunchKernelGGL((colsum_partial_grouped_kernel<float>), grid, dim3(kWg), 0, stream, g);
  *parts_out = parts;
  *total_cols_out = cols;
  return hipGetLastError();
}

hipError_t colsum_finalize_grouped(const FinalizeItem* items, int count, bool accumulate, hipStream_t stream) {
  if (!items || count < 1 || count > kFinalizeMaxItems) return hipErrorInvalidValue;
  FinalizeGroup g{};
  g.count = count;
  g.accumulate = accumulate ? 1 : 0;
  int blocks = 0;
  for (int i = 0; i < count; ++i) {
    const FinalizeItem& it = items[i];
    if (!it.partial || !it.out || it.parts <= 0 || it.n <= 0 || it.ld < it.n) return hipErrorInvalidValue;
    if (it.n % 4 || it.ld % 4 || !aligned16(it.partial) || !aligned16(it.out)) return hipErrorInvalidValue;   // 16-byte accesses
    g.partial[i] = it.partial; g.parts[i] = it.parts; g.n[i] = it.n; g.ld[i] = it.ld; g.out[i] = it.out;
    g.block0[i] = blocks;
    blocks += ceil_div(it.n, 64);
  }
  hipLaunchKernelGGL(colsum_finalize_grouped_kernel, dim3(blocks), dim3(kWg), 0, stream, g);
  return hipGetLastError();
}

}  // namespace k2bw
