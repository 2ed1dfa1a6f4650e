// Fused coalesce + Adam update writing the other weight buffer, and dtype conversions.
// HBM-bound: 16-byte accesses, one pass front to back (no grid-stride loop), every byte touched once.
//   fp32 mode: read W(t), m, v, G (16 B/param); write W(t+1), m, v (12 B/param).
//   bf16 mode: read master, m, v, G (16 B); write master, m, v, bf16 W(t+1) (14 B).
#include "kernels.hpp"

namespace k2bw {
namespace {

// One workgroup per 512 consecutive float4 (two per thread), no grid-stride loop: measured on
// MI355X, a grid that simply walks memory front to back sustains 5.4 TB/s on this 16-byte-read /
// 14-byte-write mix, against 4.4..4.7 TB/s for a capped grid with a strided loop (non-temporal
// hints, deeper unrolling and workgroup-contiguous ranges made no difference).
constexpr int kAdamPerThread = 2;
template <bool LP>
__global__ __launch_bounds__(256) void adam_kernel(AdamDesc d) {
  const int64_t n4 = d.n / 4;
  const int64_t base = (int64_t)blockIdx.x * (256 * kAdamPerThread) + threadIdx.x;
  const float omb1 = d.omb1, omb2 = d.omb2;
  float4 w[kAdamPerThread], m[kAdamPerThread], v[kAdamPerThread], gs[kAdamPerThread];
#pragma unroll
  for (int u = 0; u < kAdamPerThread; ++u) {
    const int64_t i = base + u * 256;
    if (i < n4) {
      w[u] = reinterpret_cast<const float4*>(d.w_cur)[i];
      m[u] = reinterpret_cast<const float4*>(d.m)[i];
      v[u] = reinterpret_cast<const float4*>(d.v)[i];
      gs[u] = reinterpret_cast<const float4*>(d.G)[i];
    }
  }
#pragma unroll
  for (int u = 0; u < kAdamPerThread; ++u) {
    const int64_t i = base + u * 256;
    if (i >= n4) continue;
    float wv[4] = {w[u].x, w[u].y, w[u].z, w[u].w}, mv[4] = {m[u].x, m[u].y, m[u].z, m[u].w};
    float vv[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
    const float gv[4] = {gs[u].x, gs[u].y, gs[u].z, gs[u].w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float g = gv[k] * d.inv_m;
      mv[k] = d.beta1 * mv[k] + omb1 * g;
      vv[k] = d.beta2 * vv[k] + omb2 * g * g;
      wv[k] = wv[k] - d.lr * (mv[k] * d.c1) / (sqrtf(vv[k] * d.c2) + d.eps);
    }
    reinterpret_cast<float4*>(d.m)[i] = make_float4(mv[0], mv[1], mv[2], mv[3]);
    reinterpret_cast<float4*>(d.v)[i] = make_float4(vv[0], vv[1], vv[2], vv[3]);
    reinterpret_cast<float4*>(d.w_next)[i] = make_float4(wv[0], wv[1], wv[2], wv[3]);
    if (LP) reinterpret_cast<uint2*>(d.w_next_lp)[i] = make_uint2(pack_bf16x2(wv[0], wv[1]), pack_bf16x2(wv[2], wv[3]));
  }
}

// SGD with momentum in the form Section 3.1 prints: m <- beta m + (1 - beta) g, W(t+1) = W(t) - lr m,
// with g = G / m_micro the coalesced 1-stale gradient; no bias correction, no second moment.
// 12 B/param read, 8 (+2 bf16) written.
template <bool LP>
__global__ __launch_bounds__(256) void momentum_kernel(AdamDesc d) {
  const int64_t n4 = d.n / 4;
  const int64_t base = (int64_t)blockIdx.x * (256 * kAdamPerThread) + threadIdx.x;
  const float omb1 = d.omb1;
#pragma unroll
  for (int u = 0; u < kAdamPerThread; ++u) {
    const int64_t i = base + u * 256;
    if (i >= n4) continue;
    const float4 w = reinterpret_cast<const float4*>(d.w_cur)[i];
    const float4 m = reinterpret_cast<const float4*>(d.m)[i];
    const float4 gs = reinterpret_cast<const float4*>(d.G)[i];
    float wv[4] = {w.x, w.y, w.z, w.w}, mv[4] = {m.x, m.y, m.z, m.w};
    const float gv[4] = {gs.x, gs.y, gs.z, gs.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      mv[k] = d.beta1 * mv[k] + omb1 * (gv[k] * d.inv_m);
      wv[k] = wv[k] - d.lr * mv[k];
    }
    reinterpret_cast<float4*>(d.m)[i] = make_float4(mv[0], mv[1], mv[2], mv[3]);
    reinterpret_cast<float4*>(d.w_next)[i] = make_float4(wv[0], wv[1], wv[2], wv[3]);
    if (LP) reinterpret_cast<uint2*>(d.w_next_lp)[i] = make_uint2(pack_bf16x2(wv[0], wv[1]), pack_bf16x2(wv[2], wv[3]));
  }
}

__global__ __launch_bounds__(256) void f32_to_bf16_kernel(const float* __restrict__ in, bf16_t* __restrict__ out,
                                                           int64_t n4) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
    const float4 a = reinterpret_cast<const float4*>(in)[i];
    reinterpret_cast<uint2*>(out)[i] = make_uint2(pack_bf16x2(a.x, a.y), pack_bf16x2(a.z, a.w));
  }
}

__global__ __launch_bounds__(256) void bf16_to_f32_kernel(const bf16_t* __restrict__ in, float* __restrict__ out,
                                                           int64_t n4) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
    const uint2 a = reinterpret_cast<const uint2*>(in)[i];
    reinterpret_cast<float4*>(out)[i] =
        make_float4(__uint_as_float(a.x << 16), __uint_as_float(a.x & 0xffff0000u), __uint_as_float(a.y << 16),
                    __uint_as_float(a.y & 0xffff0000u));
  }
}

__global__ __launch_bounds__(256) void copy16_kernel(const uint4* __restrict__ in, uint4* __restrict__ out, int64_t n16) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;   // one element per thread (see adam_kernel)
  if (i < n16) out[i] = in[i];
}

// dy = (y - target) * scale: the gradient of scale/2 * sum (y - target)^2, the loss the last stage of a
// multi-stage run applies to its output; 8 elements (bf16) or 4 (fp32) per thread.
template <typename T>
__global__ __launch_bounds__(256) void squared_error_grad_kernel(const T* __restrict__ y, const T* __restrict__ target,
                                                                  T* __restrict__ dy, float scale, int64_t n) {
  constexpr int V = Act<T>::kVec;
  const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * V;
  if (i >= n) return;
  float a[8], b[8], o[8];
  if (V == 8) {
    load8(reinterpret_cast<const bf16_t*>(y) + i, a);
    load8(reinterpret_cast<const bf16_t*>(target) + i, b);
#pragma unroll
    for (int k = 0; k < 8; ++k) o[k] = (a[k] - b[k]) * scale;
    store8(reinterpret_cast<bf16_t*>(dy) + i, o);
  } else {
    const float4 ya = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(y) + i);
    const float4 tb = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(target) + i);
    *reinterpret_cast<float4*>(reinterpret_cast<float*>(dy) + i) =
        make_float4((ya.x - tb.x) * scale, (ya.y - tb.y) * scale, (ya.z - tb.z) * scale, (ya.w - tb.w) * scale);
  }
}

// Transposes of up to kTransposeMaxItems bf16 matrices in one launch: dst[c][r] = src[r][c] for src [rows][cols]
// (both multiples of 8).  A workgroup moves one 64 x 64 tile through LDS: 16-byte loads along the source rows,
// 16-byte stores along the destination rows.
struct TransposeGroup {
  const bf16_t* src[kTransposeMaxItems];
  bf16_t* dst[kTransposeMaxItems];
  int rows[kTransposeMaxItems], cols[kTransposeMaxItems], tiles_c[kTransposeMaxItems], tile0[kTransposeMaxItems];
  int count;
};
__global__ __launch_bounds__(256) void transpose_bf16_grouped_kernel(TransposeGroup g) {
  __shared__ bf16_t tile[64][64 + 2];
  int q = 0;
  for (int i = 1; i < g.count; ++i)
    if ((int)blockIdx.x >= g.tile0[i]) q = i;
  const bf16_t* __restrict__ src = g.src[q];
  bf16_t* __restrict__ dst = g.dst[q];
  const int rows = g.rows[q], cols = g.cols[q];
  const int t = blockIdx.x - g.tile0[q];
  const int r0 = (t / g.tiles_c[q]) * 64, c0 = (t % g.tiles_c[q]) * 64;
  const int tid = threadIdx.x;
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    const int idx = tid + it * 256;          // 64 rows x 8 chunks of 8 elements
    const int r = idx / 8, c8 = (idx % 8) * 8;
    if (r0 + r < rows && c0 + c8 < cols) {
      const uint4 v = *reinterpret_cast<const uint4*>(src + (int64_t)(r0 + r) * cols + c0 + c8);
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        tile[r][c8 + 2 * i] = (bf16_t)(w[i] & 0xffffu);
        tile[r][c8 + 2 * i + 1] = (bf16_t)(w[i] >> 16);
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    const int idx = tid + it * 256;          // 64 destination rows (source columns) x 8 chunks
    const int c = idx / 8, r8 = (idx % 8) * 8;
    if (c0 + c < cols && r0 + r8 < rows) {
      uint32_t w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) w[i] = (uint32_t)tile[r8 + 2 * i][c] | ((uint32_t)tile[r8 + 2 * i + 1][c] << 16);
      *reinterpret_cast<uint4*>(dst + (int64_t)(c0 + c) * rows + r0 + r8) = make_uint4(w[0], w[1], w[2], w[3]);
    }
  }
}

int stream_grid(int64_t items) {
  // enough workgroups to cover 256 CUs several times over, capped so the grid-stride loop does the rest
  int64_t g = (items + 255) / 256;
  if (g > 256 * 16) g = 256 * 16;
  if (g < 1) g = 1;
  return static_cast<int>(g);
}
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

}  // namespace

hipError_t adam_step(const AdamDesc& d_in, hipStream_t stream) {
  AdamDesc d = d_in;
  d.omb1 = (float)(1.0 - (double)d.beta1);
  d.omb2 = (float)(1.0 - (double)d.beta2);
  if (d.n <= 0 || d.n % 4 || !d.w_cur || !d.w_next || !d.m || !d.v || !d.G) return hipErrorInvalidValue;
  if (!aligned16(d.w_cur) || !aligned16(d.w_next) || !aligned16(d.m) || !aligned16(d.v) || !aligned16(d.G) ||
      (reinterpret_cast<uintptr_t>(d.w_next_lp) & 7))
    return hipErrorInvalidValue;
  const int64_t blocks = (d.n / 4 + 256 * kAdamPerThread - 1) / (256 * kAdamPerThread);
  if (blocks > 0x7fffffff) return hipErrorInvalidValue;
  const int grid = (int)blocks;
  if (d.w_next_lp)
    hipLaunchKernelGGL(adam_kernel<true>, dim3(grid), dim3(256), 0, stream, d);
  else
    hipLaunchKernelGGL(adam_kernel<false>, dim3(grid), dim3(256), 0, stream, d);
  return hipGetLastError();
}

hipError_t momentum_step(const AdamDesc& d_in, hipStream_t stream) {
  AdamDesc d = d_in;
  d.omb1 = (float)(1.0 - (double)d.beta1);
  if (d.n <= 0 || d.n % 4 || !d.w_cur || !d.w_next || !d.m || !d.G) return hipErrorInvalidValue;
  if (!aligned16(d.w_cur) || !aligned16(d.w_next) || !aligned16(d.m) || !aligned16(d.G) ||
      (reinterpret_cast<uintptr_t>(d.w_next_lp) & 7))
    return hipErrorInvalidValue;
  const int64_t blocks = (d.n / 4 + 256 * kAdamPerThread - 1) / (256 * kAdamPerThread);
  if (blocks > 0x7fffffff) return hipErrorInvalidValue;
  if (d.w_next_lp)
    hipLaunchKernelGGL(momentum_kernel<true>, dim3((int)blocks), dim3(256), 0, stream, d);
  else
    hipLaunchKernelGGL(momentum_kernel<false>, dim3((int)blocks), dim3(256), 0, stream, d);
  return hipGetLastError();
}

hipError_t convert_f32_to_bf16(const float* in, bf16_t* out, int64_t n, hipStream_t stream) {
  if (n <= 0 || n % 4 || !in || !out || !aligned16(in) || (reinterpret_cast<uintptr_t>(out) & 7))
    return hipErrorInvalidValue;
  hipLaunchKernelGGL(f32_to_bf16_kernel, dim3(stream_grid(n / 4)), dim3(256), 0, stream, in, out, n / 4);
  return hipGetLastError();
}

hipError_t convert_bf16_to_f32(const bf16_t* in, float* out, int64_t n, hipStream_t stream) {
  if (n <= 0 || n % 4 || !in || !out || !aligned16(out) || (reinterpret_cast<uintptr_t>(in) & 7))
    return hipErrorInvalidValue;
  hipLaunchKernelGGL(bf16_to_f32_kernel, dim3(stream_grid(n / 4)), dim3(256), 0, stream, in, out, n / 4);
  return hipGetLastError();
}

hipError_t squared_error_grad(const void* y, const void* target, void* dy, float scale, int64_t n, int dtype,
                              hipStream_t stream) {
  const int v = dtype == kBF16 ? 8 : 4;
  if (n <= 0 || n % v || !y || !target || !dy || !aligned16(y) || !aligned16(target) || !aligned16(dy))
    return hipErrorInvalidValue;
  const int64_t blocks = (n / v + 255) / 256;
  if (blocks > 0x7fffffff) return hipErrorInvalidValue;
  if (dtype == kBF16)
    hipLaunchKernelGGL(squared_error_grad_kernel<bf16_t>, dim3((unsigned)blocks), dim3(256), 0, stream,
                       static_cast<const bf16_t*>(y), static_cast<const bf16_t*>(target), static_cast<bf16_t*>(dy), scale, n);
  else
    hipLaunchKernelGGL(squared_error_grad_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, stream,
                       static_cast<const float*>(y), static_cast<const float*>(target), static_cast<float*>(dy), scale, n);
  return hipGetLastError();
}

hipError_t transpose_bf16_grouped(const TransposeItem* items, int count, hipStream_t stream) {
  if (!items || count < 1) return hipErrorInvalidValue;
  for (int i0 = 0; i0 < count; i0 += kTransposeMaxItems) {
    TransposeGroup g{};
    g.count = count - i0 < kTransposeMaxItems ? count - i0 : kTransposeMaxItems;
    int64_t tiles = 0;
    for (int i = 0; i < g.count; ++i) {
      const TransposeItem& it = items[i0 + i];
      if (!it.src || !it.dst || it.rows <= 0 || it.cols <= 0 || it.rows % 8 || it.cols % 8 || !aligned16(it.src) ||
          !aligned16(it.dst))
        return hipErrorInvalidValue;
      g.src[i] = static_cast<const bf16_t*>(it.src); g.dst[i] = static_cast<bf16_t*>(it.dst);
      g.rows[i] = it.rows; g.cols[i] = it.cols;
      g.tiles_c[i] = ceil_div(it.cols, 64);
      g.tile0[i] = (int)tiles;
      tiles += (int64_t)ceil_div(it.rows, 64) * g.tiles_c[i];
      if (tiles > 0x7fffffff) return hipErrorInvalidValue;
    }
    hipLaunchKernelGGL(transpose_bf16_grouped_kernel, dim3((unsigned)tiles), dim3(256), 0, stream, g);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t copy_bytes(const void* in, void* out, int64_t bytes, hipStream_t stream) {
  if (bytes <= 0 || bytes % 16 || !in || !out || !aligned16(in) || !aligned16(out)) return hipErrorInvalidValue;
  if ((bytes / 16 + 255) / 256 > 0x7fffffff) return hipErrorInvalidValue;
  hipLaunchKernelGGL(copy16_kernel, dim3((unsigned)((bytes / 16 + 255) / 256)), dim3(256), 0, stream,
                     static_cast<const uint4*>(in), static_cast<uint4*>(out), bytes / 16);
  return hipGetLastError();
}

}  // namespace k2bw
