// Masked softmax attention, forward and backward, in plain fp32 arithmetic on the vector ALUs.
// Used by the fp32 mode of the stage and for any head size the MFMA kernels do not take.
//
// Forward: one thread per query row; keys and values of the (batch, head) stream through LDS
// in tiles of 32; running maximum and sum (online softmax), so no s x s matrix is stored.
// Saves lse = max + log(sum) per row.
// Backward: delta = rowsum(dO * O) first; then dQ with one thread per query row, and dK, dV
// with one thread per key row, each re-deriving P = exp(S - lse).  No atomics: the result does
// not depend on scheduling.
// Masked keys get probability exactly zero (they enter neither the maximum nor the sum).
#include "kernels.hpp"

namespace k2bw {
namespace {

constexpr int kTile = 32;  // rows staged in LDS per step
constexpr int kRowsPerWg = 64;

template <typename T, int DH>
__device__ __forceinline__ void stage_rows(const T* __restrict__ src, int64_t ld, int row0, int row_end, int dh,
                                           float* dst, int tid, int nthreads) {
  // rows [row0, row0 + kTile) x DH -> dst[r][d]; rows past row_end and columns past dh are zero
  constexpr int chunks = DH / 8;
  for (int e = tid; e < kTile * chunks; e += nthreads) {
    const int r = e / chunks, c = e % chunks;
    float v[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (row0 + r < row_end && c * 8 < dh) load8(src + (int64_t)(row0 + r) * ld + c * 8, v);
#pragma unroll
    for (int i = 0; i < 8; ++i) dst[r * DH + c * 8 + i] = v[i];
  }
}

__device__ __forceinline__ bool visible(int mask_mode, int i, int j, int len) {
  if (mask_mode == 1) return j <= i;
  if (mask_mode == 2) return j < len;
  return true;
}
// one past the last key any query of [i0, i1) may see
__device__ __forceinline__ int key_end(int mask_mode, int i1, int s, int len) {
  if (mask_mode == 1) return min(i1, s);
  if (mask_mode == 2) return len;
  return s;
}

template <typename T, int DH>
__global__ __launch_bounds__(kRowsPerWg) void attn_fwd_simple(const T* __restrict__ qkv, T* __restrict__ o,
                                                               float* __restrict__ lse, int s, int a, int dh,
                                                               int mask_mode, const int32_t* __restrict__ seqlens) {
  __shared__ float ks[kTile * DH];
  __shared__ float vs[kTile * DH];
  const int tid = threadIdx.x;
  const int n = blockIdx.z, head = blockIdx.y;
  const int h = a * dh;
  const int64_t ld = 3 * (int64_t)h;
  const int i0 = blockIdx.x * kRowsPerWg;
  const int i = i0 + tid;
  const bool row_ok = i < s;
  const int len = (mask_mode == 2) ? min(max(seqlens[n], 1), s) : s;   // clamped into [1, s]
  const T* base = qkv + (int64_t)n * s * ld + head * dh;
  const float scale = 1.0f / sqrtf((float)dh);

  float q[DH], acc[DH];
#pragma unroll
  for (int d = 0; d < DH; ++d) { q[d] = 0.f; acc[d] = 0.f; }
  if (row_ok) {
#pragma unroll
    for (int c = 0; c < DH / 8; ++c) {
      if (c * 8 < dh) {
        float v[8];
        load8(base + (int64_t)i * ld + c * 8, v);
#pragma unroll
        for (int t = 0; t < 8; ++t) q[c * 8 + t] = v[t] * scale;
      }
    }
  }
  float mx = -INFINITY, sum = 0.f;
  const int jend = key_end(mask_mode, min(i0 + kRowsPerWg, s), s, len);
  for (int j0 = 0; j0 < jend; j0 += kTile) {
    __syncthreads();
    stage_rows<T, DH>(base + h, ld, j0, jend, dh, ks, tid, kRowsPerWg);
    stage_rows<T, DH>(base + 2 * h, ld, j0, jend, dh, vs, tid, kRowsPerWg);
    __syncthreads();
    const int jn = min(kTile, jend - j0);
    for (int jj = 0; jj < jn; ++jj) {
      const int j = j0 + jj;
      if (!row_ok || !visible(mask_mode, i, j, len)) continue;
      float sc = 0.f;
#pragma unroll
      for (int d = 0; d < DH; ++d) sc = fmaf(q[d], ks[jj * DH + d], sc);
      const float mnew = fmaxf(mx, sc);
      const float corr = expf(mx - mnew);   // exp(-inf) = 0 on the first visible key
      const float pj = expf(sc - mnew);
      sum = sum * corr + pj;
#pragma unroll
      for (int d = 0; d < DH; ++d) acc[d] = fmaf(acc[d], corr, pj * vs[jj * DH + d]);
      mx = mnew;
    }
  }
  if (!row_ok) return;
  const float inv = 1.0f / sum;
  T* orow = o + ((int64_t)n * s + i) * h + head * dh;
#pragma unroll
  for (int c = 0; c < DH / 8; ++c) {
    if (c * 8 < dh) {
      float v[8];
#pragma unroll
      for (int t = 0; t < 8; ++t) v[t] = acc[c * 8 + t] * inv;
      store8(orow + c * 8, v);
    }
  }
  lse[((int64_t)n * a + head) * s + i] = mx + logf(sum);
}

// delta[n, head, i] = sum_d dO[i, d] * O[i, d]
template <typename T>
__global__ __launch_bounds__(256) void attn_delta_kernel(const T* __restrict__ o, const T* __restrict__ d_o,
                                                          float* __restrict__ delta, int b, int s, int a, int dh) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;   // over b*s*a, head fastest
  if (idx >= (int64_t)b * s * a) return;
  const int head = idx % a;
  const int64_t tok = idx / a;
  const int n = tok / s, i = tok % s;
  const T* po = o + tok * (int64_t)(a * dh) + head * dh;
  const T* pd = d_o + tok * (int64_t)(a * dh) + head * dh;
  float acc = 0.f;
  for (int c = 0; c < dh; c += 8) {
    float x[8], y[8];
    load8(po + c, x);
    load8(pd + c, y);
#pragma unroll
    for (int t = 0; t < 8; ++t) acc = fmaf(x[t], y[t], acc);
  }
  delta[((int64_t)n * a + head) * s + i] = acc;
}

// dQ: thread per query row.
template <typename T, int DH>
__global__ __launch_bounds__(kRowsPerWg) void attn_dq_simple(const T* __restrict__ qkv, const T* __restrict__ d_o,
                                                              const float* __restrict__ lse,
                                                              const float* __restrict__ delta, T* __restrict__ dqkv,
                                                              int s, int a, int dh, int mask_mode,
                                                              const int32_t* __restrict__ seqlens) {
  __shared__ float ks[kTile * DH];
  __shared__ float vs[kTile * DH];
  const int tid = threadIdx.x;
  const int n = blockIdx.z, head = blockIdx.y;
  const int h = a * dh;
  const int64_t ld = 3 * (int64_t)h;
  const int i0 = blockIdx.x * kRowsPerWg;
  const int i = i0 + tid;
  const bool row_ok = i < s;
  const int len = (mask_mode == 2) ? min(max(seqlens[n], 1), s) : s;   // clamped into [1, s]
  const T* base = qkv + (int64_t)n * s * ld + head * dh;
  const float scale = 1.0f / sqrtf((float)dh);

  float q[DH], go[DH], dq[DH];
#pragma unroll
  for (int d = 0; d < DH; ++d) { q[d] = 0.f; go[d] = 0.f; dq[d] = 0.f; }
  float l = 0.f, dl = 0.f;
  if (row_ok) {
    const T* gorow = d_o + ((int64_t)n * s + i) * h + head * dh;
#pragma unroll
    for (int c = 0; c < DH / 8; ++c) {
      if (c * 8 < dh) {
        float v[8], w[8];
        load8(base + (int64_t)i * ld + c * 8, v);
        load8(gorow + c * 8, w);
#pragma unroll
        for (int t = 0; t < 8; ++t) { q[c * 8 + t] = v[t] * scale; go[c * 8 + t] = w[t]; }
      }
    }
    l = lse[((int64_t)n * a + head) * s + i];
    dl = delta[((int64_t)n * a + head) * s + i];
  }
  const int jend = key_end(mask_mode, min(i0 + kRowsPerWg, s), s, len);
  for (int j0 = 0; j0 < jend; j0 += kTile) {
    __syncthreads();
    stage_rows<T, DH>(base + h, ld, j0, jend, dh, ks, tid, kRowsPerWg);
    stage_rows<T, DH>(base + 2 * h, ld, j0, jend, dh, vs, tid, kRowsPerWg);
    __syncthreads();
    const int jn = min(kTile, jend - j0);
    for (int jj = 0; jj < jn; ++jj) {
      const int j = j0 + jj;
      if (!row_ok || !visible(mask_mode, i, j, len)) continue;
      float sc = 0.f, dp = 0.f;
#pragma unroll
      for (int d = 0; d < DH; ++d) {
        sc = fmaf(q[d], ks[jj * DH + d], sc);
        dp = fmaf(go[d], vs[jj * DH + d], dp);
      }
      const float ds = expf(sc - l) * (dp - dl);
#pragma unroll
      for (int d = 0; d < DH; ++d) dq[d] = fmaf(ds, ks[jj * DH + d], dq[d]);
    }
  }
  if (!row_ok) return;
  T* out = dqkv + ((int64_t)n * s + i) * ld + head * dh;
#pragma unroll
  for (int c = 0; c < DH / 8; ++c) {
    if (c * 8 < dh) {
      float v[8];
#pragma unroll
      for (int t = 0; t < 8; ++t) v[t] = dq[c * 8 + t] * scale;
      store8(out + c * 8, v);
    }
  }
}

// dK, dV: thread per key row; query rows, dO, lse, delta stream through LDS.
template <typename T, int DH>
__global__ __launch_bounds__(kRowsPerWg) void attn_dkv_simple(const T* __restrict__ qkv, const T* __restrict__ d_o,
                                                               const float* __restrict__ lse,
                                                               const float* __restrict__ delta, T* __restrict__ dqkv,
                                                               int s, int a, int dh, int mask_mode,
                                                               const int32_t* __restrict__ seqlens) {
  __shared__ float qs[kTile * DH];
  __shared__ float gs[kTile * DH];
  __shared__ float ls[kTile];
  __shared__ float ds_[kTile];
  const int tid = threadIdx.x;
  const int n = blockIdx.z, head = blockIdx.y;
  const int h = a * dh;
  const int64_t ld = 3 * (int64_t)h;
  const int j0 = blockIdx.x * kRowsPerWg;
  const int j = j0 + tid;
  const int len = (mask_mode == 2) ? min(max(seqlens[n], 1), s) : s;   // clamped into [1, s]
  const bool row_ok = j < s;
  const T* base = qkv + (int64_t)n * s * ld + head * dh;
  const T* gobase = d_o + (int64_t)n * s * h + head * dh;
  const float scale = 1.0f / sqrtf((float)dh);

  float k[DH], v[DH], dk[DH], dv[DH];
#pragma unroll
  for (int d = 0; d < DH; ++d) { k[d] = 0.f; v[d] = 0.f; dk[d] = 0.f; dv[d] = 0.f; }
  if (row_ok) {
#pragma unroll
    for (int c = 0; c < DH / 8; ++c) {
      if (c * 8 < dh) {
        float x[8], y[8];
        load8(base + h + (int64_t)j * ld + c * 8, x);
        load8(base + 2 * h + (int64_t)j * ld + c * 8, y);
#pragma unroll
        for (int t = 0; t < 8; ++t) { k[c * 8 + t] = x[t]; v[c * 8 + t] = y[t]; }
      }
    }
  }
  // queries that can see any key of this block: causal -> i >= j0; otherwise all
  const int istart = (mask_mode == 1) ? (j0 / kTile) * kTile : 0;
  const bool block_dead = (mask_mode == 2) && (j0 >= len);
  for (int i0 = istart; i0 < s && !block_dead; i0 += kTile) {
    __syncthreads();
    stage_rows<T, DH>(base, ld, i0, s, dh, qs, tid, kRowsPerWg);
    stage_rows<T, DH>(gobase, (int64_t)h, i0, s, dh, gs, tid, kRowsPerWg);
    if (tid < kTile) {
      const int i = i0 + tid;
      ls[tid] = (i < s) ? lse[((int64_t)n * a + head) * s + i] : 0.f;
      ds_[tid] = (i < s) ? delta[((int64_t)n * a + head) * s + i] : 0.f;
    }
    __syncthreads();
    const int in = min(kTile, s - i0);
    for (int ii = 0; ii < in; ++ii) {
      const int i = i0 + ii;
      if (!row_ok || !visible(mask_mode, i, j, len)) continue;
      float sc = 0.f, dp = 0.f;
#pragma unroll
      for (int d = 0; d < DH; ++d) {
        sc = fmaf(qs[ii * DH + d], k[d], sc);
        dp = fmaf(gs[ii * DH + d], v[d], dp);
      }
      const float p = expf(sc * scale - ls[ii]);
      const float dsv = p * (dp - ds_[ii]) * scale;
#pragma unroll
      for (int d = 0; d < DH; ++d) {
        dv[d] = fmaf(p, gs[ii * DH + d], dv[d]);
        dk[d] = fmaf(dsv, qs[ii * DH + d], dk[d]);
      }
    }
  }
  if (!row_ok) return;
  T* outk = dqkv + ((int64_t)n * s + j) * ld + h + head * dh;
  T* outv = outk + h;
#pragma unroll
  for (int c = 0; c < DH / 8; ++c) {
    if (c * 8 < dh) {
      float x[8], y[8];
#pragma unroll
      for (int t = 0; t < 8; ++t) { x[t] = dk[c * 8 + t]; y[t] = dv[c * 8 + t]; }
      store8(outk + c * 8, x);
      store8(outv + c * 8, y);
    }
  }
}

template <typename T, int DH>
hipError_t fwd_launch(const AttnDesc& d, const void* qkv, void* o, float* lse, hipStream_t st) {
  dim3 grid(ceil_div(d.s, kRowsPerWg), d.a, d.b);
  hipLaunchKernelGGL((attn_fwd_simple<T, DH>), grid, dim3(kRowsPerWg), 0, st, static_cast<const T*>(qkv),
                     static_cast<T*>(o), lse, d.s, d.a, d.dh, d.mask_mode, d.seqlens);
  return hipGetLastError();
}

template <typename T, int DH>
hipError_t bwd_launch(const AttnDesc& d, const void* qkv, const void* o, const float* lse, const void* d_o,
                      void* dqkv, float* delta, hipStream_t st) {
  const int64_t rows = (int64_t)d.b * d.s * d.a;
  hipLaunchKernelGGL((attn_delta_kernel<T>), dim3(ceil_div(rows, 256)), dim3(256), 0, st,
                     static_cast<const T*>(o), static_cast<const T*>(d_o), delta, d.b, d.s, d.a, d.dh);
  dim3 grid(ceil_div(d.s, kRowsPerWg), d.a, d.b);
  hipLaunchKernelGGL((attn_dq_simple<T, DH>), grid, dim3(kRowsPerWg), 0, st, static_cast<const T*>(qkv),
                     static_cast<const T*>(d_o), lse, delta, static_cast<T*>(dqkv), d.s, d.a, d.dh, d.mask_mode,
                     d.seqlens);
  hipLaunchKernelGGL((attn_dkv_simple<T, DH>), grid, dim3(kRowsPerWg), 0, st, static_cast<const T*>(qkv),
                     static_cast<const T*>(d_o), lse, delta, static_cast<T*>(dqkv), d.s, d.a, d.dh, d.mask_mode,
                     d.seqlens);
  return hipGetLastError();
}

}  // namespace

hipError_t attention_delta(const AttnDesc& d, const void* o, const void* d_o, float* delta, hipStream_t st) {
  const int64_t rows = (int64_t)d.b * d.s * d.a;
  if (d.dtype == kBF16)
    hipLaunchKernelGGL((attn_delta_kernel<bf16_t>), dim3(ceil_div(rows, 256)), dim3(256), 0, st,
                       static_cast<const bf16_t*>(o), static_cast<const bf16_t*>(d_o), delta, d.b, d.s, d.a, d.dh);
  else
    hipLaunchKernelGGL((attn_delta_kernel<float>), dim3(ceil_div(rows, 256)), dim3(256), 0, st,
                       static_cast<const float*>(o), static_cast<const float*>(d_o), delta, d.b, d.s, d.a, d.dh);
  return hipGetLastError();
}

hipError_t attention_fwd_simple(const AttnDesc& d, const void* qkv, void* o, float* lse, hipStream_t st) {
  const bool bf = d.dtype == kBF16;
  if (d.dh <= 32) return bf ? fwd_launch<bf16_t, 32>(d, qkv, o, lse, st) : fwd_launch<float, 32>(d, qkv, o, lse, st);
  if (d.dh <= 64) return bf ? fwd_launch<bf16_t, 64>(d, qkv, o, lse, st) : fwd_launch<float, 64>(d, qkv, o, lse, st);
  return bf ? fwd_launch<bf16_t, 128>(d, qkv, o, lse, st) : fwd_launch<float, 128>(d, qkv, o, lse, st);
}

hipError_t attention_bwd_simple(const AttnDesc& d, const void* qkv, const void* o, const float* lse,
                                const void* d_o, void* dqkv, float* delta, hipStream_t st) {
  const bool bf = d.dtype == kBF16;
  if (d.dh <= 32)
    return bf ? bwd_launch<bf16_t, 32>(d, qkv, o, lse, d_o, dqkv, delta, st)
              : bwd_launch<float, 32>(d, qkv, o, lse, d_o, dqkv, delta, st);
  if (d.dh <= 64)
    return bf ? bwd_launch<bf16_t, 64>(d, qkv, o, lse, d_o, dqkv, delta, st)
              : bwd_launch<float, 64>(d, qkv, o, lse, d_o, dqkv, delta, st);
  return bf ? bwd_launch<bf16_t, 128>(d, qkv, o, lse, d_o, dqkv, delta, st)
            : bwd_launch<float, 128>(d, qkv, o, lse, d_o, dqkv, delta, st);
}

}  // namespace k2bw
