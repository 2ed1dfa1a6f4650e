// bf16 masked-softmax attention on the gfx950 matrix cores, forward and backward, for head
// sizes 32, 64, 80 and 128.  fp32 scores, statistics and accumulators; no s x s matrix in HBM.
//
// All three kernels keep one query (forward, dQ) or one key (dK/dV) per lane of a 32-wide MFMA
// column, so softmax statistics, lse and delta are per-lane scalars or short in-lane loops:
//
//   forward   S^T = K Q^T  (keys x queries): lane = query, registers = keys.  Row maximum and
//             sum are in-lane plus one exchange between the two 32-lane halves.  P^T in that
//             layout is directly the second MFMA operand of O^T = V^T P^T.
//   dQ        same orientation: dP^T = V dO^T, dS^T = P^T (dP^T - delta), dQ^T = K^T dS^T.
//   dK, dV    S = Q K^T (queries x keys): lane = key, registers = queries; P and dS in that
//             layout are the second operands of dV^T = dO^T P and dK^T = Q^T dS.
//
// v_mfma_f32_32x32x16_bf16: lane l gives row l%32 of the first operand and column l%32 of the
// second, k-slots 8*(l/32)..+7; it gets column l%32 of the result, rows 8*(r/4)+4*(l/32)+(r%4)
// in register r.  Re-using a result as a second operand therefore fixes which actual index
// sits in which k-slot (slot t of half hf <-> index 16*kk + 4*hf + t for t < 4, 16*kk + 8 +
// 4*hf + t - 4 otherwise); the first operand is read from a transposed LDS tile in 8-byte
// pieces of four consecutive indices to match.
//
// LDS tiles: row-major [row][dh] with 16-byte chunks and one chunk of padding per row, and
// transposed [d][64 rows] in 8-byte pieces with one piece of padding per row (odd strides:
// conflict-free for 32 consecutive rows).  Masked keys get probability exactly zero.
#include "kernels.hpp"

namespace k2bw {

hipError_t attention_delta(const AttnDesc& d, const void* o, const void* d_o, float* delta, hipStream_t st);

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kBlockRows = 128;   // rows (queries or keys) owned by a workgroup: 4 waves x 32
constexpr int kTile = 64;         // rows streamed through LDS per step
constexpr int kTP = 17;           // 8-byte pieces per row of a transposed tile (16 + 1 pad)
constexpr float kLog2e = 1.4426950408889634f;

template <int DH>
struct Cfg {
  static constexpr int KS = DH / 16;               // MFMA k-steps over the head dimension
  static constexpr int DHP = (DH + 31) / 32 * 32;  // head dimension padded to whole 32-row blocks
  static constexpr int DB = DHP / 32;
  static constexpr int KC = DH / 8 + 1;            // 16-byte chunks per row of a row-major tile
  static constexpr int kRowTile = kTile * KC;      // uint4 per row-major tile
  static constexpr int kTrTile = DHP * kTP;        // uint2 per transposed tile
};

__device__ __forceinline__ uint32_t word(const uint4& v, int i) {
  return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w;
}

// Tiles go HBM -> registers -> LDS in two steps so that the loads of the next tile are in
// flight while the current one is being consumed.
// rows [row0, row0+64) x DH of a [*, ld] matrix -> row-major LDS tile; rows >= row_end are zero
template <int DH>
struct RowFetch {
  static constexpr int C = DH / 8;
  static constexpr int N = (kTile * C + kThreads - 1) / kThreads;
  uint4 v[N];
  __device__ __forceinline__ void fetch(const bf16_t* __restrict__ src, int64_t ld, int row0, int row_end, int tid) {
#pragma unroll
    for (int it = 0; it < N; ++it) {
      const int e = tid + it * kThreads;
      const int r = e / C, c = e % C;
      v[it] = make_uint4(0, 0, 0, 0);
      if (e < kTile * C && row0 + r < row_end)
        v[it] = *reinterpret_cast<const uint4*>(src + (int64_t)(row0 + r) * ld + c * 8);
    }
  }
  __device__ __forceinline__ void commit(uint4* tile, int tid) const {
#pragma unroll
    for (int it = 0; it < N; ++it) {
      const int e = tid + it * kThreads;
      if (e < kTile * C) tile[(e / C) * Cfg<DH>::KC + e % C] = v[it];
    }
  }
};

// the same rows, transposed: tile[d][row] in 8-byte pieces of 4 consecutive rows
template <int DH>
struct TrFetch {
  static constexpr int C = DH / 8;
  static constexpr int N = (16 * C + kThreads - 1) / kThreads;
  uint4 v[N][4];
  __device__ __forceinline__ void fetch(const bf16_t* __restrict__ src, int64_t ld, int row0, int row_end, int tid) {
#pragma unroll
    for (int it = 0; it < N; ++it) {
      const int u = tid + it * kThreads;
      const int rq = u % 16, c = u / 16;   // row quad, d chunk
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int r = row0 + rq * 4 + j;
        v[it][j] = make_uint4(0, 0, 0, 0);
        if (u < 16 * C && r < row_end) v[it][j] = *reinterpret_cast<const uint4*>(src + (int64_t)r * ld + c * 8);
      }
    }
  }
  __device__ __forceinline__ void commit(uint2* tile, int tid) const {
#pragma unroll
    for (int it = 0; it < N; ++it) {
      const int u = tid + it * kThreads;
      if (u >= 16 * C) continue;
      const int rq = u % 16, c = u / 16;
#pragma unroll
      for (int ii = 0; ii < 8; ++ii) {
        const int wd = ii >> 1;
        const uint32_t w0 = word(v[it][0], wd), w1 = word(v[it][1], wd), w2 = word(v[it][2], wd), w3 = word(v[it][3], wd);
        uint2 o;
        if (ii & 1) {
          o.x = __builtin_amdgcn_perm(w1, w0, 0x07060302u);
          o.y = __builtin_amdgcn_perm(w3, w2, 0x07060302u);
        } else {
          o.x = __builtin_amdgcn_perm(w1, w0, 0x05040100u);
          o.y = __builtin_amdgcn_perm(w3, w2, 0x05040100u);
        }
        tile[(c * 8 + ii) * kTP + rq] = o;
      }
    }
  }
};

template <int DH>
__device__ __forceinline__ void zero_pad_rows(uint2* tile, int tid) {
  if (Cfg<DH>::DHP > DH)
    for (int e = tid; e < (Cfg<DH>::DHP - DH) * kTP; e += kThreads) tile[DH * kTP + e] = make_uint2(0, 0);
}

// 16-byte k-fragment of a row of a [*, ld] matrix straight from HBM (second MFMA operand)
template <int DH>
__device__ __forceinline__ void load_frags(const bf16_t* __restrict__ row_ptr, bool ok, int hf, bf16x8 (&f)[Cfg<DH>::KS]) {
#pragma unroll
  for (int ks = 0; ks < Cfg<DH>::KS; ++ks) {
    uint4 v = make_uint4(0, 0, 0, 0);
    if (ok) v = *reinterpret_cast<const uint4*>(row_ptr + ks * 16 + hf * 8);
    f[ks] = __builtin_bit_cast(bf16x8, v);
  }
}

// registers 8*half .. 8*half+7 of a result block -> second operand of the next MFMA
__device__ __forceinline__ bf16x8 pack_half(const f32x16& v, int half) {
  uint4 w;
  const int b = 8 * half;
  w.x = pack_bf16x2(v[b + 0], v[b + 1]); w.y = pack_bf16x2(v[b + 2], v[b + 3]);
  w.z = pack_bf16x2(v[b + 4], v[b + 5]); w.w = pack_bf16x2(v[b + 6], v[b + 7]);
  return __builtin_bit_cast(bf16x8, w);
}

// first operand from a transposed tile: row d, index group kk (16 indices), this lane's half
__device__ __forceinline__ bf16x8 read_tr(const uint2* tile, int d, int kk, int hf) {
  const uint2 p0 = tile[d * kTP + 4 * kk + hf];
  const uint2 p1 = tile[d * kTP + 4 * kk + 2 + hf];
  return __builtin_bit_cast(bf16x8, make_uint4(p0.x, p0.y, p1.x, p1.y));
}

__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int r = 0; r < 16; ++r) z[r] = 0.f;
  return z;
}

__device__ __forceinline__ uint2 pack4f(float a, float b, float c, float d) {
  return make_uint2(pack_bf16x2(a, b), pack_bf16x2(c, d));
}

// ------------------------------------------------------------------------------------------------
// forward
template <int DH>
__global__ __launch_bounds__(kThreads) void attn_fwd_mfma_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ o,
                                                                  float* __restrict__ lse, int s, int a, int mask_mode,
                                                                  const int32_t* __restrict__ seqlens) {
  using C = Cfg<DH>;
  extern __shared__ uint4 smem[];
  uint4* k_lds = smem;
  uint2* vt_lds = reinterpret_cast<uint2*>(smem + C::kRowTile);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, hf = lane >> 5;
  const int n = blockIdx.z, head = blockIdx.y, i0 = blockIdx.x * kBlockRows;
  const int h = a * DH;
  const int64_t ld = 3 * (int64_t)h;
  const bf16_t* base = qkv + (int64_t)n * s * ld + head * DH;
  const int kv_len = mask_mode == 2 ? seqlens[n] : s;
  const bool causal = mask_mode == 1;
  const int iw0 = i0 + wave * 32;
  const int i = iw0 + l32;
  const float scale = 1.0f / sqrtf((float)DH);
  const float c = scale * kLog2e;

  bf16x8 qf[C::KS];
  load_frags<DH>(base + (int64_t)i * ld, i < s, hf, qf);
  f32x16 oacc[C::DB];
#pragma unroll
  for (int db = 0; db < C::DB; ++db) oacc[db] = zero16();
  float m_i = -INFINITY, l_i = 0.f;

  zero_pad_rows<DH>(vt_lds, tid);
  const int jend = causal ? min(i0 + kBlockRows, s) : kv_len;
  RowFetch<DH> kfetch;
  TrFetch<DH> vfetch;
  kfetch.fetch(base + h, ld, 0, jend, tid);
  vfetch.fetch(base + 2 * h, ld, 0, jend, tid);
  for (int j0 = 0; j0 < jend; j0 += kTile) {
    __syncthreads();
    kfetch.commit(k_lds, tid);
    vfetch.commit(vt_lds, tid);
    __syncthreads();
    kfetch.fetch(base + h, ld, j0 + kTile, jend, tid);        // next tile, in flight during the MFMAs
    vfetch.fetch(base + 2 * h, ld, j0 + kTile, jend, tid);
    if (causal && j0 > iw0 + 31) continue;   // every key of the tile lies after this wave's queries

    f32x16 sacc[2] = {zero16(), zero16()};
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) {
      const bf16x8 k0 = __builtin_bit_cast(bf16x8, k_lds[l32 * C::KC + ks * 2 + hf]);
      const bf16x8 k1 = __builtin_bit_cast(bf16x8, k_lds[(32 + l32) * C::KC + ks * 2 + hf]);
      sacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k0, qf[ks], sacc[0], 0, 0, 0);
      sacc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k1, qf[ks], sacc[1], 0, 0, 0);
    }
    // masks (only tiles that touch a boundary need them) and the running maximum
    const bool need_mask = (j0 + kTile > kv_len) || (causal && j0 + kTile - 1 > iw0);
    float mloc = -INFINITY;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        if (need_mask) {
          const int key = j0 + nb * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
          const bool vis = key < kv_len && (!causal || key <= i);
          sacc[nb][r] = vis ? sacc[nb][r] : -INFINITY;
        }
        mloc = fmaxf(mloc, sacc[nb][r]);
      }
    mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));
    const float m_new = fmaxf(m_i, mloc);
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;   // row with nothing visible yet
    const float alpha = __builtin_amdgcn_exp2f((m_i - m_use) * c);
    const float mc = m_use * c;
    float rowsum = 0.f;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float pv = __builtin_amdgcn_exp2f(fmaf(sacc[nb][r], c, -mc));
        sacc[nb][r] = pv;
        rowsum += pv;
      }
    l_i = l_i * alpha + rowsum;
    m_i = m_new;
#pragma unroll
    for (int db = 0; db < C::DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
    bf16x8 pb[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) pb[kk] = pack_half(sacc[kk >> 1], kk & 1);
#pragma unroll
    for (int db = 0; db < C::DB; ++db)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_tr(vt_lds, db * 32 + l32, kk, hf), pb[kk], oacc[db], 0, 0, 0);
  }

  const float l_tot = l_i + __shfl_xor(l_i, 32, 64);
  if (i >= s) return;
  const float inv = 1.0f / l_tot;
  bf16_t* orow = o + ((int64_t)n * s + i) * h + head * DH;
#pragma unroll
  for (int db = 0; db < C::DB; ++db)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int d = db * 32 + 8 * g + 4 * hf;
      if (d < DH)
        *reinterpret_cast<uint2*>(orow + d) = pack4f(oacc[db][4 * g] * inv, oacc[db][4 * g + 1] * inv,
                                                     oacc[db][4 * g + 2] * inv, oacc[db][4 * g + 3] * inv);
    }
  if (hf == 0) lse[((int64_t)n * a + head) * s + i] = m_i * scale + logf(l_tot);
}

// ------------------------------------------------------------------------------------------------
// dQ
template <int DH>
__global__ __launch_bounds__(kThreads) void attn_dq_mfma_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ d_o,
                                                                 const float* __restrict__ lse, const float* __restrict__ delta,
                                                                 bf16_t* __restrict__ dqkv, int s, int a, int mask_mode,
                                                                 const int32_t* __restrict__ seqlens) {
  using C = Cfg<DH>;
  extern __shared__ uint4 smem[];
  uint4* k_lds = smem;
  uint4* v_lds = smem + C::kRowTile;
  uint2* kt_lds = reinterpret_cast<uint2*>(smem + 2 * C::kRowTile);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, hf = lane >> 5;
  const int n = blockIdx.z, head = blockIdx.y, i0 = blockIdx.x * kBlockRows;
  const int h = a * DH;
  const int64_t ld = 3 * (int64_t)h;
  const bf16_t* base = qkv + (int64_t)n * s * ld + head * DH;
  const int kv_len = mask_mode == 2 ? seqlens[n] : s;
  const bool causal = mask_mode == 1;
  const int iw0 = i0 + wave * 32;
  const int i = iw0 + l32;
  const bool row_ok = i < s;
  const float scale = 1.0f / sqrtf((float)DH);
  const float c = scale * kLog2e;

  bf16x8 qf[C::KS], dof[C::KS];
  load_frags<DH>(base + (int64_t)i * ld, row_ok, hf, qf);
  load_frags<DH>(d_o + ((int64_t)n * s + i) * h + head * DH, row_ok, hf, dof);
  const float lse_i = row_ok ? lse[((int64_t)n * a + head) * s + i] * kLog2e : INFINITY;
  const float delta_i = row_ok ? delta[((int64_t)n * a + head) * s + i] : 0.f;
  f32x16 dq[C::DB];
#pragma unroll
  for (int db = 0; db < C::DB; ++db) dq[db] = zero16();

  zero_pad_rows<DH>(kt_lds, tid);
  const int jend = causal ? min(i0 + kBlockRows, s) : kv_len;
  // (no register prefetch here: it would push the kernel past 256 registers per lane, and two
  // waves per SIMD hide the tile loads better than one wave with prefetch -- measured)
  for (int j0 = 0; j0 < jend; j0 += kTile) {
    __syncthreads();
    {
      RowFetch<DH> kfetch, vfetch;
      TrFetch<DH> ktfetch;
      kfetch.fetch(base + h, ld, j0, jend, tid);
      vfetch.fetch(base + 2 * h, ld, j0, jend, tid);
      ktfetch.fetch(base + h, ld, j0, jend, tid);
      kfetch.commit(k_lds, tid);
      vfetch.commit(v_lds, tid);
      ktfetch.commit(kt_lds, tid);
    }
    __syncthreads();
    if (causal && j0 > iw0 + 31) continue;

    f32x16 sacc[2] = {zero16(), zero16()}, dp[2] = {zero16(), zero16()};
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) {
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
        const bf16x8 kf = __builtin_bit_cast(bf16x8, k_lds[(nb * 32 + l32) * C::KC + ks * 2 + hf]);
        const bf16x8 vf = __builtin_bit_cast(bf16x8, v_lds[(nb * 32 + l32) * C::KC + ks * 2 + hf]);
        sacc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], sacc[nb], 0, 0, 0);
        dp[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, dof[ks], dp[nb], 0, 0, 0);
      }
    }
    const bool need_mask = (j0 + kTile > kv_len) || (causal && j0 + kTile - 1 > iw0);
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float pv = __builtin_amdgcn_exp2f(fmaf(sacc[nb][r], c, -lse_i));
        if (need_mask) {
          const int key = j0 + nb * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
          const bool vis = key < kv_len && (!causal || key <= i);
          pv = vis ? pv : 0.f;
        }
        sacc[nb][r] = pv * (dp[nb][r] - delta_i);   // dS^T (the 1/sqrt(dh) factor is applied at the end)
      }
    bf16x8 dsb[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) dsb[kk] = pack_half(sacc[kk >> 1], kk & 1);
#pragma unroll
    for (int db = 0; db < C::DB; ++db)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
        dq[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_tr(kt_lds, db * 32 + l32, kk, hf), dsb[kk], dq[db], 0, 0, 0);
  }
  if (!row_ok) return;
  bf16_t* out = dqkv + ((int64_t)n * s + i) * ld + head * DH;
#pragma unroll
  for (int db = 0; db < C::DB; ++db)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int d = db * 32 + 8 * g + 4 * hf;
      if (d < DH)
        *reinterpret_cast<uint2*>(out + d) = pack4f(dq[db][4 * g] * scale, dq[db][4 * g + 1] * scale,
                                                    dq[db][4 * g + 2] * scale, dq[db][4 * g + 3] * scale);
    }
}

// ------------------------------------------------------------------------------------------------
// dK, dV
template <int DH>
__global__ __launch_bounds__(kThreads) void attn_dkv_mfma_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ d_o,
                                                                  const float* __restrict__ lse, const float* __restrict__ delta,
                                                                  bf16_t* __restrict__ dqkv, int s, int a, int mask_mode,
                                                                  const int32_t* __restrict__ seqlens) {
  using C = Cfg<DH>;
  extern __shared__ uint4 smem[];
  uint4* q_lds = smem;
  uint4* do_lds = smem + C::kRowTile;
  uint2* qt_lds = reinterpret_cast<uint2*>(smem + 2 * C::kRowTile);
  uint2* dot_lds = qt_lds + C::kTrTile;
  float* lse_lds = reinterpret_cast<float*>(dot_lds + C::kTrTile);
  float* delta_lds = lse_lds + kTile;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, hf = lane >> 5;
  const int n = blockIdx.z, head = blockIdx.y, j0 = blockIdx.x * kBlockRows;
  const int h = a * DH;
  const int64_t ld = 3 * (int64_t)h;
  const bf16_t* base = qkv + (int64_t)n * s * ld + head * DH;
  const bf16_t* dobase = d_o + (int64_t)n * s * h + head * DH;
  const float* lse_row = lse + ((int64_t)n * a + head) * s;
  const float* delta_row = delta + ((int64_t)n * a + head) * s;
  const int kv_len = mask_mode == 2 ? seqlens[n] : s;
  const bool causal = mask_mode == 1;
  const int jw0 = j0 + wave * 32;
  const int j = jw0 + l32;
  const bool row_ok = j < s;
  const float scale = 1.0f / sqrtf((float)DH);
  const float c = scale * kLog2e;

  bf16x8 kf[C::KS], vf[C::KS];
  load_frags<DH>(base + h + (int64_t)j * ld, row_ok, hf, kf);
  load_frags<DH>(base + 2 * h + (int64_t)j * ld, row_ok, hf, vf);
  f32x16 dk[C::DB], dv[C::DB];
#pragma unroll
  for (int db = 0; db < C::DB; ++db) { dk[db] = zero16(); dv[db] = zero16(); }

  zero_pad_rows<DH>(qt_lds, tid);
  zero_pad_rows<DH>(dot_lds, tid);
  const bool wg_dead = j0 >= kv_len;                       // every key of the workgroup is padding
  const int istart = causal ? (j0 / kTile) * kTile : 0;    // earlier queries see none of these keys
  for (int i0 = istart; i0 < s && !wg_dead; i0 += kTile) {
    __syncthreads();
    {
      RowFetch<DH> qfetch, dofetch;
      TrFetch<DH> qtfetch, dotfetch;
      qfetch.fetch(base, ld, i0, s, tid);
      dofetch.fetch(dobase, (int64_t)h, i0, s, tid);
      qtfetch.fetch(base, ld, i0, s, tid);
      dotfetch.fetch(dobase, (int64_t)h, i0, s, tid);
      qfetch.commit(q_lds, tid);
      dofetch.commit(do_lds, tid);
      qtfetch.commit(qt_lds, tid);
      dotfetch.commit(dot_lds, tid);
    }
    if (tid < kTile) {
      const int i = i0 + tid;
      lse_lds[tid] = i < s ? lse_row[i] * kLog2e : INFINITY;   // +inf: probability 0 for rows past the end
      delta_lds[tid] = i < s ? delta_row[i] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const int ib = i0 + qb * 32;
      if (causal && ib + 31 < jw0) continue;   // all 32 queries lie before this wave's keys
      f32x16 sacc = zero16(), dp = zero16();
#pragma unroll
      for (int ks = 0; ks < C::KS; ++ks) {
        const bf16x8 qa = __builtin_bit_cast(bf16x8, q_lds[(qb * 32 + l32) * C::KC + ks * 2 + hf]);
        const bf16x8 da = __builtin_bit_cast(bf16x8, do_lds[(qb * 32 + l32) * C::KC + ks * 2 + hf]);
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa, kf[ks], sacc, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(da, vf[ks], dp, 0, 0, 0);
      }
      const bool need_mask = (jw0 + 32 > kv_len) || (causal && jw0 + 31 > ib);
      f32x16 pv16, ds16;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 l4 = *reinterpret_cast<const float4*>(lse_lds + qb * 32 + 8 * g + 4 * hf);
        const float4 d4 = *reinterpret_cast<const float4*>(delta_lds + qb * 32 + 8 * g + 4 * hf);
        const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dl[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int r = 4 * g + t;
          float pv = __builtin_amdgcn_exp2f(fmaf(sacc[r], c, -lv[t]));
          if (need_mask) {
            const int iq = ib + 8 * g + 4 * hf + t;
            const bool vis = j < kv_len && (!causal || j <= iq);
            pv = vis ? pv : 0.f;
          }
          pv16[r] = pv;
          ds16[r] = pv * (dp[r] - dl[t]);
        }
      }
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const bf16x8 pb = pack_half(pv16, half), dsb = pack_half(ds16, half);
        const int kk = qb * 2 + half;
#pragma unroll
        for (int db = 0; db < C::DB; ++db) {
          dv[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_tr(dot_lds, db * 32 + l32, kk, hf), pb, dv[db], 0, 0, 0);
          dk[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_tr(qt_lds, db * 32 + l32, kk, hf), dsb, dk[db], 0, 0, 0);
        }
      }
    }
  }
  if (!row_ok) return;
  bf16_t* outk = dqkv + ((int64_t)n * s + j) * ld + h + head * DH;
  bf16_t* outv = outk + h;
#pragma unroll
  for (int db = 0; db < C::DB; ++db)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int d = db * 32 + 8 * g + 4 * hf;
      if (d < DH) {
        *reinterpret_cast<uint2*>(outk + d) = pack4f(dk[db][4 * g] * scale, dk[db][4 * g + 1] * scale,
                                                     dk[db][4 * g + 2] * scale, dk[db][4 * g + 3] * scale);
        *reinterpret_cast<uint2*>(outv + d) = pack4f(dv[db][4 * g], dv[db][4 * g + 1], dv[db][4 * g + 2], dv[db][4 * g + 3]);
      }
    }
}

template <typename K>
hipError_t set_lds(K kern, size_t bytes, bool* done) {
  if (*done) return hipSuccess;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)bytes);
  if (e == hipSuccess) *done = true;
  return e;
}

template <int DH>
hipError_t fwd_launch(const AttnDesc& d, const void* qkv, void* o, float* lse, hipStream_t st) {
  using C = Cfg<DH>;
  constexpr size_t lds = C::kRowTile * sizeof(uint4) + C::kTrTile * sizeof(uint2);
  static bool done = false;
  hipError_t e = set_lds(attn_fwd_mfma_kernel<DH>, lds, &done);
  if (e != hipSuccess) return e;
  dim3 grid(ceil_div(d.s, kBlockRows), d.a, d.b);
  hipLaunchKernelGGL(attn_fwd_mfma_kernel<DH>, grid, dim3(kThreads), lds, st, static_cast<const bf16_t*>(qkv),
                     static_cast<bf16_t*>(o), lse, d.s, d.a, d.mask_mode, d.seqlens);
  return hipGetLastError();
}

template <int DH>
hipError_t bwd_launch(const AttnDesc& d, const void* qkv, const void* o, const float* lse, const void* d_o, void* dqkv,
                      float* delta, hipStream_t st) {
  using C = Cfg<DH>;
  hipError_t e = attention_delta(d, o, d_o, delta, st);
  if (e != hipSuccess) return e;
  constexpr size_t lds_dq = 2 * C::kRowTile * sizeof(uint4) + C::kTrTile * sizeof(uint2);
  constexpr size_t lds_dkv = 2 * C::kRowTile * sizeof(uint4) + 2 * C::kTrTile * sizeof(uint2) + 2 * kTile * sizeof(float);
  static bool done_dq = false, done_dkv = false;
  e = set_lds(attn_dq_mfma_kernel<DH>, lds_dq, &done_dq);
  if (e != hipSuccess) return e;
  e = set_lds(attn_dkv_mfma_kernel<DH>, lds_dkv, &done_dkv);
  if (e != hipSuccess) return e;
  dim3 grid(ceil_div(d.s, kBlockRows), d.a, d.b);
  hipLaunchKernelGGL(attn_dq_mfma_kernel<DH>, grid, dim3(kThreads), lds_dq, st, static_cast<const bf16_t*>(qkv),
                     static_cast<const bf16_t*>(d_o), lse, delta, static_cast<bf16_t*>(dqkv), d.s, d.a, d.mask_mode,
                     d.seqlens);
  hipLaunchKernelGGL(attn_dkv_mfma_kernel<DH>, grid, dim3(kThreads), lds_dkv, st, static_cast<const bf16_t*>(qkv),
                     static_cast<const bf16_t*>(d_o), lse, delta, static_cast<bf16_t*>(dqkv), d.s, d.a, d.mask_mode,
                     d.seqlens);
  return hipGetLastError();
}

}  // namespace

bool attention_mfma_supported(const AttnDesc& d) {
  return d.dtype == kBF16 && (d.dh == 32 || d.dh == 64 || d.dh == 80 || d.dh == 128);
}

hipError_t attention_fwd_mfma(const AttnDesc& d, const void* qkv, void* o, float* lse, hipStream_t st) {
  switch (d.dh) {
    case 32: return fwd_launch<32>(d, qkv, o, lse, st);
    case 64: return fwd_launch<64>(d, qkv, o, lse, st);
    case 80: return fwd_launch<80>(d, qkv, o, lse, st);
    case 128: return fwd_launch<128>(d, qkv, o, lse, st);
    default: return hipErrorInvalidValue;
  }
}

hipError_t attention_bwd_mfma(const AttnDesc& d, const void* qkv, const void* o, const float* lse, const void* d_o,
                              void* dqkv, float* delta, hipStream_t st) {
  switch (d.dh) {
    case 32: return bwd_launch<32>(d, qkv, o, lse, d_o, dqkv, delta, st);
    case 64: return bwd_launch<64>(d, qkv, o, lse, d_o, dqkv, delta, st);
    case 80: return bwd_launch<80>(d, qkv, o, lse, d_o, dqkv, delta, st);
    case 128: return bwd_launch<128>(d, qkv, o, lse, d_o, dqkv, delta, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace k2bw
