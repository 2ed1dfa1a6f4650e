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
// 4*hf + t - 4 otherwise); the transposing LDS reads deliver the first operand in that order.
//
// LDS tiles are row-major [64 rows][dh] copies of K, V, Q or dO rows, filled straight from HBM by
// global_load_lds (16 bytes per lane, no registers, no LDS store instructions), two stages deep:
// the loads of tile t+1 are in flight while tile t is consumed, one barrier per tile.  A tile
// serves both operand forms: rows as MFMA rows (16-byte reads along dh) and, through
// ds_read_b64_tr_b16, columns as MFMA rows (the transposed operands K^T, V^T, Q^T, dO^T), so no
// transposed copy is ever built.  16-byte chunks are XOR-swizzled by row so that both read
// patterns are bank-conflict free.  Masked keys get probability exactly zero.
#include <type_traits>

#include "kernels.hpp"

namespace k2bw {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef short v8i16 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) v4i16 lds_v4i16_t;
typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(3))) char lds_char_t;
typedef __attribute__((address_space(1))) const void glob_void_t;

// Waves per workgroup, 32 rows (queries or keys) each.  Measured on MI355X with 2 / 4 / 8 waves
// (s = 512, dh = 64: forward 27.9 / 20.7 / 19.5 us, backward 66.7 / 58.8 / 57.1 us; s = 2048,
// dh = 128 causal: forward 270 / 258 / 152 us): more waves share each K/V tile and each barrier.
constexpr int kWaves = 8;
constexpr int kThreads = kWaves * 64;
constexpr int kBlockRows = kWaves * 32;
constexpr int kTile = 64;         // rows streamed through LDS per step
constexpr float kLog2e = 1.4426950408889634f;

template <int DH>
struct Cfg {
  static constexpr int KS = DH / 16;               // MFMA k-steps over the head dimension
  static constexpr int DHP = (DH + 31) / 32 * 32;  // head dimension padded to whole 32-row blocks
  static constexpr int DB = DHP / 32;
  static constexpr int CH = DH / 8;                // 16-byte chunks per tile row
  static constexpr int kTileU4 = kTile * CH;       // uint4 per tile
  static constexpr int kPadU4 = 4;                 // transposing reads of the padded head columns run past a row
  // Two waves per SIMD (which 8-wave workgroups imply) cap a lane at 256 registers; the compiler
  // then keeps MFMA results in ordinary VGPRs.  With 512 available it parks them in the
  // accumulator file and copies every score to a VGPR and back around the softmax arithmetic,
  // which costs more than the MFMAs.
  static constexpr int kMinWaves = 2;
  static constexpr bool kDkvVInLds = DH == 128;   // dK/dV kernel: V fragments of the wave's keys in LDS, not registers
};

// Chunk swizzle per head size (rows are 64 / 128 / 160 / 256 bytes; the LDS has 64 banks of 4 bytes).
// Checked against a bank model for both read patterns: 16-byte reads of 16 consecutive rows at one
// logical chunk, and the transposing 8-byte reads (4 consecutive rows x 32 or 64 contiguous bytes).
template <int DH>
__device__ __forceinline__ int swz(int r) {
  if (DH == 32) return (r >> 2) & 3;
  if (DH == 64) { const int u = (r >> 1) & 7; return ((u & 1) << 2) | (u >> 1); }
  if (DH == 80) return (r >> 3) & 1;
  return ((r & 3) << 2) | ((r >> 2) & 3);
}

// s_waitcnt immediate for "at most n vector-memory operations outstanding" (gfx9 encoding)
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

// Rows [row0, row0 + 64) x DH of a [*, ld] matrix -> LDS tile; lane i of a load instruction owns
// LDS slot L0 + i and fetches the chunk that belongs there.  Rows >= row_end are fetched from row
// row_end - 1 (finite data; whatever they produce is masked or never stored).
template <int DH>
struct TileLoader {
  static constexpr int CH = DH / 8;
  static constexpr int kInstr = kTile * CH / 64;            // wave-instructions per tile
  static constexpr int NI = (kInstr + kWaves - 1) / kWaves;  // per wave
  int row[NI], coff[NI];
  int wave_;
  __device__ __forceinline__ void init(int wave, int lane) {
    wave_ = wave;
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      const int L = (j * kWaves + wave) * 64 + lane;
      const int r = L / CH, pc = L % CH;
      row[j] = r < kTile ? r : kTile - 1;
      coff[j] = (pc ^ swz<DH>(r)) * 8;
    }
  }
  __device__ __forceinline__ void issue(const bf16_t* __restrict__ src, int64_t ld, int row0, int row_end, uint4* tile) const {
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      if ((j * kWaves + wave_) < kInstr) {   // wave-uniform
        const int r = min(row0 + row[j], row_end - 1);
        __builtin_amdgcn_global_load_lds((glob_void_t*)(src + (int64_t)r * ld + coff[j]),
                                         (lds_void_t*)(tile + (j * kWaves + wave_) * 64), 16, 0, 0);
      }
    }
  }
};

// 64 floats starting at src[i0] -> LDS, by one wave (4 bytes per lane); entries past n_valid repeat the last one
__device__ __forceinline__ void issue_floats(const float* __restrict__ src, int i0, int n_valid, float* dst, int lane) {
  const int i = min(i0 + lane, n_valid - 1);
  __builtin_amdgcn_global_load_lds((glob_void_t*)(src + i), (lds_void_t*)dst, 4, 0, 0);
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

// first operand, rows of the tile as MFMA rows: row `row`, head columns 16*ks + 8*hf .. +7
template <int DH>
__device__ __forceinline__ bf16x8 read_rows(const uint4* tile, int row, int ks, int hf) {
  return __builtin_bit_cast(bf16x8, tile[row * Cfg<DH>::CH + ((ks * 2 + hf) ^ swz<DH>(row))]);
}

// registers 8*half .. 8*half+7 of a result block -> second operand of the next MFMA
__device__ __forceinline__ bf16x8 pack_half(const f32x16& v, int half) {
  uint4 w;
  const int b = 8 * half;
  w.x = pack_bf16x2(v[b + 0], v[b + 1]); w.y = pack_bf16x2(v[b + 2], v[b + 3]);
  w.z = pack_bf16x2(v[b + 4], v[b + 5]); w.w = pack_bf16x2(v[b + 6], v[b + 7]);
  return __builtin_bit_cast(bf16x8, w);
}

// First operand, head columns of the tile as MFMA rows: this lane's row is head column
// d0 + lane % 32, its k-slots are tile rows 16*kk + 4*hf + 0..3 and 16*kk + 8 + 4*hf + 0..3 (the
// order in which a 32x32 result block, re-used as second operand, holds them).
// ds_read_b64_tr_b16, measured on gfx950: within each group of 16 lanes, lane a + 4t supplies the
// address of 4 consecutive columns of row t, and lane 4a + j receives rows 0..3 of column 4a + j.
template <int DH>
__device__ __forceinline__ bf16x8 read_cols(const uint4* tile, int d0, int kk, int lane) {
  const int r16 = lane & 15, a = r16 & 3, t = r16 >> 2, hf = lane >> 5;
  const int col = d0 + ((lane >> 4) & 1) * 16 + 4 * a;
  const int r0 = 16 * kk + 4 * hf + t, r1 = r0 + 8;
  const int b0 = r0 * (DH * 2) + (((col >> 3) ^ swz<DH>(r0)) << 4) + ((col >> 2) & 1) * 8;
  const int b1 = r1 * (DH * 2) + (((col >> 3) ^ swz<DH>(r1)) << 4) + ((col >> 2) & 1) * 8;
  const lds_char_t* base = (const lds_char_t*)tile;
  const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16_t*)(base + b0));
  const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16_t*)(base + b1));
  const v8i16 w = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, w);
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

// Sum of v over the 16 lanes of a DPP row, left in every lane of the row: two quad permutes, then
// the half-row and full-row mirrors (each step adds a lane that holds the other group's sum).
__device__ __forceinline__ float row16_sum(float v) {
  auto dpp_add = [](float x, auto ctrl) {
    const int y = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), decltype(ctrl)::value, 0xF, 0xF, false);
    return x + __builtin_bit_cast(float, y);
  };
  v = dpp_add(v, std::integral_constant<int, 0xB1>{});    // quad_perm [1,0,3,2]
  v = dpp_add(v, std::integral_constant<int, 0x4E>{});    // quad_perm [2,3,0,1]
  v = dpp_add(v, std::integral_constant<int, 0x141>{});   // row_half_mirror
  v = dpp_add(v, std::integral_constant<int, 0x140>{});   // row_mirror
  return v;
}

// Column sums over the workgroup's rows of a result held as acc[db][r] (lane = row, registers =
// head columns db*32 + 8*(r/4) + 4*hf + r%4), scaled by `scale`, written to out[0 .. DH).
// red: 16 * DHP floats of LDS that no wave still reads (one partial row per 16 lanes).
template <int DH>
__device__ __forceinline__ void block_column_sums(const f32x16 (&acc)[Cfg<DH>::DB], float scale, float* red, float* out,
                                                  int tid, int lane, int wave) {
  using C = Cfg<DH>;
  const int hf = lane >> 5;
  float* mine = red + (wave * 2 + ((lane >> 4) & 1)) * C::DHP + 4 * hf;
#pragma unroll
  for (int db = 0; db < C::DB; ++db)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      float4 v;
      v.x = row16_sum(acc[db][4 * g]);
      v.y = row16_sum(acc[db][4 * g + 1]);
      v.z = row16_sum(acc[db][4 * g + 2]);
      v.w = row16_sum(acc[db][4 * g + 3]);
      if ((lane & 15) == 0) *reinterpret_cast<float4*>(mine + db * 32 + 8 * g) = v;
    }
  __syncthreads();
  for (int d = tid; d < DH; d += kThreads) {
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < 2 * kWaves; ++w) t += red[w * C::DHP + d];
    out[d] = t * scale;
  }
}

// Rows of a result held as acc[db][r] (lane % 32 = row, registers = head columns db*32 + 8*(r/4) + 4*hf + r%4),
// times `scale`, to out[row][0 .. DH) (bf16, `ld` elements between rows; `out` is row 0 of this wave's 32 rows, of
// which the first rows_valid exist).  Stored as they lie in the registers, a lane writes 8-byte pieces and one store
// instruction touches 32 rows with 16 bytes each: measured, those stores were two thirds of what the dK/dV kernel costs
// beyond its loop (8.5 of 12.5 us per workgroup at head size 128).  So the rows pass through a wave-private piece
// of LDS (rows 16 bytes apart from a multiple of 256: the 8-byte writes of 32 rows spread over the banks) and
// leave with 16 bytes per lane along a row.  No barrier: the piece belongs to the wave, whose LDS operations
// complete in order.  `strip`: 32 * (2 * DH + 16) bytes.
template <int DH>
constexpr int out_strip_u4() { return 32 * (2 * DH + 16) / 16; }
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
template <int DH>
__device__ __forceinline__ void store_rows(const f32x16 (&acc)[Cfg<DH>::DB], float scale, uint4* strip, bf16_t* out, int64_t ld,
                                           int rows_valid, int lane) {
  using C = Cfg<DH>;
  constexpr int STRIDE = 2 * DH + 16;   // bytes
  char* w = reinterpret_cast<char*>(strip);
  const int l32 = lane & 31, hf = lane >> 5;
#pragma unroll
  for (int db = 0; db < C::DB; ++db)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int d = db * 32 + 8 * g + 4 * hf;
      if (d < DH)
        *reinterpret_cast<uint2*>(w + l32 * STRIDE + d * 2) =
            pack4f(acc[db][4 * g] * scale, acc[db][4 * g + 1] * scale, acc[db][4 * g + 2] * scale, acc[db][4 * g + 3] * scale);
    }
  wave_lds_sync();
  constexpr int TOTAL = 32 * C::CH;   // 16-byte chunks of the 32 rows
#pragma unroll
  for (int it = 0; it < (TOTAL + 63) / 64; ++it) {
    const int L = it * 64 + lane;
    const int row = L / C::CH, ch = L % C::CH;
    if (L < TOTAL && row < rows_valid)
      *reinterpret_cast<uint4*>(out + row * ld + ch * 8) = *reinterpret_cast<const uint4*>(w + row * STRIDE + ch * 16);
  }
  wave_lds_sync();   // the strip may be written again
}

// ------------------------------------------------------------------------------------------------
// forward
template <int DH>
__global__ __launch_bounds__(kThreads, Cfg<DH>::kMinWaves) void attn_fwd_mfma_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ o,
                                                                  float* __restrict__ lse, int s, int a, int mask_mode,
                                                                  const int32_t* __restrict__ seqlens) {
  using C = Cfg<DH>;
  extern __shared__ uint4 smem[];   // stage st: K tile at st * 2 * kTileU4, V tile behind it

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), l32 = lane & 31, hf = lane >> 5;
  // grid = (heads, sequences, row blocks): the row block varies slowest, so all heads' copies of a block are
  // dispatched together, and under a causal mask the blocks with the most keys to visit (the last queries) go
  // first: the workgroups that take longest start earliest and the launch does not end on one of them
  const int n = blockIdx.y, head = blockIdx.x;
  const int blk = mask_mode == 1 ? (int)(gridDim.z - 1 - blockIdx.z) : (int)blockIdx.z;
  const int i0 = blk * kBlockRows;
  const int h = a * DH;
  const int64_t ld = 3 * (int64_t)h;
  const bf16_t* base = qkv + (int64_t)n * s * ld + head * DH;
  const int kv_len = mask_mode == 2 ? min(max(seqlens[n], 1), s) : s;   // lengths outside [1, s] are clamped: no read past the sequence, no empty row
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

  const int jend = causal ? min(i0 + kBlockRows, s) : kv_len;
  const int ntiles = (jend + kTile - 1) / kTile;
  TileLoader<DH> loader;
  loader.init(wave, lane);
  loader.issue(base + h, ld, 0, jend, smem);
  loader.issue(base + 2 * h, ld, 0, jend, smem + C::kTileU4);
  for (int t = 0; t < ntiles; ++t) {
    const int j0 = t * kTile;
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));   // this wave's share of tile t has landed
    __syncthreads();                            // ... and everyone's; all waves are done with tile t-1
    if (t + 1 < ntiles) {
      uint4* nxt = smem + ((t + 1) & 1) * 2 * C::kTileU4;
      loader.issue(base + h, ld, j0 + kTile, jend, nxt);
      loader.issue(base + 2 * h, ld, j0 + kTile, jend, nxt + C::kTileU4);
    }
    if (causal && j0 > iw0 + 31) continue;   // every key of the tile lies after this wave's queries
    const uint4* k_lds = smem + (t & 1) * 2 * C::kTileU4;
    const uint4* v_lds = k_lds + C::kTileU4;

    f32x16 sacc[2] = {zero16(), zero16()};
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) {
      sacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows<DH>(k_lds, l32, ks, hf), qf[ks], sacc[0], 0, 0, 0);
      sacc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows<DH>(k_lds, 32 + l32, ks, hf), qf[ks], sacc[1], 0, 0, 0);
    }
    // masks (only tiles that touch a boundary need them) and the running maximum
    const bool need_mask = (j0 + kTile > kv_len) || (causal && j0 + kTile - 1 > iw0);
    if (need_mask) {
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = j0 + nb * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
          const bool vis = key < kv_len && (!causal || key <= i);
          sacc[nb][r] = vis ? sacc[nb][r] : -INFINITY;
        }
    }
    float mloc = -INFINITY;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mloc = fmaxf(mloc, sacc[nb][r]);
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
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_cols<DH>(v_lds, db * 32, kk, lane), pb[kk], oacc[db], 0, 0, 0);
  }

  const float l_tot = l_i + __shfl_xor(l_i, 32, 64);
  __syncthreads();   // every wave is done with the K / V tiles, whose LDS the output strips re-use
  const float inv = 1.0f / l_tot;   // (rows past the sequence: never stored)
  store_rows<DH>(oacc, inv, smem + wave * out_strip_u4<DH>(), o + ((int64_t)n * s + iw0) * h + head * DH, h, s - iw0, lane);
  if (i < s && hf == 0) lse[((int64_t)n * a + head) * s + i] = m_i * scale + logf(l_tot);
}

// ------------------------------------------------------------------------------------------------
// dQ (and delta = rowsum(dO * O), which the dK/dV kernel reads afterwards)
template <int DH>
__global__ __launch_bounds__(kThreads, Cfg<DH>::kMinWaves) void attn_dq_mfma_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ o,
                                                                 const bf16_t* __restrict__ d_o, const float* __restrict__ lse,
                                                                 float* __restrict__ delta, bf16_t* __restrict__ dqkv, int s,
                                                                 int a, int mask_mode, const int32_t* __restrict__ seqlens,
                                                                 float* __restrict__ colsum) {
  using C = Cfg<DH>;
  extern __shared__ uint4 smem[];   // stage st: K tile at st * 2 * kTileU4, V tile behind it

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), l32 = lane & 31, hf = lane >> 5;
  // grid = (heads, sequences, row blocks): the row block varies slowest, so all heads' copies of a block are
  // dispatched together, and under a causal mask the blocks with the most keys to visit (the last queries) go
  // first: the workgroups that take longest start earliest and the launch does not end on one of them
  const int n = blockIdx.y, head = blockIdx.x;
  const int blk = mask_mode == 1 ? (int)(gridDim.z - 1 - blockIdx.z) : (int)blockIdx.z;
  const int i0 = blk * kBlockRows;
  const int h = a * DH;
  const int64_t ld = 3 * (int64_t)h;
  const bf16_t* base = qkv + (int64_t)n * s * ld + head * DH;
  const int kv_len = mask_mode == 2 ? min(max(seqlens[n], 1), s) : s;   // lengths outside [1, s] are clamped: no read past the sequence, no empty row
  const bool causal = mask_mode == 1;
  const int iw0 = i0 + wave * 32;
  const int i = iw0 + l32;
  const bool row_ok = i < s;
  const float scale = 1.0f / sqrtf((float)DH);
  const float c = scale * kLog2e;

  const int jend = causal ? min(i0 + kBlockRows, s) : kv_len;
  const int ntiles = (jend + kTile - 1) / kTile;
  TileLoader<DH> loader;
  loader.init(wave, lane);
  loader.issue(base + h, ld, 0, jend, smem);
  loader.issue(base + 2 * h, ld, 0, jend, smem + C::kTileU4);

  bf16x8 qf[C::KS], dof[C::KS];
  load_frags<DH>(base + (int64_t)i * ld, row_ok, hf, qf);
  load_frags<DH>(d_o + ((int64_t)n * s + i) * h + head * DH, row_ok, hf, dof);
  float delta_i;
  {
    bf16x8 of[C::KS];
    load_frags<DH>(o + ((int64_t)n * s + i) * h + head * DH, row_ok, hf, of);
    float part = 0.f;
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks)
#pragma unroll
      for (int e = 0; e < 8; ++e) part = fmaf((float)dof[ks][e], (float)of[ks][e], part);
    delta_i = part + __shfl_xor(part, 32, 64);
    if (row_ok && hf == 0) delta[((int64_t)n * a + head) * s + i] = delta_i;
  }
  const float lse_i = row_ok ? lse[((int64_t)n * a + head) * s + i] * kLog2e : INFINITY;
  f32x16 dq[C::DB];
#pragma unroll
  for (int db = 0; db < C::DB; ++db) dq[db] = zero16();

  for (int t = 0; t < ntiles; ++t) {
    const int j0 = t * kTile;
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __syncthreads();
    if (t + 1 < ntiles) {
      uint4* nxt = smem + ((t + 1) & 1) * 2 * C::kTileU4;
      loader.issue(base + h, ld, j0 + kTile, jend, nxt);
      loader.issue(base + 2 * h, ld, j0 + kTile, jend, nxt + C::kTileU4);
    }
    if (causal && j0 > iw0 + 31) continue;
    const uint4* k_lds = smem + (t & 1) * 2 * C::kTileU4;
    const uint4* v_lds = k_lds + C::kTileU4;

    f32x16 sacc[2] = {zero16(), zero16()}, dp[2] = {zero16(), zero16()};
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) {
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
        sacc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows<DH>(k_lds, nb * 32 + l32, ks, hf), qf[ks], sacc[nb], 0, 0, 0);
        dp[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows<DH>(v_lds, nb * 32 + l32, ks, hf), dof[ks], dp[nb], 0, 0, 0);
      }
    }
    const bool need_mask = (j0 + kTile > kv_len) || (causal && j0 + kTile - 1 > iw0);
    if (need_mask) {   // a masked score of -inf gives probability exactly 0
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = j0 + nb * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
          const bool vis = key < kv_len && (!causal || key <= i);
          sacc[nb][r] = vis ? sacc[nb][r] : -INFINITY;
        }
    }
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float pv = __builtin_amdgcn_exp2f(fmaf(sacc[nb][r], c, -lse_i));
        sacc[nb][r] = pv * (dp[nb][r] - delta_i);   // dS^T (the 1/sqrt(dh) factor is applied at the end)
      }
    bf16x8 dsb[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) dsb[kk] = pack_half(sacc[kk >> 1], kk & 1);
#pragma unroll
    for (int db = 0; db < C::DB; ++db)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
        dq[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_cols<DH>(k_lds, db * 32, kk, lane), dsb[kk], dq[db], 0, 0, 0);
  }
  __syncthreads();   // every wave is done with the K / V tiles
  if (colsum) {   // rows past the end of the sequence hold zeros
    float* row = colsum + ((int64_t)n * gridDim.z + blk) * ld + head * DH;
    block_column_sums<DH>(dq, scale, reinterpret_cast<float*>(smem), row, tid, lane, wave);
    __syncthreads();   // ... and with the partial rows of the sums
  }
  store_rows<DH>(dq, scale, smem + wave * out_strip_u4<DH>(), dqkv + ((int64_t)n * s + iw0) * ld + head * DH, ld, s - iw0, lane);
}

// ------------------------------------------------------------------------------------------------
// dK, dV
template <int DH>
__global__ __launch_bounds__(kThreads, Cfg<DH>::kMinWaves) void attn_dkv_mfma_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ d_o,
                                                                  const float* __restrict__ lse, const float* __restrict__ delta,
                                                                  bf16_t* __restrict__ dqkv, int s, int a, int mask_mode,
                                                                  const int32_t* __restrict__ seqlens, float* __restrict__ colsum) {
  using C = Cfg<DH>;
  extern __shared__ uint4 smem[];
  // stage st: Q tile, dO tile, 64 lse, 64 delta
  constexpr int kStageU4 = 2 * C::kTileU4 + 2 * kTile / 4;

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), l32 = lane & 31, hf = lane >> 5;
  // grid = (heads, sequences, key blocks), key block slowest: under a causal mask the first keys are seen by
  // the most queries, and those workgroups are dispatched first (see the forward kernel)
  const int n = blockIdx.y, head = blockIdx.x, blk = blockIdx.z;
  const int j0 = blk * kBlockRows;
  const int h = a * DH;
  const int64_t ld = 3 * (int64_t)h;
  const bf16_t* base = qkv + (int64_t)n * s * ld + head * DH;
  const bf16_t* dobase = d_o + (int64_t)n * s * h + head * DH;
  const float* lse_row = lse + ((int64_t)n * a + head) * s;
  const float* delta_row = delta + ((int64_t)n * a + head) * s;
  const int kv_len = mask_mode == 2 ? min(max(seqlens[n], 1), s) : s;   // lengths outside [1, s] are clamped: no read past the sequence, no empty row
  const bool causal = mask_mode == 1;
  const int jw0 = j0 + wave * 32;
  const int j = jw0 + l32;
  const bool row_ok = j < s;
  const float scale = 1.0f / sqrtf((float)DH);
  const float c = scale * kLog2e;

  bf16x8 kf[C::KS], vf[C::KS];
  load_frags<DH>(base + h + (int64_t)j * ld, row_ok, hf, kf);
  load_frags<DH>(base + 2 * h + (int64_t)j * ld, row_ok, hf, vf);
  // At head size 128 the two accumulators are 128 registers and the K and V fragments of the wave's keys 64 more: with
  // the scores on top the kernel spilled.  There the V fragments wait in a wave-private piece of LDS (16 bytes per
  // lane and k-step, read back in the order written: no bank conflicts, no barrier) and are fetched per use.
  constexpr bool kVInLds = Cfg<DH>::kDkvVInLds;
  uint4* vstore = smem + 2 * kStageU4 + C::kPadU4 + wave * (C::KS * 64);
  if (kVInLds) {
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) vstore[ks * 64 + lane] = __builtin_bit_cast(uint4, vf[ks]);
  }
  f32x16 dk[C::DB], dv[C::DB];
#pragma unroll
  for (int db = 0; db < C::DB; ++db) { dk[db] = zero16(); dv[db] = zero16(); }

  const bool wg_dead = j0 >= kv_len;                       // every key of the workgroup is padding
  const int istart = causal ? (j0 / kTile) * kTile : 0;    // earlier queries see none of these keys
  const int ntiles = wg_dead ? 0 : (s - istart + kTile - 1) / kTile;
  TileLoader<DH> loader;
  loader.init(wave, lane);
  auto issue_tile = [&](int i0, uint4* stage) {
    loader.issue(base, ld, i0, s, stage);
    loader.issue(dobase, (int64_t)h, i0, s, stage + C::kTileU4);
    float* f = reinterpret_cast<float*>(stage + 2 * C::kTileU4);
    if (wave == 0) issue_floats(lse_row, i0, s, f, lane);
    if (wave == 1) issue_floats(delta_row, i0, s, f + kTile, lane);
  };
  if (ntiles > 0) issue_tile(istart, smem);
  for (int t = 0; t < ntiles; ++t) {
    const int i0 = istart + t * kTile;
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __syncthreads();
    if (t + 1 < ntiles) issue_tile(i0 + kTile, smem + ((t + 1) & 1) * kStageU4);
    const uint4* q_lds = smem + (t & 1) * kStageU4;
    const uint4* do_lds = q_lds + C::kTileU4;
    const float* lse_lds = reinterpret_cast<const float*>(q_lds + 2 * C::kTileU4);
    const float* delta_lds = lse_lds + kTile;
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const int ib = i0 + qb * 32;
      if (causal && ib + 31 < jw0) continue;   // all 32 queries lie before this wave's keys
      if (ib >= s) continue;                   // no query of the block exists
      f32x16 sacc = zero16(), dp = zero16();
#pragma unroll
      for (int ks = 0; ks < C::KS; ++ks) {
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows<DH>(q_lds, qb * 32 + l32, ks, hf), kf[ks], sacc, 0, 0, 0);
        const bf16x8 vfr = kVInLds ? __builtin_bit_cast(bf16x8, vstore[ks * 64 + lane]) : vf[ks];
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows<DH>(do_lds, qb * 32 + l32, ks, hf), vfr, dp, 0, 0, 0);
      }
      const bool need_mask = (jw0 + 32 > kv_len) || (causal && jw0 + 31 > ib) || (ib + 32 > s);
      if (need_mask) {   // a masked score of -inf gives probability exactly 0
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int iq = ib + 8 * (r >> 2) + 4 * hf + (r & 3);
          const bool vis = j < kv_len && (!causal || j <= iq) && iq < s;
          sacc[r] = vis ? sacc[r] : -INFINITY;
        }
      }
      f32x16 pv16, ds16;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 l4 = *reinterpret_cast<const float4*>(lse_lds + qb * 32 + 8 * g + 4 * hf);
        const float4 d4 = *reinterpret_cast<const float4*>(delta_lds + qb * 32 + 8 * g + 4 * hf);
        const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dl[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
        for (int t4 = 0; t4 < 4; ++t4) {
          const int r = 4 * g + t4;
          const float pv = __builtin_amdgcn_exp2f(fmaf(sacc[r], c, -lv[t4] * kLog2e));
          pv16[r] = pv;
          ds16[r] = pv * (dp[r] - dl[t4]);
        }
      }
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const bf16x8 pb = pack_half(pv16, half), dsb = pack_half(ds16, half);
        const int kk = qb * 2 + half;
#pragma unroll
        for (int db = 0; db < C::DB; ++db) {
          dv[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_cols<DH>(do_lds, db * 32, kk, lane), pb, dv[db], 0, 0, 0);
          dk[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_cols<DH>(q_lds, db * 32, kk, lane), dsb, dk[db], 0, 0, 0);
        }
      }
    }
  }
  __syncthreads();   // every wave is done with the Q / dO tiles
  if (colsum) {   // masked and non-existent keys hold zeros
    float* row = colsum + ((int64_t)n * gridDim.z + blk) * ld + head * DH;
    float* red = reinterpret_cast<float*>(smem);
    block_column_sums<DH>(dk, scale, red, row + h, tid, lane, wave);
    __syncthreads();
    block_column_sums<DH>(dv, 1.0f, red, row + 2 * h, tid, lane, wave);
    __syncthreads();
  }
  bf16_t* outk = dqkv + ((int64_t)n * s + jw0) * ld + h + head * DH;
  uint4* strip = smem + wave * out_strip_u4<DH>();
  store_rows<DH>(dk, scale, strip, outk, ld, s - jw0, lane);
  store_rows<DH>(dv, 1.0f, strip, outk + h, ld, s - jw0, lane);
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
  constexpr size_t lds_out = (size_t)kWaves * out_strip_u4<DH>() * sizeof(uint4);   // the output strips re-use the tiles' LDS
  constexpr size_t lds_tiles = (4 * C::kTileU4 + C::kPadU4) * sizeof(uint4);
  constexpr size_t lds = lds_tiles > lds_out ? lds_tiles : lds_out;
  static bool done = false;
  hipError_t e = set_lds(attn_fwd_mfma_kernel<DH>, lds, &done);
  if (e != hipSuccess) return e;
  dim3 grid(d.a, d.b, ceil_div(d.s, kBlockRows));
  hipLaunchKernelGGL(attn_fwd_mfma_kernel<DH>, grid, dim3(kThreads), lds, st, static_cast<const bf16_t*>(qkv),
                     static_cast<bf16_t*>(o), lse, d.s, d.a, d.mask_mode, d.seqlens);
  return hipGetLastError();
}

template <int DH>
hipError_t bwd_launch(const AttnDesc& d, const void* qkv, const void* o, const float* lse, const void* d_o, void* dqkv,
                      float* delta, hipStream_t st) {
  using C = Cfg<DH>;
  constexpr size_t lds_out = (size_t)kWaves * out_strip_u4<DH>() * sizeof(uint4);   // the output strips re-use the tiles' LDS
  constexpr size_t lds_dq_tiles = (4 * C::kTileU4 + C::kPadU4) * sizeof(uint4);
  constexpr size_t lds_dq = lds_dq_tiles > lds_out ? lds_dq_tiles : lds_out;
  constexpr size_t lds_dkv_tiles = (2 * (2 * C::kTileU4 + 2 * kTile / 4) + C::kPadU4 + (C::kDkvVInLds ? kWaves * C::KS * 64 : 0)) * sizeof(uint4);
  constexpr size_t lds_dkv = lds_dkv_tiles > lds_out ? lds_dkv_tiles : lds_out;
  static_assert(lds_dkv <= 160 * 1024, "LDS of a CU");
  static bool done_dq = false, done_dkv = false;
  hipError_t e = set_lds(attn_dq_mfma_kernel<DH>, lds_dq, &done_dq);
  if (e != hipSuccess) return e;
  e = set_lds(attn_dkv_mfma_kernel<DH>, lds_dkv, &done_dkv);
  if (e != hipSuccess) return e;
  dim3 grid(d.a, d.b, ceil_div(d.s, kBlockRows));
  hipLaunchKernelGGL(attn_dq_mfma_kernel<DH>, grid, dim3(kThreads), lds_dq, st, static_cast<const bf16_t*>(qkv),
                     static_cast<const bf16_t*>(o), static_cast<const bf16_t*>(d_o), lse, delta,
                     static_cast<bf16_t*>(dqkv), d.s, d.a, d.mask_mode, d.seqlens, d.colsum_partial);
  hipLaunchKernelGGL(attn_dkv_mfma_kernel<DH>, grid, dim3(kThreads), lds_dkv, st, static_cast<const bf16_t*>(qkv),
                     static_cast<const bf16_t*>(d_o), lse, delta, static_cast<bf16_t*>(dqkv), d.s, d.a, d.mask_mode,
                     d.seqlens, d.colsum_partial);
  return hipGetLastError();
}

}  // namespace

int attention_colsum_rows(int b, int s) { return b * ceil_div(s, kBlockRows); }

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
