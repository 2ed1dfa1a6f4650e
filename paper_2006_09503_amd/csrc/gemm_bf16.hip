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
// (TN) forms.  Two LDS stages.  Per K step a wave issues the global loads of the next tile
// first, runs its MFMAs with the LDS fragment reads of sub-step ks+1 in flight behind the MFMAs
// of sub-step ks, and writes the prefetched tile to the other LDS stage during the last two
// sub-steps; one barrier per K step.  Out-of-range rows/chunks are loaded from a clamped
// address and zeroed by select, so the loop has no divergent branches.
//
// Lane layout of v_mfma_f32_32x32x16_bf16: lane l supplies row (l % 32) of the first operand and
// column (l % 32) of the second, k = 8*(l/32) .. +7; it receives column (l % 32) of D, rows
// 8*(r/4) + 4*(l/32) + (r % 4) for accumulator register r.  The kernel feeds the B tile as the
// first operand and the A tile as the second, i.e. it accumulates C^T blocks: a lane then owns
// one row m of C and four consecutive columns n per register quad, which makes the epilogue's
// global accesses 8-byte (bf16) or 16-byte (fp32 accumulator) vectors.
#include "kernels.hpp"

namespace k2bw {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kMaxGroup = 4;   // GEMMs of one form that may share a launch

struct BfParams {
  const bf16_t* A; const bf16_t* B; void* C;
  int M, N, K, lda, ldb, ldc;
  const bf16_t* bias; const bf16_t* aux; bf16_t* aux_out;
  int accumulate;
  int tiles_m, tiles_n;
};

// Up to kMaxGroup independent GEMMs of the same form in one launch: workgroup ids
// [tile_start[g], tile_start[g+1]) belong to problem g.
struct GroupParams {
  BfParams p[kMaxGroup];
  int tile_start[kMaxGroup + 1];
  int count;
};

// Chunk swizzle.  Three LDS access patterns have to avoid bank conflicts at once: fragment
// reads (32 consecutive rows, same logical chunk, 16 bytes per lane), direct stores (the 8 or 16
// chunks of a row by consecutive lanes) and transposing stores (rows 8 apart, same chunk, 8 bytes
// per lane).  Rows of 8 chunks are 128 bytes, so two rows share a 256-byte bank line: XOR the
// chunk with ((row >> 1) ^ (row >> 4)) & 7; rows of 16 chunks: (row ^ (row >> 4)) & 15.
// Measured with rocprofv3 (SQ_LDS_BANK_CONFLICT, 8192^3): 0 for the form with two direct
// operands; the transposing stores keep a 2-way conflict (4 cycles per 8-byte store wave-op).
// Other candidates tried: (row + (row>>3)) & 7, row & 7, ((row>>1) ^ (row>>3)) & 7 cost 4 extra
// cycles on every fragment read; (row >> 1) & 7 makes the transposing stores 4-way conflicted.
template <int CH>
__device__ __forceinline__ int swz(int row) {
  return CH == 8 ? ((row >> 1) ^ (row >> 4)) & 7 : (row ^ (row >> 4)) & 15;
}

__device__ __forceinline__ uint4 select_zero(bool ok, uint4 v) {
  v.x = ok ? v.x : 0u; v.y = ok ? v.y : 0u; v.z = ok ? v.z : 0u; v.w = ok ? v.w : 0u;
  return v;
}

// Operand with K contiguous in HBM: tile rows = R, CH chunks of 8 bf16 per row.
template <int R, int NT, int BK>
struct DirectLoader {
  static constexpr int CH = BK / 8;
  static constexpr int kIters = R * CH / NT;
  static_assert(R * CH % NT == 0 && NT % CH == 0, "tile/threads mismatch");
  uint4 regs[kIters];
  const bf16_t* base_;         // uniform: element (row0, k = 0)
  uint32_t off[kIters];        // (clamped row) * ld, in elements: 32-bit offsets from base_
  int lds_idx[kIters];
  bool row_ok[kIters];
  int c8;                      // this thread's k offset inside a tile (same for every iter)
  // base: element (row0, k = 0); rows_valid >= 1: rows of the tile inside the matrix
  __device__ __forceinline__ void init(const bf16_t* base, int ld, int rows_valid, int tid) {
    base_ = base;
    c8 = (tid % CH) * 8;
#pragma unroll
    for (int i = 0; i < kIters; ++i) {
      const int idx = tid + i * NT;
      const int row = idx / CH, c = idx % CH;
      row_ok[i] = row < rows_valid;
      const int rc = row_ok[i] ? row : rows_valid - 1;
      off[i] = (uint32_t)rc * (uint32_t)ld;
      lds_idx[i] = row * CH + (c ^ swz<CH>(row));
    }
  }
  // The zeroing of out-of-range data happens at store time, so that nothing waits on the
  // loads before the MFMAs of the current tile have been issued.
  bool k_ok[kIters];
  __device__ __forceinline__ void load_one(int i, int k0, int K) {
    const int k = k0 + c8;
    k_ok[i] = k < K;
    regs[i] = *reinterpret_cast<const uint4*>(base_ + (off[i] + (uint32_t)(k_ok[i] ? k : K - 8)));
  }
  __device__ __forceinline__ void load(int k0, int K) {
#pragma unroll
    for (int i = 0; i < kIters; ++i) load_one(i, k0, K);
  }
  __device__ __forceinline__ void store(uint4* tile) {
#pragma unroll
    for (int i = 0; i < kIters; ++i) tile[lds_idx[i]] = select_zero(k_ok[i] && row_ok[i], regs[i]);
  }
  // Slice `part` of `nparts` of the per-step work: store this slice of the tile held in
  // registers, then refill those registers with the tile at k0_next.  Spreading the slices over
  // the MFMA sub-steps keeps LDS stores from queueing up in front of the fragment reads.
  // Unconditional on purpose (past the end the loads read a clamped, valid address and the
  // stores fill a stage nobody reads): with no branches in the K loop the compiler can count
  // outstanding loads exactly instead of waiting for all of them before every store.
  __device__ __forceinline__ void step(int part, int nparts, uint4* tile, int k0_next, int K) {
    static_assert(kIters % 2 == 0, "");
#pragma unroll
    for (int i = 0; i < kIters; ++i) {
      if (i * nparts / kIters != part) continue;
      tile[lds_idx[i]] = select_zero(k_ok[i] && row_ok[i], regs[i]);
      load_one(i, k0_next, K);
    }
  }
};

__device__ __forceinline__ uint32_t word(const uint4& v, int i) {
  return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w;
}

// Operand with the row index contiguous in HBM (element (row, k) at base[k*ld + row]).
template <int R, int NT, int BK>
struct TransposingLoader {
  static constexpr int CH = BK / 8;
  static constexpr int kUnits = (BK / 4) * (R / 8);  // 4(k) x 8(row) patches per tile
  static constexpr int kIters = kUnits / NT;
  static_assert(kUnits % NT == 0, "tile/threads mismatch");
  uint4 regs[kIters][4];
  const bf16_t* base_;         // uniform: element (row0, k = 0)
  uint32_t off[kIters];        // (clamped) row chunk, in elements
  int kq[kIters], rc8[kIters];
  bool row_ok[kIters];
  int ld_;
  int k_left[kIters];   // K - k0 of the tile held in regs[i]
  // rows_valid: multiple of 8, >= 8
  __device__ __forceinline__ void init(const bf16_t* base, int ld, int rows_valid, int tid) {
    ld_ = ld;
    base_ = base;
#pragma unroll
    for (int i = 0; i < kIters; ++i) {
      const int u = tid + i * NT;
      const int rc = u % (R / 8);
      kq[i] = u / (R / 8);
      rc8[i] = rc * 8;
      row_ok[i] = rc * 8 < rows_valid;
      off[i] = (uint32_t)(row_ok[i] ? rc * 8 : rows_valid - 8);
    }
  }
  __device__ __forceinline__ void load_one(int i, int k0, int K) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int k = k0 + kq[i] * 4 + j;
      const int kc = k < K ? k : K - 1;
      regs[i][j] = *reinterpret_cast<const uint4*>(base_ + (off[i] + (uint32_t)kc * (uint32_t)ld_));
    }
    k_left[i] = K - k0;
  }
  __device__ __forceinline__ void load(int k0, int K) {
#pragma unroll
    for (int i = 0; i < kIters; ++i) load_one(i, k0, K);
  }
  // zero what lies outside the matrix (row chunks past the edge, k rows past K); branch-free
  __device__ __forceinline__ void mask_one(int i) {
#pragma unroll
    for (int j = 0; j < 4; ++j) regs[i][j] = select_zero(row_ok[i] && (kq[i] * 4 + j < k_left[i]), regs[i][j]);
  }
  __device__ __forceinline__ void store_piece(int i, int ii, uint2* t2) const {
    const int wd = ii >> 1;
    const uint32_t w0 = word(regs[i][0], wd), w1 = word(regs[i][1], wd);
    const uint32_t w2 = word(regs[i][2], wd), w3 = word(regs[i][3], wd);
    // v_perm_b32 picks bytes from {first operand: bytes 4..7, second operand: bytes 0..3}
    uint2 o;
    if (ii & 1) {   // (w0 >> 16) | (w1 & 0xffff0000)
      o.x = __builtin_amdgcn_perm(w1, w0, 0x07060302u);
      o.y = __builtin_amdgcn_perm(w3, w2, 0x07060302u);
    } else {        // (w0 & 0xffff) | (w1 << 16)
      o.x = __builtin_amdgcn_perm(w1, w0, 0x05040100u);
      o.y = __builtin_amdgcn_perm(w3, w2, 0x05040100u);
    }
    const int row = rc8[i] + ii;
    t2[(row * CH + ((kq[i] >> 1) ^ swz<CH>(row))) * 2 + (kq[i] & 1)] = o;
  }
  __device__ __forceinline__ void store(uint4* tile) {
    uint2* t2 = reinterpret_cast<uint2*>(tile);
#pragma unroll
    for (int i = 0; i < kIters; ++i) {
      mask_one(i);
#pragma unroll
      for (int ii = 0; ii < 8; ++ii) store_piece(i, ii, t2);
    }
  }
  // see DirectLoader::step; a patch's registers are refilled once its eighth piece is stored
  __device__ __forceinline__ void step(int part, int nparts, uint4* tile, int k0_next, int K) {
    uint2* t2 = reinterpret_cast<uint2*>(tile);
    constexpr int S = kIters * 8;
#pragma unroll
    for (int sidx = 0; sidx < S; ++sidx) {
      if (sidx * nparts / S != part) continue;
      const int i = sidx / 8, ii = sidx % 8;
      if (ii == 0) mask_one(i);
      store_piece(i, ii, t2);
      if (ii == 7) load_one(i, k0_next, K);
    }
  }
};

template <int R, int NT, int BK, bool K_CONTIGUOUS>
struct LoaderSel { using type = DirectLoader<R, NT, BK>; };
template <int R, int NT, int BK>
struct LoaderSel<R, NT, BK, false> { using type = TransposingLoader<R, NT, BK>; };

__device__ __forceinline__ uint2 pack4(const float (&v)[4]) {
  return make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
}
__device__ __forceinline__ void unpack4(uint2 w, float (&v)[4]) {
  v[0] = __uint_as_float(w.x << 16); v[1] = __uint_as_float(w.x & 0xffff0000u);
  v[2] = __uint_as_float(w.y << 16); v[3] = __uint_as_float(w.y & 0xffff0000u);
}

template <int BM, int BN, int WM, int WN, int BK, bool TA, bool TB, int EPI>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64) void gemm_bf16_kernel(GroupParams gp) {
  constexpr int NT = (BM / WM) * (BN / WN) * 64;
  constexpr int CH = BK / 8;
  constexpr int MI = WM / 32, NI = WN / 32;
  constexpr int WAVES_N = BN / WN;
  constexpr int KS = BK / 16;
  constexpr bool kFragDbuf = NT <= 256;
  extern __shared__ uint4 smem[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;

  // Workgroup -> tile: consecutive workgroup ids land on different XCDs (round-robin over 8),
  // so give each XCD a contiguous run of tiles: they share A rows / B columns in that XCD's L2.
  const int n_tiles = gp.tile_start[gp.count];
  int wg = blockIdx.x;
  {
    const int per_xcd = n_tiles / 8;
    if (wg < per_xcd * 8) wg = (wg % 8) * per_xcd + wg / 8;
  }
  int g = 0;
#pragma unroll
  for (int q = 1; q < kMaxGroup; ++q)
    if (q < gp.count && wg >= gp.tile_start[q]) g = q;
  const BfParams& p = gp.p[g];
  wg -= gp.tile_start[g];
  const int bm = wg / p.tiles_n, bn = wg % p.tiles_n;
  const int m0 = bm * BM, n0 = bn * BN;

  typename LoaderSel<BM, NT, BK, !TA>::type ld_a;
  typename LoaderSel<BN, NT, BK, TB>::type ld_b;
  ld_a.init(TA ? p.A + m0 : p.A + (int64_t)m0 * p.lda, p.lda, p.M - m0, tid);
  ld_b.init(TB ? p.B + (int64_t)n0 * p.ldb : p.B + n0, p.ldb, p.N - n0, tid);

  constexpr int kStage = (BM + BN) * CH;  // uint4 per stage
  f32x16 acc[MI][NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

  const int nk = (p.K + BK - 1) / BK;
  ld_a.load(0, p.K);
  ld_b.load(0, p.K);
  ld_a.store(smem);
  ld_b.store(smem + BM * CH);
  ld_a.load(BK, p.K);   // tile 1 stays in flight in registers during the first K step
  ld_b.load(BK, p.K);
  __syncthreads();

  const int khalf = lane >> 5;
  // fragment addresses (uint4 index inside a stage's A / B tile) for sub-step 0; sub-step ks
  // flips chunk bits: chunk = (2*ks + khalf) ^ swz(row)
  int a_row[MI], b_row[NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) a_row[mi] = wm * WM + mi * 32 + (lane & 31);
#pragma unroll
  for (int ni = 0; ni < NI; ++ni) b_row[ni] = wn * WN + ni * 32 + (lane & 31);

  // K step kt: MFMAs on stage kt&1.  In the middle of the step the tile kt+1, whose global loads
  // were issued one whole step earlier, goes from registers to the other stage, and the loads of
  // tile kt+2 are issued into the freed registers: they have a full step to arrive.
  for (int kt = 0; kt < nk; ++kt) {
    const uint4* sA = smem + (kt & 1) * kStage;
    const uint4* sB = sA + BM * CH;
    uint4* dA = smem + ((kt + 1) & 1) * kStage;
    // With one wave per SIMD (4-wave configurations) the fragments of sub-step ks+1 are read
    // while the MFMAs of sub-step ks run; with two waves per SIMD the other wave covers the LDS
    // latency and the registers are better spent elsewhere.
    constexpr int FB = kFragDbuf ? 2 : 1;
    bf16x8 af[FB][MI], bfr[FB][NI];
    if (kFragDbuf) {
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
        af[0][mi] = __builtin_bit_cast(bf16x8, sA[a_row[mi] * CH + (khalf ^ swz<CH>(a_row[mi]))]);
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
        bfr[0][ni] = __builtin_bit_cast(bf16x8, sB[b_row[ni] * CH + (khalf ^ swz<CH>(b_row[ni]))]);
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int cur = kFragDbuf ? (ks & 1) : 0, nxt = kFragDbuf ? (cur ^ 1) : 0;
      const int kr = kFragDbuf ? ks + 1 : ks;   // sub-step whose fragments are read now
      if (kr < KS) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
          af[nxt][mi] = __builtin_bit_cast(bf16x8, sA[a_row[mi] * CH + ((kr * 2 + khalf) ^ swz<CH>(a_row[mi]))]);
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
          bfr[nxt][ni] = __builtin_bit_cast(bf16x8, sB[b_row[ni] * CH + ((kr * 2 + khalf) ^ swz<CH>(b_row[ni]))]);
      }
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[cur][ni], af[cur][mi], acc[mi][ni], 0, 0, 0);
      // sub-steps 0..KS/2-1 move slices of the A tile, the rest slices of the B tile
      if (ks < KS / 2) ld_a.step(ks, KS / 2, dA, (kt + 2) * BK, p.K);
      else ld_b.step(ks - KS / 2, KS / 2, dA + BM * CH, (kt + 2) * BK, p.K);
      // keep each slice's stores and loads inside its sub-step: left alone, the scheduler sinks
      // every global load to the end of the K step and hoists the selects that wait for them
      __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();
  }

  // epilogue: lane owns row m = .. + (lane % 32) and, per register quad g, columns
  // n = .. + 8*g + 4*(lane/32) + 0..3 of each 32x32 block
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
    const int row = m0 + wm * WM + mi * 32 + (lane & 31);
    if (row >= p.M) continue;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = n0 + wn * WN + ni * 32 + 8 * g + 4 * khalf;
        if (col >= p.N) continue;   // N is a multiple of 8: a quad is inside or outside as a whole
        const int64_t idx = (int64_t)row * p.ldc + col;
        float v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = acc[mi][ni][4 * g + j];
        if (EPI == kEpiStore || EPI == kEpiGelu) {
          if (p.bias) {
            float b[4];
            unpack4(*reinterpret_cast<const uint2*>(p.bias + col), b);
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] += b[j];
          }
        }
        if (EPI == kEpiStore) {
          if (p.aux) {
            float r[4];
            unpack4(*reinterpret_cast<const uint2*>(p.aux + idx), r);
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] += r[j];
          }
          *reinterpret_cast<uint2*>(static_cast<bf16_t*>(p.C) + idx) = pack4(v);
        } else if (EPI == kEpiGelu) {
          *reinterpret_cast<uint2*>(static_cast<bf16_t*>(p.C) + idx) = pack4(v);
#pragma unroll
          for (int j = 0; j < 4; ++j) v[j] = gelu_fast(v[j]);
          *reinterpret_cast<uint2*>(p.aux_out + idx) = pack4(v);
        } else if (EPI == kEpiGeluGrad) {
          float u[4];
          unpack4(*reinterpret_cast<const uint2*>(p.aux + idx), u);
#pragma unroll
          for (int j = 0; j < 4; ++j) v[j] *= gelu_grad_fast(u[j]);
          *reinterpret_cast<uint2*>(static_cast<bf16_t*>(p.C) + idx) = pack4(v);
        } else {
          float4* c = reinterpret_cast<float4*>(static_cast<float*>(p.C) + idx);
          float4 o = make_float4(v[0], v[1], v[2], v[3]);
          if (p.accumulate) {
            const float4 old = *c;
            o.x += old.x; o.y += old.y; o.z += old.z; o.w += old.w;
          }
          *c = o;
        }
      }
    }
  }
}

template <int BM, int BN, int WM, int WN, int BK, bool TA, bool TB, int EPI>
hipError_t launch(GroupParams gp, hipStream_t s) {
  constexpr int NT = (BM / WM) * (BN / WN) * 64;
  constexpr size_t lds = 2 * (BM + BN) * (BK / 8) * sizeof(uint4);
  auto kern = gemm_bf16_kernel<BM, BN, WM, WN, BK, TA, TB, EPI>;
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    configured = true;
  }
  int total = 0;
  for (int g = 0; g < gp.count; ++g) {
    gp.p[g].tiles_m = ceil_div(gp.p[g].M, BM);
    gp.p[g].tiles_n = ceil_div(gp.p[g].N, BN);
    gp.tile_start[g] = total;
    total += gp.p[g].tiles_m * gp.p[g].tiles_n;
  }
  for (int g = gp.count; g <= kMaxGroup; ++g) gp.tile_start[g] = total;
  hipLaunchKernelGGL(kern, dim3(total), dim3(NT), lds, s, gp);
  return hipGetLastError();
}

int g_tile_override = 0;  // 0: heuristic; else force a tile shape (tuning aid)

template <bool TA, bool TB, int EPI>
hipError_t pick_tile(const GroupParams& gp, hipStream_t s) {
  int tile = g_tile_override;
  if (tile == 0) {
    // Measured on MI355X (M = 4096..8192): 128x128 tiles with two workgroups per CU win until the
    // problem fills the chip several times over with 256x256 tiles; then the 8-wave 256x256
    // kernel is fastest when both operands are K-contiguous, the 4-wave one (512 registers per
    // lane, no spills in the transposing loaders) otherwise.
    int64_t big = 0;
    for (int g = 0; g < gp.count; ++g) big += (int64_t)ceil_div(gp.p[g].M, 256) * ceil_div(gp.p[g].N, 256);
    if (!TA && TB) tile = big >= 192 ? 3 : 2;
    else tile = big >= 512 ? 1 : 2;
  }
  switch (tile) {
    case 1: return launch<256, 256, 128, 128, 64, TA, TB, EPI>(gp, s);
    case 2: return launch<128, 128, 64, 64, 64, TA, TB, EPI>(gp, s);
    case 3: return launch<256, 256, 128, 64, 64, TA, TB, EPI>(gp, s);   // 8 waves
    case 4: return launch<128, 128, 64, 64, 128, TA, TB, EPI>(gp, s);   // deeper K step
    case 5: return launch<256, 128, 128, 64, 64, TA, TB, EPI>(gp, s);
    default: return hipErrorInvalidValue;
  }
}

bool vector_ok(const GemmDesc& d) {
  // 8-byte / 16-byte vector accesses in the epilogue
  return !(d.N % 8 || d.ldc % 8 || (reinterpret_cast<uintptr_t>(d.C) & 15) || (reinterpret_cast<uintptr_t>(d.bias) & 7) ||
           (reinterpret_cast<uintptr_t>(d.aux) & 7) || (reinterpret_cast<uintptr_t>(d.aux_out) & 7));
}

BfParams to_params(const GemmDesc& d) {
  return BfParams{static_cast<const bf16_t*>(d.A), static_cast<const bf16_t*>(d.B), d.C,
                  d.M, d.N, d.K, d.lda, d.ldb, d.ldc, static_cast<const bf16_t*>(d.bias),
                  static_cast<const bf16_t*>(d.aux), static_cast<bf16_t*>(d.aux_out), d.accumulate ? 1 : 0, 0, 0};
}

}  // namespace

void gemm_bf16_set_tile(int id) { g_tile_override = id; }

// `count` GEMMs (1..4) with the same form and epilogue in one launch.
hipError_t gemm_bf16_grouped(const GemmDesc* d, int count, hipStream_t stream) {
  if (count < 1 || count > kMaxGroup) return hipErrorInvalidValue;
  GroupParams gp{};
  gp.count = count;
  for (int g = 0; g < count; ++g) {
    if (!vector_ok(d[g])) return hipErrorInvalidValue;
    if (d[g].trans_a != d[0].trans_a || d[g].trans_b != d[0].trans_b || d[g].epilogue != d[0].epilogue)
      return hipErrorInvalidValue;
    gp.p[g] = to_params(d[g]);
  }
  const GemmDesc& f = d[0];
  if (!f.trans_a && !f.trans_b) {
    if (f.epilogue == kEpiStore) return pick_tile<false, false, kEpiStore>(gp, stream);
    if (f.epilogue == kEpiGelu) return pick_tile<false, false, kEpiGelu>(gp, stream);
  } else if (!f.trans_a && f.trans_b) {
    if (f.epilogue == kEpiStore) return pick_tile<false, true, kEpiStore>(gp, stream);
    if (f.epilogue == kEpiGeluGrad) return pick_tile<false, true, kEpiGeluGrad>(gp, stream);
  } else if (f.trans_a && !f.trans_b) {
    if (f.epilogue == kEpiAccum) return pick_tile<true, false, kEpiAccum>(gp, stream);
  }
  return hipErrorInvalidValue;  // form/epilogue pair the stage never issues
}

hipError_t gemm_bf16(const GemmDesc& d, hipStream_t stream) { return gemm_bf16_grouped(&d, 1, stream); }

}  // namespace k2bw
