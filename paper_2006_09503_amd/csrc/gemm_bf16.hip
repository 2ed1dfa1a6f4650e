// bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulation.
//
// One workgroup computes a BM x BN tile of C.  Two kernel families share the tile order, the
// fragment layout and the epilogue:
//
//   * the ring kernel (gemm_bf16_ring_kernel, further down): operand tiles go from HBM straight
//     into LDS (global_load_lds) through a ring of four stages, K-strided operands stay in their
//     HBM form and are transposed by the LDS read.  It serves every launch whose K is a multiple
//     of its K tile, which is every GEMM of the workloads;
//   * the register-staged kernel (gemm_bf16_kernel): K steps of 64 through two LDS stages, any K.
//     Both operand tiles are staged in one common form -- [row][64 k] bf16, 128-byte rows, 16-byte
//     chunks XOR-swizzled by row -- whatever the operand's layout in HBM:
//       - K contiguous in HBM (activations as A, W read for the data gradient): 16-byte global
//         loads go to LDS as they are;
//       - K strided in HBM (W[K,N] read for the forward, both operands of the weight gradient):
//         each thread loads a 4(k) x 8(row) patch with four 16-byte loads along the contiguous
//         dimension, transposes it in registers and writes eight 8-byte pieces.
//     Per K step a wave issues the global loads of the next tile first, runs its MFMAs with the
//     LDS fragment reads of sub-step ks+1 in flight behind the MFMAs of sub-step ks, and writes
//     the prefetched tile to the other LDS stage during the last two sub-steps; one barrier per K
//     step.  Out-of-range rows/chunks are loaded from a clamped address and zeroed by select, so
//     the loop has no divergent branches.
// The MFMA loop is the same for the forward (NN), data-gradient (NT) and weight-gradient (TN)
// forms in both families.
//
// Lane layout of v_mfma_f32_32x32x16_bf16: lane l supplies row (l % 32) of the first operand and
// column (l % 32) of the second, k = 8*(l/32) .. +7; it receives column (l % 32) of D, rows
// 8*(r/4) + 4*(l/32) + (r % 4) for accumulator register r.  The kernel feeds the B tile as the
// first operand and the A tile as the second, i.e. it accumulates C^T blocks: a lane then owns
// one row m of C and four consecutive columns n per register quad, which makes the epilogue's
// global accesses 8-byte (bf16) or 16-byte (fp32 accumulator) vectors.
#include <cstdio>

#include <type_traits>

#include "kernels.hpp"

namespace k2bw {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kMaxGroup = kGemmMaxGroup;   // GEMMs of one form that may share a launch

struct BfParams {
  const bf16_t* A; const bf16_t* B; void* C;
  int M, N, K, lda, ldb, ldc;
  const bf16_t* bias; const bf16_t* aux; bf16_t* aux_out;
  float* colsum;   // GELU' epilogue: partial[ceil(M/32)][N] column sums of the result, or null
  int accumulate;
  int tiles_m, tiles_n;
  int tile_m;      // rows of C per tile: the kernel's BM, or BM/2 in the balanced tail of a ring launch
  const void* prefetch;        // lines to touch for a later launch, or null (ring kernels)
  uint32_t prefetch_bytes;     // multiple of 4, below 2^31
  // segmented reduction range (ring kernels): K tiles per piece (the launcher fills it in; K / tile for
  // a plain problem), the buffer index of every piece in 4-bit fields (piece 0 lowest) and the
  // distance between consecutive buffer indices in units of 256 bytes
  int seg_tiles;
  uint32_t a_seg, b_seg, a_stride256, b_stride256;
};

// Up to kMaxGroup independent GEMMs of the same form in one launch: workgroup ids
// [tile_start[g], tile_start[g+1]) belong to problem g.
constexpr int kMaxProblems = kMaxGroup + 1;   // + one problem split in two for the balanced tail
struct GroupParams {
  BfParams p[kMaxProblems];
  int tile_start[kMaxProblems + 1];
  int count;
  int n_tiles;   // = tile_start[count] = the launch's workgroups
  // workgroup id -> tile number (see select_problem): [0, seg0) in blocks of 32 tiles dealt to the XCDs in turn
  // (seg0 a multiple of 256), then [seg0, seg0 + seg1) and the seg2 ids behind them each dealt to the XCDs in
  // runs (multiples of 8), the rest as they come
  int seg0, seg1, seg2;
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
  return CH == 4 ? ((row >> 2) ^ (row >> 4)) & 3 : CH == 8 ? ((row >> 1) ^ (row >> 4)) & 7 : (row ^ (row >> 4)) & 15;
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

// Tile order inside a problem: groups of kGroupM tile rows, walked column by column, so that
// the workgroups running at the same time on an XCD (consecutive ids after the XCD remap) cover
// a kGroupM x (32 / kGroupM) block of tiles and share A row panels and B column panels in that
// XCD's L2 instead of streaming a whole row of B panels.
constexpr int kGroupM = 8;
__device__ __forceinline__ void tile_coords(int t, int tiles_m, int tiles_n, int& bm, int& bn) {
  const int per_group = kGroupM * tiles_n;
  const int group = t / per_group;
  const int first_m = group * kGroupM;
  const int gm = min(kGroupM, tiles_m - first_m);
  const int t_in = t - group * per_group;
  bm = first_m + t_in % gm;
  bn = t_in / gm;
}

// The problem and the tile of a workgroup.  Consecutive workgroup ids land on different XCDs
// (round-robin over 8).  An XCD's 32 CUs get 32 consecutive tiles at a time (8 tile rows x 4 columns in
// the order of tile_coords: they share A rows / B columns in that XCD's L2), and the eight XCDs work on
// eight consecutive such blocks: at any moment the whole chip is inside the same few operand panels, which
// the memory-side cache then serves to all XCDs from one HBM read (with each XCD on a contiguous eighth of
// the launch instead, eight distant regions of the operands compete for that cache at once: measured, the
// multi-round weight-gradient launches are 3..5 % slower that way).  What does not fill whole blocks is dealt
// to the XCDs in contiguous runs.  Kernel arguments live in device memory and every dependent round of loads
// from them costs the better part of a microsecond before the first tile can be requested: with
// one problem in the launch (all but the grouped weight-gradient launches) everything here comes
// from one round -- problem 0 is read unconditionally and replaced only in a grouped launch.
// Returns a copy of the problem for the code in front of the K loop (only the fields used there
// are kept); the epilogue reads its operands through gp.p[g], where their latency does not matter
// and they occupy no registers during the loop.
__device__ __forceinline__ BfParams select_problem(const GroupParams& gp, int& wg, int& g) {
  BfParams p = gp.p[0];
  const int count = gp.count;
  // (mask arithmetic, not branches: all the loads above stay in one round)
  const int b = blockIdx.x, seg0 = gp.seg0, seg1 = gp.seg1, seg2 = gp.seg2;
  const int in0 = -(int)(b < seg0), in1 = -(int)(b >= seg0 && b < seg0 + seg1);
  const int in2 = -(int)(b >= seg0 + seg1 && b < seg0 + seg1 + seg2);
  const int i0 = b >> 3, b1 = b - seg0, b2 = b - seg0 - seg1;
  const int w0 = ((((i0 >> 5) << 3) + (b & 7)) << 5) + (i0 & 31);
  wg = (w0 & in0) | ((seg0 + (b1 % 8) * (seg1 / 8) + b1 / 8) & in1) | ((seg0 + seg1 + (b2 % 8) * (seg2 / 8) + b2 / 8) & in2) |
       (b & ~(in0 | in1 | in2));
  g = 0;
  if (count > 1) {
#pragma unroll
    for (int q = 1; q < kMaxProblems; ++q)
      if (q < count && wg >= gp.tile_start[q]) g = q;
    if (g > 0) {
      p = gp.p[g];
      wg -= gp.tile_start[g];
    }
  }
  return p;
}

// Epilogue shared by the GEMM kernels.  A lane's accumulators are one row m = .. + (lane % 32) and,
// per register quad g, columns n = .. + 8*g + 4*(lane/32) + 0..3 of each 32x32 block: stored as they
// are, one store instruction would touch 32 rows with 16 bytes each, and HBM sees partly filled
// lines (measured: 1.7x the output bytes for the two-output GELU epilogue).  So every 32-row strip
// of the wave's sub-tile goes through a wave-private piece of LDS (fp32, 16-byte chunks
// XOR-swizzled with the row: both sides at the LDS's full rate) and leaves in row-major order:
// 8 lanes (bf16 outputs, 8 columns per lane) or 16 lanes (fp32 accumulator, 4 columns per lane)
// cover 128 / 256 contiguous bytes of a row, and the residual / pre-activation operands are read
// the same way.  The arithmetic and its order are those of a direct store: one rounding to bf16.
// v + (v of lane ^ OFF) without the LDS crossbar (ds_bpermute, which __shfl_xor compiles to, costs
// several times as much): a DPP rotation inside the 16-lane row, the row and half-wave swaps
// (of two copies of v: swapping odd rows of one with even rows of the other leaves both partners
// of every pair in the same lane of the two results) beyond it.
template <int OFF>
__device__ __forceinline__ float xor_lane_sum(float v) {
  static_assert(OFF == 8 || OFF == 16 || OFF == 32, "supported lane distances");
  const unsigned u = __builtin_bit_cast(unsigned, v);
  if constexpr (OFF == 8) {
    return v + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, (int)u, 0x128 /* row_ror:8 */, 0xF, 0xF, false));
  } else if constexpr (OFF == 16) {
    // (written as assembly: with the builtin the compiler adds the first result to itself; the
    // s_nop covers the wait states the swap needs after a VALU write of its operands)
    unsigned a = u, b = u;
    asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1" : "+v"(a), "+v"(b));
    return __builtin_bit_cast(float, a) + __builtin_bit_cast(float, b);
  } else {
    unsigned a = u, b = u;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
    return __builtin_bit_cast(float, a) + __builtin_bit_cast(float, b);
  }
}

__device__ __forceinline__ void unpack8(uint4 w, float (&v)[8]) {
  v[0] = __uint_as_float(w.x << 16); v[1] = __uint_as_float(w.x & 0xffff0000u);
  v[2] = __uint_as_float(w.y << 16); v[3] = __uint_as_float(w.y & 0xffff0000u);
  v[4] = __uint_as_float(w.z << 16); v[5] = __uint_as_float(w.z & 0xffff0000u);
  v[6] = __uint_as_float(w.w << 16); v[7] = __uint_as_float(w.w & 0xffff0000u);
}
__device__ __forceinline__ uint4 pack8(const float (&v)[8]) {
  return make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
}
__device__ __forceinline__ void wave_lds_sync() {
  // LDS serves one wave's instructions in order; this only keeps the compiler from moving the
  // strip's reads above its writes (or the next strip's writes above these reads)
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int MI, int NI, int WM, int WN, int EPI>
__device__ __forceinline__ void epilogue(const f32x16 (&acc)[MI][NI], const BfParams& p, int m0, int n0, int wm,
                                         int wn, int lane, uint4* smem, int wave, int mi_begin, int mi_count) {
  constexpr int CPR = WN / 4;   // 16-byte chunks per strip row
  static_assert(CPR >= 16, "row swizzle spans 16 chunks");
  float4* strip = reinterpret_cast<float4*>(smem) + wave * (32 * CPR);
  const int r = lane & 31, khalf = lane >> 5;
  const int col_base = n0 + wn * WN;
  // What a strip reads from HBM besides the accumulators -- the fp32 tile it adds to (kEpiAccum),
  // the residual (kEpiStore) or the pre-activation (kEpiGeluGrad) -- is fetched one strip ahead,
  // so that its latency runs under the previous strip's LDS round trip and stores.
  constexpr int NIT = EPI == kEpiAccum ? WN / 8 : WN / 16;   // row-major passes of 64 lanes over a strip
  constexpr int LPR = EPI == kEpiAccum ? CPR : WN / 8;        // lanes per strip row
  constexpr int CW = EPI == kEpiAccum ? 4 : 8;                // columns per lane
  const bool want_pre = EPI == kEpiAccum ? p.accumulate != 0 : (EPI == kEpiGeluGrad || (EPI == kEpiStore && p.aux != nullptr));
  uint4 pre[2][NIT];
  auto prefetch = [&](int mi, int buf) {
    const int row_base = m0 + wm * WM + mi * 32;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int L = it * 64 + lane;
      const int row = row_base + L / LPR, col = col_base + (L % LPR) * CW;
      if (row < p.M && col < p.N) {
        const int64_t idx = (int64_t)row * p.ldc + col;
        pre[buf][it] = EPI == kEpiAccum ? *reinterpret_cast<const uint4*>(static_cast<const float*>(p.C) + idx)
                                        : *reinterpret_cast<const uint4*>(p.aux + idx);
      }
    }
  };
  if (want_pre) {
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
      if (mi == mi_begin) prefetch(mi, mi & 1);
  }
  // the bias columns of a lane are the same in every pass and strip
  float bias8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if ((EPI == kEpiStore || EPI == kEpiGelu) && p.bias) {
    const int col = col_base + (lane % (WN / 8)) * 8;
    if (col < p.N) unpack8(*reinterpret_cast<const uint4*>(p.bias + col), bias8);
  }
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
    if (mi < mi_begin || mi >= mi_begin + mi_count) continue;   // wave-uniform
    const int row_base = m0 + wm * WM + mi * 32;
    if (want_pre && mi + 1 < MI && mi + 1 < mi_begin + mi_count) prefetch(mi + 1, (mi + 1) & 1);
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int chunk = ni * 8 + 2 * g + khalf;
        strip[r * CPR + (chunk ^ (r & 15))] =
            make_float4(acc[mi][ni][4 * g], acc[mi][ni][4 * g + 1], acc[mi][ni][4 * g + 2], acc[mi][ni][4 * g + 3]);
      }
    wave_lds_sync();
    if (EPI == kEpiAccum) {
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        const int L = it * 64 + lane;
        const int rr = L / CPR, c = L % CPR;
        const float4 v = strip[rr * CPR + (c ^ (rr & 15))];
        const int row = row_base + rr, col = col_base + c * 4;
        if (row < p.M && col < p.N) {
          float4* dst = reinterpret_cast<float4*>(static_cast<float*>(p.C) + (int64_t)row * p.ldc + col);
          float4 o = v;
          if (p.accumulate) {
            const uint4 old = pre[mi & 1][it];
            o.x += __uint_as_float(old.x); o.y += __uint_as_float(old.y);
            o.z += __uint_as_float(old.z); o.w += __uint_as_float(old.w);
          }
          *dst = o;
        }
      }
    } else {
      float cs[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        const int L = it * 64 + lane;
        const int rr = L / (WN / 8), c8 = L % (WN / 8);
        const float4 lo = strip[rr * CPR + ((2 * c8) ^ (rr & 15))];
        const float4 hi = strip[rr * CPR + ((2 * c8 + 1) ^ (rr & 15))];
        const int row = row_base + rr, col = col_base + c8 * 8;
        if (row < p.M && col < p.N) {   // N is a multiple of 8: a group of 8 columns is inside or outside as a whole
          const int64_t idx = (int64_t)row * p.ldc + col;
          float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
          if (EPI == kEpiStore || EPI == kEpiGelu) {
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] += bias8[j];
          }
          bf16_t* out = static_cast<bf16_t*>(p.C) + idx;
          if (EPI == kEpiStore) {
            if (p.aux) {
              float res[8];
              unpack8(pre[mi & 1][it], res);
#pragma unroll
              for (int j = 0; j < 8; ++j) v[j] += res[j];
            }
            *reinterpret_cast<uint4*>(out) = pack8(v);
          } else if (EPI == kEpiGelu) {
            *reinterpret_cast<uint4*>(out) = pack8(v);
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = gelu_fast(v[j]);
            *reinterpret_cast<uint4*>(p.aux_out + idx) = pack8(v);
          } else {   // kEpiGeluGrad
            float u[8];
            unpack8(pre[mi & 1][it], u);
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] *= gelu_grad_fast(u[j]);
            *reinterpret_cast<uint4*>(out) = pack8(v);
#pragma unroll
            for (int j = 0; j < 8; ++j) cs[j] += v[j];
          }
        }
      }
      if (EPI == kEpiGeluGrad && p.colsum) {
        // column sums of this 32-row strip: the lanes that share a column group are WN/8 apart
        static_assert(WN / 8 == 8 || WN / 8 == 16, "lane distance of a column group");
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          if (WN / 8 == 8) cs[j] = xor_lane_sum<8>(cs[j]);
          cs[j] = xor_lane_sum<16>(cs[j]);
          cs[j] = xor_lane_sum<32>(cs[j]);
        }
        const int col = col_base + lane * 8;
        if (lane < WN / 8 && row_base < p.M && col < p.N) {
          float* dst = p.colsum + (int64_t)(row_base >> 5) * p.N + col;
          *reinterpret_cast<float4*>(dst) = make_float4(cs[0], cs[1], cs[2], cs[3]);
          *reinterpret_cast<float4*>(dst + 4) = make_float4(cs[4], cs[5], cs[6], cs[7]);
        }
      }
    }
    wave_lds_sync();
  }
}

// Instruction order of one MFMA sub-step: the RD fragment reads of the next sub-step go between
// the first half of the NM MFMAs of the current one, so that the second half covers their
// latency.  Left to itself the scheduler sinks every read to just before its first use (fewer
// live registers), and each group of MFMAs then waits out the full LDS latency.
template <int I, int NM, int RD>
__device__ __forceinline__ void interleave_reads_with_mfma() {
  if constexpr (I < NM) {
    constexpr int H = NM / 2 > 0 ? NM / 2 : 1;
    constexpr int r = I < H ? (RD * (I + 1)) / H - (RD * I) / H : 0;
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                        // one MFMA
    if constexpr (r > 0) __builtin_amdgcn_sched_group_barrier(0x100, r, 0);   // DS reads
    interleave_reads_with_mfma<I + 1, NM, RD>();
  }
}

// KSPLIT = 2: two groups of waves share the workgroup's tile and split its K range in halves, each
// with its own pair of LDS stages; at the end the groups swap halves of their partial sums through
// LDS and each finishes half of the tile's rows.  For launches with about one tile per CU this
// doubles the waves per SIMD (the LDS and global-load latencies of one group hide behind the
// MFMAs of the other) without shrinking the tile; the sum order is fixed, so results do not
// depend on timing.
template <int BM, int BN, int WM, int WN, int BK, bool TA, bool TB, int EPI, int KSPLIT>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64 * KSPLIT) void gemm_bf16_kernel(GroupParams gp) {
  constexpr int NT = (BM / WM) * (BN / WN) * 64;   // threads of one K group
  constexpr int CH = BK / 8;
  constexpr int MI = WM / 32, NI = WN / 32;
  constexpr int WAVES_N = BN / WN;
  constexpr int KS = BK / 16;
  // fragments of sub-step ks+1 are read while the MFMAs of sub-step ks run, where the registers
  // allow it (up to 64 x 64 per wave)
  constexpr bool kFragDbuf = MI * NI <= 4;
  static_assert(KSPLIT == 1 || (KSPLIT == 2 && MI % 2 == 0), "");
  extern __shared__ uint4 smem_all[];

  const int kg = KSPLIT == 1 ? 0 : (int)threadIdx.x / NT;   // wave-uniform
  const int tid = threadIdx.x - kg * NT, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;

  int wg, g;
  const BfParams p = select_problem(gp, wg, g);
  int bm, bn;
  tile_coords(wg, p.tiles_m, p.tiles_n, bm, bn);
  const int m0 = bm * BM, n0 = bn * BN;

  typename LoaderSel<BM, NT, BK, !TA>::type ld_a;
  typename LoaderSel<BN, NT, BK, TB>::type ld_b;
  ld_a.init(TA ? p.A + m0 : p.A + (int64_t)m0 * p.lda, p.lda, p.M - m0, tid);
  ld_b.init(TB ? p.B + (int64_t)n0 * p.ldb : p.B + n0, p.ldb, p.N - n0, tid);

  constexpr int kStage = (BM + BN) * CH;  // uint4 per stage
  uint4* smem = smem_all + kg * 2 * kStage;
  f32x16 acc[MI][NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

  // this group's K tiles: [kt0, kt0 + nk) in units of BK, elements below k_hi (a group whose range
  // is short or empty runs the same number of steps on zero-filled tiles: barriers stay matched)
  const int nk_all = (p.K + BK - 1) / BK;
  const int nk = (nk_all + KSPLIT - 1) / KSPLIT;
  const int kt0 = kg * nk;
  const int k_hi = min(p.K, (kt0 + nk) * BK);
  ld_a.load(kt0 * BK, k_hi);
  ld_b.load(kt0 * BK, k_hi);
  ld_a.store(smem);
  ld_b.store(smem + BM * CH);
  ld_a.load((kt0 + 1) * BK, k_hi);   // tile 1 stays in flight in registers during the first K step
  ld_b.load((kt0 + 1) * BK, k_hi);
  __syncthreads();

  const int khalf = lane >> 5;
  // fragment addresses (uint4 index inside a stage's A / B tile) for sub-step 0; sub-step ks
  // flips chunk bits: chunk = (2*ks + khalf) ^ swz(row), i.e. index ^ (2*ks)
  int a_idx[MI], b_idx[NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
    const int row = wm * WM + mi * 32 + (lane & 31);
    a_idx[mi] = row * CH + (khalf ^ swz<CH>(row));
  }
#pragma unroll
  for (int ni = 0; ni < NI; ++ni) {
    const int row = wn * WN + ni * 32 + (lane & 31);
    b_idx[ni] = row * CH + (khalf ^ swz<CH>(row));
  }

  // K step kt: MFMAs on stage kt&1.  In the middle of the step the tile kt+1, whose global loads
  // were issued one whole step earlier, goes from registers to the other stage, and the loads of
  // tile kt+2 are issued into the freed registers: they have a full step to arrive.
  for (int kt = 0; kt < nk; ++kt) {
    const uint4* sA = smem + (kt & 1) * kStage;
    const uint4* sB = sA + BM * CH;
    uint4* dA = smem + ((kt + 1) & 1) * kStage;
    // The per-sub-step addresses are one XOR away from a_idx / b_idx; hiding the values from the
    // optimizer here keeps it from hoisting all KS x (MI + NI) of them out of the loop, where
    // they would not fit in registers next to the accumulators.
    int ai[MI], bi[NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) { ai[mi] = a_idx[mi]; asm volatile("" : "+v"(ai[mi])); }
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) { bi[ni] = b_idx[ni]; asm volatile("" : "+v"(bi[ni])); }
    // With one wave per SIMD (4-wave configurations) the fragments of sub-step ks+1 are read
    // while the MFMAs of sub-step ks run; with two waves per SIMD the other wave covers the LDS
    // latency and the registers are better spent elsewhere.
    constexpr int FB = kFragDbuf ? 2 : 1;
    bf16x8 af[FB][MI], bfr[FB][NI];
    if (kFragDbuf) {
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) af[0][mi] = __builtin_bit_cast(bf16x8, sA[ai[mi]]);
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) bfr[0][ni] = __builtin_bit_cast(bf16x8, sB[bi[ni]]);
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int cur = kFragDbuf ? (ks & 1) : 0, nxt = kFragDbuf ? (cur ^ 1) : 0;
      const int kr = kFragDbuf ? ks + 1 : ks;   // sub-step whose fragments are read now
      if (kr < KS) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) af[nxt][mi] = __builtin_bit_cast(bf16x8, sA[ai[mi] ^ (kr * 2)]);
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) bfr[nxt][ni] = __builtin_bit_cast(bf16x8, sB[bi[ni] ^ (kr * 2)]);
      }
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[cur][ni], af[cur][mi], acc[mi][ni], 0, 0, 0);
      // sub-steps 0..KS/2-1 move slices of the A tile, the rest slices of the B tile
      if (ks < KS / 2) ld_a.step(ks, KS / 2, dA, (kt0 + kt + 2) * BK, k_hi);
      else ld_b.step(ks - KS / 2, KS / 2, dA + BM * CH, (kt0 + kt + 2) * BK, k_hi);
      if (kFragDbuf) {
        if (ks + 1 < KS) interleave_reads_with_mfma<0, MI * NI, MI + NI>();
        else __builtin_amdgcn_sched_group_barrier(0x008, MI * NI, 0);
      }
      // keep each slice's stores and loads inside its sub-step: left alone, the scheduler sinks
      // every global load to the end of the K step and hoists the selects that wait for them
      __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();
  }

  if (KSPLIT == 2) {
    // group kg keeps block rows mi with mi / (MI/2) == kg and receives the other group's partial
    // sums for them: slot j of thread t of group q sits at float4 index (j * 2 + q) * NT + t
    float4* xb = reinterpret_cast<float4*>(smem_all);
    constexpr int H = MI / 2;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      if ((mi / H) == kg) continue;
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int q = 0; q < 4; ++q)
          xb[(((mi % H) * NI + ni) * 4 + q) * 2 * NT + kg * NT + tid] =
              make_float4(acc[mi][ni][4 * q], acc[mi][ni][4 * q + 1], acc[mi][ni][4 * q + 2], acc[mi][ni][4 * q + 3]);
    }
    __syncthreads();
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      if ((mi / H) != kg) continue;
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const float4 o = xb[(((mi % H) * NI + ni) * 4 + q) * 2 * NT + (1 - kg) * NT + tid];
          // fixed order: low K half + high K half
          acc[mi][ni][4 * q] = kg == 0 ? acc[mi][ni][4 * q] + o.x : o.x + acc[mi][ni][4 * q];
          acc[mi][ni][4 * q + 1] = kg == 0 ? acc[mi][ni][4 * q + 1] + o.y : o.y + acc[mi][ni][4 * q + 1];
          acc[mi][ni][4 * q + 2] = kg == 0 ? acc[mi][ni][4 * q + 2] + o.z : o.z + acc[mi][ni][4 * q + 2];
          acc[mi][ni][4 * q + 3] = kg == 0 ? acc[mi][ni][4 * q + 3] + o.w : o.w + acc[mi][ni][4 * q + 3];
        }
    }
    // strips live behind the exchange buffer: no wave overwrites partial sums another still reads
    constexpr int kXchg = H * NI * 4 * 2 * NT;   // float4 = uint4 units
    epilogue<MI, NI, WM, WN, EPI>(acc, gp.p[g], m0, n0, wm, wn, lane, smem_all + kXchg, (int)threadIdx.x >> 6, kg * H, H);
  } else {
    epilogue<MI, NI, WM, WN, EPI>(acc, gp.p[g], m0, n0, wm, wn, lane, smem_all, wave, 0, MI);
  }
}

// ------------------------------------------------------------------------------------------------
// Asynchronous kernels (K a multiple of the K tile).  Tiles go from HBM straight into LDS with
// global_load_lds (16 bytes per lane, a wave fills 1 KB of consecutive LDS), so no registers and
// no LDS store instructions are spent on staging:
//   * K-contiguous operand: LDS [row][8 chunks], chunk XOR-swizzled as above; lane i of a load
//     owns LDS slot L0 + i and fetches the global chunk that belongs there.
//   * K-strided operand: LDS keeps the HBM form [k][row] (rows contiguous), 16-byte pieces
//     XOR-swizzled with (k & 3) << 1.  The MFMA fragment is read with ds_read_b64_tr_b16: within
//     each 16-lane group, lane a + 4t supplies the address of 4 consecutive rows at k_t and lane
//     4a + j receives (k_0..k_3) of row 4a + j -- measured on gfx950 -- so two such reads give a
//     lane the 8 k-values of its row in the same slot order as a 16-byte read of the other form.
// Out-of-range rows are fetched from a clamped address (their products only reach outputs that
// are never stored).
typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) v4i16 lds_v4i16_t;
typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void glob_void_t;

// A wave-uniform pointer, moved to scalar registers.
__device__ __forceinline__ uint64_t uniform_address(const void* ptr) {
  const uint64_t bb = reinterpret_cast<uint64_t>(ptr);
  const uint32_t b_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(bb >> 32));
  const uint32_t b_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)bb);
  return ((uint64_t)b_hi << 32) | (uint64_t)b_lo;
}

template <int R, int NW, int BKA, bool K_CONTIG>
struct AsyncLoader {
  static constexpr int CHK = BKA / 8;               // chunks per row of a K-contiguous tile
  static constexpr int kSlots = R * CHK;            // 16-byte slots per tile
  static constexpr int IPW = kSlots / 64 / NW;      // load instructions per wave
  static_assert(kSlots % (64 * NW) == 0, "tile/waves mismatch");
  const bf16_t* base_;
  uint32_t voff[IPW];   // byte offsets from the tile's base
  int ld_, first_slot_;
  __device__ __forceinline__ void init(const bf16_t* base, int ld, int rows_valid, int wave, int lane) {
    base_ = base; ld_ = ld;
    first_slot_ = wave * IPW * 64;
#pragma unroll
    for (int j = 0; j < IPW; ++j) {
      const int L = first_slot_ + j * 64 + lane;
      if (K_CONTIG) {
        const int row = L / CHK, pc = L % CHK;
        const int c = pc ^ swz<CHK>(row);
        const int rc = row < rows_valid ? row : rows_valid - 1;
        voff[j] = ((uint32_t)rc * (uint32_t)ld + c * 8) * 2u;
      } else {
        constexpr int PPR = R / 8;                  // pieces per k row
        const int k = L / PPR, pp = L % PPR;
        const int piece = pp ^ ((k & 3) << 1);
        int col = piece * 8;
        if (col >= rows_valid) col = rows_valid - 8;
        voff[j] = ((uint32_t)k * (uint32_t)ld + col) * 2u;
      }
    }
  }
  // Load instruction j of the tile at k0, written as assembly so that the compiler does not see a
  // store to LDS: it would otherwise put s_waitcnt vmcnt(0) in front of every later LDS read (it
  // cannot tell the ring's stages apart), and the loads of the tiles further ahead could not stay
  // in flight.  The caller waits (vmcnt) and synchronises before anyone reads the stage.
  // Addressing: the tile's base in a scalar register pair plus this lane's 32-bit byte offset
  // (operands are smaller than 2 GiB, checked on the host): the per-tile address arithmetic stays
  // on the scalar unit and a load sends half the address data of the 64-bit form (+2..5 % on the
  // weight-gradient form).
  // lds_tile: byte address of the stage's tile in LDS, wave-uniform.
  // tile_addr: address of the tile's element (row0, k0), wave-uniform.
  __device__ __forceinline__ void issue_one_untracked(int j, uint64_t tile_addr, uint32_t lds_tile) const {
    const uint32_t dst = __builtin_amdgcn_readfirstlane(lds_tile + (uint32_t)(first_slot_ + j * 64) * 16u);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(dst), "v"(voff[j]), "s"(tile_addr)
                 : "memory");   // (M0 is reserved: the compiler keeps nothing in it)
  }
  // bytes from one K tile to the next inside a contiguous piece of the reduction range
  __device__ __forceinline__ uint32_t tile_step_bytes() const {
    return K_CONTIG ? (uint32_t)BKA * 2u : (uint32_t)BKA * (uint32_t)ld_ * 2u;
  }
};

// The addresses of successive K tiles of both operands, all in scalar registers.  The reduction
// range is made of pieces of seg_tiles tiles each; piece s of an operand lies in buffer number
// (seg >> 4s) & 15, the buffers being `stride` bytes apart (a plain problem is one piece).  Past the
// last tile the walk stays where it is: that tile is fetched again and never read.
struct TileWalk {
  uint64_t a_addr, b_addr;       // tile about to be requested
  uint64_t a_base, b_base;       // element (row0, k = 0) of buffer number 0
  uint64_t a_stride, b_stride;   // bytes between consecutive buffer numbers
  uint32_t a_step, b_step;       // bytes between consecutive tiles of a piece
  uint32_t a_rest, b_rest;       // buffer numbers of this and the later pieces (this one in the low 4 bits)
  int left;                      // tiles left in this piece, this one included
  int seg_tiles;
  int remaining;                 // tiles left in the whole range, this one included
  __device__ __forceinline__ void init(const void* a0, const void* b0, uint32_t a_step_, uint32_t b_step_, const BfParams& p,
                                       int nk) {
    a_base = uniform_address(a0); b_base = uniform_address(b0);
    a_step = a_step_; b_step = b_step_;
    a_stride = (uint64_t)p.a_stride256 << 8; b_stride = (uint64_t)p.b_stride256 << 8;
    a_rest = p.a_seg; b_rest = p.b_seg;
    seg_tiles = p.seg_tiles; left = p.seg_tiles; remaining = nk;
    a_addr = a_base + (uint64_t)(a_rest & 15u) * a_stride;
    b_addr = b_base + (uint64_t)(b_rest & 15u) * b_stride;
  }
  __device__ __forceinline__ void advance() {
    const int more = min(remaining - 1, 1);   // 1 while another tile follows, then 0 (remaining >= 1 always)
    remaining -= more;
    left -= more;
    if (left == 0) {   // wave-uniform, once per piece
      left = seg_tiles;
      a_rest >>= 4; b_rest >>= 4;
      a_addr = a_base + (uint64_t)(a_rest & 15u) * a_stride;
      b_addr = b_base + (uint64_t)(b_rest & 15u) * b_stride;
    } else {
      a_addr += a_step * (uint32_t)more;
      b_addr += b_step * (uint32_t)more;
    }
  }
};

// fragment of 32 rows starting at row0 for sub-step ks
template <int R, int BKA, bool K_CONTIG>
__device__ __forceinline__ bf16x8 read_frag(const uint4* tile, int row0, int ks, int lane) {
  if (K_CONTIG) {
    constexpr int CHK = BKA / 8;
    const int row = row0 + (lane & 31);
    return __builtin_bit_cast(bf16x8, tile[row * CHK + ((ks * 2 + (lane >> 5)) ^ swz<CHK>(row))]);
  } else {
    const int r = lane & 15, a = r & 3, t = r >> 2;
    const int k = ks * 16 + (lane >> 5) * 8 + t;
    const int col = row0 + ((lane >> 4) & 1) * 16 + 4 * a;
    const int piece = (col >> 3) ^ (t << 1);        // (k & 3) == t
    const int byte = k * (R * 2) + piece * 16 + ((col >> 2) & 1) * 8;
    const lds_v4i16_t* p0 = (const lds_v4i16_t*)((const __attribute__((address_space(3))) char*)tile + byte);
    const lds_v4i16_t* p1 = (const lds_v4i16_t*)((const __attribute__((address_space(3))) char*)tile + byte + 4 * R * 2);
    const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16_t*)p0);
    const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16_t*)p1);
    typedef short v8i16 __attribute__((ext_vector_type(8)));
    const v8i16 w = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, w);
  }
}

// s_waitcnt immediate for "at most n vector-memory operations outstanding" (gfx9 encoding:
// vmcnt = bits 3:0 and 15:14; expcnt and lgkmcnt fields left at their maxima = no wait)
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

// ------------------------------------------------------------------------------------------------
// The ring kernel: K tiles of BKA (32 or 64) in a ring of NS LDS stages (a power of 2).  A wave's 16-byte global->LDS load occupies the CU's address unit for about 16
// cycles, so the loads of a 256x256x64 step are a thousand cycles of issue; behind a barrier, back
// to back, every wave sits in that queue with no MFMA in flight (measured with s_memtime around
// the phases of the two-stage kernel: 1400 cycles for the 8 MFMAs that follow the loads, 840 for
// the other 24).  With more than two stages the stage that tile kt+NS-1 goes to is already free
// during the whole of step kt, so its loads are issued one at a time between the MFMAs of all
// sub-steps and the queue never fills; a load has NS-2 steps to land.  256x256 tiles: four stages
// of K = 32 (128 KB).  128x128 tiles: four stages of K = 64; with K = 32 (half a 128-byte line per
// row and load) that tile is 10..15 % slower once the operands come from HBM, as they do inside
// the stage, with four stages or with eight.
template <int BM, int BN, int WM, int WN, int BKA, int NS, bool TA, bool TB, int EPI>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64) void gemm_bf16_ring_kernel(GroupParams gp) {
  constexpr int CHK = BKA / 8, KS = BKA / 16;
  constexpr int NW = (BM / WM) * (BN / WN);
  constexpr int MI = WM / 32, NI = WN / 32;
  constexpr int WAVES_N = BN / WN;
  static_assert((NS & (NS - 1)) == 0 && NS >= 4 && KS % 2 == 0, "ring size, even number of sub-steps");
  extern __shared__ uint4 smem[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  int wg, g;
  const BfParams p = select_problem(gp, wg, g);
  int bm, bn;
  tile_coords(wg, p.tiles_m, p.tiles_n, bm, bn);
  // A launch may end with tiles of BM/2 rows (see launch_ring): the waves of the lower half then only
  // take part in the loads and barriers.
  constexpr bool kCanHalve = BM == 2 * WM;
  const int tile_m = kCanHalve ? p.tile_m : BM;
  const bool active = !kCanHalve || wm * WM < tile_m;   // wave-uniform
  const int m0 = bm * tile_m, n0 = bn * BN;

  AsyncLoader<BM, NW, BKA, !TA> ld_a;
  AsyncLoader<BN, NW, BKA, TB> ld_b;
  ld_a.init(TA ? p.A + m0 : p.A + (int64_t)m0 * p.lda, p.lda, min(p.M - m0, tile_m), wave, lane);
  ld_b.init(TB ? p.B + (int64_t)n0 * p.ldb : p.B + n0, p.ldb, p.N - n0, wave, lane);
  constexpr int IPA = decltype(ld_a)::IPW, NV = IPA + decltype(ld_b)::IPW;   // loads per wave and tile

  constexpr int kStage = (BM + BN) * CHK;  // uint4 per stage
  f32x16 acc[MI][NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

  const int nk = p.K / BKA;   // K is a multiple of BKA
  // tile t (past the end: the last one again, never read) goes to stage t & (NS - 1);
  // a stage's LDS byte address: the low half of a generic pointer into LDS is its LDS address
  const uint32_t lds_base = __builtin_amdgcn_readfirstlane((uint32_t)reinterpret_cast<uintptr_t>(smem));
  TileWalk walk;   // the tile the next loads fetch
  walk.init(ld_a.base_, ld_b.base_, ld_a.tile_step_bytes(), ld_b.tile_step_bytes(), p, nk);
  auto issue = [&](int v, uint32_t stage_bytes) {
    if (v < IPA) ld_a.issue_one_untracked(v, walk.a_addr, stage_bytes);
    else ld_b.issue_one_untracked(v - IPA, walk.b_addr, stage_bytes + (uint32_t)(BM * CHK) * 16u);
  };
  // Lines of the operand a later launch will read (GemmDesc::prefetch): every wave of the launch
  // touches 64 of them, 128 bytes apart, with one 4-byte load in front of its own first loads.  The
  // load is older than every tile load, so the waits below (which count the newest operations that
  // may still be outstanding) stay sufficient whenever it returns.  The compiler does not know that the
  // value arrives late: its destination register is kept out of other use up to the first wait below,
  // after which the load has returned (vector-memory loads return in order) and the register is free.
  uint32_t touched = 0;
  if (p.prefetch != nullptr) {
    const uint32_t line = ((uint32_t)blockIdx.x * NW + (uint32_t)wave) * 64u + (uint32_t)lane;
    const uint32_t off = min(line * 128u, p.prefetch_bytes - 4u);
    asm volatile("global_load_dword %0, %1, %2" : "=v"(touched) : "v"(off), "s"(uniform_address(p.prefetch)) : "memory");
  }
#pragma unroll
  for (int t = 0; t < NS - 1; ++t) {
#pragma unroll
    for (int v = 0; v < NV; ++v) issue(v, lds_base + (uint32_t)(t * kStage) * 16u);
    walk.advance();
  }
  __builtin_amdgcn_s_waitcnt(vmcnt_imm((NS - 2) * NV));
  asm volatile("" : "+v"(touched));   // the touch has landed: last use of its register
  __syncthreads();
  bf16x8 af[2][MI], bfr[2][NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) af[0][mi] = read_frag<BM, BKA, !TA>(smem, wm * WM + mi * 32, 0, lane);
#pragma unroll
  for (int ni = 0; ni < NI; ++ni) bfr[0][ni] = read_frag<BN, BKA, TB>(smem + BM * CHK, wn * WN + ni * 32, 0, lane);

  // One step = KS sub-steps of NM MFMAs.  The NV loads of tile kt+NS-1 go out every EVERY-th MFMA
  // of the step; the fragments of the following sub-step (after the last one: sub-step 0 of tile
  // kt+1) are read behind the first half of each sub-step's MFMAs.
  constexpr int NM = MI * NI, H = NM / 2, NF = MI + NI;
  static_assert((KS * NM) % NV == 0, "one load every (KS * NM / NV)-th MFMA");
  constexpr int EVERY = KS * NM / NV;
  constexpr int NV_PRE = ((KS - 1) * NM + EVERY - 1) / EVERY;   // loads issued before the barrier
  static_assert((NS - 3) * NV + NV_PRE <= 63, "vmcnt range");
  if (!active) {
    // same loads, waits and barriers as below, no fragments and no MFMAs: the step's loads follow its
    // barrier, so at the wait the tiles kt+2 .. kt+NS-2 may be outstanding
    for (int kt = 0; kt < nk; ++kt) {
      const uint32_t l_stage = lds_base + (uint32_t)(((kt + NS - 1) & (NS - 1)) * kStage) * 16u;
      __builtin_amdgcn_s_waitcnt(vmcnt_imm((NS - 3) * NV));
      __syncthreads();
#pragma unroll
      for (int v = 0; v < NV; ++v) issue(v, l_stage);
      walk.advance();
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __syncthreads();
    return;
  }
  // One step on the tile in stage st = kt & (NS - 1).  The loop below runs NS steps per trip with st a
  // constant, so that every LDS address of a step is a register of the lane plus an immediate and the
  // K loop has no vector address arithmetic left (vector ALU instructions take issue cycles from the
  // MFMAs of the same SIMD); the steps of a remainder run with st computed.
  auto step = [&](int kt, int st) __attribute__((always_inline)) {
    const uint4* sA = smem + st * kStage;
    const uint4* sB = sA + BM * CHK;
    const uint4* nA = smem + ((st + 1) & (NS - 1)) * kStage;
    const uint4* nB = nA + BM * CHK;
    const uint32_t l_stage = lds_base + (uint32_t)(((st + NS - 1) & (NS - 1)) * kStage) * 16u;
    (void)kt;   // the loads of this step fetch tile kt + NS - 1, which is where `walk` stands
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int cur = ks & 1, nxt = cur ^ 1;
      const bool last = ks == KS - 1;
      if (last) {
        // tile kt+1 has landed once at most the loads issued after it are outstanding: all of
        // tiles kt+2 .. kt+NS-2 and what this step has issued of tile kt+NS-1 so far; the barrier
        // also tells that nobody reads stage kt any more (its last fragments are in registers)
        __builtin_amdgcn_s_waitcnt(vmcnt_imm((NS - 3) * NV + NV_PRE) & ~(15 << 8));   // and lgkmcnt(0)
        __syncthreads();
      }
#pragma unroll
      for (int i = 0; i < NM; ++i) {
        const int mi = i / NI, ni = i % NI, q = ks * NM + i;
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[cur][ni], af[cur][mi], acc[mi][ni], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (q % EVERY == 0) issue(q / EVERY, l_stage);
        if (i < H) {
#pragma unroll
          for (int f = (NF * i) / H; f < (NF * (i + 1)) / H; ++f) {
            if (f < MI) af[nxt][f] = read_frag<BM, BKA, !TA>(last ? nA : sA, wm * WM + f * 32, last ? 0 : ks + 1, lane);
            else bfr[nxt][f - MI] = read_frag<BN, BKA, TB>(last ? nB : sB, wn * WN + (f - MI) * 32, last ? 0 : ks + 1, lane);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    walk.advance();
  };
  int kt = 0;
  for (; kt + NS <= nk; kt += NS) {
#pragma unroll
    for (int u = 0; u < NS; ++u) step(kt + u, u);
  }
  for (; kt < nk; ++kt) step(kt, kt & (NS - 1));
  // the last prefetches may still be landing in LDS, which the epilogue re-uses
  __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
  __syncthreads();
  epilogue<MI, NI, WM, WN, EPI>(acc, gp.p[g], m0, n0, wm, wn, lane, smem, wave, 0, MI);
}


int compute_units() {
  static int n = 0;
  if (n == 0) {
    int dev = 0;
    hipDeviceProp_t prop;
    n = (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
            ? prop.multiProcessorCount : 256;
  }
  return n;
}

// Rows [m_split, M) of problem q as a problem of its own (m_split a multiple of 32).
template <bool TA, int EPI>
BfParams lower_rows(const BfParams& q, int m_split) {
  BfParams r = q;
  r.M = q.M - m_split;
  r.A = TA ? q.A + m_split : q.A + (int64_t)m_split * q.lda;
  const int64_t c_off = (int64_t)m_split * q.ldc;
  r.C = EPI == kEpiAccum ? static_cast<void*>(static_cast<float*>(q.C) + c_off)
                         : static_cast<void*>(static_cast<bf16_t*>(q.C) + c_off);
  if (q.aux) r.aux = q.aux + c_off;
  if (q.aux_out) r.aux_out = q.aux_out + c_off;
  if (q.colsum) r.colsum = q.colsum + (int64_t)(m_split / 32) * q.N;
  return r;
}

// A launch of T tiles on n CUs takes ceil(T / n) rounds of one tile per CU.  When the last round
// would fill at most half of the CUs (T mod n in 1..n/2, T > n) the rows of its tiles are given to
// twice as many workgroups with tiles of BM/2 rows, in which half of the waves run the MFMAs: that
// round then takes about 0.6 of a full one (the B tile is still loaded whole).  The halved tiles
// are the launch's last problems, or the last tile rows of one that is split in two for this;
// they are dispatched last because the XCD remap treats them as a segment of its own.
template <int BM, int BN, int WM, int WN, int BKA, int NS, bool TA, bool TB, int EPI>
hipError_t launch_ring(GroupParams gp, hipStream_t s) {
  constexpr int NT = (BM / WM) * (BN / WN) * 64;
  constexpr size_t lds = NS * (BM + BN) * (BKA / 8) * sizeof(uint4);
  static_assert(lds <= 160 * 1024, "LDS of a CU");
  auto kern = gemm_bf16_ring_kernel<BM, BN, WM, WN, BKA, NS, TA, TB, EPI>;
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    configured = true;
  }
  int64_t full = 0;
  for (int g = 0; g < gp.count; ++g) {
    // (seg_tiles arrives as the number of pieces; choose_tile has checked that a piece is whole K tiles)
    gp.p[g].seg_tiles = gp.p[g].K / BKA / (gp.p[g].seg_tiles > 1 ? gp.p[g].seg_tiles : 1);
    gp.p[g].tile_m = BM;
    gp.p[g].tiles_m = ceil_div(gp.p[g].M, BM);
    gp.p[g].tiles_n = ceil_div(gp.p[g].N, BN);
    full += (int64_t)gp.p[g].tiles_m * gp.p[g].tiles_n;
  }
  int first_half = gp.count;   // problems [first_half, count) get tiles of BM/2 rows
  if (BM == 2 * WM) {
    const int n_cu = compute_units();
    int64_t need = full % n_cu;
    if (full > n_cu && need > 0 && need <= n_cu / 2) {
      while (need > 0 && first_half > 0) {
        BfParams& q = gp.p[first_half - 1];
        const int64_t t = (int64_t)q.tiles_m * q.tiles_n;
        const int rows = (int)ceil_div(need, (int64_t)q.tiles_n);   // tile rows of q still wanted
        if (t <= need || rows >= q.tiles_m) {
          --first_half;
          need -= t;
        } else {
          // split q: its last `rows` tile rows become a problem of their own behind it
          const int m_split = (q.tiles_m - rows) * BM;
          for (int g = gp.count; g > first_half; --g) gp.p[g] = gp.p[g - 1];
          gp.p[first_half] = lower_rows<TA, EPI>(q, m_split);
          q.M = m_split;
          q.tiles_m -= rows;
          ++gp.count;
          need = 0;
        }
      }
      for (int g = first_half; g < gp.count; ++g) {
        gp.p[g].tile_m = BM / 2;
        gp.p[g].tiles_m = ceil_div(gp.p[g].M, BM / 2);
      }
    }
  }
  int total = 0;
  for (int g = 0; g < gp.count; ++g) {
    gp.tile_start[g] = total;
    total += gp.p[g].tiles_m * gp.p[g].tiles_n;
  }
  for (int g = gp.count; g <= kMaxProblems; ++g) gp.tile_start[g] = total;
  gp.n_tiles = total;
  const int full_tiles = first_half < gp.count ? gp.tile_start[first_half] : total;
  gp.seg0 = full_tiles / 256 * 256;
  gp.seg1 = (full_tiles - gp.seg0) / 8 * 8;
  gp.seg2 = (total - gp.seg0 - gp.seg1) / 8 * 8;
  hipLaunchKernelGGL(kern, dim3(total), dim3(NT), lds, s, gp);
  return hipGetLastError();
}

template <int BM, int BN, int WM, int WN, int BK, bool TA, bool TB, int EPI, int KSPLIT = 1>
hipError_t launch(GroupParams gp, hipStream_t s) {
  constexpr int NT = (BM / WM) * (BN / WN) * 64 * KSPLIT;
  constexpr size_t lds = KSPLIT * 2 * (BM + BN) * (BK / 8) * sizeof(uint4);
  static_assert(KSPLIT == 1 || (BM * BN + NT / 64 * 32 * WN) * 4 <= lds, "exchange buffer + strips fit in the stages");
  auto kern = gemm_bf16_kernel<BM, BN, WM, WN, BK, TA, TB, EPI, KSPLIT>;
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
  for (int g = gp.count; g <= kMaxProblems; ++g) gp.tile_start[g] = total;
  gp.n_tiles = total;
  gp.seg0 = 0;
  gp.seg1 = total / 8 * 8;
  gp.seg2 = 0;
  hipLaunchKernelGGL(kern, dim3(total), dim3(NT), lds, s, gp);
  return hipGetLastError();
}

int g_tile_override = 0;  // 0: heuristic; else force a tile shape (tuning aid)

// Tile choice for a (grouped) problem; ta/tb as in GemmDesc.
int choose_tile(const BfParams* p, int count, bool ta, bool tb) {
  int tile = g_tile_override;
  if (tile == 0) {
    // Measured on MI355X (M = 2048..8192): once 256x256 tiles give about 5/8 of the CUs a tile
    // (160 tiles: N = 2560 at M = 4096) the 8-wave 256x256 kernels win, by 15..30 % at 160..192
    // tiles and more above, and among them the ring kernel by 10..25 %.  Below that, 128x128
    // tiles: with about one tile per CU the ring kernel with K tiles of 64 (a little ahead of the
    // register-staged variant with two K groups per workgroup), with more tiles two register-staged
    // workgroups per CU.  The ring kernels need K to be a multiple of their K tile and fall back to
    // the register-staged kernel of the same tile otherwise.
    int64_t big = 0, small = 0;
    for (int g = 0; g < count; ++g) {
      big += (int64_t)ceil_div(p[g].M, 256) * ceil_div(p[g].N, 256);
      small += (int64_t)ceil_div(p[g].M, 128) * ceil_div(p[g].N, 128);
    }
    tile = big >= 144 ? 23 : small <= 256 ? 22 : 2;
    (void)ta; (void)tb;
  }
  bool segmented = false;
  for (int g = 0; g < count; ++g) segmented = segmented || p[g].seg_tiles > 1;
  if (segmented && tile < 20) tile = 22;   // only the ring kernels walk a segmented reduction range
  if (tile > 20) {   // the ring kernels need whole K tiles (in every piece of a segmented range)
    const int bk = tile == 22 ? 64 : 32;
    for (int g = 0; g < count; ++g)
      if ((p[g].K / (p[g].seg_tiles > 1 ? p[g].seg_tiles : 1)) % bk) { tile = segmented ? -1 : tile == 22 ? 6 : 3; break; }
  }
  return tile;
}

template <bool TA, bool TB, int EPI>
hipError_t pick_tile(const GroupParams& gp, hipStream_t s) {
  const int tile = choose_tile(gp.p, gp.count, TA, TB);
  switch (tile) {
    case 2: return launch<128, 128, 64, 64, 64, TA, TB, EPI>(gp, s);
    case 3: return launch<256, 256, 128, 64, 64, TA, TB, EPI>(gp, s);   // 8 waves
    case 6: return launch<128, 128, 64, 64, 64, TA, TB, EPI, 2>(gp, s);   // two K groups of 4 waves
    case 22: return launch_ring<128, 128, 32, 64, 64, 4, TA, TB, EPI>(gp, s);   // 8 waves
    case 23: return launch_ring<256, 256, 128, 64, 32, 4, TA, TB, EPI>(gp, s);
    default: return hipErrorInvalidValue;
  }
}

bool vector_ok(const GemmDesc& d) {
  // 16-byte vector accesses in the epilogue
  return !(d.N % 8 || d.ldc % 8 || (reinterpret_cast<uintptr_t>(d.C) & 15) || (reinterpret_cast<uintptr_t>(d.bias) & 15) ||
           (reinterpret_cast<uintptr_t>(d.aux) & 15) || (reinterpret_cast<uintptr_t>(d.aux_out) & 15));
}

uint32_t pack_seg(const uint8_t* idx, int n) {
  uint32_t v = 0;
  for (int s = 0; s < n && s < 8; ++s) v |= (uint32_t)(idx[s] & 15) << (4 * s);
  return v;
}

BfParams to_params(const GemmDesc& d) {
  return BfParams{static_cast<const bf16_t*>(d.A), static_cast<const bf16_t*>(d.B), d.C,
                  d.M, d.N, d.K, d.lda, d.ldb, d.ldc, static_cast<const bf16_t*>(d.bias),
                  static_cast<const bf16_t*>(d.aux), static_cast<bf16_t*>(d.aux_out),
                  d.epilogue == kEpiGeluGrad ? d.colsum_partial : nullptr, d.accumulate ? 1 : 0, 0, 0, 0,
                  // (matrices beyond the reach of one launch's touches, or of the cache, are left alone)
                  d.prefetch_bytes >= 4 && d.prefetch_bytes <= (32ll << 20) ? d.prefetch : nullptr,
                  (uint32_t)(d.prefetch_bytes >= 4 && d.prefetch_bytes <= (32ll << 20) ? d.prefetch_bytes & ~3ll : 0),
                  // (a plain problem walks one piece in buffer 0: its index and stride fields are not looked at)
                  d.n_seg, d.n_seg > 1 ? pack_seg(d.a_seg_idx, d.n_seg) : 0u, d.n_seg > 1 ? pack_seg(d.b_seg_idx, d.n_seg) : 0u,
                  d.n_seg > 1 ? (uint32_t)(d.a_seg_stride >> 8) : 0u, d.n_seg > 1 ? (uint32_t)(d.b_seg_stride >> 8) : 0u};
}

// A segmented reduction range is valid for the weight-gradient form only, with pieces of equal length
// in buffers 0..15 at strides that are multiples of 256 bytes and below 2^40.
bool segments_ok(const GemmDesc& d) {
  if (d.n_seg == 1) return true;
  if (d.n_seg < 1 || d.n_seg > kGemmMaxSegments || d.epilogue != kEpiAccum || !d.trans_a || d.trans_b) return false;
  if (d.K % d.n_seg) return false;
  if (d.a_seg_stride < 0 || d.b_seg_stride < 0 || (d.a_seg_stride & 255) || (d.b_seg_stride & 255) ||
      (d.a_seg_stride >> 40) || (d.b_seg_stride >> 40))
    return false;
  for (int s = 0; s < d.n_seg; ++s)
    if (d.a_seg_idx[s] > 15 || d.b_seg_idx[s] > 15) return false;
  return true;
}

}  // namespace

void gemm_bf16_set_tile(int id) { g_tile_override = id; }

int gemm_compute_units() { return compute_units(); }

// Name of the kernel instance a (grouped) call will run, in the form profilers print template
// arguments, so that event timings can be matched with a kernel trace.
void gemm_bf16_kernel_name(const GemmDesc* d, int count, char* out, size_t cap) {
  BfParams p[kMaxGroup];
  for (int g = 0; g < count && g < kMaxGroup; ++g) p[g] = to_params(d[g]);
  const int tile = choose_tile(p, count < kMaxGroup ? count : kMaxGroup, d[0].trans_a, d[0].trans_b);
  const char* ta = d[0].trans_a ? "true" : "false";
  const char* tb = d[0].trans_b ? "true" : "false";
  switch (tile) {
    case 2: snprintf(out, cap, "gemm_bf16_kernel<128, 128, 64, 64, 64, %s, %s, %d, 1>", ta, tb, d[0].epilogue); break;
    case 3: snprintf(out, cap, "gemm_bf16_kernel<256, 256, 128, 64, 64, %s, %s, %d, 1>", ta, tb, d[0].epilogue); break;
    case 6: snprintf(out, cap, "gemm_bf16_kernel<128, 128, 64, 64, 64, %s, %s, %d, 2>", ta, tb, d[0].epilogue); break;
    case 22: snprintf(out, cap, "gemm_bf16_ring_kernel<128, 128, 32, 64, 64, 4, %s, %s, %d>", ta, tb, d[0].epilogue); break;
    case 23: snprintf(out, cap, "gemm_bf16_ring_kernel<256, 256, 128, 64, 32, 4, %s, %s, %d>", ta, tb, d[0].epilogue); break;
    default: snprintf(out, cap, "gemm_bf16 tile %d <%s, %s, %d>", tile, ta, tb, d[0].epilogue); break;
  }
}

// `count` GEMMs (1..4) with the same form and epilogue in one launch.
hipError_t gemm_bf16_grouped(const GemmDesc* d, int count, hipStream_t stream) {
  if (count < 1 || count > kMaxGroup) return hipErrorInvalidValue;
  GroupParams gp{};
  gp.count = count;
  for (int g = 0; g < count; ++g) {
    if (!vector_ok(d[g]) || !segments_ok(d[g])) return hipErrorInvalidValue;
    // the kernels address an operand with 32-bit byte offsets from its first element (of a piece)
    const int64_t a_rows = d[g].trans_a ? d[g].K / d[g].n_seg : d[g].M, b_rows = d[g].trans_b ? d[g].N : d[g].K / d[g].n_seg;
    if (a_rows * (int64_t)d[g].lda * 2 >= (1ll << 31) || b_rows * (int64_t)d[g].ldb * 2 >= (1ll << 31))
      return hipErrorInvalidValue;
    if (d[g].trans_a != d[0].trans_a || d[g].trans_b != d[0].trans_b || d[g].epilogue != d[0].epilogue)
      return hipErrorInvalidValue;
    gp.p[g] = to_params(d[g]);
  }
  const GemmDesc& f = d[0];
  if (!f.trans_a && !f.trans_b) {
    if (f.epilogue == kEpiStore) return pick_tile<false, false, kEpiStore>(gp, stream);
    if (f.epilogue == kEpiGelu) return pick_tile<false, false, kEpiGelu>(gp, stream);
    if (f.epilogue == kEpiGeluGrad) return pick_tile<false, false, kEpiGeluGrad>(gp, stream);
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
