// The 2BW stage: device state, the forward/backward/update launch sequences and the C ABI.
//
// Device state (P parameters, T = b*s tokens, E = bytes per activation element):
//   wbuf[2]   two weight versions, flat, same per-layer order as the host vector; fp32 in fp32
//             mode, bf16 in bf16 mode.  Version v lives in wbuf[v % 2].
//   master    fp32 copy updated in place (bf16 mode only; it is never read by forward/backward)
//   G         fp32 coalesced gradient accumulator
//   adam_m/v  one copy of optimizer state
//   sets      activation sets (every saved activation of every layer for one microbatch), carved at a
//             constant stride from one allocation.  Full stash: a microbatch owns a set from its
//             forward pass until the grouped weight-gradient launch that consumed it; with
//             recomputation the stash is the stage input only and the sets are scratch
//   ws        backward temporaries, reduction partials
//
// Weight gradients of `wg_j` consecutive backward passes of a batch are computed by ONE grouped launch
// whose reduction range is the concatenation of those passes' tokens (K = j*T): the fp32 accumulator is
// read and written once per j microbatches instead of once per microbatch.  The operands of the passes
// stay where they are (activation sets; per-position copies of the output gradients); the kernel walks
// the pieces.  Groups never cross a batch boundary, so the coalesced sum of Section 3.1 is unchanged up
// to the order of fp32 additions.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <algorithm>
#include <vector>

#include "../../include/stage2bw.h"
#include "kernels.hpp"
#include "schedule.hpp"

using namespace k2bw;
using s2bw::Schedule;

namespace {

struct LayerOff {  // element offsets into a flat parameter vector
  int64_t ln1_g, ln1_b, wqkv, bqkv, wo, bo, ln2_g, ln2_b, w1, b1, w2, b2;
};

struct LayerActs {  // saved activations of one layer for one microbatch
  char *x, *a, *qkv, *o, *x1, *c, *u, *g;  // activation dtype
  float *mean1, *rstd1, *mean2, *rstd2, *lse;
};

struct ActSet {
  std::vector<LayerActs> layer;
};

int64_t align_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

struct EventPair {
  hipEvent_t start, stop;
  int cls;
  double flops, bytes;
  char name[96];   // kernel instance, as a kernel trace names it
};

}  // namespace

struct stage2bw {
  stage_config_t cfg;
  hipStream_t stream = nullptr;    // forward passes (and everything else until a backward stream is set)
  hipStream_t bstream = nullptr;   // backward passes and updates
  hipStream_t cur = nullptr;       // the stream the running call enqueues on
  bool two_streams = false;
  // two-stream ordering: per stash slot "forward written" / "backward has read"; per version
  // buffer "update has written"
  std::vector<hipEvent_t> fwd_done, bwd_done, set_done;   // per slot, per slot, per activation set
  std::vector<char> bwd_pending, set_pending;
  hipEvent_t ver_ready[2] = {nullptr, nullptr};
  bool ver_pending[2] = {false, false};
  Schedule sched;
  int64_t P = 0;
  int T = 0;
  int esize = 4;  // bytes per activation / version-buffer element
  int dtype = kF32;
  std::vector<LayerOff> off;

  // device memory
  std::vector<void*> allocations;
  int64_t bytes_total = 0, bytes_weights = 0, bytes_stash = 0;
  char* wbuf[2] = {nullptr, nullptr};
  // bf16 mode: per version, the transposes of the four projection matrices of every layer ([out, in] row-major;
  // per layer WqkvT [3h,h] | WoT [h,h] | W1T [f,h] | W2T [h,f]).  The data-gradient products read these, so that
  // their weight operand has the contraction index strided like the forward's instead of contiguous: the direct-
  // to-LDS loads then fetch whole 512-byte rows, and the products with long contractions run 16..28 % faster.
  // Rewritten from wbuf after every update (4 bytes of traffic per matrix element, once per m microbatches).
  char* wT[2] = {nullptr, nullptr};
  int64_t bytes_transposed = 0;
  float* master = nullptr;
  float* G = nullptr;
  float* adam_m = nullptr;
  float* adam_v = nullptr;

  // activation sets: sets[i] lives at acts_base + i * set_stride
  std::vector<ActSet> sets;
  char* acts_base = nullptr;
  int64_t set_stride = 0;
  std::vector<int> slot_set;       // full stash: the set an in-flight slot owns
  std::vector<int> free_sets;      // full stash: sets nobody owns (oldest release first)
  int fwd_scratch_set = 0;         // recompute: the set the forward pass scribbles on
  std::vector<char*> slot_x0;      // recompute: the stashed stage input per slot
  std::vector<int32_t*> slot_lens; // per slot: key lengths (padding mask)
  // deferred weight-gradient products
  int wg_j = 1;                    // backward passes per grouped weight-gradient launch
  int n_pending = 0;               // passes whose products are still to be launched
  bool pending_overwrite = false;  // the pending group holds the batch's first pass: its launch overwrites G
  int pending_set[kGemmMaxSegments] = {};   // the set of each pending pass, in order

  // backward workspace
  // tmp_h is transient; the gradients that the weight-gradient products read (dx1, du, dqkv and
  // each layer's input gradient dchain) exist once per layer, because those products run after
  // the data-gradient chain of the whole stage
  char* tmp_h = nullptr;
  std::vector<char*> dx1, dchain, du, dqkv;   // wg_j copies each, one per position in the pending group
  char* dy_top = nullptr;     // wg_j copies of the stage's incoming gradient (only when wg_j > 1)
  float* delta = nullptr;
  // per layer: partial rows of the bias / gain / shift gradients, reduced by one launch per backward pass
  std::vector<float*> ln_partial, ln_partial2, cs_partial, du_partial, attn_partial;

  // timing
  bool timing = false;
  std::vector<EventPair> events;
  size_t events_used = 0;

  stage2bw(const stage_config_t& c) : cfg(c), sched(c.m, c.max_inflight, c.flush != 0) {}
};

namespace {

int hip_rc(hipError_t e) {
  if (e == hipSuccess) return STAGE_OK;
  if (e == hipErrorOutOfMemory) return STAGE_ERR_OOM;
  return STAGE_ERR_HIP;
}

#define HIP_TRY(expr)                       \
  do {                                      \
    hipError_t e__ = (expr);                \
    if (e__ != hipSuccess) return hip_rc(e__); \
  } while (0)

int validate(const stage_config_t* c) {
  if (!c) return STAGE_ERR_INVALID_ARG;
  if (c->n_layers < 1 || c->hidden < 8 || c->n_heads < 1 || c->ffn < 8 || c->seq < 1 || c->microbatch < 1)
    return STAGE_ERR_INVALID_ARG;
  if (c->hidden % 8 || c->ffn % 8 || c->hidden % c->n_heads) return STAGE_ERR_INVALID_ARG;
  const int dh = c->hidden / c->n_heads;
  if (dh % 8 || dh > 128 || c->hidden > 16384) return STAGE_ERR_INVALID_ARG;
  if (c->m < 1 || c->max_inflight < 1 || c->m < c->max_inflight) return STAGE_ERR_INVALID_ARG;
  if (c->mask_mode < 0 || c->mask_mode > 2) return STAGE_ERR_INVALID_ARG;
  if (c->precision != STAGE_PREC_FP32 && c->precision != STAGE_PREC_BF16) return STAGE_ERR_INVALID_ARG;
  if (c->recompute != 0 && c->recompute != 1) return STAGE_ERR_INVALID_ARG;
  if (c->flush != 0 && c->flush != 1) return STAGE_ERR_INVALID_ARG;
  if (c->optimizer != STAGE_OPT_ADAM && c->optimizer != STAGE_OPT_MOMENTUM) return STAGE_ERR_INVALID_ARG;
  if (c->wgrad_group < 0 || c->wgrad_group > kGemmMaxSegments) return STAGE_ERR_INVALID_ARG;
  if (!(c->lr >= 0.f) || !(c->beta1 >= 0.f && c->beta1 < 1.f) || !(c->beta2 >= 0.f && c->beta2 < 1.f) ||
      !(c->adam_eps >= 0.f) || !(c->ln_eps >= 0.f))
    return STAGE_ERR_INVALID_ARG;
  if ((int64_t)c->seq * c->microbatch > (1 << 24)) return STAGE_ERR_INVALID_ARG;
  // every GEMM operand below 2 GiB in bf16 (32-bit byte offsets in the kernels)
  const int64_t T = (int64_t)c->seq * c->microbatch, widest = c->ffn > 3 * c->hidden ? c->ffn : 3 * c->hidden;
  if (T * widest >= (1ll << 30) || (int64_t)c->hidden * c->ffn >= (1ll << 30)) return STAGE_ERR_INVALID_ARG;
  return STAGE_OK;
}

int64_t layer_params(int64_t h, int64_t f) { return 4 * h * h + 2 * h * f + 9 * h + f; }

std::vector<LayerOff> make_offsets(const stage_config_t& c) {
  std::vector<LayerOff> v(c.n_layers);
  const int64_t h = c.hidden, f = c.ffn;
  int64_t o = 0;
  for (int l = 0; l < c.n_layers; ++l) {
    LayerOff& L = v[l];
    L.ln1_g = o; o += h;
    L.ln1_b = o; o += h;
    L.wqkv = o; o += h * 3 * h;
    L.bqkv = o; o += 3 * h;
    L.wo = o; o += h * h;
    L.bo = o; o += h;
    L.ln2_g = o; o += h;
    L.ln2_b = o; o += h;
    L.w1 = o; o += h * f;
    L.b1 = o; o += f;
    L.w2 = o; o += f * h;
    L.b2 = o; o += h;
  }
  return v;
}

int dev_alloc(stage2bw* st, void** out, int64_t bytes, int64_t* account) {
  void* p = nullptr;
  bytes = align_up(bytes, 256);
  hipError_t e = hipMalloc(&p, (size_t)bytes);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return STAGE_ERR_OOM;
  }
  st->allocations.push_back(p);
  st->bytes_total += bytes;
  if (account) *account += bytes;
  *out = p;
  return STAGE_OK;
}

// One allocation holding n activation sets at a constant stride (a multiple of 256 bytes).
int alloc_sets(stage2bw* st, int n) {
  const stage_config_t& c = st->cfg;
  const int64_t T = st->T, h = c.hidden, f = c.ffn, E = st->esize;
  const int64_t act_h = align_up(T * h * E, 256), act_3h = align_up(T * 3 * h * E, 256), act_f = align_up(T * f * E, 256);
  const int64_t stat = align_up(T * 4, 256), lse = align_up((int64_t)c.microbatch * c.n_heads * c.seq * 4, 256);
  const int64_t per_layer = 5 * act_h + act_3h + 2 * act_f + 4 * stat + lse;
  st->set_stride = per_layer * c.n_layers;
  int rc = dev_alloc(st, reinterpret_cast<void**>(&st->acts_base), st->set_stride * n, &st->bytes_stash);
  if (rc != STAGE_OK) return rc;
  st->sets.resize(n);
  for (int i = 0; i < n; ++i) {
    st->sets[i].layer.resize(c.n_layers);
    for (int l = 0; l < c.n_layers; ++l) {
      char* p = st->acts_base + st->set_stride * i + per_layer * l;
      LayerActs& A = st->sets[i].layer[l];
      A.x = p; p += act_h;
      A.a = p; p += act_h;
      A.qkv = p; p += act_3h;
      A.o = p; p += act_h;
      A.x1 = p; p += act_h;
      A.c = p; p += act_h;
      A.u = p; p += act_f;
      A.g = p; p += act_f;
      A.mean1 = reinterpret_cast<float*>(p); p += stat;
      A.rstd1 = reinterpret_cast<float*>(p); p += stat;
      A.mean2 = reinterpret_cast<float*>(p); p += stat;
      A.rstd2 = reinterpret_cast<float*>(p); p += stat;
      A.lse = reinterpret_cast<float*>(p); p += lse;
    }
  }
  return STAGE_OK;
}

// ---- launch wrapper with optional event timing ------------------------------------------------
template <typename F>
hipError_t timed(stage2bw* st, int cls, const char* name, double flops, double bytes, F&& launch) {
  EventPair* ev = nullptr;
  if (st->timing && st->events_used < st->events.size()) {
    ev = &st->events[st->events_used++];
    ev->cls = cls; ev->flops = flops; ev->bytes = bytes;
    std::snprintf(ev->name, sizeof(ev->name), "%s", name);
    hipError_t e = hipEventRecord(ev->start, st->cur);
    if (e != hipSuccess) return e;
  }
  hipError_t e = launch();
  if (e != hipSuccess) return e;
  if (ev) return hipEventRecord(ev->stop, st->cur);
  return hipSuccess;
}

const char* wptr(const stage2bw* st, int buffer, int64_t elem_off) {
  return st->wbuf[buffer] + elem_off * st->esize;
}

enum WhichMatrix { kWqkv = 0, kWo = 1, kW1 = 2, kW2 = 3 };
// element offset of a layer's transposed matrix inside wT (per layer: 3h*h | h*h | f*h | h*f elements)
int64_t wT_offset(const stage2bw* st, int layer, int which) {
  const int64_t h = st->cfg.hidden, f = st->cfg.ffn;
  const int64_t per_layer = 4 * h * h + 2 * h * f;
  const int64_t in_layer[4] = {0, 3 * h * h, 4 * h * h, 4 * h * h + h * f};
  return per_layer * layer + in_layer[which];
}
const char* wTptr(const stage2bw* st, int buffer, int layer, int which) {
  return st->wT[buffer] + wT_offset(st, layer, which) * 2;
}

// wT[buffer] <- transposes of the matrices in wbuf[buffer] (bf16 mode), one grouped launch
hipError_t refresh_transposed(stage2bw* st, int buffer, hipStream_t stream) {
  if (st->dtype != kBF16) return hipSuccess;
  const int h = st->cfg.hidden, f = st->cfg.ffn;
  std::vector<TransposeItem> items;
  items.reserve(4 * st->cfg.n_layers);
  for (int l = 0; l < st->cfg.n_layers; ++l) {
    const LayerOff& o = st->off[l];
    char* dst = st->wT[buffer];
    items.push_back({st->wbuf[buffer] + o.wqkv * 2, dst + wT_offset(st, l, kWqkv) * 2, h, 3 * h});
    items.push_back({st->wbuf[buffer] + o.wo * 2, dst + wT_offset(st, l, kWo) * 2, h, h});
    items.push_back({st->wbuf[buffer] + o.w1 * 2, dst + wT_offset(st, l, kW1) * 2, h, f});
    items.push_back({st->wbuf[buffer] + o.w2 * 2, dst + wT_offset(st, l, kW2) * 2, f, h});
  }
  return transpose_bf16_grouped(items.data(), (int)items.size(), stream);
}

hipError_t run_gemm(stage2bw* st, int cls, const GemmDesc& d) {
  char name[96] = "";
  if (st->timing) gemm_kernel_name(&d, 1, name, sizeof(name));
  return timed(st, cls, name, 2.0 * d.M * d.N * d.K, 0.0, [&] { return gemm(d, st->cur); });
}

hipError_t run_ln_fwd(stage2bw* st, const void* x, const void* gain, const void* shift, void* y, float* mean,
                      float* rstd) {
  const double bytes = 2.0 * st->T * st->cfg.hidden * st->esize + 8.0 * st->T;
  return timed(st, STAGE_K_LN_FWD, "ln_fwd_kernel", 0.0, bytes, [&] {
    return layernorm_fwd(x, gain, shift, y, mean, rstd, st->T, st->cfg.hidden, st->cfg.ln_eps, st->dtype, st->cur);
  });
}

// LayerNorm backward; its two parameter gradients (gain | shift are adjacent in G) are left as
// per-workgroup partial rows in `partial` and reduced at the end of the layer.
hipError_t run_ln_bwd(stage2bw* st, const void* dy, const void* x, const float* mean, const float* rstd,
                      const void* gain, const void* dres, void* dx, float* partial, int* parts) {
  const int h = st->cfg.hidden;
  const double bytes = 4.0 * st->T * h * st->esize + 8.0 * st->T;
  return timed(st, STAGE_K_LN_BWD, h >= 2048 ? "ln_bwd_wide_kernel" : "ln_bwd_kernel", 0.0, bytes, [&] {
    return layernorm_bwd(dy, x, mean, rstd, gain, dres, dx, partial, parts, st->T, h, st->dtype, st->cur);
  });
}

AttnDesc attn_desc(const stage2bw* st, const int32_t* lens) {
  AttnDesc d;
  d.b = st->cfg.microbatch; d.s = st->cfg.seq; d.a = st->cfg.n_heads; d.dh = st->cfg.hidden / st->cfg.n_heads;
  d.mask_mode = st->cfg.mask_mode; d.seqlens = lens; d.dtype = st->dtype;
  return d;
}

// Forward of all layers on weight buffer `buf`.  acts.layer[0].x already holds the stage input.
// y_out == nullptr: the stage output is not wanted (the forward re-run inside a backward pass with
// recomputation): the last layer stops after FC1 + GELU, whose outputs the backward pass reads; its FC2
// product would only produce the output that was already sent on.
hipError_t run_forward(stage2bw* st, int buf, ActSet& acts, const int32_t* lens, void* y_out) {
  const stage_config_t& c = st->cfg;
  const int T = st->T, h = c.hidden, f = c.ffn;
  const double attn_flops = 4.0 * c.microbatch * (double)c.seq * c.seq * h;
  for (int l = 0; l < c.n_layers; ++l) {
    const LayerOff& o = st->off[l];
    LayerActs& A = acts.layer[l];
    void* y = (l == c.n_layers - 1) ? y_out : static_cast<void*>(acts.layer[l + 1].x);
    hipError_t e;
    e = run_ln_fwd(st, A.x, wptr(st, buf, o.ln1_g), wptr(st, buf, o.ln1_b), A.a, A.mean1, A.rstd1);
    if (e != hipSuccess) return e;
    GemmDesc g;
    g.dtype = st->dtype;
    g.A = A.a; g.lda = h; g.B = wptr(st, buf, o.wqkv); g.ldb = 3 * h; g.C = A.qkv; g.ldc = 3 * h;
    g.M = T; g.N = 3 * h; g.K = h; g.bias = wptr(st, buf, o.bqkv);
    g.prefetch = wptr(st, buf, o.wo); g.prefetch_bytes = (int64_t)h * h * st->esize;   // the next GEMM's weights
    e = run_gemm(st, STAGE_K_GEMM_FWD, g);
    if (e != hipSuccess) return e;
    e = timed(st, STAGE_K_ATTN_FWD, st->dtype == kBF16 ? "attn_fwd_mfma_kernel" : "attn_fwd_simple", attn_flops, 0.0, [&] {
      return attention_fwd(attn_desc(st, lens), A.qkv, A.o, A.lse, st->cur);
    });
    if (e != hipSuccess) return e;
    g = GemmDesc();
    g.dtype = st->dtype;
    g.A = A.o; g.lda = h; g.B = wptr(st, buf, o.wo); g.ldb = h; g.C = A.x1; g.ldc = h;
    g.M = T; g.N = h; g.K = h; g.bias = wptr(st, buf, o.bo); g.aux = A.x;
    g.prefetch = wptr(st, buf, o.w1); g.prefetch_bytes = (int64_t)h * f * st->esize;
    e = run_gemm(st, STAGE_K_GEMM_FWD, g);
    if (e != hipSuccess) return e;
    e = run_ln_fwd(st, A.x1, wptr(st, buf, o.ln2_g), wptr(st, buf, o.ln2_b), A.c, A.mean2, A.rstd2);
    if (e != hipSuccess) return e;
    g = GemmDesc();
    g.dtype = st->dtype;
    g.A = A.c; g.lda = h; g.B = wptr(st, buf, o.w1); g.ldb = f; g.C = A.u; g.ldc = f;
    g.M = T; g.N = f; g.K = h; g.bias = wptr(st, buf, o.b1); g.epilogue = kEpiGelu; g.aux_out = A.g;
    g.prefetch = wptr(st, buf, o.w2); g.prefetch_bytes = (int64_t)h * f * st->esize;
    e = run_gemm(st, STAGE_K_GEMM_FWD, g);
    if (e != hipSuccess) return e;
    if (y == nullptr) break;
    g = GemmDesc();
    g.dtype = st->dtype;
    g.A = A.g; g.lda = f; g.B = wptr(st, buf, o.w2); g.ldb = h; g.C = y; g.ldc = h;
    g.M = T; g.N = h; g.K = f; g.bias = wptr(st, buf, o.b2); g.aux = A.x1;
    if (l + 1 < c.n_layers) { g.prefetch = wptr(st, buf, st->off[l + 1].wqkv); g.prefetch_bytes = (int64_t)3 * h * h * st->esize; }
    e = run_gemm(st, STAGE_K_GEMM_FWD, g);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

// The grouped weight-gradient launch(es) for the pending backward passes: per layer the four products
// G_W (+)= [X_1; ..; X_n]^T [dY_1; ..; dY_n] over the n = n_pending passes' tokens.  The activation
// operand of pass s lies in activation set pending_set[s], its gradient operand in copy s of the
// layer's gradient buffers.
hipError_t flush_wgrad(stage2bw* st) {
  const int n = st->n_pending;
  if (n == 0) return hipSuccess;
  const stage_config_t& c = st->cfg;
  const int T = st->T, h = c.hidden, f = c.ffn;
  const int64_t E = st->esize;
  std::vector<GemmDesc> wg;
  wg.reserve(4 * c.n_layers);
  const int set0 = st->pending_set[0];
  for (int l = c.n_layers - 1; l >= 0; --l) {
    const LayerOff& o = st->off[l];
    auto product = [&](const char* act_in_set0, int M, const char* grad0, int64_t grad_copy_bytes, int N, float* out) {
      wg.emplace_back();
      GemmDesc& w = wg.back();
      w.dtype = st->dtype;
      w.lda = M; w.trans_a = true; w.ldb = N; w.C = out; w.ldc = N;
      w.M = M; w.N = N; w.K = n * T; w.epilogue = kEpiAccum; w.accumulate = !st->pending_overwrite;
      w.n_seg = n;
      if (n == 1) {   // plain operands (the only form the fp32 kernels take)
        w.A = act_in_set0 + st->set_stride * set0;
        w.B = grad0;
      } else {
        w.A = act_in_set0; w.a_seg_stride = st->set_stride;
        w.B = grad0; w.b_seg_stride = grad_copy_bytes;
        for (int s = 0; s < n; ++s) { w.a_seg_idx[s] = (uint8_t)st->pending_set[s]; w.b_seg_idx[s] = (uint8_t)s; }
      }
    };
    const LayerActs& A = st->sets[0].layer[l];   // addresses inside set number 0
    const char* dy0 = l == c.n_layers - 1 ? st->dy_top : st->dchain[l + 1];
    product(A.g, f, dy0, (int64_t)T * h * E, h, st->G + o.w2);
    product(A.c, h, st->du[l], (int64_t)T * f * E, f, st->G + o.w1);
    product(A.o, h, st->dx1[l], (int64_t)T * h * E, h, st->G + o.wo);
    product(A.a, h, st->dqkv[l], (int64_t)T * 3 * h * E, 3 * h, st->G + o.wqkv);
  }
  // One launch per run of products with at least kMinRounds rounds of 256x256 tiles on the chip's CUs (what is left
  // at the end joins the last run).  Shared launches exist to spare small products their ramp, drain and partial
  // last round; beyond a few rounds a longer launch is slower, not faster: the 32 tiles that run on an XCD at a time
  // share operand panels in its L2 only while they stay within some twenty K steps of each other, they drift apart
  // over the rounds, and nothing but the end of a launch brings them back in step (weight-gradient time per batch
  // on one box, C5: 96 rounds in one launch 390 ms, launches of 16 rounds 358 ms; C4: 48 rounds 184 ms, 8 rounds
  // 168 ms; thresholds of 4 and 16 rounds measure within 1 % of 8).
  constexpr int64_t kMinRounds = 8;
  const int64_t min_tiles = kMinRounds * gemm_compute_units();
  auto tiles_of = [](const GemmDesc& d) { return (int64_t)((d.M + 255) / 256) * ((d.N + 255) / 256); };
  for (size_t i0 = 0; i0 < wg.size();) {
    size_t i1 = i0;
    int64_t tiles = 0, rest = 0;
    while (i1 < wg.size() && i1 - i0 < (size_t)kGemmMaxGroup && tiles < min_tiles) tiles += tiles_of(wg[i1++]);
    for (size_t i = i1; i < wg.size(); ++i) rest += tiles_of(wg[i]);
    if (rest < min_tiles / 2 && wg.size() - i0 <= (size_t)kGemmMaxGroup) i1 = wg.size();
    const int cnt = (int)(i1 - i0);
    double flops = 0.0;
    for (int i = 0; i < cnt; ++i) flops += 2.0 * wg[i0 + i].M * (double)wg[i0 + i].N * wg[i0 + i].K;
    char wg_name[96] = "";
    if (st->timing) gemm_kernel_name(&wg[i0], cnt, wg_name, sizeof(wg_name));
    hipError_t e = timed(st, STAGE_K_GEMM_WGRAD, wg_name, flops, 0.0, [&] { return gemm_grouped(&wg[i0], cnt, st->cur); });
    if (e != hipSuccess) return e;
    i0 = i1;
  }
  // the sets are free again once this launch has run
  if (!c.recompute) {
    for (int s = 0; s < n; ++s) {
      const int set = st->pending_set[s];
      if (st->two_streams) {
        hipError_t e = hipEventRecord(st->set_done[set], st->cur);
        if (e != hipSuccess) return e;
        st->set_pending[set] = 1;
      }
      st->free_sets.push_back(set);
    }
  }
  st->n_pending = 0;
  st->pending_overwrite = false;
  return hipSuccess;
}

// Backward of all layers on weight buffer `buf` for the pass at position `pos` of the pending group,
// whose activations are in set `set`.  Leaves the operands of the weight-gradient products in place
// (flush_wgrad launches them); bias, gain and shift gradients go into G here (overwrite when `first`).
hipError_t run_backward(stage2bw* st, int buf, int set, int pos, const int32_t* lens, const void* dy_in, void* dx_out,
                        bool first) {
  const stage_config_t& c = st->cfg;
  const int T = st->T, h = c.hidden, f = c.ffn;
  const int64_t E = st->esize;
  const bool acc = !first;
  const double attn_flops = 10.0 * c.microbatch * (double)c.seq * c.seq * h;
  ActSet& acts = st->sets[set];
  // the top layer's weight-gradient product reads the incoming gradient after this call has returned:
  // keep a copy (one launch's worth of traffic per pass)
  char* dy_keep = st->dy_top + (int64_t)pos * T * h * E;
  {
    const int64_t bytes = (int64_t)T * h * E;
    hipError_t e = timed(st, STAGE_K_OTHER, "copy16_kernel", 0.0, 2.0 * bytes, [&] { return copy_bytes(dy_in, dy_keep, bytes, st->cur); });
    if (e != hipSuccess) return e;
  }
  const void* dy = dy_keep;
  std::vector<FinalizeItem> fin;
  fin.reserve(8 * c.n_layers);
  double fin_elems = 0.0;
  for (int l = c.n_layers - 1; l >= 0; --l) {
    const LayerOff& o = st->off[l];
    LayerActs& A = acts.layer[l];
    void* dx = (l == 0) ? dx_out : static_cast<void*>(st->dchain[l] + (int64_t)pos * T * h * E);
    char* du = st->du[l] + (int64_t)pos * T * f * E;
    char* dx1 = st->dx1[l] + (int64_t)pos * T * h * E;
    char* dqkv = st->dqkv[l] + (int64_t)pos * T * 3 * h * E;
    hipError_t e;
    // Bias gradients are column sums of the four projection-output gradients.  Three of them come
    // out of the kernels that produce those gradients: dx1 and this layer's result dx (= the next
    // lower layer's dy) from the LayerNorm backward kernels, du (bf16 mode) from the epilogue of
    // the GEMM that computes it, dqkv (bf16 mode) from the attention backward kernels; the stage's
    // incoming dy, and du and dqkv in fp32 mode, are summed by the column-sum kernel.
    const bool fused_du = st->dtype == kBF16;
    const bool bf16 = st->dtype == kBF16;
    auto dgrad = [&](const void* grad, int N, int which, int64_t w_off, int K, void* out, const void* u, int next_layer,
                     int next_which, int64_t next_off, int64_t next_elems) {
      // out[T,K] = grad[T,N] * W[K,N]^T.  Where the product runs on 256 x 256 tiles (bf16, at least 144 of them)
      // it reads the transposed copy W^T [N,K] in the forward's operand form: measured 2 % (contraction 8192) to
      // 16..28 % (16384 and up) faster there, while the 128 x 128 kernel of the small products, whose K tiles of 64
      // already fetch whole 128-byte lines, is 10 % faster on W as it is stored.  fp32: W as it is stored.
      // next_*: the weights of the chain's next data-gradient GEMM, in the form that GEMM will read
      GemmDesc d;
      d.dtype = st->dtype;
      d.A = grad; d.lda = N; d.C = out; d.ldc = K;
      d.M = T; d.N = K; d.K = N;
      auto reads_transposed = [&](int k_out) { return bf16 && (int64_t)ceil_div(T, 256) * ceil_div(k_out, 256) >= 144; };
      if (reads_transposed(K)) { d.B = wTptr(st, buf, l, which); d.ldb = K; d.trans_b = false; }
      else { d.B = wptr(st, buf, w_off); d.ldb = N; d.trans_b = true; }
      if (next_layer >= 0) {
        d.prefetch = reads_transposed(next_which == kW2 ? f : h) ? wTptr(st, buf, next_layer, next_which) : wptr(st, buf, next_off);
        d.prefetch_bytes = next_elems * st->esize;
      }
      if (u) { d.epilogue = kEpiGeluGrad; d.aux = u; if (fused_du) d.colsum_partial = st->du_partial[l]; }
      return run_gemm(st, STAGE_K_GEMM_DGRAD, d);
    };
    // y = x1 + GELU(u) W2 + b2
    e = dgrad(dy, h, kW2, o.w2, f, du, A.u, l, kW1, o.w1, (int64_t)h * f);   if (e != hipSuccess) return e;
    // u = c W1 + b1
    e = dgrad(du, f, kW1, o.w1, h, st->tmp_h, nullptr, l, kWo, o.wo, (int64_t)h * h);   if (e != hipSuccess) return e;
    // c = LN2(x1); dx1 = dy + LN2'(dc)
    int ln2_parts = 0, ln1_parts = 0;
    e = run_ln_bwd(st, st->tmp_h, A.x1, A.mean2, A.rstd2, wptr(st, buf, o.ln2_g), dy, dx1, st->ln_partial[l], &ln2_parts);
    if (e != hipSuccess) return e;
    // x1 = x + o Wo + bo
    e = dgrad(dx1, h, kWo, o.wo, h, st->tmp_h, nullptr, l, kWqkv, o.wqkv, (int64_t)3 * h * h);   if (e != hipSuccess) return e;
    // attention
    AttnDesc ad = attn_desc(st, lens);
    const bool fused_dqkv = attention_mfma_supported(ad);
    if (fused_dqkv) ad.colsum_partial = st->attn_partial[l];
    e = timed(st, STAGE_K_ATTN_BWD, "attention backward (dq + dkv kernels)", attn_flops, 0.0, [&] {
      return attention_bwd(ad, A.qkv, A.o, A.lse, st->tmp_h, dqkv, st->delta, st->cur);
    });
    if (e != hipSuccess) return e;
    // qkv = a Wqkv + bqkv
    e = dgrad(dqkv, 3 * h, kWqkv, o.wqkv, h, st->tmp_h, nullptr, l - 1, kW2, l > 0 ? st->off[l - 1].w2 : 0, (int64_t)h * f);
    if (e != hipSuccess) return e;
    // a = LN1(x); dx = dx1 + LN1'(da)
    e = run_ln_bwd(st, st->tmp_h, A.x, A.mean1, A.rstd1, wptr(st, buf, o.ln1_g), dx1, dx, st->ln_partial2[l], &ln1_parts);
    if (e != hipSuccess) return e;
    ColsumItem cs[3];
    int n_cs = 0, col_dqkv = -1, col_du = -1, col_dy = -1, cols = 0;
    if (!fused_dqkv) { col_dqkv = cols; cs[n_cs++] = {dqkv, 3 * h, 3 * h}; cols += 3 * h; }
    if (!fused_du) { col_du = cols; cs[n_cs++] = {du, f, f}; cols += f; }
    if (l == c.n_layers - 1) { col_dy = cols; cs[n_cs++] = {dy, h, h}; cols += h; }
    int cs_parts = 0, cs_cols = 0;
    if (n_cs > 0) {
      e = timed(st, STAGE_K_BIAS_GRAD, "colsum_partial_grouped_kernel", 0.0, (double)T * cols * st->esize, [&] {
        return colsum_partial_grouped(cs, n_cs, T, st->cs_partial[l], &cs_parts, &cs_cols, st->dtype, st->cur);
      });
      if (e != hipSuccess) return e;
    }
    auto add_fin = [&](const float* partial, int parts, int ld, int n, float* out) {
      fin.push_back({partial, parts, ld, n, out});
      fin_elems += (double)parts * n;
    };
    if (fused_dqkv) add_fin(st->attn_partial[l], attention_colsum_rows(c.microbatch, c.seq), 3 * h, 3 * h, st->G + o.bqkv);
    else add_fin(st->cs_partial[l] + col_dqkv, cs_parts, cs_cols, 3 * h, st->G + o.bqkv);
    if (fused_du) add_fin(st->du_partial[l], (T + 31) / 32, f, f, st->G + o.b1);
    else add_fin(st->cs_partial[l] + col_du, cs_parts, cs_cols, f, st->G + o.b1);
    if (col_dy >= 0) add_fin(st->cs_partial[l] + col_dy, cs_parts, cs_cols, h, st->G + o.b2);
    add_fin(st->ln_partial[l], ln2_parts, 3 * h, 2 * h, st->G + o.ln2_g);
    add_fin(st->ln_partial[l] + 2 * h, ln2_parts, 3 * h, h, st->G + o.bo);
    add_fin(st->ln_partial2[l], ln1_parts, 3 * h, 2 * h, st->G + o.ln1_g);
    if (l > 0) add_fin(st->ln_partial2[l] + 2 * h, ln1_parts, 3 * h, h, st->G + st->off[l - 1].b2);
    dy = dx;
  }
  // every layer left its partial rows in buffers of its own: one reduction launch finishes the
  // bias, gain and shift gradients of the whole stage
  for (size_t i0 = 0; i0 < fin.size(); i0 += kFinalizeMaxItems) {
    const int n = (int)std::min<size_t>(kFinalizeMaxItems, fin.size() - i0);
    hipError_t e = timed(st, STAGE_K_BIAS_GRAD, "colsum_finalize_grouped_kernel", 0.0, 4.0 * fin_elems * n / fin.size(), [&] {
      return colsum_finalize_grouped(&fin[i0], n, acc, st->cur);
    });
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

int free_all(stage2bw* st) {
  int rc = STAGE_OK;
  for (void* p : st->allocations)
    if (hipFree(p) != hipSuccess) rc = STAGE_ERR_HIP;
  st->allocations.clear();
  for (EventPair& e : st->events) {
    (void)hipEventDestroy(e.start);
    (void)hipEventDestroy(e.stop);
  }
  st->events.clear();
  for (hipEvent_t e : st->fwd_done) (void)hipEventDestroy(e);
  for (hipEvent_t e : st->bwd_done) (void)hipEventDestroy(e);
  for (hipEvent_t e : st->set_done) (void)hipEventDestroy(e);
  st->fwd_done.clear();
  st->bwd_done.clear();
  st->set_done.clear();
  for (hipEvent_t& e : st->ver_ready)
    if (e) { (void)hipEventDestroy(e); e = nullptr; }
  return rc;
}

hipError_t sync_all(stage2bw* st) {
  hipError_t e = hipStreamSynchronize(st->stream);
  if (e == hipSuccess && st->two_streams) e = hipStreamSynchronize(st->bstream);
  return e;
}

}  // namespace

// =============================================================================== C ABI

extern "C" {

int64_t stage_param_count(const stage_config_t* cfg) {
  int rc = validate(cfg);
  if (rc != STAGE_OK) return rc;
  return cfg->n_layers * layer_params(cfg->hidden, cfg->ffn);
}

int stage_create(const stage_config_t* cfg, const float* init_weights_host, void* hip_stream, stage_t** out) {
  if (!out) return STAGE_ERR_INVALID_ARG;
  *out = nullptr;
  int rc = validate(cfg);
  if (rc != STAGE_OK) return rc;
  if (!init_weights_host) return STAGE_ERR_INVALID_ARG;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) {
    (void)hipGetLastError();
    return STAGE_ERR_HIP;
  }
  stage2bw* st = new (std::nothrow) stage2bw(*cfg);
  if (!st) return STAGE_ERR_OOM;
  st->stream = st->bstream = st->cur = static_cast<hipStream_t>(hip_stream);
  st->P = cfg->n_layers * layer_params(cfg->hidden, cfg->ffn);
  st->T = cfg->microbatch * cfg->seq;
  st->dtype = cfg->precision == STAGE_PREC_BF16 ? kBF16 : kF32;
  st->esize = st->dtype == kBF16 ? 2 : 4;
  st->off = make_offsets(*cfg);

  const int64_t P = st->P, T = st->T, h = cfg->hidden, f = cfg->ffn, E = st->esize;
  auto fail = [&](int code) {
    free_all(st);
    delete st;
    return code;
  };
#define ALLOC(ptr, bytes, account)                                                      \
  do {                                                                                  \
    int rc__ = dev_alloc(st, reinterpret_cast<void**>(&(ptr)), (bytes), (account));     \
    if (rc__ != STAGE_OK) return fail(rc__);                                            \
  } while (0)

  ALLOC(st->wbuf[0], P * E, &st->bytes_weights);
  if (cfg->flush) st->wbuf[1] = st->wbuf[0];   // one weight version (Section 3.2)
  else ALLOC(st->wbuf[1], P * E, &st->bytes_weights);
  if (st->dtype == kBF16) ALLOC(st->master, P * 4, &st->bytes_weights);
  if (st->dtype == kBF16) {
    const int64_t tbytes = cfg->n_layers * (4 * h * h + 2 * h * f) * 2;
    ALLOC(st->wT[0], tbytes, &st->bytes_transposed);
    if (cfg->flush) st->wT[1] = st->wT[0];
    else ALLOC(st->wT[1], tbytes, &st->bytes_transposed);
  }
  ALLOC(st->G, P * 4, nullptr);
  ALLOC(st->adam_m, P * 4, nullptr);
  if (cfg->optimizer == STAGE_OPT_ADAM) ALLOC(st->adam_v, P * 4, nullptr);

  // Backward passes per grouped weight-gradient launch: the caller's choice, else what brings the reduction
  // range to 16384 tokens (4 passes of 4096 tokens, 8 of 2048 or fewer: measured, 8 instead of 4 passes of 2048
  // are +3 % on the weight-gradient launches, 8 instead of 4 of 4096 nothing); never more than m (a group stays
  // inside its batch).  The segmented product exists in the bf16 ring kernels only, whose
  // K tiles must divide a pass's tokens, and a set's number must fit the kernel's 4-bit fields.
  int j = cfg->wgrad_group > 0 ? cfg->wgrad_group : (T <= 2048 ? 8 : 4);
  if (j > cfg->m) j = cfg->m;
  if (st->dtype != kBF16 || T % 64 != 0) j = 1;
  if (!cfg->recompute && j > 1 && cfg->max_inflight + j - 1 > 16) j = std::max(1, 17 - cfg->max_inflight);
  st->wg_j = j;
  // full stash: a set per in-flight microbatch plus the j-1 that may wait for their group's launch;
  // recompute: the j sets the pending passes re-computed into, and one for the forward pass to scribble on
  const int n_sets = cfg->recompute ? j + 1 : cfg->max_inflight + j - 1;
  rc = alloc_sets(st, n_sets);
  if (rc != STAGE_OK) return fail(rc);
  st->fwd_scratch_set = cfg->recompute ? j : 0;
  st->slot_set.assign(cfg->max_inflight, -1);
  if (!cfg->recompute)
    for (int i = 0; i < n_sets; ++i) st->free_sets.push_back(i);
  st->slot_lens.resize(cfg->max_inflight, nullptr);
  st->slot_x0.resize(cfg->max_inflight, nullptr);
  for (int i = 0; i < cfg->max_inflight; ++i) {
    ALLOC(st->slot_lens[i], (int64_t)cfg->microbatch * 4, &st->bytes_stash);
    if (cfg->recompute) ALLOC(st->slot_x0[i], T * h * E, &st->bytes_stash);
  }
  ALLOC(st->tmp_h, T * h * E, nullptr);
  st->dx1.assign(cfg->n_layers, nullptr);
  st->dchain.assign(cfg->n_layers, nullptr);
  st->du.assign(cfg->n_layers, nullptr);
  st->dqkv.assign(cfg->n_layers, nullptr);
  // (T*h*E is a multiple of 256 bytes whenever j > 1: T % 64 == 0 and h % 8 == 0)
  for (int l = 0; l < cfg->n_layers; ++l) {
    ALLOC(st->dx1[l], j * T * h * E, nullptr);
    if (l > 0) ALLOC(st->dchain[l], j * T * h * E, nullptr);
    ALLOC(st->du[l], j * T * f * E, nullptr);
    ALLOC(st->dqkv[l], j * T * 3 * h * E, nullptr);
  }
  ALLOC(st->dy_top, j * T * h * E, nullptr);
  ALLOC(st->delta, (int64_t)cfg->microbatch * cfg->n_heads * cfg->seq * 4, nullptr);
  st->ln_partial.assign(cfg->n_layers, nullptr);
  st->ln_partial2.assign(cfg->n_layers, nullptr);
  st->cs_partial.assign(cfg->n_layers, nullptr);
  st->du_partial.assign(cfg->n_layers, nullptr);
  st->attn_partial.assign(cfg->n_layers, nullptr);
  for (int l = 0; l < cfg->n_layers; ++l) {
    ALLOC(st->ln_partial[l], (int64_t)ln_bwd_max_parts() * 3 * h * 4, nullptr);
    ALLOC(st->ln_partial2[l], (int64_t)ln_bwd_max_parts() * 3 * h * 4, nullptr);
    if (st->dtype == kBF16) {
      ALLOC(st->du_partial[l], (int64_t)((T + 31) / 32) * f * 4, nullptr);
      ALLOC(st->attn_partial[l], (int64_t)attention_colsum_rows(cfg->microbatch, cfg->seq) * 3 * h * 4, nullptr);
    }
    // the column-sum kernel serves the stage's incoming dy (top layer) and, in fp32 mode or for
    // head sizes without the fused attention kernels, du and dqkv of every layer
    ALLOC(st->cs_partial[l], (int64_t)colsum_max_parts() * (5 * h + f) * 4, nullptr);
  }
#undef ALLOC

  // upload W(0): fp32 mode -> both buffers; bf16 mode -> master, then both bf16 buffers
  hipError_t e;
  float* dst32 = st->dtype == kBF16 ? st->master : reinterpret_cast<float*>(st->wbuf[0]);
  e = hipMemcpyAsync(dst32, init_weights_host, (size_t)P * 4, hipMemcpyHostToDevice, st->stream);
  if (e == hipSuccess) {
    if (st->dtype == kBF16) {
      e = convert_f32_to_bf16(st->master, reinterpret_cast<bf16_t*>(st->wbuf[0]), P, st->stream);
      if (e == hipSuccess && !cfg->flush)
        e = hipMemcpyAsync(st->wbuf[1], st->wbuf[0], (size_t)P * 2, hipMemcpyDeviceToDevice, st->stream);
    } else if (!cfg->flush) {
      e = hipMemcpyAsync(st->wbuf[1], st->wbuf[0], (size_t)P * 4, hipMemcpyDeviceToDevice, st->stream);
    }
  }
  if (e == hipSuccess) e = refresh_transposed(st, 0, st->stream);
  if (e == hipSuccess && !cfg->flush) e = refresh_transposed(st, 1, st->stream);
  if (e == hipSuccess) e = hipMemsetAsync(st->G, 0, (size_t)P * 4, st->stream);
  if (e == hipSuccess) e = hipMemsetAsync(st->adam_m, 0, (size_t)P * 4, st->stream);
  if (e == hipSuccess && st->adam_v) e = hipMemsetAsync(st->adam_v, 0, (size_t)P * 4, st->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(st->stream);
  if (e != hipSuccess) return fail(hip_rc(e));
  *out = st;
  return STAGE_OK;
}

int stage_forward(stage_t* st, int64_t mb, const void* x_dev, const int32_t* seqlens_dev, void* y_dev) {
  if (!st || !x_dev || !y_dev || x_dev == y_dev) return STAGE_ERR_INVALID_ARG;
  if (st->cfg.mask_mode == STAGE_MASK_PADDING && !seqlens_dev) return STAGE_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(x_dev) & 15) || (reinterpret_cast<uintptr_t>(y_dev) & 15)) return STAGE_ERR_INVALID_ARG;
  int slot = -1;
  int rc = st->sched.check_forward(mb, &slot);
  if (rc != STAGE_OK) return rc;
  const int buf = st->sched.buffer_of(st->sched.read_version());
  const int64_t in_bytes = (int64_t)st->T * st->cfg.hidden * st->esize;
  st->cur = st->stream;
  // full stash: the microbatch takes the activation set that has been free the longest
  if (!st->cfg.recompute && st->free_sets.empty()) return STAGE_ERR_BAD_STATE;   // (cannot happen: sets = slots + wg_j - 1)
  const int set = st->cfg.recompute ? st->fwd_scratch_set : st->free_sets.front();
  if (st->two_streams) {
    // the slot's previous occupant has been read by its backward pass, the set's by the weight-gradient
    // launch of its group; the version has been written
    if (st->bwd_pending[slot]) { HIP_TRY(hipStreamWaitEvent(st->stream, st->bwd_done[slot], 0)); st->bwd_pending[slot] = 0; }
    if (st->set_pending[set]) { HIP_TRY(hipStreamWaitEvent(st->stream, st->set_done[set], 0)); st->set_pending[set] = 0; }
    if (st->ver_pending[buf]) { HIP_TRY(hipStreamWaitEvent(st->stream, st->ver_ready[buf], 0)); st->ver_pending[buf] = false; }
  }
  ActSet& acts = st->sets[set];
  // stash the stage input (with recompute it is the only thing kept)
  char* x_keep = st->cfg.recompute ? st->slot_x0[slot] : acts.layer[0].x;
  HIP_TRY(timed(st, STAGE_K_OTHER, "copy16_kernel", 0.0, 2.0 * in_bytes, [&] { return copy_bytes(x_dev, x_keep, in_bytes, st->stream); }));
  const int32_t* lens = nullptr;
  if (st->cfg.mask_mode == STAGE_MASK_PADDING) {
    HIP_TRY(hipMemcpyAsync(st->slot_lens[slot], seqlens_dev, (size_t)st->cfg.microbatch * 4, hipMemcpyDeviceToDevice,
                           st->stream));
    lens = st->slot_lens[slot];
  }
  if (st->cfg.recompute) {
    // the shared activation set is scratch here; its layer-0 input is read from the stash
    char* saved = acts.layer[0].x;
    acts.layer[0].x = x_keep;
    hipError_t e = run_forward(st, buf, acts, lens, y_dev);
    acts.layer[0].x = saved;
    HIP_TRY(e);
  } else {
    HIP_TRY(run_forward(st, buf, acts, lens, y_dev));
  }
  if (st->two_streams) HIP_TRY(hipEventRecord(st->fwd_done[slot], st->stream));
  if (!st->cfg.recompute) {
    st->free_sets.erase(st->free_sets.begin());
    st->slot_set[slot] = set;
  }
  int64_t version = 0;
  int b2 = 0;
  return st->sched.forward(mb, &slot, &version, &b2);
}

int stage_backward(stage_t* st, int64_t mb, const void* dy_dev, void* dx_dev) {
  if (!st || !dy_dev || !dx_dev || dy_dev == dx_dev) return STAGE_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(dy_dev) & 15) || (reinterpret_cast<uintptr_t>(dx_dev) & 15)) return STAGE_ERR_INVALID_ARG;
  int slot = -1;
  int rc = st->sched.check_backward(mb, &slot);
  if (rc != STAGE_OK) return rc;
  // commit the bookkeeping first to learn tag and accumulate flag (no failure path after the check)
  int64_t version = 0;
  int buf = 0, first = 0;
  rc = st->sched.backward(mb, &slot, &version, &buf, &first);
  if (rc != STAGE_OK) return rc;
  const int32_t* lens = st->cfg.mask_mode == STAGE_MASK_PADDING ? st->slot_lens[slot] : nullptr;
  st->cur = st->bstream;
  if (st->two_streams) HIP_TRY(hipStreamWaitEvent(st->bstream, st->fwd_done[slot], 0));
  const int pos = st->n_pending;
  if (pos == 0) st->pending_overwrite = first != 0;
  // the activations of this pass: the set the forward pass filled, or (recompute) set number `pos`, which
  // the re-run forward fills now
  const int set = st->cfg.recompute ? pos : st->slot_set[slot];
  if (st->cfg.recompute) {
    // re-run the forward on the version tagged at the forward pass (Section 4.1 with Section 3.1)
    ActSet& acts = st->sets[set];
    char* saved = acts.layer[0].x;
    acts.layer[0].x = st->slot_x0[slot];
    hipError_t e = run_forward(st, buf, acts, lens, nullptr);
    if (e == hipSuccess) e = run_backward(st, buf, set, pos, lens, dy_dev, dx_dev, first != 0);
    acts.layer[0].x = saved;
    HIP_TRY(e);
  } else {
    HIP_TRY(run_backward(st, buf, set, pos, lens, dy_dev, dx_dev, first != 0));
    st->slot_set[slot] = -1;
  }
  st->pending_set[st->n_pending++] = set;
  // the group is complete after wg_j passes, and at the batch's last pass whatever its size
  if (st->n_pending == st->wg_j || st->sched.accumulated() == st->cfg.m) HIP_TRY(flush_wgrad(st));
  if (st->two_streams) {
    HIP_TRY(hipEventRecord(st->bwd_done[slot], st->bstream));
    st->bwd_pending[slot] = 1;
  }
  return STAGE_OK;
}

int stage_coalesce_update(stage_t* st) {
  if (!st) return STAGE_ERR_INVALID_ARG;
  int rc = st->sched.check_update();
  if (rc != STAGE_OK) return rc;
  int rb = 0, wb = 0;
  int64_t step = 0;
  rc = st->sched.coalesce_update(&rb, &wb, &step);
  if (rc != STAGE_OK) return rc;
  st->cur = st->bstream;
  AdamDesc d;
  d.n = st->P; d.m = st->adam_m; d.v = st->adam_v; d.G = st->G;
  d.lr = st->cfg.lr; d.beta1 = st->cfg.beta1; d.beta2 = st->cfg.beta2; d.eps = st->cfg.adam_eps;
  d.inv_m = 1.0f / (float)st->cfg.m;
  d.c1 = (float)(1.0 / (1.0 - std::pow((double)st->cfg.beta1, (double)step)));
  d.c2 = (float)(1.0 / (1.0 - std::pow((double)st->cfg.beta2, (double)step)));
  double bytes;
  if (st->dtype == kBF16) {
    d.w_cur = st->master; d.w_next = st->master; d.w_next_lp = reinterpret_cast<bf16_t*>(st->wbuf[wb]);
    bytes = 30.0 * st->P;
  } else {
    d.w_cur = reinterpret_cast<const float*>(st->wbuf[rb]); d.w_next = reinterpret_cast<float*>(st->wbuf[wb]);
    bytes = 28.0 * st->P;
  }
  if (st->cfg.optimizer == STAGE_OPT_MOMENTUM) {
    bytes -= 8.0 * st->P;   // no second moment
    HIP_TRY(timed(st, STAGE_K_ADAM, "momentum_kernel", 0.0, bytes, [&] { return momentum_step(d, st->cur); }));
  } else {
    HIP_TRY(timed(st, STAGE_K_ADAM, "adam_kernel", 0.0, bytes, [&] { return adam_step(d, st->cur); }));
  }
  // the transposed copy of the version just written (the data-gradient products of its microbatches read it)
  if (st->dtype == kBF16) {
    const double tbytes = 4.0 * st->cfg.n_layers * (4.0 * st->cfg.hidden * st->cfg.hidden + 2.0 * st->cfg.hidden * st->cfg.ffn);
    HIP_TRY(timed(st, STAGE_K_OTHER, "transpose_bf16_grouped_kernel", 0.0, tbytes, [&] { return refresh_transposed(st, wb, st->cur); }));
  }
  if (st->two_streams) {
    HIP_TRY(hipEventRecord(st->ver_ready[wb], st->bstream));
    st->ver_pending[wb] = true;
  }
  return STAGE_OK;
}

int stage_set_backward_stream(stage_t* st, void* hip_stream) {
  if (!st) return STAGE_ERR_INVALID_ARG;
  if (st->sched.inflight() != 0 || st->sched.accumulated() != 0) return STAGE_ERR_BAD_STATE;
  HIP_TRY(sync_all(st));
  hipStream_t b = static_cast<hipStream_t>(hip_stream);
  if (b == st->stream) {   // back to one stream
    st->bstream = st->stream;
    st->two_streams = false;
    return STAGE_OK;
  }
  if (st->fwd_done.empty()) {
    std::vector<hipEvent_t> ev;
    const int n_sets = (int)st->sets.size();
    const int want = 2 * st->cfg.max_inflight + 2 + n_sets;
    for (int i = 0; i < want; ++i) {
      hipEvent_t e = nullptr;
      if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) {
        for (hipEvent_t x : ev) (void)hipEventDestroy(x);
        return STAGE_ERR_HIP;
      }
      ev.push_back(e);
    }
    st->fwd_done.assign(ev.begin(), ev.begin() + st->cfg.max_inflight);
    st->bwd_done.assign(ev.begin() + st->cfg.max_inflight, ev.begin() + 2 * st->cfg.max_inflight);
    st->ver_ready[0] = ev[2 * st->cfg.max_inflight];
    st->ver_ready[1] = ev[2 * st->cfg.max_inflight + 1];
    st->set_done.assign(ev.begin() + 2 * st->cfg.max_inflight + 2, ev.end());
    st->bwd_pending.assign(st->cfg.max_inflight, 0);
    st->set_pending.assign(n_sets, 0);
  }
  std::fill(st->bwd_pending.begin(), st->bwd_pending.end(), 0);
  std::fill(st->set_pending.begin(), st->set_pending.end(), 0);
  st->ver_pending[0] = st->ver_pending[1] = false;
  st->bstream = b;
  st->two_streams = true;
  return STAGE_OK;
}

int stage_swap_versions(stage_t* st) {
  if (!st) return STAGE_ERR_INVALID_ARG;
  return st->sched.swap_versions();
}

int stage_destroy(stage_t* st) {
  if (!st) return STAGE_ERR_INVALID_ARG;
  (void)sync_all(st);
  int rc = free_all(st);
  delete st;
  return rc;
}

static int read_f32(stage_t* st, const float* dev, float* host) {
  HIP_TRY(sync_all(st));
  HIP_TRY(hipMemcpy(host, dev, (size_t)st->P * 4, hipMemcpyDeviceToHost));
  return STAGE_OK;
}

int stage_read_weights(stage_t* st, int which, float* out_host) {
  if (!st || !out_host) return STAGE_ERR_INVALID_ARG;
  if (which == STAGE_WEIGHTS_MASTER) {
    if (st->dtype == kBF16) return read_f32(st, st->master, out_host);
    which = st->sched.buffer_of(st->sched.updates());
  }
  if (which != 0 && which != 1) return STAGE_ERR_INVALID_ARG;
  if (st->dtype == kF32) return read_f32(st, reinterpret_cast<const float*>(st->wbuf[which]), out_host);
  std::vector<uint16_t> tmp;
  try { tmp.resize((size_t)st->P); } catch (...) { return STAGE_ERR_OOM; }
  HIP_TRY(sync_all(st));
  HIP_TRY(hipMemcpy(tmp.data(), st->wbuf[which], (size_t)st->P * 2, hipMemcpyDeviceToHost));
  for (int64_t i = 0; i < st->P; ++i) {
    const uint32_t u = (uint32_t)tmp[i] << 16;
    std::memcpy(&out_host[i], &u, 4);
  }
  return STAGE_OK;
}

int stage_read_grad_accum(stage_t* st, float* out_host) {
  if (!st || !out_host) return STAGE_ERR_INVALID_ARG;
  // products still waiting for their group are launched first: the accumulator then holds every pass so far
  st->cur = st->bstream;
  HIP_TRY(flush_wgrad(st));
  return read_f32(st, st->G, out_host);
}

int stage_read_adam(stage_t* st, float* m_out_host, float* v_out_host) {
  if (!st) return STAGE_ERR_INVALID_ARG;
  if (m_out_host) { int rc = read_f32(st, st->adam_m, m_out_host); if (rc) return rc; }
  if (v_out_host) {
    if (!st->adam_v) return STAGE_ERR_INVALID_ARG;   // momentum SGD keeps no second moment
    int rc = read_f32(st, st->adam_v, v_out_host); if (rc) return rc;
  }
  return STAGE_OK;
}

int stage_query(stage_t* st, int what, int64_t* out) {
  if (!st || !out) return STAGE_ERR_INVALID_ARG;
  switch (what) {
    case STAGE_Q_UPDATES: *out = st->sched.updates(); break;
    case STAGE_Q_READ_VERSION: *out = st->sched.read_version(); break;
    case STAGE_Q_INFLIGHT: *out = st->sched.inflight(); break;
    case STAGE_Q_ACCUMULATED: *out = st->sched.accumulated(); break;
    case STAGE_Q_BYTES_ALLOCATED: *out = st->bytes_total; break;
    case STAGE_Q_BYTES_WEIGHTS: *out = st->bytes_weights; break;
    case STAGE_Q_BYTES_STASH: *out = st->bytes_stash; break;
    case STAGE_Q_BUFFER_OF_NEWEST: *out = st->sched.buffer_of(st->sched.updates()); break;
    case STAGE_Q_BUFFER_OF_READ: *out = st->sched.buffer_of(st->sched.read_version()); break;
    default: return STAGE_ERR_INVALID_ARG;
  }
  return STAGE_OK;
}

const char* stage_strerror(int code) {
  switch (code) {
    case STAGE_OK: return "ok";
    case STAGE_ERR_INVALID_ARG: return "invalid argument";
    case STAGE_ERR_BAD_STATE: return "call violates the 2BW schedule";
    case STAGE_ERR_OOM: return "out of memory";
    case STAGE_ERR_HIP: return "HIP runtime error";
    default: return "unknown error code";
  }
}

int stage_timing_enable(stage_t* st, int enable, int32_t capacity) {
  if (!st) return STAGE_ERR_INVALID_ARG;
  HIP_TRY(sync_all(st));
  for (EventPair& e : st->events) {
    (void)hipEventDestroy(e.start);
    (void)hipEventDestroy(e.stop);
  }
  st->events.clear();
  st->events_used = 0;
  st->timing = false;
  if (!enable) return STAGE_OK;
  if (capacity < 1) return STAGE_ERR_INVALID_ARG;
  try { st->events.reserve(capacity); } catch (...) { return STAGE_ERR_OOM; }
  for (int i = 0; i < capacity; ++i) {
    EventPair e{};
    if (hipEventCreate(&e.start) != hipSuccess) return STAGE_ERR_HIP;
    if (hipEventCreate(&e.stop) != hipSuccess) { (void)hipEventDestroy(e.start); return STAGE_ERR_HIP; }
    st->events.push_back(e);
  }
  st->timing = true;
  return STAGE_OK;
}

int stage_timing_collect_kernels(stage_t* st, int32_t capacity, char* names_out, double* ms_out,
                                 int64_t* launches_out, double* flops_out, double* bytes_out, int32_t* count_out) {
  if (!st || capacity < 1 || !names_out || !ms_out || !launches_out || !flops_out || !bytes_out || !count_out)
    return STAGE_ERR_INVALID_ARG;
  HIP_TRY(sync_all(st));
  int n = 0;
  for (size_t i = 0; i < st->events_used; ++i) {
    const EventPair& e = st->events[i];
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, e.start, e.stop));
    int k = 0;
    for (; k < n; ++k)
      if (std::strncmp(names_out + (size_t)k * 96, e.name, 96) == 0) break;
    if (k == n) {
      if (n == capacity) continue;   // more distinct kernels than the caller has room for
      std::snprintf(names_out + (size_t)k * 96, 96, "%s", e.name);
      ms_out[k] = 0; launches_out[k] = 0; flops_out[k] = 0; bytes_out[k] = 0;
      ++n;
    }
    ms_out[k] += ms; launches_out[k] += 1; flops_out[k] += e.flops; bytes_out[k] += e.bytes;
  }
  *count_out = n;
  return STAGE_OK;
}

int stage_timing_collect(stage_t* st, double* ms_out, int64_t* launches_out, double* flops_out, double* bytes_out) {
  if (!st || !ms_out || !launches_out || !flops_out || !bytes_out) return STAGE_ERR_INVALID_ARG;
  HIP_TRY(sync_all(st));
  for (int i = 0; i < STAGE_K_COUNT; ++i) { ms_out[i] = 0; launches_out[i] = 0; flops_out[i] = 0; bytes_out[i] = 0; }
  for (size_t i = 0; i < st->events_used; ++i) {
    const EventPair& e = st->events[i];
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, e.start, e.stop));
    ms_out[e.cls] += ms;
    launches_out[e.cls] += 1;
    flops_out[e.cls] += e.flops;
    bytes_out[e.cls] += e.bytes;
  }
  st->events_used = 0;
  return STAGE_OK;
}

// ---- the schedule alone -------------------------------------------------------------------

struct stage_sched {
  Schedule s;
  stage_sched(int m, int p, bool flush) : s(m, p, flush) {}
};

int stage_sched_create(int32_t m, int32_t max_inflight, int32_t flush, stage_sched_t** out) {
  if (!out || m < 1 || max_inflight < 1 || m < max_inflight || (flush != 0 && flush != 1)) return STAGE_ERR_INVALID_ARG;
  *out = new (std::nothrow) stage_sched(m, max_inflight, flush != 0);
  return *out ? STAGE_OK : STAGE_ERR_OOM;
}
int stage_sched_forward(stage_sched_t* s, int64_t mb, int32_t* slot_out, int64_t* version_out, int32_t* buffer_out) {
  if (!s || !slot_out || !version_out || !buffer_out) return STAGE_ERR_INVALID_ARG;
  int slot = 0, buf = 0;
  int64_t ver = 0;
  int rc = s->s.forward(mb, &slot, &ver, &buf);
  if (rc == STAGE_OK) { *slot_out = slot; *version_out = ver; *buffer_out = buf; }
  return rc;
}
int stage_sched_backward(stage_sched_t* s, int64_t mb, int32_t* slot_out, int64_t* version_out, int32_t* buffer_out,
                         int32_t* first_of_batch_out) {
  if (!s || !slot_out || !version_out || !buffer_out || !first_of_batch_out) return STAGE_ERR_INVALID_ARG;
  int slot = 0, buf = 0, first = 0;
  int64_t ver = 0;
  int rc = s->s.backward(mb, &slot, &ver, &buf, &first);
  if (rc == STAGE_OK) { *slot_out = slot; *version_out = ver; *buffer_out = buf; *first_of_batch_out = first; }
  return rc;
}
int stage_sched_coalesce_update(stage_sched_t* s, int32_t* read_buffer_out, int32_t* write_buffer_out,
                                int64_t* step_out) {
  if (!s || !read_buffer_out || !write_buffer_out || !step_out) return STAGE_ERR_INVALID_ARG;
  int rb = 0, wb = 0;
  int64_t step = 0;
  int rc = s->s.coalesce_update(&rb, &wb, &step);
  if (rc == STAGE_OK) { *read_buffer_out = rb; *write_buffer_out = wb; *step_out = step; }
  return rc;
}
int stage_sched_swap_versions(stage_sched_t* s) {
  if (!s) return STAGE_ERR_INVALID_ARG;
  return s->s.swap_versions();
}
int stage_sched_query(stage_sched_t* s, int what, int64_t* out) {
  if (!s || !out) return STAGE_ERR_INVALID_ARG;
  switch (what) {
    case STAGE_Q_UPDATES: *out = s->s.updates(); break;
    case STAGE_Q_READ_VERSION: *out = s->s.read_version(); break;
    case STAGE_Q_INFLIGHT: *out = s->s.inflight(); break;
    case STAGE_Q_ACCUMULATED: *out = s->s.accumulated(); break;
    case STAGE_Q_BUFFER_OF_NEWEST: *out = s->s.buffer_of(s->s.updates()); break;
    case STAGE_Q_BUFFER_OF_READ: *out = s->s.buffer_of(s->s.read_version()); break;
    default: return STAGE_ERR_INVALID_ARG;
  }
  return STAGE_OK;
}
int stage_sched_destroy(stage_sched_t* s) {
  if (!s) return STAGE_ERR_INVALID_ARG;
  delete s;
  return STAGE_OK;
}

}  // extern "C"
