/*
 * stage2bw.h -- C ABI of one PipeDream-2BW pipeline stage on one MI355X (gfx950).
 *
 * One stage is a stack of pre-LayerNorm transformer blocks.  The library keeps the stage's
 * two weight versions, the coalesced weight-gradient accumulator, one copy of Adam state and
 * the activation stashes of the in-flight microbatches, and runs the stage's share of the
 * 2BW schedule (Section 3.1 of the paper):
 *
 *   - microbatch k (1-indexed) runs forward and backward on weight version
 *     max(floor((k-1)/m) - 1, 0)                                        (Section 3.1);
 *   - weight gradients of the m microbatches of a batch are summed in place into one
 *     accumulator and averaged over m at the update                    (Section 3.1);
 *   - the update computes W(t+1) = W(t) - nu * step(grad f(W(t-1))) with Adam moments built
 *     from that 1-stale gradient, and writes W(t+1) into the buffer that held the dead
 *     version W(t-1); no second copy of optimizer state               (Section 3.1, Semantics);
 *   - with activation recomputation only the stage input is stashed and the forward is
 *     re-run, on the stashed version, inside the backward               (Section 4.1);
 *   - in flush mode (Section 3.2) the stage keeps ONE weight version: microbatch k runs on
 *     version floor((k-1)/m), so batch t+1 cannot start before update t (the pipeline is
 *     drained at every batch end), and the update is the vanilla W(t+1) = W(t) - nu *
 *     step(grad f(W(t))) in place.
 *
 * All pointers named *_dev are device pointers owned by the caller, *_host are host pointers
 * owned by the caller.  Everything else is owned by the library and freed by stage_destroy.
 * The five hot calls only enqueue work on the stream given to stage_create and return; the
 * stage_read_* calls synchronise that stream.  Calls on one stage must not overlap, and calls on
 * different stages from several host threads must be serialised by the caller: the library sets
 * up process-wide state on first use (kernel attributes, the device's CU count) without locks.
 *
 * Every function returns STAGE_OK (0) or a negative error code.  A call that returns an
 * error has enqueued nothing and changed no state.
 */
#ifndef STAGE2BW_H
#define STAGE2BW_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  STAGE_OK = 0,
  STAGE_ERR_INVALID_ARG = -1, /* NULL pointer, bad dimension, unsupported shape            */
  STAGE_ERR_BAD_STATE = -2,   /* the call would violate the 2BW schedule (see each call)   */
  STAGE_ERR_OOM = -3,         /* device or host allocation failed                          */
  STAGE_ERR_HIP = -4          /* a HIP runtime call or a kernel launch failed              */
};

enum { STAGE_MASK_NONE = 0, STAGE_MASK_CAUSAL = 1, STAGE_MASK_PADDING = 2 };
enum { STAGE_PREC_FP32 = 0, STAGE_PREC_BF16 = 1 };
enum { STAGE_OPT_ADAM = 0, STAGE_OPT_MOMENTUM = 1 };

typedef struct stage2bw stage_t; /* opaque */

typedef struct {
  int32_t n_layers;     /* L >= 1                                                           */
  int32_t hidden;       /* h, multiple of 8 and of n_heads                                  */
  int32_t n_heads;      /* a; head size h/a must be a multiple of 8, at most 128            */
  int32_t ffn;          /* f, multiple of 8                                                 */
  int32_t seq;          /* s                                                                */
  int32_t microbatch;   /* b sequences per microbatch; tokens T = b*s                       */
                        /* T <= 2^24; T*max(f, 3h) and h*f below 2^30 elements (the kernels  */
                        /* address an operand with 32-bit byte offsets); h <= 16384          */
  int32_t m;            /* microbatches per coalesced update; m >= max_inflight (Sec. 3.1:  */
                        /* a new version every m >= d microbatches)                         */
  int32_t max_inflight; /* activation stash slots = microbatches in flight at this stage    */
  int32_t mask_mode;    /* STAGE_MASK_*; causal: key j visible to query i iff j <= i;       */
                        /* padding: key j of sequence n visible iff j < seqlens[n]          */
  int32_t precision;    /* STAGE_PREC_FP32: everything fp32, the two weight buffers are the */
                        /* versions.  STAGE_PREC_BF16: two bf16 weight buffers, one fp32    */
                        /* master copy, bf16 activations, fp32 accumulation/statistics      */
  int32_t recompute;    /* 0: stash every saved activation; 1: stash the stage input only   */
  float lr, beta1, beta2, adam_eps; /* Adam with bias correction, eps outside the root      */
  float ln_eps;                     /* added to the biased variance under the root           */
  int32_t flush;        /* 0: 2BW (two versions, Section 3.1); 1: one version with a pipeline    */
                        /* flush per batch (Section 3.2)                                      */
  int32_t optimizer;    /* STAGE_OPT_ADAM, or STAGE_OPT_MOMENTUM: m <- beta1 m + (1-beta1) g,    */
                        /* W(t+1) = W(t) - lr m, the form Section 3.1 prints (beta2, adam_eps    */
                        /* unused; the second-moment array is not allocated)                  */
  int32_t wgrad_group;  /* backward passes whose weight-gradient products share one launch with the  */
                        /* reduction range j*T (the accumulator of Section 3.1 is then read and       */
                        /* written once per j microbatches; a group never crosses a batch end, so the */
                        /* coalesced sum is the same up to the order of fp32 additions).  0: the      */
                        /* library's choice (4; 8 if b*s <= 2048); 1..8: at most this many.  Always 1  */
                        /* in fp32 mode and when b*s is not a multiple of 64.  Each unit above 1 keeps */
                        /* one more set of activations alive (with recompute: one more scratch set)    */
} stage_config_t;

/*
 * Flat parameter vector (init_weights_host, stage_read_*): per layer, in order,
 *   ln1.gain[h] ln1.shift[h] Wqkv[h,3h] bqkv[3h] Wo[h,h] bo[h]
 *   ln2.gain[h] ln2.shift[h] W1[h,f] b1[f] W2[f,h] b2[h]
 * matrices row-major [in,out] (y = x W + b); Wqkv columns are Q|K|V, each head-major.
 * Length P = L*(4h^2 + 2hf + 9h + f).
 */

/* Number of parameters P for a configuration, or a negative error code. */
int64_t stage_param_count(const stage_config_t* cfg);

/*
 * Build a stage.  init_weights_host: P floats; both weight versions start as W(0)
 * (the version rule's max(.,0) makes batches 0 and 1 both run on W(0), Section 3.1).
 * hip_stream: a hipStream_t (NULL = the null stream) on the current device; it must outlive
 * the stage.  Errors: INVALID_ARG, OOM, HIP.
 */
int stage_create(const stage_config_t* cfg, const float* init_weights_host, void* hip_stream,
                 stage_t** out);

/*
 * Forward pass of microbatch mb (1-indexed, global count) on the version the rule assigns it
 * (Section 3.1).  x_dev, y_dev: [b, s, h] contiguous, bf16 in bf16 mode, fp32 in fp32 mode
 * (y_dev may not alias x_dev).  seqlens_dev: b int32 key lengths in [1, s] (values outside are
 * clamped into that range by the kernels) for STAGE_MASK_PADDING, ignored (may be NULL) otherwise.  The microbatch becomes in flight: its
 * activations (or just x, with recompute) are stashed with the version tag.
 * BAD_STATE if mb is already in flight, if no stash slot is free, or if the version the rule
 * assigns to mb is not the one new forwards currently read (call stage_swap_versions first,
 * or the needed version has not been generated yet; in flush mode: the update of the previous
 * batch has not been applied yet).
 */
int stage_forward(stage_t* st, int64_t mb, const void* x_dev, const int32_t* seqlens_dev,
                  void* y_dev);

/*
 * Backward pass of in-flight microbatch mb on the version tagged at its forward
 * (Section 3.1: same version for both passes).  dy_dev: gradient wrt the stage output,
 * dx_dev: receives the gradient wrt the stage input, both [b, s, h], dtype as in forward.
 * Weight gradients are added in place into the coalesced accumulator (the first backward of a
 * batch overwrites it), at the latest when the batch's last backward pass is enqueued (see
 * wgrad_group).  Frees the stash slot.  BAD_STATE if mb is not in flight or m
 * backward passes are already waiting for stage_coalesce_update.
 */
int stage_backward(stage_t* st, int64_t mb, const void* dy_dev, void* dx_dev);

/*
 * Apply the coalesced gradient of the batch just completed: g = G/m, Adam moments, and
 * W(t+1) = W(t) - lr * mhat/(sqrt(vhat) + eps) written into the other weight buffer
 * (Section 3.1, Semantics; Adam "similarly" to the printed momentum form).  t counts updates.
 * BAD_STATE unless exactly m backward passes have run since the last update, or if an
 * in-flight microbatch still reads the buffer about to be overwritten.
 */
int stage_coalesce_update(stage_t* st);

/*
 * Make the next-newer weight version the one new forward passes read; the version they read
 * so far stays available to microbatches already in flight until their backward passes are
 * done (the "shadow" version of Section 1).  BAD_STATE if no newer version exists (always, in
 * flush mode: there the update itself makes the new version current).
 */
int stage_swap_versions(stage_t* st);

/*
 * Run backward passes and updates on a stream of their own, so that in 1F1B steady state
 * (Section 3.1, Figure 2: a stage alternates forward and backward passes of different
 * microbatches) the two passes overlap on the GPU instead of taking turns.  After this call
 * stage_backward and stage_coalesce_update enqueue on hip_stream, stage_forward stays on the
 * stream given to stage_create.  The stage orders its own state across the two streams: a
 * backward pass after the forward pass of its microbatch, the reuse of a stash slot after the
 * backward pass that read it, a forward pass after the update that wrote the version it
 * reads.  The caller orders its own buffers: dy_dev must be complete on hip_stream when
 * stage_backward is called, dx_dev is complete there; x_dev / y_dev likewise on the forward
 * stream.  Results are the same as with one stream.  hip_stream equal to the creation stream
 * returns to one stream.  With recompute this allocates one more activation set (the forward
 * pass needs scratch of its own).  BAD_STATE while microbatches are in flight or gradients
 * wait for an update; the call synchronises both streams.  Errors: INVALID_ARG, BAD_STATE, OOM,
 * HIP.
 */
int stage_set_backward_stream(stage_t* st, void* hip_stream);

int stage_destroy(stage_t* st);

/* ---- inspection, for parity tests; each synchronises the stage's streams ---------------- */

enum { STAGE_WEIGHTS_BUF0 = 0, STAGE_WEIGHTS_BUF1 = 1, STAGE_WEIGHTS_MASTER = 2 };
/* which: one of the two version buffers (converted to fp32), or the fp32 master (in fp32 mode
 * the master is the buffer holding W(t)).  out_host: P floats. */
int stage_read_weights(stage_t* st, int which, float* out_host);
/* The coalesced accumulator (sum over the backward passes since the last update); weight-gradient
 * products still waiting for their group (wgrad_group) are launched first. */
int stage_read_grad_accum(stage_t* st, float* out_host);
/* Adam first and second moments (momentum SGD: its one moment; v_out_host must then be NULL);
 * either pointer may be NULL. */
int stage_read_adam(stage_t* st, float* m_out_host, float* v_out_host);

enum {
  STAGE_Q_UPDATES = 0,        /* t: updates applied                                        */
  STAGE_Q_READ_VERSION = 1,   /* r: version new forwards read                              */
  STAGE_Q_INFLIGHT = 2,       /* microbatches in flight                                    */
  STAGE_Q_ACCUMULATED = 3,    /* backward passes since the last update                     */
  STAGE_Q_BYTES_ALLOCATED = 4,/* device bytes owned by the stage                           */
  STAGE_Q_BYTES_WEIGHTS = 5,  /* of which: both weight versions (+ master)                 */
  STAGE_Q_BYTES_STASH = 6,    /* of which: activation stashes                              */
  STAGE_Q_BUFFER_OF_NEWEST = 7,  /* index (0/1) of the buffer holding W(t)                  */
  STAGE_Q_BUFFER_OF_READ = 8     /* index (0/1) of the buffer new forwards read             */
};
int stage_query(stage_t* st, int what, int64_t* out);

const char* stage_strerror(int code);

/* ---- per-kernel-class timing (HIP events on the stage's stream) -------------------------- */

enum {
  STAGE_K_GEMM_FWD = 0, STAGE_K_GEMM_DGRAD = 1, STAGE_K_GEMM_WGRAD = 2,
  STAGE_K_ATTN_FWD = 3, STAGE_K_ATTN_BWD = 4, STAGE_K_LN_FWD = 5, STAGE_K_LN_BWD = 6,
  STAGE_K_BIAS_GRAD = 7, STAGE_K_ADAM = 8, STAGE_K_OTHER = 9, STAGE_K_COUNT = 10
};
/* enable != 0: bracket every kernel launch with events from a pool of `capacity` pairs
 * (launches beyond the pool are not timed).  enable == 0: stop and free the pool. */
int stage_timing_enable(stage_t* st, int enable, int32_t capacity);
/* Synchronise, then add up elapsed milliseconds and launch counts per class since the last
 * call, and the FLOPs / bytes the launches were issued for.  Arrays of STAGE_K_COUNT. */
int stage_timing_collect(stage_t* st, double* ms_out, int64_t* launches_out, double* flops_out,
                         double* bytes_out);

/* The same events grouped by kernel instance (name as a kernel trace prints it, 96 bytes per
 * entry in names_out, which must hold capacity*96 bytes).  Does not reset the events: call it
 * before stage_timing_collect.  count_out receives the number of entries filled. */
int stage_timing_collect_kernels(stage_t* st, int32_t capacity, char* names_out, double* ms_out,
                                 int64_t* launches_out, double* flops_out, double* bytes_out,
                                 int32_t* count_out);

/* ---- the schedule alone (host only, no device needed) ------------------------------------ */
/*
 * The state machine the stage calls use, exposed so that the 2BW bookkeeping can be checked
 * without a GPU.  Same preconditions and error codes as the stage calls.
 */
typedef struct stage_sched stage_sched_t;
int stage_sched_create(int32_t m, int32_t max_inflight, int32_t flush, stage_sched_t** out);
/* slot_out: stash slot taken; version_out: version tag; buffer_out: weight buffer to read. */
int stage_sched_forward(stage_sched_t* s, int64_t mb, int32_t* slot_out, int64_t* version_out,
                        int32_t* buffer_out);
/* first_of_batch_out: 1 if this backward must overwrite the accumulator instead of adding. */
int stage_sched_backward(stage_sched_t* s, int64_t mb, int32_t* slot_out, int64_t* version_out,
                         int32_t* buffer_out, int32_t* first_of_batch_out);
/* read_buffer_out holds W(t); write_buffer_out receives W(t+1); step_out = t+1. */
int stage_sched_coalesce_update(stage_sched_t* s, int32_t* read_buffer_out,
                                int32_t* write_buffer_out, int64_t* step_out);
int stage_sched_swap_versions(stage_sched_t* s);
int stage_sched_query(stage_sched_t* s, int what, int64_t* out); /* STAGE_Q_* 0..3, 7, 8 */
int stage_sched_destroy(stage_sched_t* s);

#ifdef __cplusplus
}
#endif
#endif /* STAGE2BW_H */
