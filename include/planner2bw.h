/*
 * planner2bw.h -- C ABI of the PipeDream-2BW planner (Section 3.4 and the appendix "Planner,
 * Additional Details": closed-form THROUGHPUT and MEMORY cost functions and the partitioning
 * algorithm).  Host only: no device is touched.
 *
 * The model is a chain of n_blocks identical blocks (transformer layers).  A configuration is a
 * pipeline of d equal stages (d divides n_blocks) replicated w times (w * d <= n_gpus), a per-GPU
 * microbatch size b and an execution mode.  Readings of the appendix taken here:
 *   - T_comp of a stage = (n_blocks / d) * block_time(b); with recomputation it is multiplied by
 *     c_extra (4/3 in the paper);
 *   - every stage pays 2 * boundary_bytes(b) / bw_depth of activation / gradient traffic when
 *     d > 1, and (2 (w-1)/w) * weight_bytes/d / bw_width of all-reduce traffic every
 *     m(b) = B / (w b) microbatches when w > 1;
 *   - a group of GPUs talks at bw_high when it fits inside one server (size <= gpus_per_server),
 *     at bw_low otherwise.  This departs from the appendix's printed case expression, which is
 *     strict (w < number of GPUs in a server): a group that fills a server exactly still stays
 *     inside it.  The pipelines are oriented whichever way (replicas of a stage inside a
 *     server, or the stages of a pipeline inside a server) gives the higher throughput;
 *   - the throughput returned is that of the whole job, w * b / t samples per second;
 *   - degree of gradient accumulation g = B / (w d b): the partitioning algorithm's last line
 *     prints B / (N b), N being all GPUs, and Section 5.2 gives the batch size as b w d g with
 *     m = d g microbatches averaged per update; a (w, d, b) is admissible iff g is a whole number
 *     >= 1, so that m = d g >= d as Section 3.1 requires for two weight versions;
 *   - MEMORY: pipelined: 2|W|/d + A_total(b) + d*A_input(b); pipelined with recomputation:
 *     2|W|/d + A_total(b)/d + d*A_input(b); without pipelining one weight version and one
 *     activation set: |W|/d + A_total(b)/d.  state_bytes/d (optimizer state, master copies) is
 *     added to each; the paper's formulas are the case state_bytes = 0.
 *
 * Every function returns 0 or a negative error code (-1: invalid argument, -2: no configuration
 * fits).
 */
#ifndef PLANNER2BW_H
#define PLANNER2BW_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { PLANNER_MODE_NO_PIPELINE = 0, PLANNER_MODE_PIPELINE = 1, PLANNER_MODE_PIPELINE_RECOMPUTE = 2 };

typedef struct {
  int32_t n_blocks;               /* blocks in the whole model                                   */
  int32_t n_gpus;                 /* N                                                            */
  int32_t gpus_per_server;
  int32_t n_sizes;                /* candidate per-GPU microbatch sizes                           */
  const int32_t* microbatch_sizes;/* host, ascending, each >= 1                                   */
  const double* block_time_s;     /* host, per candidate: forward + backward seconds of one block */
  double weight_bytes;            /* |W|, one version of all parameters                           */
  double state_bytes;             /* optimizer state + master copies of the whole model (0: paper)*/
  double act_bytes_per_sample;    /* |A_total(1)|: saved activations of the whole model           */
  double input_bytes_per_sample;  /* |A_input(1)|: input activations of one stage                 */
  double boundary_bytes_per_sample; /* |A_inp+out(1)|: a block's input plus output activations    */
  double bw_high, bw_low;         /* bytes/s inside a server / between servers                    */
  double memory_capacity;         /* M, bytes per GPU                                             */
  int64_t global_batch;           /* B, the maximum safe global batch size                        */
  double c_extra;                 /* compute multiplier of recomputation (paper: 4/3)             */
} planner_input_t;

typedef struct {
  int32_t w, d, b, mode;
  int64_t g;                      /* degree of gradient accumulation B / (w d b); m = d * g       */
  double throughput;              /* samples/s of the whole job                                   */
  double memory;                  /* bytes per GPU                                                */
} planner_choice_t;

/* THROUGHPUT(w, d, b, mode) in samples/s; b must be one of the candidates. */
int planner_throughput(const planner_input_t* in, int32_t w, int32_t d, int32_t b, int32_t mode, double* out);
/* MEMORY(w, d, b, mode) in bytes per GPU. */
int planner_memory(const planner_input_t* in, int32_t w, int32_t d, int32_t b, int32_t mode, double* out);
/* SEARCH(w, d, B): the candidate b (with w*d*b dividing B) and mode of highest throughput that fit in
 * memory_capacity; -2 if none fits. */
int planner_search(const planner_input_t* in, int32_t w, int32_t d, planner_choice_t* out);
/* The partitioning algorithm: sweep of all (w, d) with w*d <= n_gpus and d dividing n_blocks. */
int planner_partition(const planner_input_t* in, planner_choice_t* out);

#ifdef __cplusplus
}
#endif
#endif /* PLANNER2BW_H */
