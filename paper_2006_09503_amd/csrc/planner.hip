// The planner of Section 3.4 / appendix: closed-form cost functions and the exhaustive sweep over
// pipeline width and depth.  Host code only (it lives in the library so that one C ABI covers the
// stage and the choice of its shape).
#include <algorithm>
#include <cmath>

#include "../../include/planner2bw.h"

namespace {

constexpr int kOk = 0, kInvalid = -1, kNoFit = -2;

bool valid(const planner_input_t* in) {
  if (!in || in->n_blocks < 1 || in->n_gpus < 1 || in->gpus_per_server < 1 || in->n_sizes < 1) return false;
  if (!in->microbatch_sizes || !in->block_time_s) return false;
  for (int i = 0; i < in->n_sizes; ++i) {
    if (in->microbatch_sizes[i] < 1 || !(in->block_time_s[i] > 0.0)) return false;
    if (i > 0 && in->microbatch_sizes[i] <= in->microbatch_sizes[i - 1]) return false;
  }
  return in->weight_bytes >= 0 && in->state_bytes >= 0 && in->act_bytes_per_sample >= 0 &&
         in->input_bytes_per_sample >= 0 && in->boundary_bytes_per_sample >= 0 && in->bw_high > 0 &&
         in->bw_low > 0 && in->memory_capacity > 0 && in->global_batch >= 1 && in->c_extra >= 1.0;
}

int size_index(const planner_input_t* in, int b) {
  for (int i = 0; i < in->n_sizes; ++i)
    if (in->microbatch_sizes[i] == b) return i;
  return -1;
}

bool config_ok(const planner_input_t* in, int w, int d, int mode) {
  return w >= 1 && d >= 1 && (int64_t)w * d <= in->n_gpus && in->n_blocks % d == 0 &&
         mode >= PLANNER_MODE_NO_PIPELINE && mode <= PLANNER_MODE_PIPELINE_RECOMPUTE;
}

// seconds per microbatch of size b for one orientation of the pipelines over the servers
double time_per_microbatch(const planner_input_t* in, int w, int d, int bi, int mode, double bw_depth, double bw_width) {
  const double b = in->microbatch_sizes[bi];
  double comp = (double)(in->n_blocks / d) * in->block_time_s[bi];
  if (mode == PLANNER_MODE_PIPELINE_RECOMPUTE) comp *= in->c_extra;
  const double stage_comm = d > 1 ? 2.0 * in->boundary_bytes_per_sample * b / bw_depth : 0.0;
  const double m_b = (double)in->global_batch / ((double)w * b);
  const double allreduce = w > 1 ? 2.0 * (w - 1) / w * (in->weight_bytes / d) / bw_width : 0.0;
  const double per_stage = std::max(comp + stage_comm, allreduce / m_b);
  // the stages are equal: the sum over stages without pipelining is d times, the maximum with it once
  return mode == PLANNER_MODE_NO_PIPELINE ? d * per_stage : per_stage;
}

double throughput(const planner_input_t* in, int w, int d, int bi, int mode) {
  const int gps = in->gpus_per_server;
  auto bw = [&](int64_t group) { return group <= gps ? in->bw_high : in->bw_low; };
  // replicas of a stage inside a server, or the stages of a pipeline inside a server
  const double t_a = time_per_microbatch(in, w, d, bi, mode, bw((int64_t)w * d), bw(w));
  const double t_b = time_per_microbatch(in, w, d, bi, mode, bw(d), bw((int64_t)w * d));
  return (double)w * in->microbatch_sizes[bi] / std::min(t_a, t_b);
}

double memory(const planner_input_t* in, int d, int bi, int mode) {
  const double b = in->microbatch_sizes[bi];
  const double a_total = in->act_bytes_per_sample * b, a_in = in->input_bytes_per_sample * b;
  const double state = in->state_bytes / d;
  switch (mode) {
    case PLANNER_MODE_NO_PIPELINE: return in->weight_bytes / d + a_total / d + state;
    case PLANNER_MODE_PIPELINE: return 2.0 * in->weight_bytes / d + a_total + d * a_in + state;
    default: return 2.0 * in->weight_bytes / d + a_total / d + d * a_in + state;
  }
}

int search(const planner_input_t* in, int w, int d, planner_choice_t* out) {
  bool found = false;
  for (int bi = 0; bi < in->n_sizes; ++bi) {
    // g = B / (w d b) (partitioning algorithm, last line; Section 5.2: batch size b w d g, m = d g) must be
    // a whole number >= 1, which also gives m >= d (Section 3.1)
    const int64_t wdb = (int64_t)w * d * in->microbatch_sizes[bi];
    if (in->global_batch % wdb) continue;
    for (int mode = PLANNER_MODE_NO_PIPELINE; mode <= PLANNER_MODE_PIPELINE_RECOMPUTE; ++mode) {
      const double mem = memory(in, d, bi, mode);
      if (mem > in->memory_capacity) continue;
      const double thr = throughput(in, w, d, bi, mode);
      if (!found || thr > out->throughput) {
        found = true;
        *out = planner_choice_t{w, d, in->microbatch_sizes[bi], mode, in->global_batch / wdb, thr, mem};
      }
    }
  }
  return found ? kOk : kNoFit;
}

}  // namespace

extern "C" {

int planner_throughput(const planner_input_t* in, int32_t w, int32_t d, int32_t b, int32_t mode, double* out) {
  if (!valid(in) || !out || !config_ok(in, w, d, mode)) return kInvalid;
  const int bi = size_index(in, b);
  if (bi < 0 || (int64_t)w * b > in->global_batch) return kInvalid;
  *out = throughput(in, w, d, bi, mode);
  return kOk;
}

int planner_memory(const planner_input_t* in, int32_t w, int32_t d, int32_t b, int32_t mode, double* out) {
  if (!valid(in) || !out || !config_ok(in, w, d, mode)) return kInvalid;
  const int bi = size_index(in, b);
  if (bi < 0) return kInvalid;
  *out = memory(in, d, bi, mode);
  return kOk;
}

int planner_search(const planner_input_t* in, int32_t w, int32_t d, planner_choice_t* out) {
  if (!valid(in) || !out || !config_ok(in, w, d, PLANNER_MODE_PIPELINE)) return kInvalid;
  return search(in, w, d, out);
}

int planner_partition(const planner_input_t* in, planner_choice_t* out) {
  if (!valid(in) || !out) return kInvalid;
  bool found = false;
  planner_choice_t best{};
  for (int w = 1; w <= in->n_gpus; ++w)
    for (int d = 1; d <= in->n_gpus / w; ++d) {
      if (in->n_blocks % d) continue;
      planner_choice_t c{};
      if (search(in, w, d, &c) != kOk) continue;
      if (!found || c.throughput > best.throughput) { found = true; best = c; }
    }
  if (!found) return kNoFit;
  *out = best;
  return kOk;
}

}  // extern "C"
