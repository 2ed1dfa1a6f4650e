// Host-side bookkeeping of the 2BW schedule at one stage (Section 3.1 of the paper).
//
// Versions are numbered by the update that produced them (version 0 = initial weights).
// Version v lives in weight buffer v % 2; both buffers start as version 0, which is what the
// rule's max(., 0) asks for (batches 0 and 1 both run on the initial weights).
//
//   t  updates applied = id of the newest version
//   r  version new forward passes read (r <= t)
//
// At most two versions are alive: t and t-1.  Update t -> t+1 reads buffer t % 2 and writes
// buffer (t+1) % 2, which held t-1; it is refused while an in-flight microbatch is tagged
// t-1.
//
// Flush variant (Section 3.2): one weight version.  Microbatch k runs on version floor((k-1)/m),
// i.e. no forward pass of batch t+1 is admitted before update t has been applied (the pipeline
// is drained at every batch end), the update reads and writes the one buffer, and new forward
// passes read the newest version at once (no swap).
// Pure host code: no device calls here.
#pragma once
#include <cstdint>
#include <vector>

namespace s2bw {

enum : int { kOk = 0, kInvalidArg = -1, kBadState = -2, kOom = -3, kHip = -4 };

class Schedule {
 public:
  struct Slot {
    int64_t mb = 0;       // 0 = free
    int64_t version = 0;  // tag taken at the forward pass
  };

  Schedule(int m, int max_inflight, bool flush = false) : m_(m), flush_(flush), slots_(max_inflight) {}

  static int64_t version_rule(int64_t k, int64_t m) {
    int64_t v = (k - 1) / m - 1;
    return v > 0 ? v : 0;
  }
  static int64_t version_rule_flush(int64_t k, int64_t m) { return (k - 1) / m; }
  int64_t rule(int64_t k) const { return flush_ ? version_rule_flush(k, m_) : version_rule(k, m_); }
  int buffer_of(int64_t version) const { return flush_ ? 0 : static_cast<int>(version & 1); }
  bool flush() const { return flush_; }

  // Checks only; no state change.  slot: the free slot forward would take.
  int check_forward(int64_t mb, int* slot) const {
    if (mb < 1) return kInvalidArg;
    if (rule(mb) != r_) return kBadState;              // needs a swap, or runs ahead of the updates
    if (r_ + 1 < t_) return kBadState;                 // version r is dead (buffer overwritten)
    int free_slot = -1;
    for (size_t i = 0; i < slots_.size(); ++i) {
      if (slots_[i].mb == mb) return kBadState;        // already in flight
      if (slots_[i].mb == 0 && free_slot < 0) free_slot = static_cast<int>(i);
    }
    if (free_slot < 0) return kBadState;               // more in flight than stash slots
    *slot = free_slot;
    return kOk;
  }
  int forward(int64_t mb, int* slot, int64_t* version, int* buffer) {
    int s = -1;
    int rc = check_forward(mb, &s);
    if (rc != kOk) return rc;
    slots_[s].mb = mb;
    slots_[s].version = r_;
    *slot = s;
    *version = r_;
    *buffer = buffer_of(r_);
    return kOk;
  }

  int check_backward(int64_t mb, int* slot) const {
    if (mb < 1) return kInvalidArg;
    int found = -1;
    for (size_t i = 0; i < slots_.size(); ++i)
      if (slots_[i].mb == mb) found = static_cast<int>(i);
    if (found < 0) return kBadState;                   // not in flight
    if (n_acc_ >= m_) return kBadState;                // a full batch awaits its update
    if ((mb - 1) / m_ != t_) return kBadState;         // belongs to another batch than the one coalescing
    *slot = found;
    return kOk;
  }
  int backward(int64_t mb, int* slot, int64_t* version, int* buffer, int* first_of_batch) {
    int s = -1;
    int rc = check_backward(mb, &s);
    if (rc != kOk) return rc;
    *slot = s;
    *version = slots_[s].version;
    *buffer = buffer_of(slots_[s].version);
    *first_of_batch = (n_acc_ == 0);
    slots_[s].mb = 0;
    ++n_acc_;
    return kOk;
  }

  int check_update() const {
    if (n_acc_ != m_) return kBadState;
    if (t_ >= 1)
      for (const Slot& s : slots_)
        if (s.mb != 0 && s.version == t_ - 1) return kBadState;  // its buffer is about to be overwritten
    return kOk;
  }
  int coalesce_update(int* read_buffer, int* write_buffer, int64_t* step) {
    int rc = check_update();
    if (rc != kOk) return rc;
    *read_buffer = buffer_of(t_);
    *write_buffer = buffer_of(t_ + 1);
    ++t_;
    if (flush_) r_ = t_;
    *step = t_;
    n_acc_ = 0;
    return kOk;
  }

  int swap_versions() {
    if (r_ >= t_) return kBadState;                    // nothing newer has been generated
    ++r_;
    return kOk;
  }

  int64_t updates() const { return t_; }
  int64_t read_version() const { return r_; }
  int accumulated() const { return n_acc_; }
  int inflight() const {
    int n = 0;
    for (const Slot& s : slots_) n += (s.mb != 0);
    return n;
  }
  int m() const { return m_; }
  int n_slots() const { return static_cast<int>(slots_.size()); }

 private:
  int m_;
  bool flush_;
  std::vector<Slot> slots_;
  int64_t t_ = 0;
  int64_t r_ = 0;
  int n_acc_ = 0;
};

}  // namespace s2bw
