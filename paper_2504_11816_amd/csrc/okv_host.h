// Host-side integer logic: the offload plan and the copy-pipeline scheduler.
// No GPU calls in this file; the runtime and the trace entry point both walk
// the scheduler below, so what tests replay is what the GPU is given.
#pragma once

#include <stdint.h>

#include <vector>

namespace okv {

// ---- offload plan (paper §IV-C, Case 3) -------------------------------------

// Smallest integer >= num * n_layers / den, in 128-bit integers so that byte
// counts can be used as num / den.
inline int32_t plan_count(int32_t n_layers, int64_t num, int64_t den) {
  __int128 x = (__int128)num * n_layers;
  return (int32_t)((x + den - 1) / den);
}

// Even spread: layer l goes to the host when the integer part of
// (l + 1) * n_off / n_layers exceeds that of l * n_off / n_layers.
inline void plan_place(int32_t n_layers, int32_t n_off, uint8_t *on_host) {
  for (int32_t l = 0; l < n_layers; ++l) {
    int64_t hi = ((int64_t)(l + 1) * n_off) / n_layers;
    int64_t lo = ((int64_t)l * n_off) / n_layers;
    on_host[l] = (uint8_t)(hi - lo);
  }
}

// ---- copy pipeline (paper §II-B: offloaded KV is fetched back before use) ----
//
// Host layers are consumed in layer order, step after step; the j-th consumption
// overall ("copy index" j) is of host layer hl[j % k] in step j / k and uses
// staging buffer j % depth, depth = min(n_staging, k).  Copy j may start once
// the consumer of copy j - depth has released the buffer; because depth <= k
// that consumer ran after the previous step's append to the same layer, so the
// host pool the copy reads is up to date.  Each release immediately enqueues
// copy j + depth, which keeps `depth` copies in flight, across step boundaries.

enum OpKind : int32_t { OP_COPY = 0, OP_APPEND = 1, OP_ATTN = 2, OP_RELEASE = 3 };

struct Op {
  int32_t kind, step, layer, buf, copy_idx, wait_idx;
};

class Scheduler {
 public:
  void reset(int32_t n_layers, const uint8_t *on_host, int32_t n_staging) {
    n_layers_ = n_layers;
    on_host_.assign(on_host, on_host + n_layers);
    host_layers_.clear();
    rank_.assign(n_layers, -1);
    for (int32_t l = 0; l < n_layers; ++l)
      if (on_host[l]) {
        rank_[l] = (int32_t)host_layers_.size();
        host_layers_.push_back(l);
      }
    k_ = (int32_t)host_layers_.size();
    depth_ = k_ < n_staging ? k_ : n_staging;
    primed_ = false;
  }

  int32_t depth() const { return depth_; }
  int32_t n_host() const { return k_; }
  bool is_host(int32_t layer) const { return on_host_[layer] != 0; }
  bool primed() const { return primed_; }

  // Copy index of (step, host layer).
  int64_t copy_index(int64_t step, int32_t layer) const { return step * k_ + rank_[layer]; }

  Op make_copy(int64_t j, int64_t wait) const {
    Op op;
    op.kind = OP_COPY;
    op.step = (int32_t)(j / k_);
    op.layer = host_layers_[j % k_];
    op.buf = (int32_t)(j % depth_);
    op.copy_idx = (int32_t)j;
    op.wait_idx = (int32_t)wait;
    return op;
  }

  // First copies, issued once before the first step of a batch.
  void prime(std::vector<Op> &out) {
    if (primed_) return;
    primed_ = true;
    for (int32_t j = 0; j < depth_; ++j) out.push_back(make_copy(j, -1));
  }

  void on_append(int64_t step, int32_t layer, std::vector<Op> &out) const {
    Op op{OP_APPEND, (int32_t)step, layer, -1, -1, -1};
    if (is_host(layer)) {
      int64_t j = copy_index(step, layer);
      op.buf = (int32_t)(j % depth_);
      op.wait_idx = (int32_t)j;
    }
    out.push_back(op);
  }

  void on_attn(int64_t step, int32_t layer, std::vector<Op> &out) const {
    Op op{OP_ATTN, (int32_t)step, layer, -1, -1, -1};
    if (!is_host(layer)) {
      out.push_back(op);
      return;
    }
    int64_t j = copy_index(step, layer);
    op.buf = (int32_t)(j % depth_);
    out.push_back(op);
    out.push_back(Op{OP_RELEASE, (int32_t)step, layer, op.buf, (int32_t)j, -1});
    out.push_back(make_copy(j + depth_, j));
  }

 private:
  int32_t n_layers_ = 0, k_ = 0, depth_ = 0;
  bool primed_ = false;
  std::vector<uint8_t> on_host_;
  std::vector<int32_t> host_layers_, rank_;
};

// ---- split-K work list ------------------------------------------------------
//
// Sequence b with n_b keys is cut into items of equal size: with split size S it gets
// c0 = ceil(n_b / S) pieces of ceil(n_b / c0) keys, the piece size rounded up to a
// multiple of 16 (so that items start on tile boundaries), which leaves
// count = ceil(n_b / size) items.  Equal pieces matter when the launch is a single
// round of wavefronts: the longest item sets the time.  chunk_prefix[b] = number of
// items of sequences 0 .. b-1; chunk c of sequence b is item chunk_prefix[b] + c and
// covers keys [c * size_b, min((c + 1) * size_b, n_b)).  The same arithmetic runs on
// the host (item count, checks) and in the kernel that builds the item list.
struct ItemRange {
  int32_t b, lo, hi;
};

__host__ __device__ inline void seq_chunks(int32_t n, int32_t S, int32_t *count, int32_t *size) {
  if (n <= 0) {
    *count = 0;
    *size = 16;
    return;
  }
  const int32_t c0 = (n + S - 1) / S;
  const int32_t sz = (((n + c0 - 1) / c0) + 15) & ~15;
  *size = sz;
  *count = (n + sz - 1) / sz;
}

// Chunk c of sequence b with n keys and chunk size sz.
__host__ __device__ inline ItemRange chunk_range(int32_t b, int32_t c, int32_t sz, int32_t n) {
  ItemRange r;
  r.b = b;
  r.lo = c * sz;
  r.hi = r.lo + sz < n ? r.lo + sz : n;
  return r;
}

}  // namespace okv
