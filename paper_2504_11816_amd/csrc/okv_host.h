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
// The streamed unit is a chunk of a layer's host pool: the whole pool when whole layers
// are offloaded (one chunk per host layer), a run of consecutive blocks when a share of
// every layer's blocks is.  Chunks are consumed layer by layer, chunk by chunk, step
// after step; the j-th consumption overall ("copy index" j) is of unit j % k (k units per
// step) in step j / k and uses staging buffer j % depth, depth = min(n_staging, k).  Copy
// j may start once the consumer of copy j - depth has released the buffer; because
// depth <= k that consumer is no earlier than the previous step's attention over the same
// chunk, which is the launch that stored new rows into that chunk of the host pool, so
// what the copy reads is up to date.  Each release immediately enqueues copy j + depth,
// which keeps `depth` copies in flight, across step boundaries.

enum OpKind : int32_t { OP_COPY = 0, OP_APPEND = 1, OP_ATTN = 2, OP_RELEASE = 3, OP_MERGE = 4 };

struct Op {
  int32_t kind, step, layer, chunk, buf;   // chunk = -1, buf = -1: the keys that stay in HBM
  int64_t copy_idx, wait_idx;
};

class Scheduler {
 public:
  // host_chunks[l]: streamed chunks of layer l; has_resident[l]: layer l has keys in HBM.
  void reset(int32_t n_layers, const int32_t *host_chunks, const uint8_t *has_resident, int32_t n_staging) {
    n_layers_ = n_layers;
    chunks_.assign(host_chunks, host_chunks + n_layers);
    resident_.assign(has_resident, has_resident + n_layers);
    first_unit_.assign(n_layers, 0);
    unit_layer_.clear();
    unit_chunk_.clear();
    for (int32_t l = 0; l < n_layers; ++l) {
      first_unit_[l] = (int32_t)unit_layer_.size();
      for (int32_t c = 0; c < chunks_[l]; ++c) {
        unit_layer_.push_back(l);
        unit_chunk_.push_back(c);
      }
    }
    k_ = (int32_t)unit_layer_.size();
    depth_ = k_ < n_staging ? k_ : n_staging;
    primed_ = false;
  }

  int32_t depth() const { return depth_; }
  int32_t n_units() const { return k_; }
  bool primed() const { return primed_; }

  Op make_copy(int64_t j, int64_t wait) const {
    Op op;
    op.kind = OP_COPY;
    op.step = (int32_t)(j / k_);
    op.layer = unit_layer_[j % k_];
    op.chunk = unit_chunk_[j % k_];
    op.buf = (int32_t)(j % depth_);
    op.copy_idx = j;
    op.wait_idx = wait;
    return op;
  }

  // First copies, issued once before the first step of a batch.
  void prime(std::vector<Op> &out) {
    if (primed_) return;
    primed_ = true;
    for (int32_t j = 0; j < depth_; ++j) out.push_back(make_copy(j, -1));
  }

  void on_append(int64_t step, int32_t layer, std::vector<Op> &out) const {
    out.push_back(Op{OP_APPEND, (int32_t)step, layer, -1, -1, -1, -1});
  }

  void on_attn(int64_t step, int32_t layer, std::vector<Op> &out) const {
    if (resident_[layer]) out.push_back(Op{OP_ATTN, (int32_t)step, layer, -1, -1, -1, -1});
    for (int32_t c = 0; c < chunks_[layer]; ++c) {
      const int64_t j = step * k_ + first_unit_[layer] + c;
      const int32_t buf = (int32_t)(j % depth_);
      out.push_back(Op{OP_ATTN, (int32_t)step, layer, c, buf, j, j});
      out.push_back(Op{OP_RELEASE, (int32_t)step, layer, c, buf, j, -1});
      out.push_back(make_copy(j + depth_, j));
    }
    out.push_back(Op{OP_MERGE, (int32_t)step, layer, -1, -1, -1, -1});
  }

 private:
  int32_t n_layers_ = 0, k_ = 0, depth_ = 0;
  bool primed_ = false;
  std::vector<int32_t> chunks_, first_unit_, unit_layer_, unit_chunk_;
  std::vector<uint8_t> resident_;
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

// ---- equal stretches -----------------------------------------------------------
//
// Unless the caller fixes a split size, the keys of a launch are shared out evenly: the 16-key tiles of
// all sequences, laid end to end in sequence order, are cut into stretches of `span` tiles, one stretch
// per wavefront and KV head, and a sequence is cut wherever a stretch ends inside it.  The items (pieces
// of sequences) that start in stretch j form group j.  There are at most max_groups stretches and none
// is shorter than min_span tiles unless the whole launch is.  The same arithmetic runs on the host (item
// count, checks) and in the kernel that builds the item list.
struct SpanPlan {
  int64_t span;        // tiles per stretch (>= 1)
  int32_t n_groups;    // stretches that hold at least one tile
};

__host__ __device__ inline SpanPlan span_plan(int64_t total_tiles, int32_t max_groups, int32_t min_span) {
  int64_t g = total_tiles / (min_span > 0 ? min_span : 1);
  if (g > max_groups) g = max_groups;
  if (g < 1) g = 1;
  SpanPlan p;
  p.span = (total_tiles + g - 1) / g;
  if (p.span < 1) p.span = 1;
  p.n_groups = (int32_t)((total_tiles + p.span - 1) / p.span);
  return p;
}

// Pieces of a sequence whose tiles are [first, first + tiles) of the stream: it is cut at the multiples
// of span strictly inside that range.  *k0 receives the first such multiple's index, so that piece c >= 1
// starts at tile (k0 + c - 1) * span of the stream and piece c ends where piece c + 1 starts.
__host__ __device__ inline int32_t span_pieces(int64_t first, int64_t tiles, int64_t span, int64_t *k0) {
  *k0 = first / span + 1;
  if (tiles <= 0) return 0;
  const int64_t k_last = (first + tiles - 1) / span;
  return 1 + (k_last >= *k0 ? (int32_t)(k_last - *k0 + 1) : 0);
}

// Piece c of a sequence with n keys: keys [lo, hi) and the stretch it starts in.
__host__ __device__ inline ItemRange span_piece(int32_t b, int32_t c, int32_t n, int64_t first, int64_t tiles,
                                                int64_t span, int64_t k0, int64_t *group) {
  const int64_t s = c == 0 ? first : (k0 + c - 1) * span;
  int64_t e = (k0 + c) * span;
  if (e > first + tiles) e = first + tiles;
  *group = s / span;
  ItemRange r;
  r.b = b;
  r.lo = (int32_t)((s - first) << 4);
  const int64_t hi = (e - first) << 4;
  r.hi = hi < n ? (int32_t)hi : n;
  return r;
}

// ---- block classes (paper §IV-C: a share C_off of the cache lives in host memory) ----
//
// With block-granular offload, block ids below `resident` are in HBM (class 0); the others
// are in the host pool, streamed in chunks of `chunk` consecutive blocks (host block i is in
// class 1 + i / chunk).  Every class is attended by a launch of its own, so a sequence is
// first cut into runs of consecutive positions whose blocks share a class, and each run is
// cut into equal pieces by seq_chunks with the run's length in place of the sequence's.
// KV heads per group inside a 16-token tile slab: the largest divisor of G whose K rows of one tile
// (gg * 16 * d * 2 bytes) fit in 32 KiB.  Measured on MI355X with 4 KiB tiles (d = 128): a wavefront that
// reads its K tile and its V tile 32 or 64 KiB apart runs at 6.4-6.6 TB/s, at 4-16 KiB or at a multiple of
// 128 KiB apart at 5.5-6.1.
inline int32_t kv_head_group(int32_t G, int32_t d) {
  int32_t gg = 1;
  for (int32_t c = 1; c <= G; ++c)
    if (G % c == 0 && (int64_t)c * d <= 1024) gg = c;
  return gg;
}

// 16-token tiles per slab, St: the largest power of two for which the K rows of a head group of St tiles
// (St * gg * 16 * d * 2 bytes) fit in 32 KiB and St divides the tiles of a pool slice (a block, or a
// sequence's slice of a contiguous pool).  With fewer than 8 KV heads at d = 128 the K rows of one tile are
// less than 32 KiB, the K tile and the V tile a wavefront reads together would lie 4-16 KiB apart, and the
// kernel ran at 71-72 % of the HBM peak where 8 KV heads reach 81 %; taking St tiles together puts them
// 32 KiB apart again wherever the block size allows it.
inline int32_t slab_tiles_log2(int32_t G, int32_t d, int32_t slice_tokens) {
  const int32_t gg = kv_head_group(G, d);
  int32_t lg = 0;
  while ((int64_t)(2 << lg) * gg * d <= 1024 && (slice_tokens >> 4) % (2 << lg) == 0) ++lg;
  return lg;
}

inline int32_t block_class(int64_t id, int64_t resident, int64_t chunk) {
  return id < resident ? 0 : 1 + (int32_t)((id - resident) / chunk);
}

struct Run {
  int32_t b, lo, hi_cap, cls;   // positions [lo, hi_cap) of sequence b lie in blocks of class cls
};

// Runs over the allocated prefix of every table row, sorted by (class, sequence, position);
// pair_first[cls * B + b] .. pair_first[cls * B + b + 1] are the runs of sequence b in class cls.
inline void build_runs(const int32_t *table, int32_t B, int32_t max_blocks, int32_t T, int64_t resident,
                       int64_t chunk, int32_t n_cls, std::vector<Run> &runs, std::vector<int32_t> &pair_first) {
  std::vector<Run> found;
  std::vector<int32_t> count((size_t)n_cls * B + 1, 0);
  for (int32_t b = 0; b < B; ++b) {
    const int32_t *row = table + (size_t)b * max_blocks;
    int32_t j = 0;
    while (j < max_blocks && row[j] >= 0) {
      const int32_t cls = block_class(row[j], resident, chunk);
      int32_t e = j + 1;
      while (e < max_blocks && row[e] >= 0 && block_class(row[e], resident, chunk) == cls) ++e;
      found.push_back(Run{b, j * T, e * T, cls});
      count[(size_t)cls * B + b] += 1;
      j = e;
    }
  }
  pair_first.assign((size_t)n_cls * B + 1, 0);
  for (size_t p = 0; p < (size_t)n_cls * B; ++p) pair_first[p + 1] = pair_first[p] + count[p];
  std::vector<int32_t> at(pair_first.begin(), pair_first.end() - 1);
  runs.resize(found.size());
  for (const Run &r : found) runs[at[(size_t)r.cls * B + r.b]++] = r;   // rows were walked in position order
}

// Items of one run when its sequence holds n keys.
__host__ __device__ inline int32_t run_items(int32_t lo, int32_t hi_cap, int32_t n, int32_t S, int32_t *size) {
  const int32_t len = (hi_cap < n ? hi_cap : n) - lo;
  int32_t cnt;
  seq_chunks(len, S, &cnt, size);
  return cnt;
}

// ---- the newest blocks kept in HBM (block-granular offload) ----------------------------------------
//
// Rows appended to a block of the host pool stay in a slot in HBM until the block is full.  For a step
// after which sequence b holds n[b] keys (from[b] = the length it had when the batch was described:
// rows before that are in the pools already):
//   tail_patch_chunks: host chunk c (blocks resident + c * chunk .. ) gets patch[c] = 1 if the newest
//     block of some sequence (that of position n[b] - 1) or the one before it lies in the chunk and holds
//     a position >= from[b]: before the chunk is attended those rows are copied into it from the slots;
//   tail_fills: the step fills a block of sequence b that belongs to the host pool and holds rows from
//     from[b] on: after the step the block is written out.
inline void tail_patch_chunks(const int32_t *table, int32_t B, int32_t max_blocks, int32_t log2_T, const int32_t *n,
                              const int32_t *from, int64_t resident, int64_t chunk, std::vector<uint8_t> &patch) {
  for (int32_t b = 0; b < B; ++b) {
    const int32_t jn = (n[b] - 1) >> log2_T;
    for (int32_t j = jn > 0 ? jn - 1 : 0; j <= jn; ++j) {
      if (((j + 1) << log2_T) <= from[b]) continue;          // all of it was in the pool from the start
      const int64_t id = table[(size_t)b * max_blocks + j];
      if (id < resident) continue;
      const int64_t c = (id - resident) / chunk;
      if (c < (int64_t)patch.size()) patch[(size_t)c] = 1;
    }
  }
}

inline bool tail_fills(const int32_t *table, int32_t b, int32_t max_blocks, int32_t log2_T, int32_t n, int32_t from,
                       int64_t resident) {
  if (n <= 0 || (n & ((1 << log2_T) - 1)) || from >= n) return false;
  return table[(size_t)b * max_blocks + (n >> log2_T) - 1] >= resident;
}

}  // namespace okv
