// C ABI of the okv library: argument checks, batch / step bookkeeping and the
// copy pipeline for host layers.  All arithmetic on K/V/q happens in the kernels
// (okv_kernels.hip); nothing here touches tensor values.
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <chrono>
#include <string>
#include <utility>
#include <vector>

#include "../../include/okv.h"
#include "../../include/okv_layer.h"
#include "okv_host.h"
#include "okv_kernels.h"

using okv::Op;

namespace {

constexpr int kEventRing = 8;            // > copies in flight (at most OKV_MAX_STAGING)
// Wavefronts of the persistent attention launch per compute unit: one per SIMD.  The kernel keeps about
// 8 KiB in flight per wavefront (16 when wavefronts take many units each), and about 1000 wavefronts
// saturate the memory system: with 2048 equal units, 4 per compute unit working through two units each
// reach 6.5 TB/s and 8 per compute unit with one unit each 6.1-6.3; ragged batches gain less (0-4 %).
// Kept apart by query-group size (1 head per KV head, 2..7, 8 and more) for tuning; all 4 at present.
#ifndef OKV_WAVES_PER_CU_MHA
#define OKV_WAVES_PER_CU_MHA 4
#endif
#ifndef OKV_WAVES_PER_CU_GQA
#define OKV_WAVES_PER_CU_GQA 4
#endif
#ifndef OKV_WAVES_PER_CU_MFMA
#define OKV_WAVES_PER_CU_MFMA 4
#endif
constexpr int32_t kMinAutoSplit = 128;   // smallest stretch of keys the library cuts a launch into by itself
constexpr int32_t kMinSpanTiles = kMinAutoSplit / 16;
// Records of the per-pair look-up table an attention launch with max_waves wavefronts may read: its grid is
// whole workgroups of four.
inline int32_t max_pairs(int32_t max_waves) { return std::max(max_waves, 4); }
constexpr int32_t kClassSplit = 512;     // split size with block classes unless the caller sets one
constexpr int64_t kMaxClasses = 4096;
// Workgroups of a bulk store that writes into host memory: the link, not the GPU, sets its
// pace, so it is kept small enough to leave the compute units to whatever runs beside it.
#ifndef OKV_BULK_WORKGROUPS
#define OKV_BULK_WORKGROUPS 16384
#endif
#ifndef OKV_HOST_WRITE_WORKGROUPS
#define OKV_HOST_WRITE_WORKGROUPS 64
#endif
// With a share of every layer's blocks on the host, how many steps the host may have enqueued that the
// compute stream has not finished when a new one begins (0 = no limit).  Steps enqueued several deep made the
// chunked copy pipeline slower and erratic (cfg3 shape in 256 MiB chunks: 608.7 ms a step in every process
// with 1, 610 with 2, 615 without a limit on a quiet machine and 624-695 from process to process on others);
// the compute stream waits for copies most of the time anyway.  Whole layers on the host are the other way
// round (606.9 ms a step without a limit, 608.5 with 2, 610.8 with 1) and never were erratic: no limit there.
#ifndef OKV_STEPS_AHEAD
#define OKV_STEPS_AHEAD 1
#endif
#ifndef OKV_STEPS_AHEAD_LAYERS
#define OKV_STEPS_AHEAD_LAYERS 0
#endif
constexpr int kAheadRing = (OKV_STEPS_AHEAD > OKV_STEPS_AHEAD_LAYERS ? OKV_STEPS_AHEAD : OKV_STEPS_AHEAD_LAYERS) > 0
                               ? (OKV_STEPS_AHEAD > OKV_STEPS_AHEAD_LAYERS ? OKV_STEPS_AHEAD : OKV_STEPS_AHEAD_LAYERS) : 1;
// Blocks bound for the host are gathered in a staging buffer and moved by hipMemcpyAsync when, on
// average, at least this many bytes of them are adjacent in the host pool; below that the per-copy
// cost is too high and the rows are written by a kernel through the mapped pointer instead.
constexpr int64_t kMinStagedRunBytes = 1 << 20;

thread_local std::string g_error;        // failures that have no context to live in

}  // namespace

struct okv_ctx {
  okv_config cfg;
  std::vector<void *> dev_pool, host_pool;
  okv::PoolShape shape;
  int64_t pool_bytes = 0, block_bytes = 0;
  int32_t cap_tokens = 0;                // per sequence
  bool any_host = false;
  int32_t n_staging = 0;
  hipStream_t compute = nullptr, h2d = nullptr;
  hipStream_t h2d_odd = nullptr;         // library-owned second copy stream (odd staging buffers)

  // block classes (a share of every layer's blocks on the host); n_cls == 1 otherwise
  bool by_class = false;
  int64_t resident_blocks = 0, chunk_blocks = 0;
  int32_t n_cls = 1;
  std::vector<okv::Run> h_runs;          // sorted by (class, sequence, position)
  std::vector<int32_t> h_pair_first;     // [n_cls * B + 1]
  std::vector<int32_t> cls_first, cls_count;   // items of each class in the current work list
  std::vector<int32_t> active_chunks;    // chunks of the host pool that hold blocks of the batch
  std::vector<int64_t> unit_offset, unit_bytes;   // per streamed chunk: where it starts in the host pool, its size
  bool has_resident = false;
  int4 *d_runs = nullptr;
  int32_t *d_pair_first = nullptr, *d_seq_total = nullptr;
  int64_t runs_cap = 0;

  // The sequences' newest blocks kept in HBM (cfg.tail_blocks): positions from tail_from[b] on were
  // appended through this context and, where their block belongs to the host pool, reach it only when
  // the block is full (or on okv_flush_tails).
  bool tail_on = false;
  bool tail_dirty = false;               // some appended row may not have reached the host pool yet
  int64_t tail_layer_stride = 0;         // numbers between two layers' slots
  int32_t *d_tail_from = nullptr;
  void **d_host_ptrs = nullptr;          // device array [L] of the host pools' device-visible addresses
  std::vector<int32_t> h_tail_from;
  std::vector<uint8_t> patch_chunk;      // per active chunk: a newest or second-newest block of the batch lies in it
  hipEvent_t flush_ev = nullptr;
  bool flush_recorded = false;
  // host layers or blocks: the ends of the last steps on the compute stream (a ring)
  hipEvent_t step_done_ev[kAheadRing] = {};
  int64_t steps_recorded = 0;
  int32_t steps_ahead = 0;               // the limit that applies to this context's kind of offload (0 = none)

  int32_t *d_block_table = nullptr, *d_ctx_lens = nullptr, *d_chunk_prefix = nullptr;
  int4 *d_item_desc = nullptr;
  int32_t *d_group_first = nullptr;      // equal stretches: first item of every stretch (+ 1 entry)
  void *d_pair_head = nullptr;           // equal stretches: what every (stretch, KV head) pair starts with
  int32_t *d_plan = nullptr;             // equal stretches: (stretches in use, items, tiles per stretch x 2)
  int32_t max_groups = 1;                // wavefronts of a launch per KV head
  int32_t *d_items_dump = nullptr;
  int32_t max_waves = 0;                 // wavefronts of the persistent attention launch
  int64_t max_items = 0;
  float *part_o = nullptr, *part_ml = nullptr;

  std::vector<int32_t> h_block_table, h_ctx_lens;
  int32_t B = 0, split = 0, split_override = 0, n_items = 0;
  bool need_merge = false;
  bool spans = false;                    // the work list is cut into equal stretches (no split size given)
  int32_t n_groups = 0;                  // stretches in use
  int64_t span_tiles = 0;                // tiles per stretch
  int64_t copy_bytes = 0;

  // bulk store of prompts (prefill side)
  bool in_prefill = false;
  int32_t prefill_next_layer = 0;
  std::vector<int32_t> h_n_new;
  int4 *d_tiles = nullptr;
  int32_t *d_row_base = nullptr;
  int64_t tiles_cap = 0;
  // d_tiles = [tiles of a layer that is all in HBM][tiles bound for HBM blocks][tiles written straight
  //            into host memory][tiles of staged group 0][group 1] ...
  struct TileSpan { int32_t first = 0, count = 0; };
  struct CopyRun { int64_t host_off, staging_off, bytes; };
  struct StagedGroup { TileSpan tiles; std::vector<CopyRun> runs; };
  TileSpan tiles_all, tiles_hbm, tiles_direct;
  std::vector<StagedGroup> groups;
  int64_t group_counter = 0;                         // staged groups issued since okv_create (picks buffer and events)
  hipEvent_t filled_ev[kEventRing] = {}, copied_ev[kEventRing] = {};
  hipStream_t d2h = nullptr;                         // library-owned stream of the stores into host memory
  hipEvent_t rows_ready_ev = nullptr, prefill_done_ev = nullptr;
  std::vector<hipEvent_t> stored_ev;                 // per layer: its rows have left the caller's buffers
  std::vector<uint8_t> stored_set;

  bool batch_set = false, in_step = false, appended = false;
  const void *pending_k = nullptr, *pending_v = nullptr;   // rows of the current layer's kv_append
  int64_t step = 0;
  int32_t next_layer = 0;
  okv::Scheduler sched;
  hipEvent_t ready_ev[kEventRing] = {}, consumed_ev[kEventRing] = {};

  int profile = 0;                       // 0 off, 1 a bracket per split-K launch, 2 a bracket per step
  std::vector<std::pair<hipEvent_t, hipEvent_t>> prof_events;
  size_t prof_used = 0;
  int64_t prof_launches = 0;             // split-K launches inside the brackets
  bool prof_open = false;                // per-step mode: the step's bracket has begun

  std::string err;
};

namespace {

int fail(okv_ctx *ctx, int code, const char *fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  (ctx ? ctx->err : g_error) = buf;
  return code;
}

#define OKV_HIP(ctx, expr)                                                                  \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess) return fail(ctx, OKV_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

bool is_pow2(int64_t x) { return x > 0 && (x & (x - 1)) == 0; }
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// Checks the shape fields; returns a message or NULL.
const char *shape_problem(const okv_config *c) {
  if (!c) return "cfg is NULL";
  if (c->n_layers < 1) return "n_layers < 1";
  if (c->n_kv_heads < 1 || c->n_q_heads < 1 || c->n_q_heads % c->n_kv_heads) return "n_q_heads must be a multiple of n_kv_heads";
  int r = c->n_q_heads / c->n_kv_heads;
  if (r < 1 || r > 16) return "n_q_heads / n_kv_heads must be between 1 and 16";
  if (c->n_kv_heads > 65535) return "n_kv_heads too large";
  if (c->head_dim != 64 && c->head_dim != 128) return "head_dim must be 64 or 128";
  if (c->max_batch < 1 || c->max_batch > 65535) return "max_batch out of range";
  if (c->out_dtype != 0 && c->out_dtype != 1) return "out_dtype must be 0 or 1";
  if (c->split_tokens < 0) return "split_tokens < 0";
  if (c->block_tokens == 0) {
    if (c->max_ctx < 16 || c->max_ctx % 16) return "contiguous pools need max_ctx >= 16 and a multiple of 16";
  } else {
    if (!is_pow2(c->block_tokens) || c->block_tokens < 16 || c->block_tokens > 1024) return "block_tokens must be 0 or a power of two in [16, 1024]";
    if (c->max_blocks_per_seq < 1) return "max_blocks_per_seq < 1";
    if (c->blocks_per_layer < 1 || c->blocks_per_layer > 0x7fffffff) return "blocks_per_layer out of range";
    if ((int64_t)c->max_blocks_per_seq * c->block_tokens > 0x3fffffff) return "capacity per sequence too large";
  }
  if (c->chunk_blocks < 0) return "chunk_blocks < 0";
  if (c->chunk_blocks > 0) {
    if (c->block_tokens == 0) return "block classes (chunk_blocks > 0) need paged pools";
    if (c->resident_blocks < 0 || c->resident_blocks > c->blocks_per_layer) return "resident_blocks outside [0, blocks_per_layer]";
    if ((c->blocks_per_layer - c->resident_blocks + c->chunk_blocks - 1) / c->chunk_blocks + 1 > kMaxClasses)
      return "too many chunks: raise chunk_blocks";
  }
  return nullptr;
}

int64_t cap_tokens_of(const okv_config *c) {
  return c->block_tokens ? (int64_t)c->max_blocks_per_seq * c->block_tokens : c->max_ctx;
}

int64_t pool_bytes_of(const okv_config *c) {
  int64_t row = (int64_t)c->head_dim * 2;
  if (c->block_tokens) return c->blocks_per_layer * 2 * c->n_kv_heads * c->block_tokens * row;
  return (int64_t)c->max_batch * 2 * c->n_kv_heads * c->max_ctx * row;
}

int64_t block_bytes_of(const okv_config *c) {
  int64_t tcap = c->block_tokens ? c->block_tokens : c->max_ctx;
  return (int64_t)2 * c->n_kv_heads * tcap * c->head_dim * 2;
}

// Classes a context can meet: the blocks in HBM plus every chunk of the host pool.
int32_t max_classes_of(const okv_config *c) {
  if (c->chunk_blocks <= 0) return 1;
  return 1 + (int32_t)((c->blocks_per_layer - c->resident_blocks + c->chunk_blocks - 1) / c->chunk_blocks);
}

int64_t bytes_per_item(const okv_config *c) { return (int64_t)c->n_q_heads * (c->head_dim + 2) * 4; }

int64_t count_items(const int32_t *ctx, int32_t B, int32_t S) {
  int64_t n = 0;
  for (int32_t b = 0; b < B; ++b) {
    int32_t cnt, sz;
    okv::seq_chunks(ctx[b], S, &cnt, &sz);
    n += cnt;
  }
  return n;
}

// The split size the caller fixed (okv_set_split_tokens, else cfg.split_tokens), or 0: the library
// shares the launch's keys out in equal stretches.
int32_t fixed_split(const okv_ctx *ctx) { return ctx->split_override ? ctx->split_override : ctx->cfg.split_tokens; }

hipStream_t copy_stream(okv_ctx *ctx, int buf) { return (buf & 1) && ctx->h2d_odd ? ctx->h2d_odd : ctx->h2d; }

okv::AttnLaunch base_launch(okv_ctx *ctx) {
  okv::AttnLaunch a;
  a.shape = ctx->shape;
  a.batch = okv::BatchState{ctx->d_block_table, ctx->d_ctx_lens, ctx->d_chunk_prefix, ctx->d_item_desc,
                            ctx->B, ctx->split, ctx->n_items, ctx->n_cls};
  a.q = nullptr;
  a.pool = nullptr;
  a.k_new = a.v_new = nullptr;
  a.pool_mirror = nullptr;
  a.out = nullptr;
  a.part_o = ctx->part_o;
  a.part_ml = ctx->part_ml;
  a.out_fp32 = ctx->cfg.out_dtype;
  a.need_merge = ctx->need_merge;
  if (ctx->spans) {
    a.pair_head = ctx->d_pair_head;
    a.n_groups = ctx->n_groups;
  }
  a.max_waves = ctx->max_waves;
  a.item_first = 0;
  a.item_count = ctx->n_items;
  a.id_base = a.mirror_base = 0;
  return a;
}

void reset_schedule(okv_ctx *ctx);

// A stream whose hardware queue no other stream of the process uses.  The runtime spreads ordinary streams
// over a few hardware queues (4 by default) and works each queue through in order, so a copy stream that
// happens to share a queue with the compute stream holds the attention kernels back behind the marker of
// every copy (seen in the copy trace: kernels that waited for nothing started only when the other stream's
// 2 GiB copy had finished).  A stream created with a compute-unit mask is given a queue of its own; the mask
// names every compute unit.  Default priority.
hipError_t own_queue_stream(hipStream_t *out) {
  int dev = 0, cus = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return e;
  std::vector<uint32_t> mask((size_t)(std::max(cus, 1) + 31) / 32, 0xFFFFFFFFu);
  e = hipExtStreamCreateWithCUMask(out, (uint32_t)mask.size(), mask.data());
  if (e == hipSuccess) return e;
  (void)hipGetLastError();                               // an ordinary stream still works, it may only share a queue
  return hipStreamCreateWithFlags(out, hipStreamNonBlocking);
}

// The host's lead over the compute stream, in steps (OKV_STEPS_AHEAD): the step about to be enqueued may
// not begin before the one that many steps back has finished.
int wait_for_earlier_steps(okv_ctx *ctx) {
  const int64_t kAhead = ctx->steps_ahead;
  if (kAhead <= 0 || !ctx->step_done_ev[0] || ctx->steps_recorded < kAhead) return OKV_OK;
  OKV_HIP(ctx, hipEventSynchronize(ctx->step_done_ev[ctx->steps_recorded % kAhead]));   // the oldest of the ring
  return OKV_OK;
}

int mark_step_done(okv_ctx *ctx) {
  const int64_t kAhead = ctx->steps_ahead;
  if (kAhead <= 0 || !ctx->step_done_ev[0]) return OKV_OK;
  OKV_HIP(ctx, hipEventRecord(ctx->step_done_ev[ctx->steps_recorded % kAhead], ctx->compute));
  ctx->steps_recorded += 1;
  return OKV_OK;
}

okv::TailLaunch tail_launch(okv_ctx *ctx, int32_t mode) {
  okv::TailLaunch t;
  t.staged = nullptr;
  t.host_pools = ctx->d_host_ptrs;
  t.tail = ctx->cfg.tail_blocks;
  t.block_table = ctx->d_block_table;
  t.ctx_lens = ctx->d_ctx_lens;
  t.tail_from = ctx->d_tail_from;
  t.block_elems = ctx->block_bytes / 2;
  t.layer_stride = ctx->tail_layer_stride;
  t.B = ctx->B;
  t.n_layers = ctx->cfg.n_layers;
  t.max_blocks = ctx->shape.max_blocks;
  t.log2_T = ctx->shape.log2_T;
  t.D = ctx->shape.D;
  t.gg = ctx->shape.gg;
  t.st_log2 = ctx->shape.st_log2;
  t.id_lo = (int32_t)ctx->resident_blocks;
  t.id_hi = (int32_t)ctx->cfg.blocks_per_layer;
  t.mode = mode;
  return t;
}

// Positions from the current lengths on are the ones whose rows the slots will hold.
int tail_restart(okv_ctx *ctx) {
  if (!ctx->tail_on) return OKV_OK;
  ctx->h_tail_from.assign(ctx->h_ctx_lens.begin(), ctx->h_ctx_lens.begin() + ctx->B);
  OKV_HIP(ctx, hipMemcpy(ctx->d_tail_from, ctx->h_tail_from.data(), (size_t)ctx->B * sizeof(int32_t), hipMemcpyHostToDevice));
  ctx->tail_dirty = false;
  return OKV_OK;
}

// Every row still only in a slot goes to the host pool; afterwards the pools are complete, the copies
// already made of them are not, so the pipeline starts afresh.  Synchronous.
int tail_flush_all(okv_ctx *ctx) {
  if (!ctx->tail_on || !ctx->tail_dirty || !ctx->batch_set) return OKV_OK;
  int rc = okv_synchronize(ctx);
  if (rc) return rc;
  OKV_HIP(ctx, okv::launch_tail_rows(tail_launch(ctx, 2), ctx->compute));
  rc = okv_synchronize(ctx);
  if (rc) return rc;
  rc = tail_restart(ctx);
  reset_schedule(ctx);
  return rc;
}

// Chunks in which some sequence's newest or second-newest block lies at the lengths the host holds.
void tail_mark_chunks(okv_ctx *ctx) {
  const okv::PoolShape &s = ctx->shape;
  std::vector<uint8_t> by_chunk((size_t)std::max(0, ctx->n_cls - 1), 0);
  okv::tail_patch_chunks(ctx->h_block_table.data(), ctx->B, s.max_blocks, s.log2_T, ctx->h_ctx_lens.data(),
                         ctx->h_tail_from.data(), ctx->resident_blocks, ctx->chunk_blocks, by_chunk);
  ctx->patch_chunk.assign(ctx->active_chunks.size(), 0);
  for (size_t u = 0; u < ctx->active_chunks.size(); ++u) ctx->patch_chunk[u] = by_chunk[(size_t)ctx->active_chunks[u]];
}

int exec_op(okv_ctx *ctx, const Op &op, const void *a0, const void *a1, void *out) {
  switch (op.kind) {
    case okv::OP_COPY: {
      // Copies into different staging buffers go to different streams: they need no order among
      // themselves, and the marker that follows a copy (its cost grows with the bytes copied,
      // about 2 % of the copy time) then overlaps with the next copy instead of delaying it.
      hipStream_t cs = copy_stream(ctx, op.buf);
      if (op.wait_idx >= 0) OKV_HIP(ctx, hipStreamWaitEvent(cs, ctx->consumed_ev[op.wait_idx % kEventRing], 0));
      // a block written out to the host pool at the end of a step is in every copy enqueued after that
      if (ctx->flush_recorded) OKV_HIP(ctx, hipStreamWaitEvent(cs, ctx->flush_ev, 0));
      const char *src = static_cast<const char *>(ctx->host_pool[op.layer]) + ctx->unit_offset[op.chunk];
      OKV_HIP(ctx, hipMemcpyAsync(ctx->cfg.staging[op.buf], src, (size_t)ctx->unit_bytes[op.chunk],
                                  hipMemcpyHostToDevice, cs));
      OKV_HIP(ctx, hipEventRecord(ctx->ready_ev[op.copy_idx % kEventRing], cs));
      return OKV_OK;
    }
    case okv::OP_APPEND:
      // The rows are stored by the attention launch that meets each sequence's newest position
      // (one kernel instead of two); here they are only noted.
      ctx->pending_k = a0;
      ctx->pending_v = a1;
      return OKV_OK;
    case okv::OP_ATTN: {
      if (op.wait_idx >= 0) OKV_HIP(ctx, hipStreamWaitEvent(ctx->compute, ctx->ready_ev[op.wait_idx % kEventRing], 0));
      okv::AttnLaunch a = base_launch(ctx);
      if (ctx->by_class) {
        int32_t cls = 0;
        if (op.chunk >= 0) {
          const int32_t chunk = ctx->active_chunks[op.chunk];
          cls = 1 + chunk;
          a.id_base = (int32_t)(ctx->resident_blocks + (int64_t)chunk * ctx->chunk_blocks);
          a.mirror_base = (int32_t)ctx->resident_blocks;
        }
        a.item_first = ctx->cls_first[cls];
        a.item_count = ctx->cls_count[cls];
      }
      if (a.item_count == 0) return OKV_OK;              // no key of the batch lies in this class at this step
      a.q = a0;
      a.pool = op.buf >= 0 ? ctx->cfg.staging[op.buf] : ctx->dev_pool[op.layer];
      a.k_new = ctx->pending_k;
      a.v_new = ctx->pending_v;
      a.pool_mirror = op.buf >= 0 ? ctx->host_pool[op.layer] : nullptr;
      if (ctx->tail_on && op.buf >= 0 && op.chunk >= 0) {
        // rows appended to blocks of this chunk live in the layer's slots: the new ones go there, and
        // those of earlier steps are put into the staged chunk before it is attended
        uint16_t *slots = static_cast<uint16_t *>(ctx->cfg.tail_blocks) + (int64_t)op.layer * ctx->tail_layer_stride;
        a.pool_mirror = slots;
        a.mirror_is_tail = 1;
        if (ctx->patch_chunk[op.chunk]) {
          okv::TailLaunch t = tail_launch(ctx, 0);
          t.staged = ctx->cfg.staging[op.buf];
          t.tail = slots;
          t.id_lo = a.id_base;
          t.id_hi = (int32_t)std::min<int64_t>((int64_t)a.id_base + ctx->chunk_blocks, ctx->cfg.blocks_per_layer);
          OKV_HIP(ctx, okv::launch_tail_rows(t, ctx->compute));
        }
      }
      a.out = out;
      hipEvent_t e0 = nullptr, e1 = nullptr;
      if (ctx->profile == 1 || (ctx->profile == 2 && !ctx->prof_open)) {
        if (ctx->prof_used == ctx->prof_events.size()) {
          hipEvent_t x, y;
          OKV_HIP(ctx, hipEventCreate(&x));
          OKV_HIP(ctx, hipEventCreate(&y));
          ctx->prof_events.emplace_back(x, y);
        }
        e0 = ctx->prof_events[ctx->prof_used].first;
        if (ctx->profile == 1) {
          e1 = ctx->prof_events[ctx->prof_used].second;
          ++ctx->prof_used;
        } else {
          ctx->prof_open = true;                         // okv_step_end records the closing event
        }
      }
      if (ctx->profile) ++ctx->prof_launches;
      OKV_HIP(ctx, okv::launch_decode_attn(a, ctx->compute, e0, e1));
      return OKV_OK;
    }
    case okv::OP_RELEASE:
      OKV_HIP(ctx, hipEventRecord(ctx->consumed_ev[op.copy_idx % kEventRing], ctx->compute));
      return OKV_OK;
    case okv::OP_MERGE: {
      ctx->pending_k = ctx->pending_v = nullptr;
      if (!ctx->need_merge) return OKV_OK;
      okv::AttnLaunch a = base_launch(ctx);
      a.out = out;
      OKV_HIP(ctx, okv::launch_merge(a, ctx->compute));
      return OKV_OK;
    }
  }
  return fail(ctx, OKV_ESTATE, "unknown pipeline op %d", op.kind);
}

int exec_ops(okv_ctx *ctx, const std::vector<Op> &ops, const void *a0, const void *a1, void *out) {
  for (const Op &op : ops) {
    int rc = exec_op(ctx, op, a0, a1, out);
    if (rc) return rc;
  }
  return OKV_OK;
}

// Recomputes split size, item count and merge flag from the host lengths and
// rebuilds the device work list (adding `inc` to every device length first).
int rebuild_worklist(okv_ctx *ctx, int32_t inc, bool upload_lens = false) {
  if (upload_lens) {
    // the device lengths are replaced by the host's (after a bulk store); h_ctx_lens is pageable
    // memory, so the copy is over when the call returns, and the kernels below are enqueued after it
    OKV_HIP(ctx, hipStreamSynchronize(ctx->compute));
    OKV_HIP(ctx, hipMemcpy(ctx->d_ctx_lens, ctx->h_ctx_lens.data(), (size_t)ctx->B * sizeof(int32_t), hipMemcpyHostToDevice));
  }
  if (ctx->by_class) {
    ctx->split = ctx->split_override ? ctx->split_override : ctx->cfg.split_tokens ? ctx->cfg.split_tokens : kClassSplit;
    std::vector<int32_t> per_seq(ctx->B, 0);
    ctx->cls_count.assign(ctx->n_cls, 0);
    int64_t n = 0;
    for (const okv::Run &r : ctx->h_runs) {
      int32_t sz;
      const int32_t cnt = okv::run_items(r.lo, r.hi_cap, ctx->h_ctx_lens[r.b], ctx->split, &sz);
      ctx->cls_count[r.cls] += cnt;
      per_seq[r.b] += cnt;
      n += cnt;
    }
    if (n > ctx->max_items)
      return fail(ctx, OKV_ENOSPC, "split size %d needs %lld work items, workspace holds %lld", ctx->split,
                  (long long)n, (long long)ctx->max_items);
    ctx->n_items = (int32_t)n;
    ctx->cls_first.assign(ctx->n_cls + 1, 0);
    for (int32_t c = 0; c < ctx->n_cls; ++c) ctx->cls_first[c + 1] = ctx->cls_first[c] + ctx->cls_count[c];
    ctx->need_merge = false;
    ctx->spans = false;
    for (int32_t b = 0; b < ctx->B; ++b) ctx->need_merge |= per_seq[b] > 1;
    OKV_HIP(ctx, okv::launch_step_advance_classes(ctx->d_ctx_lens, ctx->d_runs, ctx->d_pair_first, ctx->d_chunk_prefix,
                                                  ctx->d_item_desc, ctx->d_seq_total, ctx->B, ctx->n_cls, ctx->split, inc,
                                                  ctx->compute));
    return OKV_OK;
  }
  if (const int32_t S = fixed_split(ctx)) {
    // a split size fixed by the caller: every sequence in equal pieces of at most S keys
    int64_t n = count_items(ctx->h_ctx_lens.data(), ctx->B, S);
    if (n > ctx->max_items)
      return fail(ctx, OKV_ENOSPC, "split size %d needs %lld work items, workspace holds %lld", S, (long long)n,
                  (long long)ctx->max_items);
    ctx->split = S;
    ctx->spans = false;
    ctx->n_items = (int32_t)n;
    ctx->need_merge = false;
    for (int32_t b = 0; b < ctx->B; ++b) {
      int32_t cnt, sz;
      okv::seq_chunks(ctx->h_ctx_lens[b], S, &cnt, &sz);
      if (cnt > 1) ctx->need_merge = true;
    }
    OKV_HIP(ctx, okv::launch_step_advance(ctx->d_ctx_lens, ctx->d_chunk_prefix, ctx->d_item_desc, ctx->B, S, inc,
                                          ctx->compute));
    return OKV_OK;
  }
  // equal stretches: the host walks the same arithmetic as the kernel for the counts it needs
  int64_t total = 0;
  for (int32_t b = 0; b < ctx->B; ++b) total += (ctx->h_ctx_lens[b] + 15) >> 4;
  const okv::SpanPlan plan = okv::span_plan(total, ctx->max_groups, kMinSpanTiles);
  int64_t n = 0, first = 0;
  bool merge = false;
  for (int32_t b = 0; b < ctx->B; ++b) {
    const int64_t tiles = (ctx->h_ctx_lens[b] + 15) >> 4;
    int64_t k0;
    const int32_t cnt = okv::span_pieces(first, tiles, plan.span, &k0);
    merge |= cnt > 1;
    n += cnt;
    first += tiles;
  }
  if (n > ctx->max_items)
    return fail(ctx, OKV_ENOSPC, "the batch needs %lld work items, workspace holds %lld", (long long)n, (long long)ctx->max_items);
  ctx->spans = true;
  ctx->n_groups = plan.n_groups;
  ctx->span_tiles = plan.span;
  ctx->split = (int32_t)std::min<int64_t>(plan.span * 16, 0x7fffffff);
  ctx->n_items = (int32_t)n;
  ctx->need_merge = merge;
  OKV_HIP(ctx, okv::launch_step_advance_spans(ctx->d_ctx_lens, ctx->d_chunk_prefix, ctx->d_item_desc, ctx->d_group_first,
                                              ctx->d_plan, ctx->B, ctx->max_groups, kMinSpanTiles, inc, ctx->d_pair_head,
                                              okv::head_geom(ctx->shape, ctx->d_block_table, max_pairs(ctx->max_waves)),
                                              ctx->compute));
  return OKV_OK;
}

// Restarts the copy pipeline for the batch just described.
void reset_schedule(okv_ctx *ctx) {
  const int32_t L = ctx->cfg.n_layers;
  std::vector<int32_t> chunks(L, 0);
  std::vector<uint8_t> resident(L, 0);
  for (int32_t l = 0; l < L; ++l) {
    if (ctx->by_class) {
      chunks[l] = (int32_t)ctx->active_chunks.size();
      resident[l] = ctx->has_resident;
    } else {
      chunks[l] = ctx->host_pool[l] != nullptr;
      resident[l] = ctx->host_pool[l] == nullptr;
    }
  }
  ctx->sched.reset(L, chunks.data(), resident.data(), ctx->n_staging);
  ctx->step = 0;                                       // copy indices count from the restart
}

}  // namespace

extern "C" {

int64_t okv_layer_pool_bytes(const okv_config *cfg) {
  if (const char *why = shape_problem(cfg)) return fail(nullptr, OKV_EINVAL, "%s", why);
  return pool_bytes_of(cfg);
}

int64_t okv_workspace_bytes(const okv_config *cfg) {
  if (const char *why = shape_problem(cfg)) return fail(nullptr, OKV_EINVAL, "%s", why);
  int64_t S = cfg->split_tokens ? cfg->split_tokens : kMinAutoSplit;
  if (S < 16) S = 16;                                  // items never hold fewer than 16 keys
  int64_t cap = cap_tokens_of(cfg);
  if (cfg->chunk_blocks > 0 && !cfg->split_tokens) S = kClassSplit;
  // with block classes a sequence has at least one item per class it has blocks in; the
  // figure assumes one run per class (an allocator that keeps a sequence's blocks of a
  // class together); a batch that needs more is refused by okv_set_batch
  // (equal stretches cut a batch into at most one item per sequence plus one per stretch, and a stretch
  // is at least kMinAutoSplit keys unless the batch is a single one: one more item per sequence covers it)
  int64_t items = (int64_t)cfg->max_batch * ((cap + S - 1) / S + (cfg->chunk_blocks > 0 ? 0 : 1) + (max_classes_of(cfg) - 1));
  return items * bytes_per_item(cfg);
}

int64_t okv_tail_bytes(const okv_config *cfg) {
  if (const char *why = shape_problem(cfg)) return fail(nullptr, OKV_EINVAL, "%s", why);
  if (cfg->chunk_blocks <= 0) return 0;
  return (int64_t)cfg->n_layers * 2 * cfg->max_batch * block_bytes_of(cfg);
}

int okv_tail_plan(int32_t B, const int32_t *block_table, int32_t max_blocks_per_seq, int32_t block_tokens,
                  const int32_t *ctx_lens_after, const int32_t *tail_from, int64_t resident_blocks, int64_t chunk_blocks,
                  int32_t n_chunks, uint8_t *patch_chunk, uint8_t *fills_block) {
  if (B < 1 || !block_table || !ctx_lens_after || !tail_from || !patch_chunk || !fills_block)
    return fail(nullptr, OKV_EINVAL, "okv_tail_plan: NULL argument or B < 1");
  if (max_blocks_per_seq < 1 || block_tokens < 16 || (block_tokens & (block_tokens - 1)) || resident_blocks < 0 || chunk_blocks < 1 ||
      n_chunks < 0)
    return fail(nullptr, OKV_EINVAL, "okv_tail_plan: bad shape");
  int32_t log2_T = 0;
  while ((1 << log2_T) < block_tokens) ++log2_T;
  for (int32_t b = 0; b < B; ++b)
    if (ctx_lens_after[b] < 1 || ctx_lens_after[b] > (int64_t)max_blocks_per_seq * block_tokens || tail_from[b] < 0)
      return fail(nullptr, OKV_EINVAL, "okv_tail_plan: sequence %d: length %d outside [1, %lld] or tail_from < 0", b, ctx_lens_after[b],
                  (long long)max_blocks_per_seq * block_tokens);
  std::vector<uint8_t> patch((size_t)n_chunks, 0);
  okv::tail_patch_chunks(block_table, B, max_blocks_per_seq, log2_T, ctx_lens_after, tail_from, resident_blocks, chunk_blocks, patch);
  for (int32_t c = 0; c < n_chunks; ++c) patch_chunk[c] = patch[(size_t)c];
  for (int32_t b = 0; b < B; ++b)
    fills_block[b] = okv::tail_fills(block_table, b, max_blocks_per_seq, log2_T, ctx_lens_after[b], tail_from[b], resident_blocks);
  return OKV_OK;
}

int kv_offload_plan(int32_t n_layers, int64_t coff_num, int64_t coff_den, uint8_t *on_host, int32_t *n_off) {
  if (n_layers < 1 || !on_host) return fail(nullptr, OKV_EINVAL, "kv_offload_plan: n_layers < 1 or on_host NULL");
  if (coff_den <= 0 || coff_num < 0 || coff_num > coff_den)
    return fail(nullptr, OKV_EINVAL, "kv_offload_plan: C_off must lie in [0, 1]");
  int32_t k = okv::plan_count(n_layers, coff_num, coff_den);
  okv::plan_place(n_layers, k, on_host);
  if (n_off) *n_off = k;
  return OKV_OK;
}

int okv_plan_from_bytes(int32_t n_layers, int64_t layer_bytes, int64_t mem_avail_bytes, uint8_t *on_host,
                        int32_t *n_off, int32_t *n_staging) {
  if (n_layers < 1 || layer_bytes < 1 || mem_avail_bytes < 0 || !on_host)
    return fail(nullptr, OKV_EINVAL, "okv_plan_from_bytes: bad argument");
  int32_t k = 0, ns = 0;
  if ((__int128)mem_avail_bytes >= (__int128)layer_bytes * n_layers) {
    k = 0;                                                      // Case 1
  } else if (layer_bytes > mem_avail_bytes) {
    return fail(nullptr, OKV_ENOSPC, "one layer's KV (%lld B) exceeds the available memory (%lld B)",
                (long long)layer_bytes, (long long)mem_avail_bytes);   // Case 2
  } else {
    int64_t fit = mem_avail_bytes / layer_bytes;                // Case 3: 1 <= fit < n_layers
    ns = fit >= 2 ? 2 : 1;
    k = n_layers - (int32_t)(fit - ns);
  }
  okv::plan_place(n_layers, k, on_host);
  if (n_off) *n_off = k;
  if (n_staging) *n_staging = ns;
  return OKV_OK;
}

int okv_schedule_trace(int32_t n_layers, const int32_t *host_chunks, const uint8_t *has_resident, int32_t n_staging,
                       int32_t n_steps, int32_t *ops, int64_t max_ops, int64_t *n_ops) {
  if (n_layers < 1 || !host_chunks || n_steps < 0 || !ops || !n_ops || n_staging < 0 || n_staging > OKV_MAX_STAGING)
    return fail(nullptr, OKV_EINVAL, "okv_schedule_trace: bad argument");
  std::vector<uint8_t> res(n_layers);
  bool any = false;
  for (int32_t l = 0; l < n_layers; ++l) {
    if (host_chunks[l] < 0) return fail(nullptr, OKV_EINVAL, "okv_schedule_trace: host_chunks[%d] < 0", l);
    res[l] = has_resident ? has_resident[l] != 0 : host_chunks[l] == 0;
    if (!res[l] && host_chunks[l] == 0) return fail(nullptr, OKV_EINVAL, "okv_schedule_trace: layer %d holds nothing", l);
    any |= host_chunks[l] > 0;
  }
  if (any && n_staging < 1) return fail(nullptr, OKV_EINVAL, "streamed chunks need a staging buffer");
  okv::Scheduler s;
  s.reset(n_layers, host_chunks, res.data(), n_staging);
  std::vector<Op> v;
  if (n_steps > 0) s.prime(v);
  for (int32_t step = 0; step < n_steps; ++step)
    for (int32_t l = 0; l < n_layers; ++l) {
      s.on_append(step, l, v);
      s.on_attn(step, l, v);
    }
  *n_ops = (int64_t)v.size();
  if ((int64_t)v.size() > max_ops) return fail(nullptr, OKV_ENOSPC, "trace needs %zu records", v.size());
  for (size_t i = 0; i < v.size(); ++i) {
    int32_t *o = ops + i * 7;
    o[0] = v[i].kind, o[1] = v[i].step, o[2] = v[i].layer, o[3] = v[i].chunk, o[4] = v[i].buf;
    o[5] = (int32_t)v[i].copy_idx, o[6] = (int32_t)v[i].wait_idx;
  }
  return OKV_OK;
}

int okv_plan_block_split(int64_t n_blocks, int64_t coff_num, int64_t coff_den, int64_t *resident_blocks,
                         int64_t *host_blocks) {
  if (n_blocks < 0 || !resident_blocks || !host_blocks) return fail(nullptr, OKV_EINVAL, "okv_plan_block_split: bad argument");
  if (coff_den <= 0 || coff_num < 0 || coff_num > coff_den)
    return fail(nullptr, OKV_EINVAL, "okv_plan_block_split: C_off must lie in [0, 1]");
  const __int128 x = (__int128)coff_num * n_blocks;
  const int64_t host = (int64_t)((x + coff_den - 1) / coff_den);
  *host_blocks = host;
  *resident_blocks = n_blocks - host;
  return OKV_OK;
}

int okv_equal_stretches(const int32_t *ctx_lens, int32_t B, int32_t max_groups, int32_t *items, int64_t max_items,
                        int64_t *n_items, int32_t *group_first, int32_t *n_groups, int64_t *span_tiles) {
  if (!ctx_lens || B < 1 || max_groups < 1 || !items || !n_items || !group_first || !n_groups || !span_tiles)
    return fail(nullptr, OKV_EINVAL, "okv_equal_stretches: bad argument");
  int64_t total = 0;
  for (int32_t b = 0; b < B; ++b) {
    if (ctx_lens[b] < 0) return fail(nullptr, OKV_EINVAL, "okv_equal_stretches: ctx_lens[%d] < 0", b);
    total += (ctx_lens[b] + 15) >> 4;
  }
  const okv::SpanPlan plan = okv::span_plan(total, max_groups, kMinSpanTiles);
  *span_tiles = plan.span;
  *n_groups = plan.n_groups;
  int64_t it = 0, first = 0;
  for (int32_t b = 0; b < B; ++b) {
    const int64_t tiles = (ctx_lens[b] + 15) >> 4;
    int64_t k0, group;
    const int32_t cnt = okv::span_pieces(first, tiles, plan.span, &k0);
    for (int32_t c = 0; c < cnt; ++c, ++it) {
      const okv::ItemRange r = okv::span_piece(b, c, ctx_lens[b], first, tiles, plan.span, k0, &group);
      if (it < max_items) items[it * 3 + 0] = r.b, items[it * 3 + 1] = r.lo, items[it * 3 + 2] = r.hi;
      if (c > 0 || first % plan.span == 0) group_first[group] = (int32_t)it;
    }
    first += tiles;
  }
  group_first[plan.n_groups] = (int32_t)it;
  *n_items = it;
  if (it > max_items) return fail(nullptr, OKV_ENOSPC, "okv_equal_stretches: %lld items", (long long)it);
  return OKV_OK;
}

int32_t okv_slab_tiles(int32_t n_kv_heads, int32_t head_dim, int32_t slice_tokens) {
  if (n_kv_heads < 1 || (head_dim != 64 && head_dim != 128) || slice_tokens < 16 || slice_tokens % 16)
    return fail(nullptr, OKV_EINVAL, "okv_slab_tiles: bad argument");
  return 1 << okv::slab_tiles_log2(n_kv_heads, head_dim, slice_tokens);
}

int32_t okv_kv_head_group(int32_t n_kv_heads, int32_t head_dim) {
  if (n_kv_heads < 1 || (head_dim != 64 && head_dim != 128)) return OKV_EINVAL;
  return okv::kv_head_group(n_kv_heads, head_dim);
}

int64_t okv_block_bytes(const okv_config *cfg) {
  if (const char *why = shape_problem(cfg)) return fail(nullptr, OKV_EINVAL, "%s", why);
  return block_bytes_of(cfg);
}

int okv_create(const okv_config *cfg, okv_ctx **out) {
  if (!out) return fail(nullptr, OKV_EINVAL, "okv_create: out is NULL");
  *out = nullptr;
  if (const char *why = shape_problem(cfg)) return fail(nullptr, OKV_EINVAL, "okv_create: %s", why);
  const int32_t L = cfg->n_layers;
  if (!cfg->dev_pool) return fail(nullptr, OKV_EINVAL, "okv_create: dev_pool is NULL");
  const bool by_class = cfg->chunk_blocks > 0;
  const int64_t host_blocks = by_class ? cfg->blocks_per_layer - cfg->resident_blocks : 0;
  bool any_host = false;
  for (int32_t l = 0; l < L; ++l) {
    void *d = cfg->dev_pool[l], *h = cfg->host_pool ? cfg->host_pool[l] : nullptr;
    if (by_class) {
      if ((cfg->resident_blocks > 0) != (d != nullptr))
        return fail(nullptr, OKV_EINVAL, "okv_create: layer %d: dev_pool must be set exactly when resident_blocks > 0", l);
      if ((host_blocks > 0) != (h != nullptr))
        return fail(nullptr, OKV_EINVAL, "okv_create: layer %d: host_pool must be set exactly when blocks live on the host", l);
    } else if ((d != nullptr) == (h != nullptr)) {
      return fail(nullptr, OKV_EINVAL, "okv_create: layer %d needs exactly one of dev_pool / host_pool", l);
    }
    if (!aligned16(d) || !aligned16(h)) return fail(nullptr, OKV_EINVAL, "okv_create: layer %d pool not 16-byte aligned", l);
    any_host |= h != nullptr;
  }
  const int64_t pool_bytes = pool_bytes_of(cfg);
  int32_t n_staging = 0;
  if (any_host) {
    if (!cfg->staging[0]) return fail(nullptr, OKV_EINVAL, "okv_create: host layers need staging[0]");
    const int64_t need_staging = by_class ? std::min(cfg->chunk_blocks, host_blocks) * block_bytes_of(cfg) : pool_bytes;
    if (cfg->staging_bytes < need_staging)
      return fail(nullptr, OKV_ENOSPC, "okv_create: staging_bytes %lld < %lld (what is streamed at once must fit on the GPU)",
                  (long long)cfg->staging_bytes, (long long)need_staging);
    for (int i = 0; i < OKV_MAX_STAGING; ++i)
      if (!aligned16(cfg->staging[i])) return fail(nullptr, OKV_EINVAL, "okv_create: staging not 16-byte aligned");
    if (cfg->h2d_stream == cfg->compute_stream) return fail(nullptr, OKV_EINVAL, "okv_create: h2d_stream must differ from compute_stream");
    while (n_staging < OKV_MAX_STAGING && cfg->staging[n_staging]) ++n_staging;
  }
  if (cfg->tail_blocks) {
    if (!by_class || host_blocks == 0)
      return fail(nullptr, OKV_EINVAL, "okv_create: tail_blocks is for block-granular offload (chunk_blocks > 0, blocks on the host)");
    if (!aligned16(cfg->tail_blocks)) return fail(nullptr, OKV_EINVAL, "okv_create: tail_blocks not 16-byte aligned");
    const int64_t need_tail = okv_tail_bytes(cfg);
    if (cfg->tail_bytes < need_tail)
      return fail(nullptr, OKV_ENOSPC, "okv_create: tail_bytes %lld < %lld", (long long)cfg->tail_bytes, (long long)need_tail);
  }
  const int64_t need_ws = okv_workspace_bytes(cfg);
  if (!cfg->workspace || !aligned16(cfg->workspace)) return fail(nullptr, OKV_EINVAL, "okv_create: workspace NULL or misaligned");
  if (cfg->workspace_bytes < need_ws)
    return fail(nullptr, OKV_ENOSPC, "okv_create: workspace_bytes %lld < %lld", (long long)cfg->workspace_bytes, (long long)need_ws);

  okv_ctx *ctx = new (std::nothrow) okv_ctx();
  if (!ctx) return fail(nullptr, OKV_ENOSPC, "okv_create: out of host memory");
  ctx->cfg = *cfg;
  ctx->dev_pool.assign(cfg->dev_pool, cfg->dev_pool + L);
  if (cfg->host_pool) ctx->host_pool.assign(cfg->host_pool, cfg->host_pool + L);
  else ctx->host_pool.assign(L, nullptr);
  ctx->cfg.dev_pool = ctx->dev_pool.data();
  ctx->cfg.host_pool = ctx->host_pool.data();
  ctx->any_host = any_host;
  ctx->n_staging = n_staging;
  ctx->pool_bytes = pool_bytes;
  ctx->cap_tokens = (int32_t)cap_tokens_of(cfg);
  ctx->compute = static_cast<hipStream_t>(cfg->compute_stream);
  ctx->h2d = static_cast<hipStream_t>(cfg->h2d_stream);
  okv::PoolShape &s = ctx->shape;
  s.H = cfg->n_q_heads, s.G = cfg->n_kv_heads, s.D = cfg->head_dim;
  s.paged = cfg->block_tokens != 0;
  s.log2_T = 0;
  while (s.paged && (1 << s.log2_T) < cfg->block_tokens) ++s.log2_T;
  s.tcap = s.paged ? cfg->block_tokens : cfg->max_ctx;
  s.gg = okv::kv_head_group(s.G, s.D);
  s.st_log2 = okv::slab_tiles_log2(s.G, s.D, s.tcap);
  s.max_blocks = s.paged ? cfg->max_blocks_per_seq : 1;
  ctx->block_bytes = (int64_t)2 * s.G * s.tcap * s.D * 2;
  ctx->by_class = by_class;
  ctx->resident_blocks = cfg->resident_blocks;
  ctx->chunk_blocks = cfg->chunk_blocks;
  ctx->n_cls = max_classes_of(cfg);

  // workspace: [max_items * H][D] floats of weighted sums, then [max_items * H][2] floats
  const int64_t per_item = bytes_per_item(cfg);
  int64_t max_items = cfg->workspace_bytes / per_item;
  max_items = std::min<int64_t>(max_items, (int64_t)cfg->max_batch * ctx->cap_tokens);
  max_items = std::min<int64_t>(max_items, 0x7fffffff / (3 * (int64_t)std::max(1, s.H)));
  ctx->max_items = max_items;
  ctx->part_o = static_cast<float *>(cfg->workspace);
  ctx->part_ml = ctx->part_o + max_items * s.H * s.D;

  auto bail = [&](int code) {
    std::string msg = ctx->err;
    okv_destroy(ctx);
    g_error = msg;
    return code;
  };
#define OKV_TRY_CREATE(expr)                                                   \
  do {                                                                         \
    hipError_t e_ = (expr);                                                    \
    if (e_ != hipSuccess) {                                                    \
      fail(ctx, OKV_EHIP, "okv_create: %s: %s", #expr, hipGetErrorString(e_)); \
      return bail(OKV_EHIP);                                                   \
    }                                                                          \
  } while (0)
  const size_t tbl = (size_t)cfg->max_batch * s.max_blocks * sizeof(int32_t);
  OKV_TRY_CREATE(hipMalloc(&ctx->d_block_table, tbl));
  OKV_TRY_CREATE(hipMemset(ctx->d_block_table, 0, tbl));
  OKV_TRY_CREATE(hipMalloc(&ctx->d_ctx_lens, (size_t)cfg->max_batch * sizeof(int32_t)));
  OKV_TRY_CREATE(hipMalloc(&ctx->d_chunk_prefix, ((size_t)cfg->max_batch * ctx->n_cls + 1) * sizeof(int32_t)));
  if (by_class) {
    OKV_TRY_CREATE(hipMalloc(&ctx->d_pair_first, ((size_t)cfg->max_batch * ctx->n_cls + 1) * sizeof(int32_t)));
    OKV_TRY_CREATE(hipMalloc(&ctx->d_seq_total, (size_t)cfg->max_batch * sizeof(int32_t)));
  }
  OKV_TRY_CREATE(hipMalloc(&ctx->d_item_desc, (size_t)std::max<int64_t>(1, max_items) * sizeof(int4)));
  if (cfg->tail_blocks) {
    ctx->tail_on = true;
    ctx->tail_layer_stride = (int64_t)2 * cfg->max_batch * (ctx->block_bytes / 2);
    OKV_TRY_CREATE(hipMalloc(&ctx->d_tail_from, (size_t)cfg->max_batch * sizeof(int32_t)));
    OKV_TRY_CREATE(hipMalloc(&ctx->d_host_ptrs, (size_t)L * sizeof(void *)));
    OKV_TRY_CREATE(hipMemcpy(ctx->d_host_ptrs, ctx->host_pool.data(), (size_t)L * sizeof(void *), hipMemcpyHostToDevice));
    OKV_TRY_CREATE(hipEventCreateWithFlags(&ctx->flush_ev, hipEventDisableTiming));
  }
  {
    int dev = 0, cus = 0;
    OKV_TRY_CREATE(hipGetDevice(&dev));
    OKV_TRY_CREATE(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    const int group = cfg->n_q_heads / cfg->n_kv_heads;
    ctx->max_waves = std::max(1, cus) * (group == 1 ? OKV_WAVES_PER_CU_MHA : group < 8 ? OKV_WAVES_PER_CU_GQA : OKV_WAVES_PER_CU_MFMA);
    ctx->max_groups = std::min(std::max(1, ctx->max_waves / cfg->n_kv_heads), okv::kHeadGroupsMax);
    if (cfg->n_kv_heads > ctx->max_waves) {              // a stretch needs a wavefront per KV head
      fail(ctx, OKV_EINVAL, "okv_create: %d KV heads, a launch on this device has %d wavefronts", cfg->n_kv_heads, ctx->max_waves);
      return bail(OKV_EINVAL);
    }
  }
  OKV_TRY_CREATE(hipMalloc(&ctx->d_group_first, ((size_t)ctx->max_groups + 1) * sizeof(int32_t)));
  OKV_TRY_CREATE(hipMemset(ctx->d_group_first, 0, ((size_t)ctx->max_groups + 1) * sizeof(int32_t)));
  OKV_TRY_CREATE(hipMalloc(&ctx->d_pair_head, (size_t)max_pairs(ctx->max_waves) * okv::kPairHeadBytes));
  OKV_TRY_CREATE(hipMemset(ctx->d_pair_head, 0, (size_t)max_pairs(ctx->max_waves) * okv::kPairHeadBytes));
  OKV_TRY_CREATE(hipMalloc(&ctx->d_plan, 4 * sizeof(int32_t)));
  if (n_staging >= 2) OKV_TRY_CREATE(own_queue_stream(&ctx->h2d_odd));
  ctx->steps_ahead = !any_host ? 0 : by_class ? OKV_STEPS_AHEAD : OKV_STEPS_AHEAD_LAYERS;
  if (ctx->steps_ahead > 0)
    for (hipEvent_t &e : ctx->step_done_ev) OKV_TRY_CREATE(hipEventCreateWithFlags(&e, hipEventDisableTiming));
  for (int i = 0; i < kEventRing; ++i) {
    OKV_TRY_CREATE(hipEventCreateWithFlags(&ctx->ready_ev[i], hipEventDisableTiming));
    OKV_TRY_CREATE(hipEventCreateWithFlags(&ctx->consumed_ev[i], hipEventDisableTiming));
  }
#undef OKV_TRY_CREATE
  *out = ctx;
  return OKV_OK;
}

int okv_destroy(okv_ctx *ctx) {
  if (!ctx) return OKV_OK;
  if (ctx->h2d) (void)hipStreamSynchronize(ctx->h2d);
  if (ctx->h2d_odd) {
    (void)hipStreamSynchronize(ctx->h2d_odd);
    (void)hipStreamDestroy(ctx->h2d_odd);
  }
  (void)hipStreamSynchronize(ctx->compute);
  (void)hipFree(ctx->d_tail_from);
  (void)hipFree(ctx->d_host_ptrs);
  if (ctx->flush_ev) (void)hipEventDestroy(ctx->flush_ev);
  for (hipEvent_t e : ctx->step_done_ev)
    if (e) (void)hipEventDestroy(e);
  (void)hipFree(ctx->d_block_table);
  (void)hipFree(ctx->d_ctx_lens);
  (void)hipFree(ctx->d_chunk_prefix);
  (void)hipFree(ctx->d_item_desc);
  (void)hipFree(ctx->d_group_first);
  (void)hipFree(ctx->d_pair_head);
  (void)hipFree(ctx->d_plan);
  (void)hipFree(ctx->d_items_dump);
  if (ctx->d2h) {
    (void)hipStreamSynchronize(ctx->d2h);
    (void)hipStreamDestroy(ctx->d2h);
  }
  for (int i = 0; i < kEventRing; ++i) {
    if (ctx->filled_ev[i]) (void)hipEventDestroy(ctx->filled_ev[i]);
    if (ctx->copied_ev[i]) (void)hipEventDestroy(ctx->copied_ev[i]);
  }
  if (ctx->rows_ready_ev) (void)hipEventDestroy(ctx->rows_ready_ev);
  if (ctx->prefill_done_ev) (void)hipEventDestroy(ctx->prefill_done_ev);
  for (hipEvent_t e : ctx->stored_ev)
    if (e) (void)hipEventDestroy(e);
  (void)hipFree(ctx->d_tiles);
  (void)hipFree(ctx->d_row_base);
  (void)hipFree(ctx->d_runs);
  (void)hipFree(ctx->d_pair_first);
  (void)hipFree(ctx->d_seq_total);
  for (int i = 0; i < kEventRing; ++i) {
    if (ctx->ready_ev[i]) (void)hipEventDestroy(ctx->ready_ev[i]);
    if (ctx->consumed_ev[i]) (void)hipEventDestroy(ctx->consumed_ev[i]);
  }
  for (auto &p : ctx->prof_events) {
    (void)hipEventDestroy(p.first);
    (void)hipEventDestroy(p.second);
  }
  delete ctx;
  return OKV_OK;
}

const char *okv_last_error(const okv_ctx *ctx) { return ctx ? ctx->err.c_str() : g_error.c_str(); }

int okv_synchronize(okv_ctx *ctx) {
  if (!ctx) return fail(nullptr, OKV_EINVAL, "ctx is NULL");
  if (ctx->any_host) OKV_HIP(ctx, hipStreamSynchronize(ctx->h2d));
  if (ctx->h2d_odd) OKV_HIP(ctx, hipStreamSynchronize(ctx->h2d_odd));
  if (ctx->d2h) OKV_HIP(ctx, hipStreamSynchronize(ctx->d2h));
  OKV_HIP(ctx, hipStreamSynchronize(ctx->compute));
  return OKV_OK;
}

int okv_set_batch(okv_ctx *ctx, int32_t B, const int32_t *block_table, const int32_t *ctx_lens) {
  if (!ctx) return fail(nullptr, OKV_EINVAL, "ctx is NULL");
  if (ctx->in_step || ctx->in_prefill) return fail(ctx, OKV_ESTATE, "okv_set_batch inside a step or a prefill");
  if (B < 1 || B > ctx->cfg.max_batch) return fail(ctx, OKV_EINVAL, "B = %d outside [1, %d]", B, ctx->cfg.max_batch);
  if (!ctx_lens) return fail(ctx, OKV_EINVAL, "ctx_lens is NULL");
  const okv::PoolShape &s = ctx->shape;
  if (s.paged && !block_table) return fail(ctx, OKV_EINVAL, "block_table is NULL");
  int64_t max_blk = -1;
  if (s.paged) {
    std::vector<uint8_t> seen((size_t)ctx->cfg.blocks_per_layer, 0);
    for (int32_t b = 0; b < B; ++b)
      for (int32_t i = 0; i < s.max_blocks; ++i) {
        int32_t id = block_table[(size_t)b * s.max_blocks + i];
        if (id == -1) continue;
        if (id < 0 || id >= ctx->cfg.blocks_per_layer)
          return fail(ctx, OKV_EINVAL, "block_table[%d][%d] = %d outside [0, %lld)", b, i, id, (long long)ctx->cfg.blocks_per_layer);
        if (seen[id]) return fail(ctx, OKV_EINVAL, "block %d appears twice in the block table", id);
        seen[id] = 1;
        max_blk = std::max<int64_t>(max_blk, id);
      }
  }
  for (int32_t b = 0; b < B; ++b) {
    if (ctx_lens[b] < 0 || ctx_lens[b] > ctx->cap_tokens)
      return fail(ctx, OKV_EINVAL, "ctx_lens[%d] = %d outside [0, %d]", b, ctx_lens[b], ctx->cap_tokens);
    if (s.paged) {
      int32_t need = (ctx_lens[b] + ctx->cfg.block_tokens - 1) >> s.log2_T;
      for (int32_t i = 0; i < need; ++i)
        if (block_table[(size_t)b * s.max_blocks + i] < 0)
          return fail(ctx, OKV_EINVAL, "sequence %d holds %d tokens but block %d is not allocated", b, ctx_lens[b], i);
    }
  }
  int rc = tail_flush_all(ctx);                          // rows of the batch that is being replaced
  if (rc) return rc;
  rc = okv_synchronize(ctx);
  if (rc) return rc;
  ctx->batch_set = false;
  ctx->B = B;
  ctx->h_ctx_lens.assign(ctx_lens, ctx_lens + B);
  if (s.paged) {
    ctx->h_block_table.assign(block_table, block_table + (size_t)B * s.max_blocks);
    OKV_HIP(ctx, hipMemcpy(ctx->d_block_table, block_table, (size_t)B * s.max_blocks * sizeof(int32_t), hipMemcpyHostToDevice));
    ctx->copy_bytes = (max_blk + 1) * ctx->block_bytes;
  } else {
    ctx->copy_bytes = (int64_t)B * ctx->block_bytes;
  }
  OKV_HIP(ctx, hipMemcpy(ctx->d_ctx_lens, ctx_lens, (size_t)B * sizeof(int32_t), hipMemcpyHostToDevice));
  ctx->unit_offset.assign(1, 0);
  ctx->unit_bytes.assign(1, ctx->copy_bytes);
  if (ctx->by_class) {
    // runs of one class per sequence, and the chunks of the host pool the batch touches
    okv::build_runs(block_table, B, s.max_blocks, ctx->cfg.block_tokens, ctx->resident_blocks, ctx->chunk_blocks,
                    ctx->n_cls, ctx->h_runs, ctx->h_pair_first);
    std::vector<int64_t> used(ctx->n_cls, 0);            // blocks of each class up to the highest id in the table
    for (int32_t b = 0; b < B; ++b)
      for (int32_t i = 0; i < s.max_blocks; ++i) {
        const int64_t id = block_table[(size_t)b * s.max_blocks + i];
        if (id < ctx->resident_blocks) continue;          // in HBM, or not allocated
        const int64_t local = id - ctx->resident_blocks;
        const int64_t chunk = local / ctx->chunk_blocks;
        used[1 + chunk] = std::max(used[1 + chunk], local - chunk * ctx->chunk_blocks + 1);
      }
    ctx->active_chunks.clear();
    ctx->unit_offset.clear();
    ctx->unit_bytes.clear();
    for (int32_t c = 1; c < ctx->n_cls; ++c)
      if (used[c] > 0) {
        ctx->active_chunks.push_back(c - 1);
        ctx->unit_offset.push_back((int64_t)(c - 1) * ctx->chunk_blocks * ctx->block_bytes);
        ctx->unit_bytes.push_back(used[c] * ctx->block_bytes);
      }
    ctx->has_resident = ctx->h_pair_first[B] > 0;         // some run of class 0
    const int64_t n_runs = (int64_t)ctx->h_runs.size();
    if (n_runs > ctx->runs_cap) {
      (void)hipFree(ctx->d_runs);
      ctx->d_runs = nullptr;
      ctx->runs_cap = 0;
      OKV_HIP(ctx, hipMalloc(&ctx->d_runs, (size_t)n_runs * sizeof(int4)));
      ctx->runs_cap = n_runs;
    }
    static_assert(sizeof(okv::Run) == sizeof(int4), "runs are uploaded as they are");
    if (n_runs) OKV_HIP(ctx, hipMemcpy(ctx->d_runs, ctx->h_runs.data(), (size_t)n_runs * sizeof(int4), hipMemcpyHostToDevice));
    OKV_HIP(ctx, hipMemcpy(ctx->d_pair_first, ctx->h_pair_first.data(), ctx->h_pair_first.size() * sizeof(int32_t),
                           hipMemcpyHostToDevice));
  }
  reset_schedule(ctx);
  ctx->next_layer = 0;
  ctx->appended = false;
  rc = tail_restart(ctx);
  if (rc) return rc;
  ctx->batch_set = true;
  rc = rebuild_worklist(ctx, 0);
  if (rc) { ctx->batch_set = false; return rc; }
  return OKV_OK;
}

int okv_step_begin(okv_ctx *ctx) {
  if (!ctx) return fail(nullptr, OKV_EINVAL, "ctx is NULL");
  if (!ctx->batch_set) return fail(ctx, OKV_ESTATE, "okv_step_begin before okv_set_batch");
  if (ctx->in_step || ctx->in_prefill) return fail(ctx, OKV_ESTATE, "okv_step_begin inside a step or a prefill");
  const okv::PoolShape &s = ctx->shape;
  for (int32_t b = 0; b < ctx->B; ++b) {
    int32_t n = ctx->h_ctx_lens[b];
    if (n + 1 > ctx->cap_tokens) return fail(ctx, OKV_ENOSPC, "sequence %d is at its capacity of %d tokens", b, ctx->cap_tokens);
    if (s.paged && ctx->h_block_table[(size_t)b * s.max_blocks + (n >> s.log2_T)] < 0)
      return fail(ctx, OKV_ENOSPC, "sequence %d has no block allocated for token %d", b, n);
  }
  if (int rc = wait_for_earlier_steps(ctx)) return rc;
  // The first copies go out before anything is advanced: a failure here leaves the lengths as they were.
  // What it does leave is a copy pipeline in an unknown state, so the batch has to be described again.
  if (ctx->sched.n_units() > 0 && !ctx->sched.primed()) {
    std::vector<Op> ops;
    ctx->sched.prime(ops);
    const int rc = exec_ops(ctx, ops, nullptr, nullptr, nullptr);
    if (rc) {
      ctx->batch_set = false;
      return rc;
    }
  }
  for (int32_t b = 0; b < ctx->B; ++b) ctx->h_ctx_lens[b] += 1;
  const int rc = rebuild_worklist(ctx, 1);
  if (rc) {
    for (int32_t b = 0; b < ctx->B; ++b) ctx->h_ctx_lens[b] -= 1;
    // OKV_ENOSPC is found on the host before anything is enqueued; any other failure may have left the
    // device lengths advanced, and only okv_set_batch uploads them again
    if (rc != OKV_ENOSPC) ctx->batch_set = false;
    return rc;
  }
  if (ctx->tail_on) {
    tail_mark_chunks(ctx);
    ctx->tail_dirty = true;
  }
  ctx->in_step = true;
  ctx->next_layer = 0;
  ctx->appended = false;
  return OKV_OK;
}

int okv_step_abort(okv_ctx *ctx) {
  if (!ctx) return fail(nullptr, OKV_EINVAL, "ctx is NULL");
  if (!ctx->in_step) return fail(ctx, OKV_ESTATE, "okv_step_abort outside a step");
  // the layers visited so far hold this step's rows, the others do not, and the lengths have advanced:
  // nothing of that can be taken back, so the batch counts as not described
  ctx->in_step = false;
  ctx->appended = false;
  ctx->pending_k = ctx->pending_v = nullptr;
  ctx->prof_open = false;
  ctx->batch_set = false;
  return okv_synchronize(ctx);
}

int okv_step_end(okv_ctx *ctx) {
  if (!ctx) return fail(nullptr, OKV_EINVAL, "ctx is NULL");
  if (!ctx->in_step) return fail(ctx, OKV_ESTATE, "okv_step_end outside a step");
  if (ctx->next_layer != ctx->cfg.n_layers)
    return fail(ctx, OKV_ESTATE, "okv_step_end after %d of %d layers", ctx->next_layer, ctx->cfg.n_layers);
  if (ctx->prof_open) {
    OKV_HIP(ctx, hipEventRecord(ctx->prof_events[ctx->prof_used].second, ctx->compute));
    ++ctx->prof_used;
    ctx->prof_open = false;
  }
  if (ctx->tail_on) {
    const okv::PoolShape &s = ctx->shape;
    bool filled = false;
    for (int32_t b = 0; b < ctx->B && !filled; ++b)
      filled = okv::tail_fills(ctx->h_block_table.data(), b, s.max_blocks, s.log2_T, ctx->h_ctx_lens[b], ctx->h_tail_from[b],
                               ctx->resident_blocks);
    if (filled) {
      // after every layer's attention of this step (same stream); copies of the host pools enqueued
      // from now on wait for it, those already enqueued are made good from the slots
      OKV_HIP(ctx, okv::launch_tail_rows(tail_launch(ctx, 1), ctx->compute));
      OKV_HIP(ctx, hipEventRecord(ctx->flush_ev, ctx->compute));
      ctx->flush_recorded = true;
    }
  }
  if (int rc = mark_step_done(ctx)) return rc;
  ctx->in_step = false;
  ctx->step += 1;
  return OKV_OK;
}

int okv_flush_tails(okv_ctx *ctx) {
  if (!ctx) return fail(nullptr, OKV_EINVAL, "ctx is NULL");
  if (ctx->in_step || ctx->in_prefill) return fail(ctx, OKV_ESTATE, "okv_flush_tails inside a step or a prefill");
  if (!ctx->batch_set) return fail(ctx, OKV_ESTATE, "okv_flush_tails: no batch set");
  if (!ctx->tail_on) return okv_synchronize(ctx);
  if (!ctx->tail_dirty) return okv_synchronize(ctx);
  return tail_flush_all(ctx);
}

int kv_append(okv_ctx *ctx, int32_t layer, const void *k_new, const void *v_new) {
  if (!ctx) return fail(nullptr, OKV_EINVAL, "ctx is NULL");
  if (!ctx->in_step) return fail(ctx, OKV_ESTATE, "kv_append outside a step");
  if (layer < 0 || layer >= ctx->cfg.n_layers) return fail(ctx, OKV_EINVAL, "layer %d outside [0, %d)", layer, ctx->cfg.n_layers);
  if (layer != ctx->next_layer || ctx->appended)
    return fail(ctx, OKV_ESTATE, "kv_append(%d) out of order: expected %s(%d)", layer,
                ctx->appended ? "decode_attn" : "kv_append", ctx->next_layer);
  if (!k_new || !v_new || !aligned16(k_new) || !aligned16(v_new)) return fail(ctx, OKV_EINVAL, "k_new / v_new NULL or not 16-byte aligned");
  std::vector<Op> ops;
  ctx->sched.on_append(ctx->step, layer, ops);
  int rc = exec_ops(ctx, ops, k_new, v_new, nullptr);
  if (rc) return rc;
  ctx->appended = true;
  return OKV_OK;
}

int decode_attn(okv_ctx *ctx, int32_t layer, const void *q, void *out) {
  if (!ctx) return fail(nullptr, OKV_EINVAL, "ctx is NULL");
  if (!ctx->in_step) return fail(ctx, OKV_ESTATE, "decode_attn outside a step");
  if (layer < 0 || layer >= ctx->cfg.n_layers) return fail(ctx, OKV_EINVAL, "layer %d outside [0, %d)", layer, ctx->cfg.n_layers);
  if (layer != ctx->next_layer || !ctx->appended)
    return fail(ctx, OKV_ESTATE, "decode_attn(%d) out of order: expected %s(%d)", layer,
                ctx->appended ? "decode_attn" : "kv_append", ctx->next_layer);
  if (!q || !out || !aligned16(q) || !aligned16(out)) return fail(ctx, OKV_EINVAL, "q / out NULL or not 16-byte aligned");
  std::vector<Op> ops;
  ctx->sched.on_attn(ctx->step, layer, ops);
  int rc = exec_ops(ctx, ops, q, nullptr, out);
  if (rc) return rc;
  ctx->appended = false;
  ctx->next_layer = layer + 1;
  return OKV_OK;
}

int okv_decode_step(okv_ctx *ctx, const void *const *q, const void *const *k_new, const void *const *v_new,
                    void *const *out) {
  if (!ctx) return fail(nullptr, OKV_EINVAL, "ctx is NULL");
  if (!q || !k_new || !v_new || !out) return fail(ctx, OKV_EINVAL, "okv_decode_step: NULL pointer array");
  int rc = okv_step_begin(ctx);
  for (int32_t l = 0; rc == OKV_OK && l < ctx->cfg.n_layers; ++l) {
    rc = kv_append(ctx, l, k_new[l], v_new[l]);
    if (rc == OKV_OK) rc = decode_attn(ctx, l, q[l], out[l]);
  }
  return rc == OKV_OK ? okv_step_end(ctx) : rc;
}

// ---- bulk store of prompts ------------------------------------------------------------

int okv_prefill_begin(okv_ctx *ctx, const int32_t *n_new) {
  if (!ctx) return fail(nullptr, OKV_EINVAL, "ctx is NULL");
  if (!n_new) return fail(ctx, OKV_EINVAL, "n_new is NULL");
  if (!ctx->batch_set) return fail(ctx, OKV_ESTATE, "okv_prefill_begin before okv_set_batch");
  if (ctx->in_step || ctx->in_prefill) return fail(ctx, OKV_ESTATE, "okv_prefill_begin inside a step or a prefill");
  const okv::PoolShape &s = ctx->shape;
  const int32_t B = ctx->B;
  for (int32_t b = 0; b < B; ++b) {
    if (n_new[b] < 0) return fail(ctx, OKV_EINVAL, "n_new[%d] < 0", b);
    const int64_t end = (int64_t)ctx->h_ctx_lens[b] + n_new[b];
    if (end > ctx->cap_tokens) return fail(ctx, OKV_ENOSPC, "sequence %d would hold %lld tokens, capacity %d", b, (long long)end, ctx->cap_tokens);
    if (s.paged && n_new[b] > 0)
      for (int32_t i = ctx->h_ctx_lens[b] >> s.log2_T; i <= (int32_t)((end - 1) >> s.log2_T); ++i)
        if (ctx->h_block_table[(size_t)b * s.max_blocks + i] < 0)
          return fail(ctx, OKV_ENOSPC, "sequence %d has no block allocated for token %d", b, i << s.log2_T);
  }
  int rc = tail_flush_all(ctx);                         // the prompt's rows go to the pools, past what decode steps left in the slots
  if (rc) return rc;
  rc = okv_synchronize(ctx);                            // a change of phase: nothing of a decode step is left in flight
  if (rc) return rc;
  // 16-position tiles that receive rows.  A tile is (sequence, tile, first and last position
  // inside it, destination block relative to the pool the launch writes into).
  auto tile_desc = [](int32_t b, int32_t t, int32_t lo, int32_t hi, int32_t dest) {
    return make_int4(b, t, (lo - (t << 4)) | ((hi - (t << 4)) << 8), dest);
  };
  struct HostTile { int32_t b, t, lo, hi; int64_t blk; };   // blk: index in the host pool
  std::vector<int4> all, hbm;
  std::vector<HostTile> host;
  std::vector<int32_t> row_base(B);
  const bool any_resident_layer = !ctx->by_class && std::any_of(ctx->dev_pool.begin(), ctx->dev_pool.end(), [](void *p) { return p != nullptr; });
  const bool any_host_layer = !ctx->by_class && ctx->any_host;
  int64_t row = 0;
  for (int32_t b = 0; b < B; ++b) {
    const int32_t lo = ctx->h_ctx_lens[b], hi = lo + n_new[b];
    row_base[b] = (int32_t)(row - lo);
    row += n_new[b];
    for (int32_t t = lo >> 4; (t << 4) < hi; ++t) {
      const int32_t t_lo = std::max(lo, t << 4), t_hi = std::min(hi, (t << 4) + 16);
      const int64_t id = s.paged ? ctx->h_block_table[(size_t)b * s.max_blocks + ((t << 4) >> s.log2_T)] : b;
      if (ctx->by_class) {
        if (id < ctx->resident_blocks) hbm.push_back(tile_desc(b, t, t_lo, t_hi, (int32_t)id));
        else host.push_back(HostTile{b, t, t_lo, t_hi, id - ctx->resident_blocks});
      } else {
        if (any_resident_layer) all.push_back(tile_desc(b, t, t_lo, t_hi, (int32_t)id));
        if (any_host_layer) host.push_back(HostTile{b, t, t_lo, t_hi, id});
      }
    }
  }
  if (row > 0x7fffffff) return fail(ctx, OKV_EINVAL, "too many new rows");
  // Host side.  A block whose first stored position is its first slot holds nothing old, so it may
  // be assembled in a staging buffer and copied over whole (slots past the new rows are unused and
  // may hold anything).  Such blocks are sorted by id; neighbours in the host pool become one copy.
  // Everything else (a prompt that continues in the middle of a block, contiguous pools, blocks
  // scattered one by one) is written by the kernel straight through the mapped pointer.
  std::vector<int4> direct;
  std::vector<std::vector<int4>> group_tiles;
  ctx->groups.clear();
  if (!host.empty()) {
    std::vector<int64_t> fresh;                          // host blocks that are written from their first slot
    if (s.paged) {
      for (const HostTile &h : host)
        if (((h.t << 4) & (s.tcap - 1)) == 0 && h.lo == (h.t << 4)) fresh.push_back(h.blk);
      std::sort(fresh.begin(), fresh.end());
    }
    int64_t n_runs = 0;
    for (size_t i = 0; i < fresh.size(); ++i) n_runs += i == 0 || fresh[i] != fresh[i - 1] + 1;
    const int64_t cap_blocks = ctx->n_staging > 0 ? ctx->cfg.staging_bytes / ctx->block_bytes : 0;
    const bool staged = n_runs > 0 && cap_blocks > 0 && (int64_t)fresh.size() * ctx->block_bytes >= n_runs * kMinStagedRunBytes;
    if (!staged) fresh.clear();
    auto rank_of = [&](int64_t blk) -> int64_t {
      auto it = std::lower_bound(fresh.begin(), fresh.end(), blk);
      return it != fresh.end() && *it == blk ? it - fresh.begin() : -1;
    };
    const int64_t n_groups = staged ? ((int64_t)fresh.size() + cap_blocks - 1) / cap_blocks : 0;
    group_tiles.resize(n_groups);
    ctx->groups.resize(n_groups);
    for (const HostTile &h : host) {
      const int64_t r = rank_of(h.blk);
      if (r < 0) direct.push_back(tile_desc(h.b, h.t, h.lo, h.hi, (int32_t)h.blk));
      else group_tiles[r / cap_blocks].push_back(tile_desc(h.b, h.t, h.lo, h.hi, (int32_t)(r % cap_blocks)));
    }
    for (int64_t g = 0; g < n_groups; ++g) {
      const int64_t first = g * cap_blocks, last = std::min<int64_t>((int64_t)fresh.size(), first + cap_blocks);
      for (int64_t i = first; i < last;) {
        int64_t e = i + 1;
        while (e < last && fresh[e] == fresh[e - 1] + 1) ++e;
        ctx->groups[g].runs.push_back(okv_ctx::CopyRun{fresh[i] * ctx->block_bytes, (i - first) * ctx->block_bytes,
                                                      (e - i) * ctx->block_bytes});
        i = e;
      }
    }
  }
  // one device array, one span per launch
  std::vector<int4> flat;
  auto add_span = [&](const std::vector<int4> &v) {
    okv_ctx::TileSpan sp;
    sp.first = (int32_t)flat.size();
    sp.count = (int32_t)v.size();
    flat.insert(flat.end(), v.begin(), v.end());
    return sp;
  };
  ctx->tiles_all = add_span(all);
  ctx->tiles_hbm = add_span(hbm);
  ctx->tiles_direct = add_span(direct);
  for (size_t g = 0; g < group_tiles.size(); ++g) ctx->groups[g].tiles = add_span(group_tiles[g]);
  const int64_t n_tiles = (int64_t)flat.size();
  if (n_tiles > ctx->tiles_cap) {
    (void)hipFree(ctx->d_tiles);
    ctx->d_tiles = nullptr;
    ctx->tiles_cap = 0;
    OKV_HIP(ctx, hipMalloc(&ctx->d_tiles, (size_t)n_tiles * sizeof(int4)));
    ctx->tiles_cap = n_tiles;
  }
  if (!ctx->d_row_base) OKV_HIP(ctx, hipMalloc(&ctx->d_row_base, (size_t)ctx->cfg.max_batch * sizeof(int32_t)));
  if (n_tiles) OKV_HIP(ctx, hipMemcpy(ctx->d_tiles, flat.data(), (size_t)n_tiles * sizeof(int4), hipMemcpyHostToDevice));
  OKV_HIP(ctx, hipMemcpy(ctx->d_row_base, row_base.data(), (size_t)B * sizeof(int32_t), hipMemcpyHostToDevice));
  if (!ctx->d2h) {
    OKV_HIP(ctx, own_queue_stream(&ctx->d2h));
    OKV_HIP(ctx, hipEventCreateWithFlags(&ctx->rows_ready_ev, hipEventDisableTiming));
    OKV_HIP(ctx, hipEventCreateWithFlags(&ctx->prefill_done_ev, hipEventDisableTiming));
    for (int i = 0; i < kEventRing; ++i) {
      OKV_HIP(ctx, hipEventCreateWithFlags(&ctx->filled_ev[i], hipEventDisableTiming));
      OKV_HIP(ctx, hipEventCreateWithFlags(&ctx->copied_ev[i], hipEventDisableTiming));
    }
    ctx->stored_ev.assign(ctx->cfg.n_layers, nullptr);
    for (int32_t l = 0; l < ctx->cfg.n_layers; ++l)
      OKV_HIP(ctx, hipEventCreateWithFlags(&ctx->stored_ev[l], hipEventDisableTiming));
  }
  ctx->stored_set.assign(ctx->cfg.n_layers, 0);
  ctx->h_n_new.assign(n_new, n_new + B);
  ctx->group_counter = 0;                                // okv_synchronize above: no staged group is in flight
  ctx->in_prefill = true;
  ctx->prefill_next_layer = 0;
  return OKV_OK;
}

int kv_append_bulk(okv_ctx *ctx, int32_t layer, const void *k_rows, const void *v_rows) {
  if (!ctx) return fail(nullptr, OKV_EINVAL, "ctx is NULL");
  if (!ctx->in_prefill) return fail(ctx, OKV_ESTATE, "kv_append_bulk outside a prefill");
  if (layer < 0 || layer >= ctx->cfg.n_layers) return fail(ctx, OKV_EINVAL, "layer %d outside [0, %d)", layer, ctx->cfg.n_layers);
  if (layer != ctx->prefill_next_layer) return fail(ctx, OKV_ESTATE, "kv_append_bulk(%d) out of order: expected layer %d", layer, ctx->prefill_next_layer);
  if (!k_rows || !v_rows || !aligned16(k_rows) || !aligned16(v_rows)) return fail(ctx, OKV_EINVAL, "k_rows / v_rows NULL or not 16-byte aligned");
  okv::BulkLaunch a;
  a.shape = ctx->shape;
  a.row_base = ctx->d_row_base;
  a.k_rows = k_rows;
  a.v_rows = v_rows;
  // A bounded grid of wavefronts that each walk several tiles: with one short-lived workgroup per
  // four tiles the store ran at full speed alone (0.77 ms per 2 GiB layer) but took 3.2 ms on
  // average whenever a device-to-host copy was running beside it; bounded to 16384 workgroups 1.1 ms.
  a.max_workgroups = OKV_BULK_WORKGROUPS;
  a.throttle = 0;
  auto launch = [&](const okv_ctx::TileSpan &sp, void *pool, hipStream_t stream) -> hipError_t {
    a.tiles = ctx->d_tiles + sp.first;
    a.n_tiles = sp.count;
    a.pool = pool;
    return okv::launch_bulk_append(a, stream);
  };
  const bool host_layer = !ctx->by_class && ctx->host_pool[layer] != nullptr;
  // rows bound for HBM, on the compute stream
  if (!ctx->by_class && !host_layer) OKV_HIP(ctx, launch(ctx->tiles_all, ctx->dev_pool[layer], ctx->compute));
  if (ctx->by_class && ctx->tiles_hbm.count) OKV_HIP(ctx, launch(ctx->tiles_hbm, ctx->dev_pool[layer], ctx->compute));
  if (!ctx->by_class && !host_layer) {
    ctx->prefill_next_layer = layer + 1;
    return OKV_OK;
  }
  // blocks gathered in a staging buffer (compute stream) and copied over by hipMemcpyAsync
  for (const okv_ctx::StagedGroup &g : ctx->groups) {
    const int64_t n = ctx->group_counter++;
    const int buf = (int)(n % ctx->n_staging);
    if (n >= ctx->n_staging) OKV_HIP(ctx, hipStreamWaitEvent(ctx->compute, ctx->copied_ev[(n - ctx->n_staging) % kEventRing], 0));
    OKV_HIP(ctx, launch(g.tiles, ctx->cfg.staging[buf], ctx->compute));
    OKV_HIP(ctx, hipEventRecord(ctx->filled_ev[n % kEventRing], ctx->compute));
    OKV_HIP(ctx, hipStreamWaitEvent(ctx->d2h, ctx->filled_ev[n % kEventRing], 0));
    for (const okv_ctx::CopyRun &r : g.runs)
      OKV_HIP(ctx, hipMemcpyAsync(static_cast<char *>(ctx->host_pool[layer]) + r.host_off,
                                  static_cast<const char *>(ctx->cfg.staging[buf]) + r.staging_off, (size_t)r.bytes,
                                  hipMemcpyDeviceToHost, ctx->d2h));
    OKV_HIP(ctx, hipEventRecord(ctx->copied_ev[n % kEventRing], ctx->d2h));
  }
  // the rest straight into host memory, by a small kernel on the library's own stream once the rows are there
  if (ctx->tiles_direct.count) {
    OKV_HIP(ctx, hipEventRecord(ctx->rows_ready_ev, ctx->compute));
    OKV_HIP(ctx, hipStreamWaitEvent(ctx->d2h, ctx->rows_ready_ev, 0));
    a.max_workgroups = OKV_HOST_WRITE_WORKGROUPS;
    a.throttle = 1;
    OKV_HIP(ctx, launch(ctx->tiles_direct, ctx->host_pool[layer], ctx->d2h));
    OKV_HIP(ctx, hipEventRecord(ctx->stored_ev[layer], ctx->d2h));
    ctx->stored_set[layer] = 1;
  }
  ctx->prefill_next_layer = layer + 1;
  return OKV_OK;
}

int okv_prefill_plan(const okv_ctx *ctx, int64_t *staged_groups, int64_t *copies, int64_t *staged_tiles, int64_t *direct_tiles) {
  if (!ctx || !staged_groups || !copies || !staged_tiles || !direct_tiles) return OKV_EINVAL;
  *staged_groups = (int64_t)ctx->groups.size();
  *copies = 0;
  *staged_tiles = 0;
  for (const okv_ctx::StagedGroup &g : ctx->groups) {
    *copies += (int64_t)g.runs.size();
    *staged_tiles += g.tiles.count;
  }
  *direct_tiles = ctx->tiles_direct.count;
  return OKV_OK;
}

int okv_prefill_release(okv_ctx *ctx, int32_t layer) {
  if (!ctx) return fail(nullptr, OKV_EINVAL, "ctx is NULL");
  if (!ctx->in_prefill) return fail(ctx, OKV_ESTATE, "okv_prefill_release outside a prefill");
  if (layer < 0 || layer >= ctx->prefill_next_layer) return fail(ctx, OKV_EINVAL, "layer %d has not been stored in this prefill", layer);
  if (ctx->stored_set[layer]) OKV_HIP(ctx, hipStreamWaitEvent(ctx->compute, ctx->stored_ev[layer], 0));
  return OKV_OK;
}

int okv_prefill_end(okv_ctx *ctx) {
  if (!ctx) return fail(nullptr, OKV_EINVAL, "ctx is NULL");
  if (!ctx->in_prefill) return fail(ctx, OKV_ESTATE, "okv_prefill_end outside a prefill");
  if (ctx->prefill_next_layer != ctx->cfg.n_layers)
    return fail(ctx, OKV_ESTATE, "okv_prefill_end after %d of %d layers", ctx->prefill_next_layer, ctx->cfg.n_layers);
  // what follows (attention, copies of host pools) comes after every store of the prefill
  OKV_HIP(ctx, hipEventRecord(ctx->prefill_done_ev, ctx->d2h));
  OKV_HIP(ctx, hipStreamWaitEvent(ctx->compute, ctx->prefill_done_ev, 0));
  if (ctx->h2d != ctx->compute) OKV_HIP(ctx, hipStreamWaitEvent(ctx->h2d, ctx->prefill_done_ev, 0));
  if (ctx->h2d_odd) OKV_HIP(ctx, hipStreamWaitEvent(ctx->h2d_odd, ctx->prefill_done_ev, 0));
  for (int32_t b = 0; b < ctx->B; ++b) ctx->h_ctx_lens[b] += ctx->h_n_new[b];
  ctx->in_prefill = false;
  reset_schedule(ctx);
  if (int rc = tail_restart(ctx)) return rc;
  return rebuild_worklist(ctx, 0, /*upload_lens=*/true);
}

int okv_set_split_tokens(okv_ctx *ctx, int32_t split_tokens) {
  if (!ctx) return fail(nullptr, OKV_EINVAL, "ctx is NULL");
  if (split_tokens < 0) return fail(ctx, OKV_EINVAL, "split_tokens < 0");
  if (ctx->in_step) return fail(ctx, OKV_ESTATE, "okv_set_split_tokens inside a step");
  if (split_tokens > 0) {
    const int64_t S = std::max(split_tokens, 16);
    int64_t worst = (int64_t)ctx->cfg.max_batch * (((int64_t)ctx->cap_tokens + S - 1) / S);
    if (worst > ctx->max_items)
      return fail(ctx, OKV_ENOSPC, "split size %d can need %lld work items, workspace holds %lld", split_tokens,
                  (long long)worst, (long long)ctx->max_items);
  }
  ctx->split_override = split_tokens;
  if (ctx->batch_set) return rebuild_worklist(ctx, 0);
  return OKV_OK;
}

int32_t okv_get_split_tokens(const okv_ctx *ctx) { return ctx ? ctx->split : 0; }

int okv_get_ctx_lens(okv_ctx *ctx, int32_t *out) {
  if (!ctx || !out) return fail(ctx, OKV_EINVAL, "ctx or out is NULL");
  if (!ctx->batch_set) return fail(ctx, OKV_ESTATE, "no batch set");
  OKV_HIP(ctx, hipStreamSynchronize(ctx->compute));
  OKV_HIP(ctx, hipMemcpy(out, ctx->d_ctx_lens, (size_t)ctx->B * sizeof(int32_t), hipMemcpyDeviceToHost));
  return OKV_OK;
}

int okv_worklist(okv_ctx *ctx, int32_t from_device, int32_t *items, int64_t max_items, int64_t *n_items) {
  if (!ctx || !items || !n_items) return fail(ctx, OKV_EINVAL, "NULL argument");
  if (!ctx->batch_set) return fail(ctx, OKV_ESTATE, "no batch set");
  *n_items = ctx->n_items;
  if (ctx->n_items > max_items) return fail(ctx, OKV_ENOSPC, "work list has %d items", ctx->n_items);
  if (ctx->n_items == 0) return OKV_OK;
  if (from_device) {
    if (!ctx->d_items_dump) OKV_HIP(ctx, hipMalloc(&ctx->d_items_dump, (size_t)ctx->max_items * 3 * sizeof(int32_t)));
    okv::BatchState bs{ctx->d_block_table, ctx->d_ctx_lens, ctx->d_chunk_prefix, ctx->d_item_desc, ctx->B, ctx->split,
                       ctx->n_items, ctx->n_cls};
    OKV_HIP(ctx, okv::launch_worklist_dump(bs, ctx->d_items_dump, ctx->compute));
    OKV_HIP(ctx, hipStreamSynchronize(ctx->compute));
    OKV_HIP(ctx, hipMemcpy(items, ctx->d_items_dump, (size_t)ctx->n_items * 3 * sizeof(int32_t), hipMemcpyDeviceToHost));
    return OKV_OK;
  }
  // host walk: the same arithmetic the device kernel runs
  int64_t it = 0;
  if (ctx->by_class) {
    for (const okv::Run &r : ctx->h_runs) {               // sorted by (class, sequence, position)
      int32_t sz;
      const int32_t n = ctx->h_ctx_lens[r.b];
      const int32_t cnt = okv::run_items(r.lo, r.hi_cap, n, ctx->split, &sz);
      const int32_t end = std::min(r.hi_cap, n);
      for (int32_t c = 0; c < cnt; ++c, ++it) {
        items[it * 3 + 0] = r.b, items[it * 3 + 1] = r.lo + c * sz, items[it * 3 + 2] = std::min(r.lo + (c + 1) * sz, end);
      }
    }
    return OKV_OK;
  }
  if (ctx->spans) {
    int64_t first = 0;
    for (int32_t b = 0; b < ctx->B; ++b) {
      const int32_t n = ctx->h_ctx_lens[b];
      const int64_t tiles = (n + 15) >> 4;
      int64_t k0, group;
      const int32_t cnt = okv::span_pieces(first, tiles, ctx->span_tiles, &k0);
      for (int32_t c = 0; c < cnt; ++c, ++it) {
        okv::ItemRange r = okv::span_piece(b, c, n, first, tiles, ctx->span_tiles, k0, &group);
        items[it * 3 + 0] = r.b, items[it * 3 + 1] = r.lo, items[it * 3 + 2] = r.hi;
      }
      first += tiles;
    }
    return OKV_OK;
  }
  for (int32_t b = 0; b < ctx->B; ++b) {
    int32_t cnt, sz;
    okv::seq_chunks(ctx->h_ctx_lens[b], ctx->split, &cnt, &sz);
    for (int32_t c = 0; c < cnt; ++c, ++it) {
      okv::ItemRange r = okv::chunk_range(b, c, sz, ctx->h_ctx_lens[b]);
      items[it * 3 + 0] = r.b, items[it * 3 + 1] = r.lo, items[it * 3 + 2] = r.hi;
    }
  }
  return OKV_OK;
}

int okv_pair_heads(okv_ctx *ctx, int32_t *records, int64_t max_records, int64_t *n_records) {
  if (!ctx || !records || !n_records) return fail(ctx, OKV_EINVAL, "NULL argument");
  if (!ctx->batch_set) return fail(ctx, OKV_ESTATE, "no batch set");
  if (!ctx->spans) return fail(ctx, OKV_ESTATE, "okv_pair_heads: the work list is not cut into equal stretches");
  const int64_t n = std::min<int64_t>((int64_t)ctx->n_groups * ctx->shape.G, max_pairs(ctx->max_waves));
  *n_records = n;
  if (n > max_records) return fail(ctx, OKV_ENOSPC, "okv_pair_heads: %lld records", (long long)n);
  OKV_HIP(ctx, hipStreamSynchronize(ctx->compute));
  OKV_HIP(ctx, hipMemcpy(records, ctx->d_pair_head, (size_t)n * okv::kPairHeadBytes, hipMemcpyDeviceToHost));
  return OKV_OK;
}

int okv_worklist_classes(okv_ctx *ctx, int32_t from_device, int32_t *class_first, int32_t max_classes, int32_t *n_classes) {
  if (!ctx || !class_first || !n_classes) return fail(ctx, OKV_EINVAL, "NULL argument");
  if (!ctx->batch_set) return fail(ctx, OKV_ESTATE, "no batch set");
  *n_classes = ctx->n_cls;
  if (ctx->n_cls + 1 > max_classes) return fail(ctx, OKV_ENOSPC, "%d classes", ctx->n_cls);
  if (from_device) {
    OKV_HIP(ctx, hipStreamSynchronize(ctx->compute));
    for (int32_t c = 0; c <= ctx->n_cls; ++c)             // chunk_prefix[cls * B] = items before class cls
      OKV_HIP(ctx, hipMemcpy(class_first + c, ctx->d_chunk_prefix + (size_t)c * ctx->B, sizeof(int32_t), hipMemcpyDeviceToHost));
    return OKV_OK;
  }
  if (ctx->by_class) {
    for (int32_t c = 0; c <= ctx->n_cls; ++c) class_first[c] = ctx->cls_first[c];
  } else {
    class_first[0] = 0;
    class_first[1] = ctx->n_items;
  }
  return OKV_OK;
}

int okv_profile_enable(okv_ctx *ctx, int32_t on) {
  if (!ctx) return fail(nullptr, OKV_EINVAL, "ctx is NULL");
  if (on < 0 || on > 2) return fail(ctx, OKV_EINVAL, "okv_profile_enable: mode %d outside 0..2", on);
  if (ctx->in_step) return fail(ctx, OKV_ESTATE, "okv_profile_enable inside a step");
  ctx->profile = on;
  return OKV_OK;
}

int okv_profile_read(okv_ctx *ctx, double *attn_ms, int64_t *attn_launches) {
  if (!ctx || !attn_ms || !attn_launches) return fail(ctx, OKV_EINVAL, "NULL argument");
  OKV_HIP(ctx, hipStreamSynchronize(ctx->compute));
  double total = 0;
  for (size_t i = 0; i < ctx->prof_used; ++i) {
    float ms = 0;
    OKV_HIP(ctx, hipEventElapsedTime(&ms, ctx->prof_events[i].first, ctx->prof_events[i].second));
    total += ms;
  }
  // What a pair of event records costs with nothing between them (median of 15 pairs)
  // is taken off every bracket, so that the sum is kernel time, not kernel + markers.
  double overhead = 0;
  if (ctx->prof_used > 0) {
    hipEvent_t a, b;
    OKV_HIP(ctx, hipEventCreate(&a));
    OKV_HIP(ctx, hipEventCreate(&b));
    std::vector<float> gaps;
    for (int i = 0; i < 15; ++i) {
      hipError_t e = hipEventRecord(a, ctx->compute);
      if (e == hipSuccess) e = hipEventRecord(b, ctx->compute);
      if (e == hipSuccess) e = hipEventSynchronize(b);
      float ms = 0;
      if (e == hipSuccess) e = hipEventElapsedTime(&ms, a, b);
      if (e != hipSuccess) {
        (void)hipEventDestroy(a);
        (void)hipEventDestroy(b);
        return fail(ctx, OKV_EHIP, "okv_profile_read: %s", hipGetErrorString(e));
      }
      gaps.push_back(ms);
    }
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    std::sort(gaps.begin(), gaps.end());
    overhead = gaps[gaps.size() / 2];
  }
  total -= overhead * (double)ctx->prof_used;
  *attn_ms = total > 0 ? total : 0;
  *attn_launches = ctx->prof_launches;
  ctx->prof_used = 0;
  ctx->prof_launches = 0;
  return OKV_OK;
}

int okv_measure_h2d(void *dst, const void *src, int64_t bytes, int32_t reps, void *stream, double *gbps_median) {
  if (!dst || !src || bytes < 1 || reps < 1 || !gbps_median) return fail(nullptr, OKV_EINVAL, "okv_measure_h2d: bad argument");
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipEvent_t e0, e1;
  OKV_HIP(nullptr, hipEventCreate(&e0));
  OKV_HIP(nullptr, hipEventCreate(&e1));
  std::vector<double> rates;
  int rc = OKV_OK;
  for (int32_t i = 0; i < reps + 1 && rc == OKV_OK; ++i) {            // the first copy is a warm-up
    hipError_t e = hipEventRecord(e0, st);
    if (e == hipSuccess) e = hipMemcpyAsync(dst, src, (size_t)bytes, hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipEventRecord(e1, st);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (e != hipSuccess) rc = fail(nullptr, OKV_EHIP, "okv_measure_h2d: %s", hipGetErrorString(e));
    else if (i > 0) rates.push_back((double)bytes / (ms * 1e-3) / 1e9);
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc) return rc;
  std::sort(rates.begin(), rates.end());
  *gbps_median = rates[rates.size() / 2];
  return OKV_OK;
}

int okv_measure_d2h(void *dst, const void *src, int64_t bytes, int32_t reps, void *stream, double *gbps_median) {
  if (!dst || !src || bytes < 1 || reps < 1 || !gbps_median) return fail(nullptr, OKV_EINVAL, "okv_measure_d2h: bad argument");
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipEvent_t e0, e1;
  OKV_HIP(nullptr, hipEventCreate(&e0));
  OKV_HIP(nullptr, hipEventCreate(&e1));
  std::vector<double> rates;
  int rc = OKV_OK;
  for (int32_t i = 0; i < reps + 1 && rc == OKV_OK; ++i) {            // the first copy is a warm-up
    hipError_t e = hipEventRecord(e0, st);
    if (e == hipSuccess) e = hipMemcpyAsync(dst, src, (size_t)bytes, hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipEventRecord(e1, st);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (e != hipSuccess) rc = fail(nullptr, OKV_EHIP, "okv_measure_d2h: %s", hipGetErrorString(e));
    else if (i > 0) rates.push_back((double)bytes / (ms * 1e-3) / 1e9);
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc) return rc;
  std::sort(rates.begin(), rates.end());
  *gbps_median = rates[rates.size() / 2];
  return OKV_OK;
}

int okv_time_copies(okv_ctx *ctx, int32_t as_pipelined, int32_t n_steps, double *ms) {
  if (!ctx || !ms) return fail(ctx, OKV_EINVAL, "NULL argument");
  if (n_steps < 1) return fail(ctx, OKV_EINVAL, "okv_time_copies: n_steps < 1");
  if (!ctx->batch_set) return fail(ctx, OKV_ESTATE, "no batch set");
  if (ctx->in_step) return fail(ctx, OKV_ESTATE, "okv_time_copies inside a step");
  *ms = 0;
  if (ctx->sched.n_units() == 0) return OKV_OK;
  int rc = okv_synchronize(ctx);
  if (rc) return rc;
  hipEvent_t e0, e1;
  OKV_HIP(ctx, hipEventCreate(&e0));
  OKV_HIP(ctx, hipEventCreate(&e1));
  hipError_t e = hipSuccess;
  float t = 0;
  if (!as_pipelined) {
    e = hipEventRecord(e0, ctx->h2d);
    int buf = 0;
    for (int32_t step = 0; step < n_steps; ++step)
      for (int32_t l = 0; l < ctx->cfg.n_layers && e == hipSuccess; ++l) {
        if (!ctx->host_pool[l]) continue;
        for (size_t u = 0; u < ctx->unit_bytes.size() && e == hipSuccess; ++u) {
          const char *src = static_cast<const char *>(ctx->host_pool[l]) + ctx->unit_offset[u];
          e = hipMemcpyAsync(ctx->cfg.staging[buf], src, (size_t)ctx->unit_bytes[u], hipMemcpyHostToDevice, ctx->h2d);
          buf = (buf + 1) % ctx->n_staging;
        }
      }
    if (e == hipSuccess) e = hipEventRecord(e1, ctx->h2d);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    if (e == hipSuccess) e = hipEventElapsedTime(&t, e0, e1);
  } else {
    // the copy half of the steps exactly as the pipeline issues it: same streams, same waits for a buffer's
    // release and same records after every copy; where a step launches attention, the compute stream only
    // waits for the copy and hands the buffer back.  Like a step in the middle of a generation, the first one
    // finds its first copies done and the last one leaves those of the step after it in flight, so n_steps
    // steps move exactly n_steps times the offloaded bytes between the two synchronisations that bracket them.
    reset_schedule(ctx);
    std::vector<Op> ops;
    ctx->sched.prime(ops);
    for (const Op &op : ops)
      if (e == hipSuccess && op.kind == okv::OP_COPY && exec_op(ctx, op, nullptr, nullptr, nullptr) != OKV_OK) e = hipErrorUnknown;
    if (e == hipSuccess && okv_synchronize(ctx) != OKV_OK) e = hipErrorUnknown;
    ops.clear();
    const auto t0 = std::chrono::steady_clock::now();
    for (int32_t step = 0; step < n_steps && e == hipSuccess; ++step) {
      if (wait_for_earlier_steps(ctx) != OKV_OK) e = hipErrorUnknown;   // the host leads by as much as in real steps
      ops.clear();
      for (int32_t l = 0; l < ctx->cfg.n_layers; ++l) ctx->sched.on_attn(step, l, ops);
      for (const Op &op : ops) {
        if (e != hipSuccess) break;
        if (op.kind == okv::OP_COPY) {
          if (exec_op(ctx, op, nullptr, nullptr, nullptr) != OKV_OK) e = hipErrorUnknown;
        } else if (op.kind == okv::OP_ATTN && op.wait_idx >= 0) {
          e = hipStreamWaitEvent(ctx->compute, ctx->ready_ev[op.wait_idx % kEventRing], 0);
        } else if (op.kind == okv::OP_RELEASE) {
          e = hipEventRecord(ctx->consumed_ev[op.copy_idx % kEventRing], ctx->compute);
        }
      }
      if (e == hipSuccess && mark_step_done(ctx) != OKV_OK) e = hipErrorUnknown;
    }
    if (e == hipSuccess && okv_synchronize(ctx) != OKV_OK) e = hipErrorUnknown;
    t = (float)std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (e != hipSuccess) return fail(ctx, OKV_EHIP, "okv_time_copies: %s", hipGetErrorString(e));
  *ms = t / n_steps;
  // the staging buffers no longer hold what the pipeline had prefetched: start it afresh
  rc = okv_synchronize(ctx);
  reset_schedule(ctx);
  return rc;
}

// ---- linear layers ---------------------------------------------------------------------------

int okv_pack_linear_weight(void *dst, const void *src, int32_t n_out, int32_t n_in, void *stream) {
  if (!dst || !src || !aligned16(dst) || !aligned16(src)) return fail(nullptr, OKV_EINVAL, "okv_pack_linear_weight: NULL or misaligned pointer");
  if (n_out < 16 || n_out % 16 || n_in < 32 || n_in % 32) return fail(nullptr, OKV_EINVAL, "okv_pack_linear_weight: n_out must be a multiple of 16 and n_in of 32");
  OKV_HIP(nullptr, okv::launch_pack_weight(dst, src, n_out, n_in, static_cast<hipStream_t>(stream)));
  return OKV_OK;
}

namespace {
int device_cus() {
  static int cus = 0;                                   // one device per process in practice; re-read if it ever reports 0
  if (cus <= 0) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
      cus = 256;
  }
  return cus;
}
}  // namespace

namespace {
// Rows per launch for a batch of m rows: the fewest launches of (nearly) equal size, a multiple of 16 rows each
// but the last.  A launch takes OKV_LINEAR_MAX_ROWS_STAGED rows if the staged kernel takes the shape (with
// the workspace at hand: unknown = as much as okv_linear_workspace_bytes would ask for), else OKV_LINEAR_MAX_ROWS.
int32_t rows_per_launch(int32_t m, int32_t n_out, int32_t n_in, bool workspace_known, bool have_workspace, int64_t workspace_bytes) {
  if (m <= OKV_LINEAR_MAX_ROWS) return m;
  for (int32_t cap : {OKV_LINEAR_MAX_ROWS_STAGED, OKV_LINEAR_MAX_ROWS}) {
    const int32_t launches = (m + cap - 1) / cap;
    const int32_t rows = std::min(m, ((m + launches - 1) / launches + 15) / 16 * 16);
    const int32_t last = m % rows ? m % rows : rows;
    if (cap == OKV_LINEAR_MAX_ROWS) return rows;
    auto takes = [&](int32_t r) {
      return r <= OKV_LINEAR_MAX_ROWS ||
             okv::linear_staged_takes(r, n_out, n_in, device_cus(), workspace_known ? have_workspace : true,
                                      workspace_known ? workspace_bytes : INT64_MAX);
    };
    if (takes(rows) && takes(last)) return rows;
  }
  return m;
}
}  // namespace

int64_t okv_linear_workspace_bytes(int32_t m, int32_t n_out, int32_t n_in) {
  if (m < 1 || m > OKV_LINEAR_MAX_BATCH || n_out < 16 || n_out % 16 || n_in < 32 || n_in % 32)
    return fail(nullptr, OKV_EINVAL, "okv_linear_workspace_bytes: bad shape");
  const int32_t rows = rows_per_launch(m, n_out, n_in, false, false, 0), last = m % rows ? m % rows : rows;
  return std::max(okv::linear_workspace_bytes(rows, n_out, n_in, device_cus()), okv::linear_workspace_bytes(last, n_out, n_in, device_cus()));
}

namespace {
int linear_impl(const void *x, const void *w_packed, const void *bias, const void *residual, void *const *out, int32_t n_seg,
                int32_t m, int32_t n_out, int32_t n_in, int32_t relu, void *workspace, int64_t workspace_bytes,
                const void *ln_gamma, const void *ln_beta, void *ln_out, float ln_eps, void *stream, int32_t first_cols = 0) {
  if (!x || !w_packed || !out || !aligned16(x) || !aligned16(w_packed)) return fail(nullptr, OKV_EINVAL, "okv_linear: NULL or misaligned pointer");
  if (m < 1 || m > OKV_LINEAR_MAX_BATCH) return fail(nullptr, OKV_EINVAL, "okv_linear: m = %d outside [1, %d]", m, OKV_LINEAR_MAX_BATCH);
  if (n_out < 16 || n_out % 16 || n_in < 32 || n_in % 32 || n_in > (1 << 20))
    return fail(nullptr, OKV_EINVAL, "okv_linear: n_out must be a multiple of 16 and n_in of 32");
  if (n_seg < 1 || n_seg > 3 || (!first_cols && n_out % (16 * n_seg)))
    return fail(nullptr, OKV_EINVAL, "okv_linear: n_seg must be 1..3 and divide n_out / 16");
  if (residual && n_seg != 1) return fail(nullptr, OKV_EINVAL, "okv_linear: a residual needs n_seg = 1");
  if (first_cols && (n_seg < 2 || first_cols < 16 || first_cols % 16 || first_cols >= n_out || (n_out - first_cols) % (16 * (n_seg - 1))))
    return fail(nullptr, OKV_EINVAL, "okv_linear: widths of the output tensors must be multiples of 16 that add up to n_out");
  if (!aligned16(bias) || !aligned16(residual)) return fail(nullptr, OKV_EINVAL, "okv_linear: bias / residual misaligned");
  if (relu != 0 && relu != 1) return fail(nullptr, OKV_EINVAL, "okv_linear: relu must be 0 or 1");
  okv::LinearLaunch l;
  l.x = x, l.w_packed = w_packed, l.bias = bias, l.residual = residual;
  for (int s = 0; s < 3; ++s) {
    l.out[s] = s < n_seg ? out[s] : nullptr;
    if (s < n_seg && (!out[s] || !aligned16(out[s]))) return fail(nullptr, OKV_EINVAL, "okv_linear: out[%d] is NULL or misaligned", s);
  }
  l.n_seg = n_seg, l.m = m, l.n_out = n_out, l.n_in = n_in, l.relu = relu;
  l.first_cols = first_cols;
  if (workspace && (!aligned16(workspace) || workspace_bytes < 0)) return fail(nullptr, OKV_EINVAL, "okv_linear: workspace misaligned");
  l.workspace = workspace;
  l.workspace_bytes = workspace_bytes;
  l.n_cus = device_cus();
  l.ln_gamma = ln_gamma, l.ln_beta = ln_beta, l.ln_out = ln_out, l.ln_eps = ln_eps;
  // more rows than one launch takes: launches of (nearly) equal size, one after the other on the stream (they
  // share the workspace); each reads the weights again
  const int32_t rows = rows_per_launch(m, n_out, n_in, true, workspace != nullptr, workspace_bytes);
  const int64_t seg0 = first_cols ? first_cols : n_out / n_seg, seg = n_seg > 1 ? (n_out - seg0) / (n_seg - 1) : n_out;
  auto at = [](const void *p, int64_t halves) -> const void * { return p ? static_cast<const char *>(p) + halves * 2 : nullptr; };
  for (int32_t r0 = 0; r0 < m; r0 += rows) {
    okv::LinearLaunch part = l;
    part.m = std::min(rows, m - r0);
    part.x = at(x, (int64_t)r0 * n_in);
    part.residual = at(residual, (int64_t)r0 * n_out);
    part.ln_out = const_cast<void *>(at(ln_out, (int64_t)r0 * n_out));
    for (int s2 = 0; s2 < n_seg; ++s2) part.out[s2] = const_cast<void *>(at(out[s2], (int64_t)r0 * (s2 == 0 ? seg0 : seg)));
    OKV_HIP(nullptr, okv::launch_linear(part, static_cast<hipStream_t>(stream)));
  }
  return OKV_OK;
}
}  // namespace

int okv_linear(const void *x, const void *w_packed, const void *bias, const void *residual, void *const *out, int32_t n_seg,
               int32_t m, int32_t n_out, int32_t n_in, int32_t relu, void *workspace, int64_t workspace_bytes, void *stream) {
  return linear_impl(x, w_packed, bias, residual, out, n_seg, m, n_out, n_in, relu, workspace, workspace_bytes, nullptr, nullptr,
                     nullptr, 0.f, stream);
}

int okv_linear_qkv(const void *x, const void *w_packed, const void *bias, void *q, void *k, void *v, int32_t m, int32_t q_cols,
                   int32_t kv_cols, int32_t n_in, void *workspace, int64_t workspace_bytes, void *stream) {
  if (q_cols < 16 || kv_cols < 16 || q_cols % 16 || kv_cols % 16) return fail(nullptr, OKV_EINVAL, "okv_linear_qkv: widths must be multiples of 16");
  void *outs[3] = {q, k, v};
  return linear_impl(x, w_packed, bias, nullptr, outs, 3, m, q_cols + 2 * kv_cols, n_in, 0, workspace, workspace_bytes, nullptr, nullptr,
                     nullptr, 0.f, stream, q_cols == kv_cols ? 0 : q_cols);
}

int okv_linear_layernorm(const void *x, const void *w_packed, const void *bias, const void *residual, void *out, const void *gamma,
                         const void *beta, float eps, void *out_norm, int32_t m, int32_t n_out, int32_t n_in, int32_t relu,
                         void *workspace, int64_t workspace_bytes, void *stream) {
  if (!out || !gamma || !beta || !out_norm || !aligned16(out) || !aligned16(gamma) || !aligned16(beta) || !aligned16(out_norm))
    return fail(nullptr, OKV_EINVAL, "okv_linear_layernorm: NULL or misaligned pointer");
  if (n_out > 16384 || !(eps >= 0)) return fail(nullptr, OKV_EINVAL, "okv_linear_layernorm: n_out > 16384 or eps < 0");
  if (out == out_norm) return fail(nullptr, OKV_EINVAL, "okv_linear_layernorm: out and out_norm must differ");
  void *outs[1] = {out};
  return linear_impl(x, w_packed, bias, residual, outs, 1, m, n_out, n_in, relu, workspace, workspace_bytes, gamma, beta, out_norm,
                     eps, stream);
}

int okv_layernorm(const void *x, const void *gamma, const void *beta, void *out, int32_t m, int32_t h, float eps, void *stream) {
  if (!x || !gamma || !beta || !out || !aligned16(x) || !aligned16(gamma) || !aligned16(beta) || !aligned16(out))
    return fail(nullptr, OKV_EINVAL, "okv_layernorm: NULL or misaligned pointer");
  if (m < 1 || h < 8 || h % 8 || h > 16384 || !(eps >= 0)) return fail(nullptr, OKV_EINVAL, "okv_layernorm: bad shape or eps");
  OKV_HIP(nullptr, okv::launch_layernorm(x, gamma, beta, out, m, h, eps, static_cast<hipStream_t>(stream)));
  return OKV_OK;
}

namespace {
// the intermediate tensors of a decoder layer inside the scratch buffer, each rounded up to 256 bytes
struct DecoderScratch {
  char *a, *q, *k, *v, *t, *y, *z, *u;
  int64_t bytes;
};
DecoderScratch decoder_scratch(void *base, int32_t m, int32_t h1, int32_t kvw, int32_t h2) {
  DecoderScratch d;
  int64_t at = 0;
  auto take = [&](int64_t cols) {
    char *p = static_cast<char *>(base) + at;
    at += ((int64_t)m * cols * 2 + 255) / 256 * 256;
    return p;
  };
  d.a = take(h1), d.q = take(h1), d.k = take(kvw), d.v = take(kvw), d.t = take(h1), d.y = take(h1), d.z = take(h1), d.u = take(h2);
  d.bytes = at;
  return d;
}
}  // namespace

int64_t okv_decoder_scratch_bytes(const okv_ctx *ctx, int32_t m, int32_t h2) {
  if (!ctx) return fail(nullptr, OKV_EINVAL, "ctx is NULL");
  if (m < 1 || m > OKV_LINEAR_MAX_BATCH || h2 < 32 || h2 % 32) return fail(nullptr, OKV_EINVAL, "okv_decoder_scratch_bytes: bad shape");
  return decoder_scratch(nullptr, m, ctx->cfg.n_q_heads * ctx->cfg.head_dim, ctx->cfg.n_kv_heads * ctx->cfg.head_dim, h2).bytes;
}

int okv_decoder_step(okv_ctx *ctx, const okv_decoder_layer *layers, int32_t n_layers, int32_t h2, void *x, float eps,
                     void *scratch, int64_t scratch_bytes, void *workspace, int64_t workspace_bytes) {
  if (!ctx) return fail(nullptr, OKV_EINVAL, "ctx is NULL");
  if (!layers || !x || !scratch) return fail(ctx, OKV_EINVAL, "okv_decoder_step: NULL pointer");
  if (n_layers != ctx->cfg.n_layers) return fail(ctx, OKV_EINVAL, "okv_decoder_step: %d layers, the context has %d", n_layers, ctx->cfg.n_layers);
  if (ctx->cfg.out_dtype != 0) return fail(ctx, OKV_EINVAL, "okv_decoder_step: the attention output must be fp16 (out_dtype 0)");
  if (!ctx->batch_set) return fail(ctx, OKV_ESTATE, "okv_decoder_step before okv_set_batch");
  const int32_t m = ctx->B, h1 = ctx->cfg.n_q_heads * ctx->cfg.head_dim, kvw = ctx->cfg.n_kv_heads * ctx->cfg.head_dim;
  if (m < 1 || m > OKV_LINEAR_MAX_BATCH) return fail(ctx, OKV_EINVAL, "okv_decoder_step: batch %d outside [1, %d]", m, OKV_LINEAR_MAX_BATCH);
  if (h2 < 32 || h2 % 32 || h2 > 16384 * 8) return fail(ctx, OKV_EINVAL, "okv_decoder_step: bad feed-forward width %d", h2);
  if (((uintptr_t)scratch & 255) || !aligned16(x)) return fail(ctx, OKV_EINVAL, "okv_decoder_step: scratch or x misaligned");
  const DecoderScratch d = decoder_scratch(scratch, m, h1, kvw, h2);
  if (scratch_bytes < d.bytes) return fail(ctx, OKV_ENOSPC, "okv_decoder_step: scratch holds %lld bytes, %lld needed", (long long)scratch_bytes, (long long)d.bytes);
  for (int32_t l = 0; l < n_layers; ++l) {
    const okv_decoder_layer &w = layers[l];
    if (!w.ln1_gamma || !w.ln1_beta || !w.w_qkv || !w.w_o || !w.ln2_gamma || !w.ln2_beta || !w.w_ff1 || !w.w_ff2)
      return fail(ctx, OKV_EINVAL, "okv_decoder_step: layer %d has a NULL matrix or norm vector", l);
  }
  void *stream = ctx->compute;
  int rc = okv_step_begin(ctx);
  if (rc != OKV_OK) return rc;
  // from here on a failure leaves the step open, as it does when the calls are made one by one
  rc = okv_layernorm(x, layers[0].ln1_gamma, layers[0].ln1_beta, d.a, m, h1, eps, stream);
  for (int32_t l = 0; rc == OKV_OK && l < n_layers; ++l) {
    const okv_decoder_layer &w = layers[l];
    rc = okv_linear_qkv(d.a, w.w_qkv, w.b_qkv, d.q, d.k, d.v, m, h1, kvw, h1, workspace, workspace_bytes, stream);
    if (rc == OKV_OK) rc = kv_append(ctx, l, d.k, d.v);
    if (rc == OKV_OK) rc = decode_attn(ctx, l, d.q, d.t);
    // output projection + residual, and the second norm of its result on the same share reduction
    if (rc == OKV_OK)
      rc = okv_linear_layernorm(d.t, w.w_o, w.b_o, x, d.y, w.ln2_gamma, w.ln2_beta, eps, d.z, m, h1, h1, 0, workspace, workspace_bytes, stream);
    void *hidden[1] = {d.u};
    if (rc == OKV_OK) rc = okv_linear(d.z, w.w_ff1, w.b_ff1, nullptr, hidden, 1, m, h2, h1, 1, workspace, workspace_bytes, stream);
    if (rc != OKV_OK) break;
    if (l + 1 < n_layers) {                                // the next layer's first norm rides on the feed-forward block
      rc = okv_linear_layernorm(d.u, w.w_ff2, w.b_ff2, d.y, x, layers[l + 1].ln1_gamma, layers[l + 1].ln1_beta, eps, d.a, m, h1, h2, 0,
                                workspace, workspace_bytes, stream);
    } else {
      void *outs[1] = {x};
      rc = okv_linear(d.u, w.w_ff2, w.b_ff2, d.y, outs, 1, m, h1, h2, 0, workspace, workspace_bytes, stream);
    }
  }
  return rc == OKV_OK ? okv_step_end(ctx) : rc;
}

// ---- decode attention without any allocation ------------------------------------------------
//
// The work list, the stretch table and the split-K partial results of okv_decode_attn_static live in
// one array of device memory that is part of the library's code object: every GPU that loads the
// library holds its own copy until the process ends.  The name below stands for it in host code only;
// its device address is looked up once per device (hipGetSymbolAddress) and everything uses that.
}  // extern "C"

static __device__ __align__(256) unsigned char scratch[OKV_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
unsigned char *g_scratch_ptr[kMaxDevices] = {};
int g_scratch_cus[kMaxDevices] = {};

struct StaticLayout {            // offsets into the scratch array, each a multiple of 256
  int64_t item_desc, chunk_prefix, group_first, pair_head, plan, part_o, part_ml, bytes;
};
StaticLayout static_layout(int64_t max_items, int32_t B, int32_t max_groups, int32_t max_waves, int32_t H, int32_t D) {
  StaticLayout l;
  int64_t at = 0;
  auto take = [&](int64_t bytes) {
    const int64_t here = at;
    at += (bytes + 255) / 256 * 256;
    return here;
  };
  l.item_desc = take(max_items * (int64_t)sizeof(int4));
  l.chunk_prefix = take(((int64_t)B + 1) * 4);
  l.group_first = take(((int64_t)max_groups + 1) * 4);
  l.pair_head = take((int64_t)max_pairs(max_waves) * okv::kPairHeadBytes);
  l.plan = take(16);
  l.part_o = take(max_items * H * D * 4);
  l.part_ml = take(max_items * H * 2 * 4);
  l.bytes = at;
  return l;
}
}  // namespace

extern "C" {

int okv_decode_attn_static(const okv_static_attn *a) {
  if (!a) return fail(nullptr, OKV_EINVAL, "okv_decode_attn_static: NULL argument");
  okv_config c;
  memset(&c, 0, sizeof c);
  c.n_layers = 1, c.n_q_heads = a->n_q_heads, c.n_kv_heads = a->n_kv_heads, c.head_dim = a->head_dim;
  c.block_tokens = a->block_tokens, c.max_batch = a->B > 0 ? a->B : 1, c.max_blocks_per_seq = a->max_blocks_per_seq;
  c.max_ctx = a->max_ctx, c.blocks_per_layer = a->block_tokens ? 1 : 0, c.out_dtype = a->out_dtype;
  if (const char *why = shape_problem(&c)) return fail(nullptr, OKV_EINVAL, "okv_decode_attn_static: %s", why);
  if (a->B < 1 || a->B > OKV_STATIC_MAX_BATCH)
    return fail(nullptr, OKV_EINVAL, "okv_decode_attn_static: B = %d outside [1, %d]", a->B, OKV_STATIC_MAX_BATCH);
  if (!a->pool || !a->ctx_lens || !a->q || !a->out || (a->block_tokens && !a->block_table))
    return fail(nullptr, OKV_EINVAL, "okv_decode_attn_static: NULL pointer");
  if (!aligned16(a->pool) || !aligned16(a->q) || !aligned16(a->out) || !aligned16(a->k_new) || !aligned16(a->v_new))
    return fail(nullptr, OKV_EINVAL, "okv_decode_attn_static: pointer not 16-byte aligned");
  if ((a->k_new == nullptr) != (a->v_new == nullptr))
    return fail(nullptr, OKV_EINVAL, "okv_decode_attn_static: k_new and v_new go together");
  int dev = 0;
  OKV_HIP(nullptr, hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(nullptr, OKV_EINVAL, "okv_decode_attn_static: device %d not supported", dev);
  if (!g_scratch_ptr[dev]) {                             // first call on this device: where its copy of the array is
    void *p = nullptr;
    OKV_HIP(nullptr, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    int cus = 0;
    OKV_HIP(nullptr, hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    g_scratch_cus[dev] = cus > 0 ? cus : 256;
    g_scratch_ptr[dev] = static_cast<unsigned char *>(p);
  }
  unsigned char *base = g_scratch_ptr[dev];
  const int32_t H = a->n_q_heads, G = a->n_kv_heads, D = a->head_dim;
  const int32_t max_waves = g_scratch_cus[dev] * OKV_WAVES_PER_CU_MHA;
  if (G > max_waves)
    return fail(nullptr, OKV_EINVAL, "okv_decode_attn_static: %d KV heads, a launch on this device has %d wavefronts", G, max_waves);
  const int32_t max_groups = std::min(std::max(1, max_waves / G), okv::kHeadGroupsMax);
  // the lengths are on the device only: room for the most items any lengths can give (one per
  // sequence and one per stretch)
  const int64_t max_items = (int64_t)a->B + max_groups;
  const StaticLayout lay = static_layout(max_items, a->B, max_groups, max_waves, H, D);
  if (lay.bytes > (int64_t)OKV_STATIC_SCRATCH_BYTES)
    return fail(nullptr, OKV_ENOSPC,
                "okv_decode_attn_static: batch %d with %d query heads of %d needs %lld bytes of work space, the library holds %lld",
                a->B, H, D, (long long)lay.bytes, (long long)OKV_STATIC_SCRATCH_BYTES);
  hipStream_t stream = static_cast<hipStream_t>(a->stream);
  int32_t *chunk_prefix = reinterpret_cast<int32_t *>(base + lay.chunk_prefix);
  int4 *item_desc = reinterpret_cast<int4 *>(base + lay.item_desc);
  int32_t *group_first = reinterpret_cast<int32_t *>(base + lay.group_first);
  int32_t *plan = reinterpret_cast<int32_t *>(base + lay.plan);
  void *pair_head = base + lay.pair_head;
  okv::AttnLaunch l;
  okv::PoolShape &s = l.shape;
  s.H = H, s.G = G, s.D = D;
  s.paged = a->block_tokens != 0;
  s.log2_T = 0;
  while (s.paged && (1 << s.log2_T) < a->block_tokens) ++s.log2_T;
  s.tcap = s.paged ? a->block_tokens : a->max_ctx;
  s.gg = okv::kv_head_group(G, D);
  s.st_log2 = okv::slab_tiles_log2(G, D, s.tcap);
  s.max_blocks = s.paged ? a->max_blocks_per_seq : 1;
  OKV_HIP(nullptr, okv::launch_step_advance_spans(const_cast<int32_t *>(a->ctx_lens), chunk_prefix, item_desc, group_first, plan, a->B,
                                                  max_groups, kMinSpanTiles, 0, pair_head,
                                                  okv::head_geom(s, a->block_table, max_pairs(max_waves)), stream));
  l.batch = okv::BatchState{a->block_table, a->ctx_lens, chunk_prefix, item_desc, a->B, 0, (int32_t)max_items, 1};
  l.q = a->q;
  l.pool = const_cast<void *>(a->pool);
  l.k_new = a->k_new, l.v_new = a->v_new;
  l.pool_mirror = nullptr;
  l.out = a->out;
  l.part_o = reinterpret_cast<float *>(base + lay.part_o);
  l.part_ml = reinterpret_cast<float *>(base + lay.part_ml);
  l.out_fp32 = a->out_dtype;
  l.need_merge = 1;
  l.pair_head = pair_head;
  l.n_groups = max_groups;
  l.n_groups_dev = plan;                                 // the kernel reads how many stretches are in use
  l.max_waves = max_waves;
  l.item_first = 0, l.item_count = (int32_t)max_items;
  l.id_base = l.mirror_base = 0;
  OKV_HIP(nullptr, okv::launch_decode_attn(l, stream, nullptr, nullptr));
  OKV_HIP(nullptr, okv::launch_merge(l, stream));         // leaves at once for sequences that were not cut
  return OKV_OK;
}

int okv_probe_copy(void *dst, const void *src, int64_t bytes, void *stream) {
  if (!dst || !src || bytes < 0 || bytes % 16 || !aligned16(dst) || !aligned16(src))
    return fail(nullptr, OKV_EINVAL, "okv_probe_copy: bad argument");
  OKV_HIP(nullptr, okv::launch_probe_copy(dst, src, bytes, static_cast<hipStream_t>(stream)));
  return OKV_OK;
}

int okv_probe_read(const void *src, int64_t bytes, void *sink, void *stream) {
  if (!src || !sink || bytes < 0 || bytes % 16 || !aligned16(src)) return fail(nullptr, OKV_EINVAL, "okv_probe_read: bad argument");
  OKV_HIP(nullptr, okv::launch_probe_read(src, bytes, sink, static_cast<hipStream_t>(stream)));
  return OKV_OK;
}

}  // extern "C"
