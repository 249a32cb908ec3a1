// Kernel launchers of the okv library (gfx950).  Plain structs and pointers;
// the C ABI in okv_api.hip validates shapes before anything here is called.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace okv {

// Shape of one layer's pool and of the batch, shared by all kernels.
struct PoolShape {
  int32_t H, G, D;         // query heads, KV heads, head dim
  int32_t paged;           // 1: block table lookup, 0: sequence b owns slice b
  int32_t log2_T;          // paged: log2(block tokens)
  int32_t tcap;            // tokens per pool slice: T (paged) or max_ctx (contiguous); a multiple of 16
  int32_t gg;              // KV heads per group inside a slab (divides G)
  int32_t st_log2;         // log2 of the 16-token tiles per slab (okv_host.h: slab_tiles); tcap / 16 is a multiple
  int32_t max_blocks;      // paged: columns of the block table
};

struct BatchState {        // device arrays owned by the context
  const int32_t *block_table;   // [B][max_blocks]
  const int32_t *ctx_lens;      // [B]
  const int32_t *chunk_prefix;  // [n_cls * B + 1] items before those of (class, sequence), class-major
  const int4 *item_desc;        // [n_items] (sequence, first key, one past last key, flags)
  int32_t B;
  int32_t split_tokens;
  int32_t n_items;              // over all classes
  int32_t n_cls;                // block classes: 1 unless a share of every layer's blocks is on the host
};

struct AttnLaunch {
  PoolShape shape;
  BatchState batch;
  const void *q;           // fp16 [B][H][D]
  void *pool;              // the layer's KV pool (HBM: resident pool or staging buffer)
  const void *k_new;       // fp16 [B][G][D] rows to store at position ctx_len - 1, or NULL
  const void *v_new;
  void *pool_mirror;       // host layer: the pinned host pool that gets the same rows, else NULL
  void *out;               // [B][H][D] fp16 or fp32
  float *part_o;           // [n_items * H][D]
  float *part_ml;          // [n_items * H][2]  (max in log2 units, sum)
  int32_t out_fp32;
  int32_t need_merge;      // some sequence has more than one item
  // How the launch's items are shared out.  pair_head NULL: every item is a group of its own, and the (item, KV
  // head) pairs are dealt out to the wavefronts round robin.  Else the records launch_step_advance_spans wrote
  // for pools of this shape: stretch j is a group of consecutive items, record j * G + g says what the wavefront
  // for KV head g of it starts with, and every pair has a wavefront of its own (n_groups * G <= max_waves); the
  // launch must cover the whole list (item_first 0) from a pool that holds the blocks as the table numbers
  // them (id_base 0).
  const void *pair_head = nullptr;        // device
  int32_t n_groups = 0;                   // stretches in use (with pair_head)
  const int32_t *n_groups_dev = nullptr;  // device: the same number when the host does not know it (the grid is
                           // then max_waves wavefronts)
  int32_t max_waves;       // wavefronts of the persistent launch (a multiple of 4)
  // The launch covers items [item_first, item_first + item_count) of the list: all of them, or
  // those of one block class.  `pool` then holds the blocks with ids from id_base on, and
  // `pool_mirror` those from mirror_base on.
  int32_t item_first, item_count;
  int32_t id_base, mirror_base;
  // pool_mirror holds the layer's tail slots instead (two blocks per sequence: block j of sequence b
  // in slot 2 b + (j & 1)); the appended rows go there and not across the link.
  int32_t mirror_is_tail = 0;
};

// Store of the step's K/V rows and split-K partial attention over the launch's items.
hipError_t launch_decode_attn(const AttnLaunch &a, hipStream_t stream,
                              hipEvent_t ev_begin, hipEvent_t ev_end);

// Merge of the partial results of every sequence that has more than one item (reads
// shape, batch, out, part_o, part_ml, out_fp32 of `a`).
hipError_t launch_merge(const AttnLaunch &a, hipStream_t stream);

// ctx_lens[b] += inc; rebuilds chunk_prefix and the item list for split size S (every sequence cut
// into equal pieces of at most S keys).
hipError_t launch_step_advance(int32_t *ctx_lens, int32_t *chunk_prefix, int4 *item_desc, int32_t B, int32_t S,
                               int32_t inc, hipStream_t stream);

// The same with the keys of the batch shared out in equal stretches (okv_host.h: span_plan): at most
// max_groups stretches of at least min_span tiles; group_first[j] = first item of stretch j (one more
// entry closes the last); plan_out[0..3] = stretches in use, items, tiles per stretch (low 31 bits, rest).
// pair_head (may be NULL): [geom.max_pairs] records of kPairHeadBytes, one per (stretch, KV head) pair, pair =
// stretch * G + head, written for the stretches the step has: the stretch's first item and how many it has,
// that item's descriptor, and where the head's K rows of its first two tiles lie in a pool of the geometry
// given (the same for every layer).  An attention launch with max_waves wavefronts looks at the records of
// the pairs below max(max_waves, 4) (and ignores those past the last stretch): geom.max_pairs is at least that.
// The bookkeeping kernel keeps what opens each stretch in LDS, for at most kHeadGroupsMax stretches: callers
// keep max_groups at or below that.
constexpr int kPairHeadBytes = 32, kHeadGroupsMax = 1024;
struct HeadGeom {
  const int32_t *block_table = nullptr;   // device; NULL: contiguous pools (a sequence's slice is its block)
  int32_t max_blocks = 1, log2_T = 0;
  int32_t tiles = 1;                      // 16-token tiles of a pool slice (tcap / 16)
  int32_t st_log2 = 0, G = 1, gg = 1;     // slab geometry, as in PoolShape
  int32_t max_pairs = 0;                  // records to write
};
inline HeadGeom head_geom(const PoolShape &s, const int32_t *block_table, int32_t max_pairs) {
  HeadGeom g;
  g.block_table = s.paged ? block_table : nullptr;
  g.max_blocks = s.max_blocks, g.log2_T = s.log2_T, g.tiles = s.tcap >> 4;
  g.st_log2 = s.st_log2, g.G = s.G, g.gg = s.gg, g.max_pairs = max_pairs;
  return g;
}
hipError_t launch_step_advance_spans(int32_t *ctx_lens, int32_t *chunk_prefix, int4 *item_desc, int32_t *group_first,
                                     int32_t *plan_out, int32_t B, int32_t max_groups, int32_t min_span, int32_t inc,
                                     void *pair_head, const HeadGeom &geom, hipStream_t stream);

// The same for block classes: runs[r] = (sequence, first position, one past the last position
// the run can hold, class), sorted by (class, sequence, position); pair_first[cls * B + b] is the
// first run of (class, sequence).  Items are listed class by class; chunk_prefix[cls * B + b]
// counts the items before those of (class, sequence).  seq_total[b] receives the sequence's
// item count.
hipError_t launch_step_advance_classes(int32_t *ctx_lens, const int4 *runs, const int32_t *pair_first,
                                       int32_t *chunk_prefix, int4 *item_desc, int32_t *seq_total, int32_t B,
                                       int32_t n_cls, int32_t S, int32_t inc, hipStream_t stream);

// Bulk store of new K/V rows (a prompt).  tiles[i] = (sequence, 16-position tile, first slot of
// the tile to store | one past the last << 8, destination block); the row of position p of
// sequence b is row row_base[b] + p of k_rows / v_rows, which are [rows][G][D] fp16.  The
// destination block counts in blocks of `pool` (an HBM pool, a host pool through its mapped
// pointer, or a staging buffer in which blocks are being gathered); for contiguous pools it
// is the sequence's slice.  max_workgroups bounds the grid (0 = as many as there is work);
// throttle = 1 holds each wavefront to one tile's stores in flight.
struct BulkLaunch {
  PoolShape shape;
  const int4 *tiles;
  const int32_t *row_base;
  int32_t n_tiles;
  const void *k_rows, *v_rows;
  void *pool;
  int32_t max_workgroups;
  int32_t throttle;
};
hipError_t launch_bulk_append(const BulkLaunch &a, hipStream_t stream);

// Rows of the sequences' newest blocks between their slots in HBM and where they are read or kept.
// mode 0: for every sequence, the rows [tail_from[b], ctx_lens[b] - 1) that lie in the block of position
//         ctx_lens[b] - 1 or in the block before it go from the slots to `staged` (which holds the blocks
//         with ids id_lo .. id_hi - 1), if the block's id is in that range.
// mode 1: for every sequence whose length is a multiple of the block size, the rows from tail_from[b]
//         on of the block just filled go to the host pool of every layer (ids id_lo .. id_hi - 1 = the
//         host pool's blocks).
// mode 2: the same for the newest block of every sequence, as far as it is filled.
struct TailLaunch {
  void *staged;
  void *const *host_pools;       // device array [n_layers]
  const void *tail;              // mode 0: the layer's slots; else layer 0's
  const int32_t *block_table, *ctx_lens, *tail_from;
  int64_t block_elems, layer_stride;
  int32_t B, n_layers, max_blocks, log2_T, D;
  int32_t gg, st_log2;           // of the pools' layout (PoolShape)
  int32_t id_lo, id_hi;
  int32_t mode;
};
hipError_t launch_tail_rows(const TailLaunch &t, hipStream_t stream);

// items[it] = (b, lo, hi) decoded on the device.
hipError_t launch_worklist_dump(const BatchState &batch, int32_t *items, hipStream_t stream);

// ---- linear layers of a decoder layer (okv_layer.hip) ----------------------------------------
struct LinearLaunch {
  const void *x, *w_packed, *bias, *residual;
  void *out[3];
  int32_t n_seg, m, n_out, n_in, relu;
  int32_t first_cols = 0;      // width of out[0] when it differs from the others' (n_out - first_cols) / (n_seg - 1); 0: all equal
  void *workspace;             // fp32 shares of the cuts of the input dimension, or NULL
  int64_t workspace_bytes;
  const void *ln_gamma, *ln_beta;   // with ln_out: layer norm of the result (n_seg = 1) written there as well
  void *ln_out;
  float ln_eps;
  int32_t n_cus;               // compute units of the device (decides how the input dimension is cut)
};
hipError_t launch_linear(const LinearLaunch &l, hipStream_t stream);
int64_t linear_workspace_bytes(int32_t m, int32_t n_out, int32_t n_in, int32_t n_cus);
bool linear_staged_takes(int32_t m, int32_t n_out, int32_t n_in, int32_t n_cus, bool have_workspace, int64_t workspace_bytes);
hipError_t launch_pack_weight(void *dst, const void *src, int32_t n_out, int32_t n_in, hipStream_t stream);
hipError_t launch_layernorm(const void *x, const void *gamma, const void *beta, void *out, int32_t m, int32_t h, float eps,
                            hipStream_t stream);

hipError_t launch_probe_copy(void *dst, const void *src, int64_t bytes, hipStream_t stream);
hipError_t launch_probe_read(const void *src, int64_t bytes, void *sink, hipStream_t stream);

}  // namespace okv
