/*
 * okv -- decode attention over a partly offloaded KV cache, for one MI355X (gfx950).
 *
 * The workload (paper §II-A, §II-B, §IV-C, §IV-D): in the decode stage every new
 * token attends over the keys and values of all earlier tokens of its sequence,
 * which are kept per layer in a KV cache.  When that cache does not fit in GPU
 * memory a share C_off of it lives in host memory and is brought back to the
 * GPU layer by layer, because attention runs on the GPU and therefore needs the
 * layer's KV in GPU memory.  This library is that hot loop and nothing else:
 *
 *   kv_offload_plan   which layers live on the host for a given C_off
 *                     (okv_plan_block_split: which share of every layer's blocks)
 *   kv_append         store this step's K/V rows of one layer
 *   decode_attn       softmax(q K^T / sqrt(d)) V of one layer for a batch
 *   kv_append_bulk    store a whole prompt's K/V rows of one layer (prefill side)
 *
 * plus the small amount of state around them (batch description, step
 * bookkeeping, the copy pipeline for host layers).
 *
 * General conventions
 *   - C ABI, no C++ or framework types.  Every pointer is labelled HOST or DEVICE.
 *   - The caller owns every large buffer (KV pools, staging buffers, workspace,
 *     q / k / v / out) and keeps it alive until okv_destroy; the library never
 *     frees or reallocates them.  The library itself allocates only small
 *     bookkeeping arrays (O(max_batch * max_blocks_per_seq) integers, a few events).
 *   - Work is enqueued on the two streams given at creation and the calls return
 *     without waiting for the GPU unless stated otherwise.  q / k_new / v_new / out
 *     may be reused once the work enqueued on the compute stream has finished.
 *   - Every function returns OKV_OK (0) or a negative OKV_E* code and never aborts
 *     or throws.  okv_last_error gives a readable message for the last failure.
 *   - A context is not thread-safe: one host thread drives it.
 *
 * KV pool layouts (fp16; kv = 0 keys, kv = 1 values; G = n_kv_heads, d = head_dim).
 * A pool is a row of SLABS.  A slab holds the K and V rows of 16 * St consecutive tokens
 * (St tiles of 16) for all G KV heads, the heads taken in groups of Gg consecutive heads,
 * each group as its K rows and then its V rows, tile after tile, row-major:
 *   slab[g / Gg][kv][tile in slab][g % Gg][slot][d]    slot < 16;  2 * G * 16 * St * d * 2 bytes
 * Gg is the largest divisor of G with Gg * d <= 1024 (8 heads at d = 128, 16 at d = 64, all
 * G heads when there are fewer; okv_kv_head_group returns it).  St is the largest power of
 * two with St * Gg * d <= 1024 that divides the number of 16-token tiles of a pool slice (a
 * block, or a sequence's slice of a contiguous pool; okv_slab_tiles returns it): 1 for 8 or
 * more KV heads at d = 128, else as many tiles as it takes to make the K rows of a group one
 * run of 32 KiB, if the slice has them.  The K rows (and the V rows) of 16 consecutive tokens
 * of one KV head are one contiguous run of 16 * d * 2 bytes, which is what a wavefront reads
 * at a time; with this grouping the K run and the V run it reads together are 32 KiB apart and
 * those of neighbouring heads adjoin, which measured 8-10 % faster on MI355X than keeping all
 * K rows of a block before all its V rows, and with fewer than 8 KV heads 10 % faster than
 * slabs of a single tile (their K and V runs are 4-16 KiB apart).
 *   contiguous (block_tokens == 0):  sequence b < max_batch owns the max_ctx / (16 St) slabs
 *     from b * (max_ctx / (16 St)) on; token i is in slab i / (16 St) of them, tile
 *     (i / 16) % St of it, slot i % 16.
 *   paged (block_tokens == T):  block blk < blocks_per_layer is the T / (16 St) slabs from
 *     blk * (T / (16 St)) on; token i of sequence b is in block block_table[b][i / T], at
 *     token i % T of it: slab (i % T) / (16 St), tile ((i % T) / 16) % St, slot i % 16.
 */
#ifndef OKV_H
#define OKV_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define OKV_OK       0
#define OKV_EINVAL  (-1)  /* bad argument: NULL, shape, range, empty context        */
#define OKV_ENOSPC  (-2)  /* no room: block table / capacity / workspace / staging  */
#define OKV_ESTATE  (-3)  /* call out of order                                      */
#define OKV_EHIP    (-4)  /* a HIP runtime call failed; see okv_last_error          */

#define OKV_MAX_STAGING 4

typedef struct okv_ctx okv_ctx;   /* opaque */

typedef struct okv_config {
  int32_t n_layers;            /* L >= 1                                                     */
  int32_t n_q_heads;           /* H; H % G == 0 and 1 <= H / G <= 16                         */
  int32_t n_kv_heads;          /* G, at most 4 x the device's compute units (1024 here)      */
  int32_t head_dim;            /* d in {64, 128}                                             */
  int32_t block_tokens;        /* T: 0 = contiguous pools, else a power of two in [16, 1024] */
  int32_t max_batch;           /* largest B okv_set_batch will see                           */
  int32_t max_blocks_per_seq;  /* paged: columns of the block table; contiguous: ignored     */
  int32_t max_ctx;             /* contiguous: capacity in tokens per sequence, multiple of 16;
                                  paged: ignored (capacity is max_blocks_per_seq * T)        */
  int64_t blocks_per_layer;    /* paged: blocks in each layer's pool; contiguous: ignored    */
  int32_t out_dtype;           /* 0 = fp16 (round to nearest even), 1 = fp32                 */
  int32_t split_tokens;        /* upper bound on the keys of one split-K work item (a sequence
                                  of n keys is cut into ceil(n / split_tokens) equal pieces,
                                  rounded up to multiples of 16); 0 lets the library share the
                                  keys of every launch out in equal stretches over its
                                  wavefronts (okv_equal_stretches), which is what to use      */
  void  **dev_pool;            /* HOST array [L] of DEVICE pointers: the pool of each layer
                                  that stays in HBM, NULL for a layer kept on the host       */
  void  **host_pool;           /* HOST array [L] of HOST pointers to PINNED, device-mapped
                                  memory (hipHostMalloc): the pool of each host layer, NULL
                                  for a resident layer.  Exactly one of dev_pool[l],
                                  host_pool[l] is non-NULL.  May be NULL if no layer is on
                                  the host.                                                   */
  void   *staging[OKV_MAX_STAGING]; /* DEVICE: buffers host layers are copied into, each at least
                                  okv_layer_pool_bytes.  The leading non-NULL entries are used:
                                  one = no overlap of copy and compute; two = the copy of the next
                                  host layer runs during this one's attention (more than two
                                  measured no faster).  All NULL if no layer is on the host      */
  int64_t staging_bytes;       /* size of each staging buffer                                */
  void   *workspace;           /* DEVICE: split-K partial results                            */
  int64_t workspace_bytes;     /* at least okv_workspace_bytes(cfg)                          */
  void   *compute_stream;      /* hipStream_t for kernels (NULL = the default stream)        */
  void   *h2d_stream;          /* hipStream_t for host-to-device copies; must differ from
                                  compute_stream when any layer is on the host.  With two or
                                  more staging buffers the library creates one more copy
                                  stream of its own (default priority) for the odd-numbered
                                  buffers; okv_synchronize waits for it as well.
                                  The two streams should not share a hardware queue: the
                                  runtime spreads ordinary streams over a few queues and works
                                  each through in order, and kernels queued behind a copy's
                                  completion marker wait for that copy (measured: no overlap
                                  of attention and copies, 2-3 % of a step).  A stream made
                                  with hipExtStreamCreateWithCUMask and a mask of all compute
                                  units has a queue to itself; the library's own streams are
                                  made that way.                                             */
  /* Block-granular offload (paper §IV-C: C_off is a share of the cache, not a number of
   * layers).  chunk_blocks == 0: off, whole layers are resident or on the host as
   * described above.  chunk_blocks > 0 (paged pools only): in EVERY layer the blocks with
   * ids below resident_blocks are in dev_pool[l] (resident_blocks blocks; NULL if that is
   * 0) and the blocks with ids from resident_blocks on are in host_pool[l] at index
   * id - resident_blocks (blocks_per_layer - resident_blocks blocks; NULL if none).  The
   * host part is streamed in chunks of chunk_blocks consecutive blocks through the
   * staging buffers, each of which then only has to hold one chunk
   * (chunk_blocks * okv_block_bytes); every chunk and the resident part are attended by
   * a launch of their own and merged afterwards.  Which blocks a sequence gets is up to
   * the caller's block table; the fewer stretches of one class a sequence has, the
   * fewer work items. */
  int64_t resident_blocks;
  int64_t chunk_blocks;
  /* Block-granular offload only, optional (paper §IV-C Case 3 keeps what does not fit in host
   * memory; which rows travel when is left open).  DEVICE memory of okv_tail_bytes(cfg) bytes: two
   * block-sized slots per sequence and layer.  With it, the rows that decode steps append to a
   * block of the HOST pool are kept in a slot in HBM and the block is written to the host pool
   * once, when it is full (after the step that fills it; okv_flush_tails, okv_set_batch and
   * okv_prefill_begin write out what is left).  Until then the host pool lacks those rows: read it
   * only after okv_flush_tails.  NULL: every appended row is stored through the mapped pointer of
   * the host pool in the step that appends it, and the host pool is complete after every step. */
  void   *tail_blocks;
  int64_t tail_bytes;
} okv_config;

/* ---- sizes ------------------------------------------------------------------ */

/* Bytes of one layer's pool under cfg (both layouts); < 0 on a bad cfg.  Only the
 * shape fields of cfg are read.  This is the paper's Mem_KVcache,per_layer
 * (Table II) for the pool's capacity. */
int64_t okv_layer_pool_bytes(const okv_config *cfg);

/* Bytes of one block of a paged pool (K and V of block_tokens tokens for every KV
 * head), or of one sequence's slice of a contiguous pool; < 0 on a bad cfg. */
int64_t okv_block_bytes(const okv_config *cfg);

/* Gg of the pool layout above for n_kv_heads KV heads of head_dim numbers; < 0 unless
 * n_kv_heads >= 1 and head_dim is 64 or 128.  Pure host function. */
int32_t okv_kv_head_group(int32_t n_kv_heads, int32_t head_dim);

/* St of the pool layout above for a pool slice of slice_tokens tokens (block_tokens, or max_ctx
 * of a contiguous pool); < 0 unless n_kv_heads >= 1, head_dim is 64 or 128 and slice_tokens is a
 * positive multiple of 16.  Pure host function. */
int32_t okv_slab_tiles(int32_t n_kv_heads, int32_t head_dim, int32_t slice_tokens);

/* Bytes of workspace the split-K partials need in the worst case under cfg (every
 * sequence at full capacity, the smallest split size the library would choose or
 * cfg->split_tokens if set); < 0 on a bad cfg. */
int64_t okv_workspace_bytes(const okv_config *cfg);

/* Bytes that cfg->tail_blocks has to hold (n_layers * 2 * max_batch * okv_block_bytes), 0 if
 * cfg->chunk_blocks == 0; < 0 on a bad cfg.  Only the shape fields are read. */
int64_t okv_tail_bytes(const okv_config *cfg);

/* What keeping the newest blocks in HBM (cfg->tail_blocks) asks of a decode step, as a pure host
 * function (the context runs the same code; tests replay it against a model of the pools).
 * ctx_lens_after[b] = keys sequence b holds once the step's row is stored; tail_from[b] = the length
 * it had when the batch was described (okv_set_batch, okv_prefill_end, okv_flush_tails).
 *   patch_chunk[c] (HOST, [n_chunks]) = 1 if, before chunk c of the host pool (blocks resident_blocks +
 *     c * chunk_blocks ..) is attended in this step, rows have to be copied into its staged copy from the
 *     slots: the newest block of some sequence, or the one before it, lies in the chunk and holds a
 *     position >= tail_from[b];
 *   fills_block[b] (HOST, [B]) = 1 if the step fills a block of sequence b that belongs to the host pool
 *     and holds such positions: the block is written to the host pool after the step.
 * OKV_EINVAL on NULL pointers, a block size that is not a power of two >= 16, or lengths outside the table. */
int okv_tail_plan(int32_t B, const int32_t *block_table, int32_t max_blocks_per_seq, int32_t block_tokens,
                  const int32_t *ctx_lens_after, const int32_t *tail_from, int64_t resident_blocks, int64_t chunk_blocks,
                  int32_t n_chunks, uint8_t *patch_chunk, uint8_t *fills_block);

/* ---- offload plan (pure host functions, no GPU, no context) ------------------- */

/* Which layers live on the host for an offload ratio C_off = coff_num / coff_den
 * (paper §IV-C, Case 3: C_off is the share of the KV cache that has to leave the
 * GPU).  Whole layers are moved; their number is the smallest integer that is at
 * least C_off * n_layers; they are spread evenly: on_host[l] = 1 exactly when
 * floor((l+1) * n_off / n_layers) > floor(l * n_off / n_layers).
 *   on_host  HOST out, [n_layers], 1 = host, 0 = HBM
 *   n_off    HOST out, number of host layers (may be NULL)
 * OKV_EINVAL unless n_layers >= 1, coff_den > 0 and 0 <= coff_num <= coff_den. */
int kv_offload_plan(int32_t n_layers, int64_t coff_num, int64_t coff_den,
                    uint8_t *on_host, int32_t *n_off);

/* The same decision from memory sizes (paper §IV-C and Algorithm 1):
 *   mem_avail_bytes >= n_layers * layer_bytes       -> Case 1, nothing moves
 *   layer_bytes > mem_avail_bytes                   -> Case 2, OKV_ENOSPC
 *   otherwise Case 3: staging buffers (two if two layers fit, else one) come out
 *   of mem_avail_bytes, the layers that still fit stay resident, the rest go to
 *   the host, placed as kv_offload_plan places them.  The share moved is never
 *   below 1 - mem_avail / (n_layers * layer_bytes).  Two buffers are preferred to a
 *   resident layer: when exactly two layers fit, both become staging buffers and
 *   every layer is streamed, although one resident layer beside one buffer would
 *   move one layer less per step.  With one buffer a copy cannot start before the
 *   attention over the previous one has ended, so the link idles during every
 *   attention launch and the attention during every copy; with two the copies run
 *   back to back, which is worth more than a layer's bytes unless there are very
 *   few layers.
 *   n_staging HOST out: 0, 1 or 2 (may be NULL). */
int okv_plan_from_bytes(int32_t n_layers, int64_t layer_bytes, int64_t mem_avail_bytes,
                        uint8_t *on_host, int32_t *n_off, int32_t *n_staging);

/* The same rule at block granularity (paper §IV-C): of n_blocks blocks the smallest
 * whole number that is at least C_off * n_blocks goes to the host.
 *   resident_blocks, host_blocks  HOST out; their sum is n_blocks. */
int okv_plan_block_split(int64_t n_blocks, int64_t coff_num, int64_t coff_den,
                         int64_t *resident_blocks, int64_t *host_blocks);

/* How the keys of a batch are shared out over the wavefronts of a launch when no split size is
 * fixed (split_tokens == 0): the 16-key tiles of all sequences, laid end to end in sequence order, are
 * cut into n = min(max_groups, max(1, tiles / 8)) stretches of ceil(tiles / n) tiles, and a sequence is
 * cut wherever a stretch ends inside it.  Every wavefront of a launch streams at the same rate, so
 * equal shares end together (this is the split-K work list of a3 in §IV-D's terms: bookkeeping only,
 * any partition of the keys merges to the same softmax).  Pure host function.
 *   ctx_lens     HOST int32 [B], keys per sequence (>= 0)
 *   max_groups   wavefronts per KV head (a context uses 4 per compute unit / n_kv_heads)
 *   items        HOST int32 [max_items][3]: (sequence, first key, one past the last key), in order
 *   group_first  HOST int32 [max_groups + 1]: first item of every stretch, then the item count
 *   n_groups, span_tiles  HOST out: stretches in use, tiles per stretch
 * OKV_ENOSPC if max_items is too small (*n_items still receives the count). */
int okv_equal_stretches(const int32_t *ctx_lens, int32_t B, int32_t max_groups, int32_t *items, int64_t max_items,
                        int64_t *n_items, int32_t *group_first, int32_t *n_groups, int64_t *span_tiles);

/* The order of operations the copy pipeline enqueues, without a GPU (the runtime
 * walks the same scheduler).
 *   host_chunks   HOST int32 [n_layers]: streamed chunks of each layer (whole-layer
 *                 offload: 1 for a host layer, 0 for a resident one)
 *   has_resident  HOST uint8 [n_layers]: 1 if the layer also has keys in HBM; NULL
 *                 means "exactly the layers without chunks"
 * ops is a HOST array of max_ops records of seven int32:
 * kind, step, layer, chunk, buf, copy_idx, wait_idx with
 *   kind 0 COPY     copy stream: wait consumed[wait_idx] if >= 0, copy chunk `chunk` of
 *                   `layer`'s host pool into staging `buf`, signal ready[copy_idx]
 *   kind 1 APPEND   the step's K/V rows of `layer` are noted for the launches below
 *   kind 2 ATTN     compute stream: wait ready[wait_idx] if >= 0; attention over the
 *                   keys of chunk `chunk` in staging `buf` (chunk = buf = -1: the keys
 *                   in HBM); stores the new rows of the sequences whose newest
 *                   position it meets
 *   kind 3 RELEASE  compute stream: signal consumed[copy_idx]
 *   kind 4 MERGE    compute stream: combine the layer's partial results
 * n_ops receives the number of records written.  OKV_ENOSPC if max_ops is too small. */
int okv_schedule_trace(int32_t n_layers, const int32_t *host_chunks, const uint8_t *has_resident,
                       int32_t n_staging, int32_t n_steps, int32_t *ops, int64_t max_ops,
                       int64_t *n_ops);

/* ---- context -------------------------------------------------------------------- */

/* Validates cfg, copies it, allocates the bookkeeping arrays on the current
 * device.  *out is NULL on failure (then okv_last_error(NULL) has the reason). */
int okv_create(const okv_config *cfg, okv_ctx **out);

/* Waits for both streams, frees what okv_create allocated.  Caller buffers are
 * untouched. */
int okv_destroy(okv_ctx *ctx);

/* Message of the last failure on ctx (or of the last failure without a context
 * when ctx is NULL).  The pointer stays valid until the next call on ctx. */
const char *okv_last_error(const okv_ctx *ctx);

/* Describes the batch that the following steps decode.
 *   B            1 <= B <= max_batch
 *   block_table  HOST int32 [B][max_blocks_per_seq]; block ids in
 *                [0, blocks_per_layer), -1 = not allocated; no block may appear
 *                twice.  The same table serves every layer.  With block-granular
 *                offload the id also says where the block lives (see okv_config),
 *                and OKV_ENOSPC is returned if the batch is cut into more work
 *                items than the workspace holds.  Ignored (may be
 *                NULL) for contiguous pools, where sequence b owns slice b.
 *   ctx_lens     HOST int32 [B]: tokens already stored per sequence (>= 0), the
 *                same in every layer.
 * Synchronous: waits for both streams, uploads the tables, restarts the copy
 * pipeline.  Must not be called between okv_step_begin and okv_step_end. */
int okv_set_batch(okv_ctx *ctx, int32_t B, const int32_t *block_table, const int32_t *ctx_lens);

/* Opens a decode step: every sequence's length grows by one (the slot kv_append
 * fills), the split-K work list is rebuilt on the device, and for host layers
 * the first copies are enqueued if none are in flight.  With block-granular offload
 * (chunk_blocks > 0, blocks on the host) the call first waits until the previous step's
 * kernels have finished: letting the host enqueue several steps ahead made those steps
 * up to 10 % slower and erratic, and the compute stream waits for copies most of the
 * time anyway.
 * OKV_ENOSPC if a sequence would outgrow its capacity or reach an unallocated
 * block (nothing is changed then).  After any other failure (OKV_EHIP) the state on the
 * device is unknown and the batch has to be described again with okv_set_batch; until then
 * the calls of a step return OKV_ESTATE. */
int okv_step_begin(okv_ctx *ctx);

/* Closes the step.  OKV_ESTATE unless every layer had its decode_attn.  With cfg->tail_blocks, the
 * blocks of the host pools that this step filled are written out (one kernel on the compute stream,
 * after the step's attention; copies of the host pools enqueued later wait for it). */
int okv_step_end(okv_ctx *ctx);

/* Writes every appended row that is still only in a slot of cfg->tail_blocks to the host pools, so
 * that they are complete; waits for it, and restarts the copy pipeline (copies made before lack
 * those rows).  Without tail_blocks it only synchronises.  Needs a batch; not inside a step or a
 * prefill (OKV_ESTATE). */
int okv_flush_tails(okv_ctx *ctx);

/* Gives up an open step (after a call inside it failed, say, and the remaining layers cannot be
 * supplied): waits for everything enqueued, closes the step and forgets the batch.  The layers visited
 * so far hold the step's rows and the lengths have advanced on the device, which cannot be taken back,
 * so the next call must be okv_set_batch with the lengths the caller wants to go on from.  With
 * cfg->tail_blocks, rows appended since the last block was written out and still only in the slots are
 * not written to the host pools.  OKV_ESTATE outside a step. */
int okv_step_abort(okv_ctx *ctx);

/* Stores this step's key and value rows of `layer` at position ctx_len - 1 of each
 * sequence (paper §II-A: K/V of every processed token are kept for the following
 * decode steps).  For a host layer the rows are written both into the staged copy
 * (so this step's attention sees them) and into the host pool (so later steps do).
 *   k_new, v_new  DEVICE fp16 [B][G][d]
 * The store is carried out by the same kernel launch as the layer's decode_attn:
 * kv_append makes the compute stream wait for the layer's copy (host layers) and
 * hands the rows to that launch, so k_new / v_new must stay valid until the work of
 * decode_attn(layer) has finished, and the pool holds the rows from then on.  A row whose
 * block is on the host (block-granular offload) is written to the host pool directly.
 * Within a step layers are visited in order 0 .. L-1, kv_append(l) before
 * decode_attn(l); anything else is OKV_ESTATE. */
int kv_append(okv_ctx *ctx, int32_t layer, const void *k_new, const void *v_new);

/* Attention of the step's query over all stored keys of `layer`, including the one
 * just appended (paper §II-A; cost model §IV-D: 4 flops per cached K/V element):
 *   out[b][h] = sum_i softmax_i(q[b][h] . k_i / sqrt(d)) v_i,  i < ctx_len[b],
 * query head h reading KV head h / (H / G).
 *   q    DEVICE fp16 [B][H][d]
 *   out  DEVICE [B][H][d], fp16 or fp32 as cfg.out_dtype says
 * Arithmetic: q, K and V enter the matrix cores as the fp16 numbers they are stored as, both
 * products accumulate in fp32, the softmax (maximum, exponentials, their sum) is fp32, and
 * the weights 2^(s - max), which lie in [0, 1], are rounded to fp16 on their way into the
 * second product (the normalising sum keeps them in fp32).  That rounding is relative to
 * the running maximum of the work item a key falls in, so results depend on how the keys
 * are cut into items at the 1e-4 level (relative); against an fp64 evaluation the error is
 * about 3e-4 relative per output vector.
 * For a host layer the call first makes the compute stream wait for the layer's
 * copy, and afterwards hands the staging buffer back and enqueues the next copy.
 * With block-granular offload it launches once over the keys in HBM and once per
 * chunk of the host pool (waiting for that chunk's copy, releasing its buffer and
 * enqueueing the next copy each time), then merges. */
int decode_attn(okv_ctx *ctx, int32_t layer, const void *q, void *out);

/* One whole decode step in one call: okv_step_begin, then kv_append(l) and decode_attn(l)
 * for l = 0 .. L-1, then okv_step_end -- exactly those calls, made from inside the library,
 * for callers that have every layer's inputs ready (attention over a cache with no linear
 * layers in between, benchmarks) and do not want to cross the ABI 2 L + 2 times a step.
 *   q, k_new, v_new, out  HOST arrays [n_layers] of DEVICE pointers, each as in kv_append /
 *                         decode_attn
 * Stops at the first error and returns its code; the step is then left open as the failing
 * call left it. */
int okv_decode_step(okv_ctx *ctx, const void *const *q, const void *const *k_new,
                    const void *const *v_new, void *const *out);

/* ---- storing prompts (the prefill side) ---------------------------------------------
 *
 * The prefill stage produces the keys and values of every prompt token, layer by
 * layer; with offloading, a layer's share for the host is moved there while the next
 * layer computes, so that a layer costs the longer of the two (paper §II-A, §IV-D
 * T_pre = max(compute, T_trans^p)).  The computation itself is the caller's; these
 * calls store its K/V output:
 *
 *   okv_prefill_begin(n_new)              sequence b will receive n_new[b] tokens
 *   for l = 0 .. L-1:  kv_append_bulk(l, k_rows, v_rows)
 *                      ... okv_prefill_release(l) before k_rows / v_rows of l are reused
 *   okv_prefill_end()                     lengths grow by n_new; decode steps may follow
 */

/* Opens a prefill.  n_new: HOST int32 [B], tokens to add per sequence (>= 0), at
 * positions ctx_len[b] .. ctx_len[b] + n_new[b] - 1.  Synchronous (waits for all
 * streams, uploads a small tile list).  OKV_ENOSPC if a sequence would outgrow its
 * capacity or reach an unallocated block; OKV_ESTATE inside a step or a prefill. */
int okv_prefill_begin(okv_ctx *ctx, const int32_t *n_new);

/* Stores the new rows of `layer` (layers in order 0 .. L-1, once each).
 *   k_rows, v_rows  DEVICE fp16 [sum(n_new)][G][d]: the rows of sequence 0 first, then
 *                   those of sequence 1, ..., each in position order (token-major, as
 *                   a projection writes them).
 * Rows whose block is in HBM are stored by a kernel on the compute stream.  Rows whose
 * block (or whole layer) is on the host take one of two routes (okv_prefill_plan tells
 * which): blocks that are filled from their first slot and lie next to each other in
 * the host pool are gathered, in pool layout, in the staging buffers by a kernel on the
 * compute stream and moved by hipMemcpyAsync on a stream of the library's own (measured
 * to slow kernels running beside it by a few percent, where a kernel writing through
 * the mapped pointer slowed an HBM-bound neighbour several times over); slots of such a block past
 * the new rows are unused and receive unspecified bits.  Everything else (a prompt that
 * continues in the middle of a block, contiguous pools, blocks scattered singly) is
 * written straight into the pinned pool by a small kernel on that stream, which first
 * waits for the work enqueued so far on the compute stream (the producer of k_rows /
 * v_rows).  k_rows / v_rows must stay untouched until the kernels that read them have
 * finished: see okv_prefill_release. */
int kv_append_bulk(okv_ctx *ctx, int32_t layer, const void *k_rows, const void *v_rows);

/* How the last okv_prefill_begin routes the rows bound for host memory, per layer that has
 * any: blocks written from their first slot whose neighbours in the host pool add up to
 * 1 MiB per stretch on average are gathered in the staging buffers and copied over by
 * the runtime (staged_groups buffer fills, `copies` hipMemcpyAsync calls, staged_tiles 16-token
 * tiles); the rest is written by a kernel through the mapped pointer (direct_tiles). */
int okv_prefill_plan(const okv_ctx *ctx, int64_t *staged_groups, int64_t *copies,
                     int64_t *staged_tiles, int64_t *direct_tiles);

/* Makes the compute stream wait until the rows given to kv_append_bulk(layer) have been
 * stored, so that work enqueued on the compute stream afterwards may overwrite
 * k_rows / v_rows of that layer.  Returns at once (no host wait). */
int okv_prefill_release(okv_ctx *ctx, int32_t layer);

/* Closes the prefill: OKV_ESTATE unless every layer was stored.  Waits for the stores,
 * adds n_new to the sequence lengths, rebuilds the work list and restarts the copy
 * pipeline.  Synchronous. */
int okv_prefill_end(okv_ctx *ctx);

/* ---- for callers that cannot allocate ------------------------------------------------------
 *
 * decode_attn for one layer with no context and no allocation of any kind, for callers that must not
 * reach hipMalloc: code under HIP graph capture, tight serving loops, harnesses that forbid it.  The
 * split-K work list and partial results, which the entry points above keep in the context and in the
 * caller's workspace, live here in OKV_STATIC_SCRATCH_BYTES of device memory that are part of the
 * library itself (every GPU the library runs on holds them until the process ends).  The call makes
 * no hipMalloc / hipFree and no library call that allocates; its first call on a device looks up the
 * array's address on that device.  It enqueues three kernels on `stream` (work list from the device
 * lengths, split-K attention with the store of k_new / v_new folded in, merge) and returns.
 *
 * The batch's lengths are read on the device, so the host never needs them: ctx_lens[b] is the number
 * of keys sequence b attends to, INCLUDING the row stored by this call when k_new / v_new are given
 * (that row goes to position ctx_lens[b] - 1).  Pool layout, block table and the meaning of every
 * other argument are those of okv_config / kv_append / decode_attn; the keys of the batch are shared
 * out in equal stretches exactly as a context does with split_tokens = 0, so the results equal
 * decode_attn's bit for bit.
 *
 * Every call on a GPU uses that GPU's one array: calls that may overlap on one GPU (two streams, two
 * host threads) race and must be ordered by the caller.  Nothing in the array has to be cleared
 * between calls: each call's first kernel rewrites what the others read.
 * OKV_EINVAL: NULL / misaligned pointer, bad shape, B outside [1, OKV_STATIC_MAX_BATCH].
 * OKV_ENOSPC: (B + wavefronts per KV head) work items of n_q_heads * (head_dim + 2) floats, plus the
 * item list, exceed OKV_STATIC_SCRATCH_BYTES (32 query heads of 128: B up to about 1900). */
#define OKV_STATIC_SCRATCH_BYTES (32 << 20)
#define OKV_STATIC_MAX_BATCH 4096

typedef struct okv_static_attn {
  int32_t n_q_heads, n_kv_heads, head_dim;   /* as in okv_config                                  */
  int32_t block_tokens;                      /* 0 = contiguous pool, else T                       */
  int32_t max_blocks_per_seq;                /* paged: columns of block_table                     */
  int32_t max_ctx;                           /* contiguous: capacity per sequence, multiple of 16 */
  int32_t out_dtype;                         /* 0 = fp16, 1 = fp32                                */
  int32_t B;                                 /* sequences                                         */
  const void    *pool;                       /* DEVICE: the layer's pool (written if k_new given) */
  const int32_t *block_table;                /* DEVICE int32 [B][max_blocks_per_seq]; paged only  */
  const int32_t *ctx_lens;                   /* DEVICE int32 [B], each >= 1                       */
  const void    *q;                          /* DEVICE fp16 [B][H][d]                             */
  void          *out;                        /* DEVICE [B][H][d], fp16 or fp32                    */
  const void    *k_new, *v_new;              /* DEVICE fp16 [B][G][d], or both NULL               */
  void          *stream;                     /* hipStream_t (NULL = the default stream)           */
} okv_static_attn;

int okv_decode_attn_static(const okv_static_attn *a);

/* Blocks until everything enqueued on the library's streams has finished. */
int okv_synchronize(okv_ctx *ctx);

/* ---- introspection used by tests and the benchmark -------------------------------- */

/* Overrides the split size (0 = back to cfg.split_tokens, or to the library's choice
 * if that is 0 too).  The work list is rebuilt at once.  OKV_ENOSPC if the workspace
 * is too small for it. */
int okv_set_split_tokens(okv_ctx *ctx, int32_t split_tokens);

/* The split size in use (after the last okv_step_begin / okv_set_batch); when the library shares the
 * keys out in equal stretches (no split size given), the length of a stretch in keys. */
int32_t okv_get_split_tokens(const okv_ctx *ctx);

/* Copies the device-side sequence lengths back.  out: HOST int32 [B].  Synchronous. */
int okv_get_ctx_lens(okv_ctx *ctx, int32_t *out);

/* The current split-K work list as (sequence, first key, one-past-last key) triples,
 * in launch order: sequence by sequence, each cut into equal pieces that start at
 * multiples of 16 keys.  from_device = 0 walks the host copy of the tables;
 * from_device = 1 runs a small kernel that decodes every item exactly as the
 * attention kernel does and copies the result back (synchronous).
 * With block-granular offload the list is class by class (class 0 = the blocks in
 * HBM, class 1 + c = chunk c of the host pool); inside a class sequence by sequence;
 * a sequence is cut where its blocks change class and each stretch into equal pieces.
 *   items  HOST int32 [max_items][3];  n_items HOST out. */
int okv_worklist(okv_ctx *ctx, int32_t from_device, int32_t *items, int64_t max_items,
                 int64_t *n_items);

/* With equal stretches (no split size fixed), what the wavefronts of a launch start from: one record of
 * eight int32 per (stretch, KV head) pair, pair = stretch * G + head, as the bookkeeping kernel of the last
 * okv_step_begin / okv_set_batch wrote them on the device (synchronous copy):
 *   [0] the stretch's first item (index into okv_worklist's list)   [1] items of the stretch
 *   [2] that item's sequence   [3] its first key   [4] one past its last key
 *   [5] bit 0: the item ends its sequence, bit 1: it is the whole sequence; the KV head in the bits from 8 up
 *   [6], [7] where the head's K rows of the item's first and second 16-key tile begin in a layer's pool, in
 *            units of 16 * head_dim elements (the second clamped to the item's last tile)
 *   records  HOST int32 [max_records][8];  n_records HOST out (stretches in use * G).
 * OKV_ESTATE when the work list is cut otherwise (a fixed split size, block classes). */
int okv_pair_heads(okv_ctx *ctx, int32_t *records, int64_t max_records, int64_t *n_records);

/* Where each class starts in that list: class_first[c] .. class_first[c + 1] are the
 * items of class c; *n_classes receives the number of classes (1 without
 * block-granular offload).  from_device = 1 reads the prefix the kernels use.
 *   class_first  HOST int32 [max_classes], needs n_classes + 1 entries. */
int okv_worklist_classes(okv_ctx *ctx, int32_t from_device, int32_t *class_first,
                         int32_t max_classes, int32_t *n_classes);

/* Kernel timing with HIP events on the compute stream.
 *   on = 1  every split-K launch is bracketed by a pair of events of its own.  The
 *           markers leave the GPU idle for some microseconds before each kernel.
 *   on = 2  one bracket per decode step, from just before the step's first split-K
 *           launch (after the step's bookkeeping kernel) to okv_step_end: the
 *           kernels run back to back as they do untimed; merge passes, where a
 *           step needs them, and the copy waits of host layers fall inside it.
 *   on = 0  off.  Not to be changed inside a step.
 * okv_profile_read waits for the stream, returns the summed bracket time (ms) and the
 * number of split-K launches inside the brackets since the last read, and resets both.
 * The time an empty pair of event records takes on the same stream (median of 15,
 * measured at the read) is subtracted per bracket. */
int okv_profile_enable(okv_ctx *ctx, int32_t on);
int okv_profile_read(okv_ctx *ctx, double *attn_ms, int64_t *attn_launches);

/* Measured host-to-device rate: `reps` plain hipMemcpyAsync copies of `bytes` from
 * pinned HOST memory `src` to DEVICE memory `dst` on `stream`, each timed with HIP
 * events; *gbps_median receives the median in GB/s (1e9 bytes).  Synchronous. */
int okv_measure_h2d(void *dst, const void *src, int64_t bytes, int32_t reps, void *stream,
                    double *gbps_median);

/* The same for the other direction: DEVICE `src` to pinned HOST `dst`. */
int okv_measure_d2h(void *dst, const void *src, int64_t bytes, int32_t reps, void *stream,
                    double *gbps_median);

/* The copy half of n_steps decode steps alone, nothing else running: every host layer's pool (every
 * streamed chunk of every layer) is copied into the staging buffers; *ms receives the time per step.
 * The yardstick for how well real steps hide their compute behind the copies (paper §IV-D: a decode
 * layer costs compute plus transfer, Eq. 6; here the two overlap).
 *   as_pipelined = 0  the copies back to back on the h2d stream, alternating over the staging buffers,
 *                     timed with events: what the link gives when nothing orders the copies
 *   as_pipelined = 1  issued exactly as real steps issue them: the same copy streams, every copy waiting
 *                     for the release of its staging buffer and followed by its record, the compute
 *                     stream waiting for each copy and handing the buffer back where a step would
 *                     launch attention; timed on the host between two synchronisations, from the
 *                     pipeline's running state (the first copies are done before the clock starts, the
 *                     copies prefetched for the step after the last are inside it), so that n_steps steps
 *                     move exactly n_steps times the offloaded bytes
 * Needs a batch (okv_set_batch), must not be called inside a step.  Synchronous; restarts the pipeline. */
int okv_time_copies(okv_ctx *ctx, int32_t as_pipelined, int32_t n_steps, double *ms);

/* A plain device-to-device copy kernel (16 bytes per lane, grid-stride), the
 * yardstick the attention kernel's HBM traffic and rate are compared with.
 * bytes must be a multiple of 16.  Asynchronous on `stream`. */
int okv_probe_copy(void *dst, const void *src, int64_t bytes, void *stream);

/* A plain read kernel over `bytes` of DEVICE memory (sums into a 4-byte sink so the
 * loads are kept): the read-only yardstick.  Asynchronous on `stream`. */
int okv_probe_read(const void *src, int64_t bytes, void *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* OKV_H */
