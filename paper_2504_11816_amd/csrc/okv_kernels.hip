// HIP kernels of the okv library, written for gfx950 (64-wide wavefronts).
//
// Decode attention (paper §II-A; cost §IV-D: two multiply-adds per cached K and
// V element) reads every KV byte exactly once and does about one flop per byte,
// so the kernel is organised around the memory system:
//
//   * one wavefront owns one work item = (sequence, KV head, a run of keys) and
//     all H/G query heads that share the KV head, so K/V is read once per group;
//   * a K or V tile of 16 tokens is one contiguous run of 16*d*2 bytes; every
//     load instruction moves 16 bytes per lane, 1 KiB per wavefront;
//   * tiles are loaded PIPE deep ahead of their use into registers, 8 KiB in flight
//     per wavefront at d = 128 (16 KiB at d = 64, see base_depth), one wavefront per
//     SIMD: a thousand such streams is where the memory system runs best;
//   * the arithmetic of a tile (scores, online softmax, weighted sum of V rows) runs
//     on the matrix cores, which takes it off the vector ALU; the tile passes through
//     LDS that belongs to the wavefront alone to reach the operand layouts;
//   * the wavefront that reaches a sequence's last key also stores the step's new K/V
//     rows (kv_append is folded into the attention launch);
//   * items of a sequence are combined by a small merge kernel (skipped when
//     every sequence has a single item).
#include "okv_kernels.h"

#include <algorithm>

#include "okv_host.h"

namespace okv {

namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef const int32_t __attribute__((address_space(4))) *const_i32_ptr;   // never written while a kernel runs

#ifndef OKV_WAVES_PER_BLOCK
#define OKV_WAVES_PER_BLOCK 4
#endif

constexpr int kWavesPerBlock = OKV_WAVES_PER_BLOCK;   // independent work items per workgroup
constexpr float kNegBig = -1.0e30f;   // "no key seen yet"; finite so that differences stay finite
constexpr int kItemLast = 1, kItemWhole = 2;   // flags of a work item (item_desc.w)

// Where the rows of a 16-token tile live.  A pool is a sequence of slabs: the K and V rows of 16 * St
// consecutive tokens for every KV head, 2 * G * 16 * St * D elements.  Block blk of a paged pool is the
// tcap / (16 St) slabs from blk * (tcap / (16 St)) on; sequence b of a contiguous pool owns as many from
// b * (tcap / (16 St)) on.  Inside a slab the KV heads come in groups of gg: the K rows of the group (for each
// of the slab's St tiles in turn, the 16 * D elements of each of its heads), then its V rows likewise.
// St = 1 << st_log2 is 1 when a group's K rows of one tile already fill 32 KiB.
struct TileAddr {
  int64_t slab_elems;    // elements of one slab
  int64_t head_k;        // offset of this KV head's K rows of the slab's first tile inside a slab
  int64_t head_v;        // and of its V rows
  int32_t tile_stride;   // elements between a head's rows of one tile of a slab and of the next
  int32_t tiles;         // 16-token tiles per block (paged) or per sequence (contiguous): a multiple of St
  int32_t st_log2;
};

template <int D>
__device__ __forceinline__ TileAddr tile_addr(int G, int gg, int tcap, int st_log2, int g) {
  TileAddr t;
  t.slab_elems = ((int64_t)2 * G * 16 * D) << st_log2;
  t.tile_stride = gg * (16 * D);
  const int grp = g / gg;
  t.head_k = (((int64_t)grp * 2 * gg) << st_log2) * (16 * D) + (int64_t)(g - grp * gg) * (16 * D);
  t.head_v = t.head_k + ((int64_t)t.tile_stride << st_log2);
  t.tiles = tcap >> 4;
  t.st_log2 = st_log2;
  return t;
}

// First element of 16-token tile `tile` of pool slice `blk` (a block, or a sequence's slice), before the
// head's offset: the slab the tile lies in, and the tile's place among the slab's St.
template <bool PAGED>
__device__ __forceinline__ int64_t slab_base(const TileAddr &t, int blk, int tile) {
  const int64_t lin = (int64_t)blk * t.tiles + (PAGED ? tile & (t.tiles - 1) : tile);
  return (lin >> t.st_log2) * t.slab_elems + (int64_t)((int)lin & ((1 << t.st_log2) - 1)) * t.tile_stride;
}

// What a wavefront needs to know to ask for its first tiles, in one aligned 32-byte record per (stretch, KV
// head) pair: the bookkeeping kernel writes the records once per step, for all layers, and the attention
// kernel fetches its own with a single scalar load instead of walking group_first -> item descriptor ->
// block table and working out the tile's place in the pool, all of it while nothing is in flight yet and
// from an instruction cache that every launch finds cold.
struct alignas(32) PairHead {
  int32_t item;              // the stretch's first item (relative to the launch's first)
  int32_t count;             // items of the stretch (0: none, which only a batch without keys has)
  int32_t b, lo, hi;         // that item's sequence and keys
  int32_t flags_g;           // its flags, and the KV head in the bits from 8 up
  int32_t base0, base1;      // where the head's K rows of the item's first two tiles begin (the second clamped to the
                             // item's last tile), in units of 16 * D elements from the pool's start, block ids as the
                             // table has them
};
typedef int32_t int32x8_t __attribute__((ext_vector_type(8)));
typedef const int32x8_t __attribute__((address_space(4))) *const_head_ptr;   // a record as one scalar load

template <int LPT>
struct Tile {
  uint4 k[LPT];
  uint4 v[LPT];
};

struct AttnArgs {
  const uint16_t *q;
  const uint16_t *pool;
  const uint16_t *k_new, *v_new;   // this step's rows [B][G][D] to store, or NULL
  uint16_t *pool_store;            // where they go: the same pool as `pool`
  uint16_t *pool_mirror;           // and, for a host layer, its pinned host pool (else NULL)
  void *out;
  float *part_o;
  float *part_ml;
  const int32_t *block_table, *chunk_prefix;
  const int4 *item_desc;           // [n_items] (sequence, first key, one past last key, flags)
  const int32_t *n_groups_dev;     // NULL, or where the number of groups is to be read (n_groups is then ignored)
  const PairHead *pair_head;       // what every (stretch, KV head) pair starts with: pair p is wavefront p's; or
                                   // NULL: group j is item j of the launch
  int32_t n_groups;
  int32_t H, G, R, log2_T, tcap, max_blocks, out_fp32;   // R = H / G
  int32_t gg;                      // KV heads per group inside a slab
  int32_t st_log2;                 // log2 of the 16-token tiles per slab
  int32_t item_first;              // the launch's first item in item_desc (and in the partial slots)
  int32_t id_base;                 // `pool` holds the blocks with ids id_base, id_base + 1, ...
  int32_t mirror_shift;            // id_base minus the id of the first block of pool_mirror
  int32_t mirror_is_tail;          // pool_mirror is the layer's tail slots: block (2 b + (block index & 1)) of it
  int32_t B, n_cls;                // merge: chunk_prefix is [n_cls][B] (+ 1)
  float scale_log2e;
};

// ---- split-K attention on the matrix cores ---------------------------------------------------
//
// A wavefront owns one work unit: a run of keys of one sequence (an item) for one KV head, for all
// the R = H / G query heads that share it (1 <= R <= 16).  It loads the unit's K and V in 16-token
// tiles, whole rows, 16 bytes per lane, a few tiles ahead of the one it reduces.  The scores of a tile
// are a 16 x 16 x D product and the weighted sum of its V rows a D x 16 x 16 one:
//   S^T[key][head]  = K[key][:] . q[head][:]      v_mfma_f32_16x16x32_f16, A = K tile, B = q
//   O^T[dim][head] += V^T[dim][key] P^T[key][head] v_mfma_f32_16x16x16_f16, A = V^T,   B = P^T
// Each tile passes through a piece of LDS that belongs to the wavefront alone (no barriers) to get
// from the load layout to the operand layouts.  The score tile comes out with lane l holding head
// l % 16 and keys 4 (l / 16) .. + 3, which is the layout of the B operand of the second product as
// it stands, so the weights never move between lanes; max and sum over the keys need the lanes 16,
// 32 and 48 apart only.  Columns past the group's heads carry zeros and are never stored; the matrix
// cores are nowhere near busy and need not be: the path is bound by reading the cache, and what they
// take over (a lane-by-lane form of the same arithmetic ran at 4.7 TB/s with 8 heads per KV head,
// against 6.5 here) is the vector ALU's and the DPP network's work.

typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));

// Rows of a tile in LDS are 16 bytes further apart than they are long: the 16 lanes that read
// 16 bytes of 16 different rows, and the 64 lanes that read one dword of rows 4 apart, then fall
// on different banks.
template <int D>
constexpr int lds_row_bytes() {
  return D * 2 + 16;
}
template <int D>
constexpr int lds_tile_bytes() {
  return 16 * lds_row_bytes<D>();
}
// 16-key tiles that are reduced together: two at d = 64 (see tile_update_pair), one at d = 128
template <int D>
constexpr int lds_tiles() {
  return D == 64 ? 2 : 1;
}

// A tile on its way from the load registers (row-major, as loaded) into the wavefront's LDS.  masked
// (wavefront-uniform; only an item's last tiles need it): V rows of tokens outside [lo, hi) are stored
// as zeros, since unused slots may hold NaN bit patterns and a weight of zero would not remove those.
// There is one copy of this code and of tile_update_mfma in the kernel, masks applied by selects: what a
// launch pays for at its start and end is fetching instructions it runs once, so code size counts, and
// the selects cost nothing measurable (a wavefront waits for its loads, not for its arithmetic).
template <int D>
__device__ __forceinline__ void tile_stage(const Tile<D / 32> &t, char *ks, char *vs, const int lane,
                                           const int tok_tile, const int lo, const int hi, const bool masked) {
  constexpr int LPR = D / 8, RPL = 64 / LPR, LPT = D / 32, S = lds_row_bytes<D>();
  const int row = lane / LPR, col = lane % LPR;
#pragma unroll
  for (int j = 0; j < LPT; ++j) {
    const int r = row + j * RPL;
    *reinterpret_cast<uint4 *>(ks + r * S + col * 16) = t.k[j];
    *reinterpret_cast<uint4 *>(vs + r * S + col * 16) = t.v[j];
  }
  if (masked) {                                          // zeros over the V rows that are not the item's
#pragma unroll
    for (int j = 0; j < LPT; ++j) {
      const int r = row + j * RPL;
      if (tok_tile + r < lo || tok_tile + r >= hi) *reinterpret_cast<uint4 *>(vs + r * S + col * 16) = make_uint4(0u, 0u, 0u, 0u);
    }
  }
}

// Online-softmax update of one wavefront with the 16-token tile that tile_stage put into LDS
// (tok_tile = its first token).  masked: tokens outside [lo, hi) get score -inf (weight exactly 0; the
// running maximum stays finite because it starts at kNegBig).
template <int D>
__device__ __forceinline__ void tile_update_mfma(const half8_t (&qb)[D / 32], float &m,
                                                 float &l, floatx4_t (&o)[D / 16], const char *ks, const char *vs,
                                                 const int lane, const int tok_tile, const int lo,
                                                 const int hi, const float scale, const bool masked) {
  constexpr int S = lds_row_bytes<D>();
  const int quarter = lane >> 4, rho = lane & 15;
  // scores: A = K, lane (quarter, rho) supplies key rho, dims 32 c + 8 quarter .. + 7, as q does
  floatx4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int c = 0; c < D / 32; ++c) {
    const half8_t ka = *reinterpret_cast<const half8_t *>(ks + rho * S + c * 64 + quarter * 16);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka, qb[c], acc, 0, 0, 0);
  }
  float s[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int tok = tok_tile + 4 * quarter + r;
    s[r] = (!masked || (tok >= lo && tok < hi)) ? acc[r] * scale : -__builtin_inff();
  }
  float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
  mx = fmaxf(mx, __shfl_xor(mx, 16));
  mx = fmaxf(mx, __shfl_xor(mx, 32));
  const float m_new = fmaxf(m, mx);
  if (__any(m_new != m)) {                          // some head's maximum moved: rescale what is summed so far
    const float alpha = __builtin_amdgcn_exp2f(m - m_new);
    l *= alpha;
#pragma unroll
    for (int i = 0; i < D / 16; ++i) o[i] *= alpha;
    m = m_new;
  }
  float p[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    p[r] = __builtin_amdgcn_exp2f(s[r] - m);
    l += p[r];
  }
  const half4_t pb = {(_Float16)p[0], (_Float16)p[1], (_Float16)p[2], (_Float16)p[3]};
  // weighted sum: A = V^T.  Lane (quarter, rho) reads, for keys 4 quarter .. + 3, the dword that holds
  // dims 32 u + 2 rho and + 1; the low halves feed product 2 u (whose row rho is dim 32 u + 2 rho),
  // the high halves product 2 u + 1 (dim 32 u + 2 rho + 1).
#pragma unroll
  for (int u = 0; u < D / 32; ++u) {
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 4; ++e)
      w[e] = *reinterpret_cast<const uint32_t *>(vs + (4 * quarter + e) * S + (16 * u + rho) * 4);
    const uint2 even = make_uint2(__builtin_amdgcn_perm(w[1], w[0], 0x05040100u),
                                  __builtin_amdgcn_perm(w[3], w[2], 0x05040100u));
    const uint2 odd = make_uint2(__builtin_amdgcn_perm(w[1], w[0], 0x07060302u),
                                 __builtin_amdgcn_perm(w[3], w[2], 0x07060302u));
    o[2 * u] = __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(half4_t, even), pb, o[2 * u], 0, 0, 0);
    o[2 * u + 1] = __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(half4_t, odd), pb, o[2 * u + 1], 0, 0, 0);
  }
}

// Two 16-key tiles at once (d = 64, where a tile is half the bytes of one at d = 128 behind the same chain of
// waits): the tiles sit in rows 0-15 and 16-31 of ks / vs; one maximum, one rescaling and one pass of weights
// for the 32 keys, and the weighted sum as 16 x 16 x 32 products.  Lane (quarter, rho) holds, of head rho, the
// scores of keys 4 quarter .. + 3 of either tile; taken in that order (first tile's four, then the second's) they
// are the eight key slots 8 quarter .. + 7 of the B operand of the second product, and its A operand, V^T,
// is gathered from the same rows in the same order.  valid1 = 0: the second tile is not the item's (its
// buffer holds the last tile once more): every key of it is masked out.
__device__ __forceinline__ void tile_update_pair(const half8_t (&qb)[2], float &m, float &l, floatx4_t (&o)[4],
                                                 const char *ks, const char *vs, const int lane, const int tok_tile,
                                                 const bool valid1, const int lo, const int hi, const float scale,
                                                 const bool masked) {
  constexpr int D = 64, S = lds_row_bytes<D>();
  const int quarter = lane >> 4, rho = lane & 15;
  float s[8];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    floatx4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < D / 32; ++c) {
      const half8_t ka = *reinterpret_cast<const half8_t *>(ks + (16 * h + rho) * S + c * 64 + quarter * 16);
      acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka, qb[c], acc, 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int tok = tok_tile + 16 * h + 4 * quarter + r;
      const bool in = (!masked || (tok >= lo && tok < hi)) && (h == 0 || valid1);
      s[4 * h + r] = in ? acc[r] * scale : -__builtin_inff();
    }
  }
  float mx = fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])), fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7])));
  mx = fmaxf(mx, __shfl_xor(mx, 16));
  mx = fmaxf(mx, __shfl_xor(mx, 32));
  const float m_new = fmaxf(m, mx);
  if (__any(m_new != m)) {
    const float alpha = __builtin_amdgcn_exp2f(m - m_new);
    l *= alpha;
#pragma unroll
    for (int i = 0; i < D / 16; ++i) o[i] *= alpha;
    m = m_new;
  }
  float p[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    p[j] = __builtin_amdgcn_exp2f(s[j] - m);
    l += p[j];
  }
  const half8_t pb = {(_Float16)p[0], (_Float16)p[1], (_Float16)p[2], (_Float16)p[3],
                      (_Float16)p[4], (_Float16)p[5], (_Float16)p[6], (_Float16)p[7]};
#pragma unroll
  for (int u = 0; u < D / 32; ++u) {
    uint32_t w[8];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int e = 0; e < 4; ++e)
        w[4 * h + e] = *reinterpret_cast<const uint32_t *>(vs + (16 * h + 4 * quarter + e) * S + (16 * u + rho) * 4);
    const uint4 even = make_uint4(__builtin_amdgcn_perm(w[1], w[0], 0x05040100u), __builtin_amdgcn_perm(w[3], w[2], 0x05040100u),
                                  __builtin_amdgcn_perm(w[5], w[4], 0x05040100u), __builtin_amdgcn_perm(w[7], w[6], 0x05040100u));
    const uint4 odd = make_uint4(__builtin_amdgcn_perm(w[1], w[0], 0x07060302u), __builtin_amdgcn_perm(w[3], w[2], 0x07060302u),
                                 __builtin_amdgcn_perm(w[5], w[4], 0x07060302u), __builtin_amdgcn_perm(w[7], w[6], 0x07060302u));
    o[2 * u] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, even), pb, o[2 * u], 0, 0, 0);
    o[2 * u + 1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, odd), pb, o[2 * u + 1], 0, 0, 0);
  }
}

// A work unit as a wavefront sees it: an item (a run of keys of one sequence) for one KV head.  All
// fields are wavefront-uniform and come through the scalar cache (constant address space: nothing
// writes the item list or the block table while this kernel runs).
template <int PIPE>
struct Unit {
  int it, g;                 // item (index in item_desc and in the partial slots), KV head
  int b, lo, hi, flags;      // sequence, keys [lo, hi) with lo a multiple of 16, kItemLast / kItemWhole
  int blk0[PIPE];            // pool slices of the first PIPE tiles (clamped to the last tile)
};

// Persistent wavefronts, each with a share of the launch that was fixed before it started.  The host
// (or the bookkeeping kernel) cuts the launch's keys, all sequences laid end to end, into as many equal
// stretches as there are wavefronts per KV head; a stretch is a group of consecutive items (the pieces
// of the sequences it covers), and the wavefront for (group, head), pair p = group * G + head, reduces
// them one after the other.  (Without stretches every item is a group and wavefront w takes the pairs w,
// w + n_waves, ...)  Every wavefront
// streams at the same rate (each is bound by the round trip of its own loads: measured within 1.3 % of
// each other over all compute units, where wavefronts that keep a load in flight all the time differed
// by 8 % from XCD to XCD and were no faster on average), so equal shares end together; nothing is drawn
// from a counter and nothing waits.
//
// A wavefront treats its items as ONE stream of tiles: PIPE tile buffers in registers, each refilled
// right after the tile in it has been reduced, and when the current item has no tile left to ask for,
// the refill is the first tile of the next one.  So the loads of the next item are in flight while the
// results of this one are written, and a wavefront's stream does not stop at an item boundary.  For
// that the next item is looked up a whole item ahead (descriptor and first block ids, scalar loads).
//
// The body is one loop with one copy of everything -- [A] ask for the next item's first tiles and q,
// [B] write the current item's results, [C] switch to the next item and reduce its tiles -- entered at
// [A] for the first item: a launch fetches every instruction it runs from a cold instruction cache
// (about 0.1 us per 64 bytes where the fetch does not run straight on), which at 50 us a launch is worth
// keeping short.
//
// The start of a launch is the other fixed cost: until a wavefront's first tile arrives nothing hides the
// round trips in front of it (a scalar load right after the launch takes 1-2 us).  With HEADS the
// wavefront's own (stretch, KV head) pair comes from a table the bookkeeping kernel wrote (PairHead): one
// look-up, whose address needs only arguments that arrive in registers, then the first tile loads, and
// everything else (the other arguments, the LDS addresses, the zeroed sums) is set up behind them.  Without
// it (a split size fixed by the caller, block classes, more pairs than wavefronts) pairs are dealt out
// round robin and the first item is found through group_first, the item list and the block table.
template <int D, bool PAGED, int PIPE, bool HEADS>
__global__ __launch_bounds__(kWavesPerBlock * 64) void attn_split_mfma_kernel(
    const PairHead *pair_head, const uint16_t *pool, const uint16_t *q, const int32_t *n_groups_dev, const int32_t n_groups,
    const int32_t G, const int32_t H, const int32_t R, const int32_t v_tiles, const AttnArgs a) {
  __shared__ __attribute__((aligned(16))) char lds_all[kWavesPerBlock][2 * lds_tiles<D>() * lds_tile_bytes<D>()];
  constexpr int LPR = D / 8, RPL = 64 / LPR, LPT = D / 32;
  const int lane = threadIdx.x & 63;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t n_waves = gridDim.x * kWavesPerBlock;
  uint32_t pair = blockIdx.x * kWavesPerBlock + wave;    // of the unit N below
  // With a table of heads every (stretch, KV head) pair has a wavefront of its own and its head says what
  // the pair starts with; otherwise pairs are dealt out round robin.  The number of groups is a launch
  // argument, or (for callers that do not know the batch's lengths on the host) what the bookkeeping kernel
  // left in device memory.
  //
  // The parameters in front of `a` are the ones the first loads need: the build asks for the leading kernel
  // arguments to be in scalar registers when a wavefront starts, so the pair's record can be asked for at
  // once, and the first tiles as soon as it is there.
  constexpr bool by_head = HEADS;                        // (pair_head is not NULL then)
  int32x8_t w = {0, 0, 0, 0, 0, 0, 0, 0};
  if (by_head) w = *(const_head_ptr)(uintptr_t)(pair_head + pair);
  const uint32_t n_pairs = (n_groups_dev ? (uint32_t)((const_i32_ptr)(uintptr_t)n_groups_dev)[0] : (uint32_t)n_groups) * (uint32_t)G;
  asm volatile("" ::"s"(w[0]), "s"(n_pairs));           // (both asked for before either is waited for)
  if (pair >= n_pairs) return;
  PairHead head = {};
  if (by_head) {
    head.item = w[0], head.count = w[1], head.b = w[2], head.lo = w[3], head.hi = w[4], head.flags_g = w[5];
    head.base0 = w[6], head.base1 = w[7];
    if (head.count <= 0) return;                         // (records past the last pair are not written)
  }

  const int row = lane / LPR, col = lane % LPR;
  const int quarter = lane >> 4, rho = lane & 15;
  char *ks = lds_all[wave], *vs = ks + lds_tiles<D>() * lds_tile_bytes<D>();

  // Block id of a tile: a wavefront-uniform (scalar) load from the block table.  The table is read
  // through the constant address space: the kernel also stores (outputs, appended rows) and without
  // that promise the compiler would turn these look-ups into vector loads, which share the tile loads'
  // counter and would drain the pipeline.
  auto blk_of = [&](int b, int tile) -> int {
    if (!PAGED) return b;
    const const_i32_ptr tbl = (const_i32_ptr)(uintptr_t)(a.block_table + (size_t)b * a.max_blocks);
    int bi = (tile << 4) >> a.log2_T;
    bi = bi < a.max_blocks ? bi : a.max_blocks - 1;
    return tbl[bi] - a.id_base;
  };
  auto load_tile = [&](Tile<LPT> &t, const TileAddr &ta, int tile, int blk) {
    const int64_t base = slab_base<PAGED>(ta, blk, tile);
    const uint4 *kp = reinterpret_cast<const uint4 *>(pool + base + ta.head_k) + lane;
    const uint4 *vp = reinterpret_cast<const uint4 *>(pool + base + ta.head_v) + lane;
#pragma unroll
    for (int j = 0; j < LPT; ++j) t.k[j] = kp[j * 64];
#pragma unroll
    for (int j = 0; j < LPT; ++j) t.v[j] = vp[j * 64];
  };

  // the items of the pair: item .. item_end - 1 (relative to the launch's first item)
  int item, item_end;
  if (by_head) {
    item = head.item, item_end = head.item + head.count;
  } else {
    item = (int)(pair / (uint32_t)G), item_end = item + 1;
  }
  bool has_next = true;                                  // N is a unit (else the wavefront's share is done)
  Unit<PIPE> N, C;                                       // the unit whose first tiles are asked for next; the one being reduced
  bool live = false;                                     // C holds a unit whose results are still to be written
  TileAddr ta = tile_addr<D>(G, a.gg, a.tcap, a.st_log2, 0);
  Tile<LPT> buf[PIPE];
  uint4 q_next[D / 32];                                  // q of N: the B operand of the score product, lane (quarter, rho) holds
                                                         // head rho, dims 32 c + 8 quarter .. + 7 (columns past the group's heads:
                                                         // head 0's, zeroed where the unit takes q over)
  if (by_head) {
    // the first unit's first tiles and its q straight from the head, before anything else is set up
#pragma unroll
    for (int i = 0; i < (PIPE < 2 ? PIPE : 2); ++i) {
      const uint4 *kp = reinterpret_cast<const uint4 *>(pool + (size_t)(uint32_t)(i ? head.base1 : head.base0) * (16 * D)) + lane;
      const uint4 *vp = kp + ((size_t)v_tiles * (16 * D) * 2 / 16);
#pragma unroll
      for (int j = 0; j < LPT; ++j) buf[i].k[j] = kp[j * 64];
#pragma unroll
      for (int j = 0; j < LPT; ++j) buf[i].v[j] = vp[j * 64];
    }
    if (PIPE > 2) {                                      // the record holds two places: the deeper buffers the long way
      const int g0 = head.flags_g >> 8, last0 = (head.hi - 1) >> 4;
      const TileAddr ta0 = tile_addr<D>(G, a.gg, a.tcap, a.st_log2, g0);
#pragma unroll
      for (int i = 2; i < PIPE; ++i) {
        const int tile = min((head.lo >> 4) + i, last0);
        load_tile(buf[i], ta0, tile, blk_of(head.b, tile));
      }
    }
    const uint4 *qp = reinterpret_cast<const uint4 *>(q + ((size_t)head.b * H + (size_t)(head.flags_g >> 8) * R + (rho < R ? rho : 0)) * D + 8 * quarter);
#pragma unroll
    for (int c = 0; c < D / 32; ++c) q_next[c] = qp[4 * c];
    __builtin_amdgcn_sched_barrier(0);
  }
  // All the other launch arguments are asked for here, in one batch of scalar loads (with a table of heads:
  // behind the first tile loads).  Left to itself the compiler fetches each where it is first used, which
  // makes three or four dependent round trips to the argument segment of them.
  asm volatile("" ::"s"(gridDim.x), "s"(a.gg), "s"(a.st_log2), "s"(a.k_new), "s"(a.v_new), "s"(a.pool_store),
               "s"(a.pool_mirror), "s"(a.out), "s"(a.part_o), "s"(a.part_ml), "s"(a.block_table), "s"(a.item_desc),
               "s"(a.log2_T), "s"(a.tcap), "s"(a.max_blocks), "s"(a.out_fp32), "s"(a.item_first),
               "s"(a.id_base), "s"(a.mirror_shift), "s"(a.mirror_is_tail), "s"(a.scale_log2e));
  float m = kNegBig, l = 0.f;
  floatx4_t o[D / 16];
  uint4 k_row = make_uint4(0u, 0u, 0u, 0u), v_row = k_row;
  C.it = C.g = C.b = C.lo = C.hi = C.flags = 0;

  for (;;) {
    // N's descriptor and first block ids: for the first unit waited for here; for the others asked for
    // a whole item earlier ([C] below)
    if (!live) {
      N.it = a.item_first + item;
      if (by_head) {                                     // its first tiles are on their way already
        N.g = head.flags_g >> 8;
        N.b = head.b, N.lo = head.lo, N.hi = head.hi, N.flags = head.flags_g & 0xff;
#pragma unroll
        for (int i = 0; i < PIPE; ++i) N.blk0[i] = 0;
      } else {
        N.g = (int)(pair % (uint32_t)G);
        const const_i32_ptr dp = (const_i32_ptr)(uintptr_t)(a.item_desc + N.it);
        N.b = dp[0], N.lo = dp[1], N.hi = dp[2], N.flags = dp[3];
#pragma unroll
        for (int i = 0; i < PIPE; ++i) N.blk0[i] = blk_of(N.b, min((N.lo >> 4) + i, (N.hi - 1) >> 4));
      }
    }
    // [A] the next unit's first tiles and its q
    // (with a table of heads a wavefront stays with one KV head: nothing to work out again)
    const TileAddr ta_next = by_head && live ? ta : tile_addr<D>(G, a.gg, a.tcap, a.st_log2, N.g);
    if (has_next && (live || !by_head)) {
#pragma unroll
      for (int i = 0; i < PIPE; ++i) load_tile(buf[i], ta_next, min((N.lo >> 4) + i, (N.hi - 1) >> 4), N.blk0[i]);
      // (lanes past the group's heads read head 0's piece, which is dropped where q is taken over: no branch
      // around each load)
      const uint4 *qp = reinterpret_cast<const uint4 *>(q + ((size_t)N.b * H + (size_t)N.g * R + (rho < R ? rho : 0)) * D + 8 * quarter);
#pragma unroll
      for (int c = 0; c < D / 32; ++c) q_next[c] = qp[4 * c];
    }
    __builtin_amdgcn_sched_barrier(0);

    // [B] the results of C.  The four quarters of the wavefront saw different keys of every tile: their
    // sums add up (the maximum is common to them already).  Lane (quarter, rho) holds, of head rho, the
    // dims 32 u + 8 quarter .. + 7 for every u: dim 32 u + 8 quarter + 2 r + par sits in o[2 u + par][r].
    // A sequence that is a single item is normalised and written to `out`; otherwise the item's sums,
    // maximum and weight go to its slot of the partial results, as floats.
    if (live) {
      const bool seq_whole = (C.flags & kItemWhole) != 0;
      float lt = l;
      lt += __shfl_xor(lt, 16);
      lt += __shfl_xor(lt, 32);
      if (rho < R) {
        const int h = C.g * R + rho;
        const float inv = seq_whole ? 1.0f / lt : 1.0f;
        const bool as_float = !seq_whole || a.out_fp32;
        float *fdst = seq_whole ? reinterpret_cast<float *>(a.out) + ((size_t)C.b * H + h) * D
                                : a.part_o + ((size_t)C.it * H + h) * D;
        uint16_t *hdst = reinterpret_cast<uint16_t *>(a.out) + ((size_t)C.b * H + h) * D;
#pragma unroll
        for (int u = 0; u < D / 32; ++u) {
          float ot[8];
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            ot[2 * r] = o[2 * u][r] * inv;
            ot[2 * r + 1] = o[2 * u + 1][r] * inv;
          }
          const int dim0 = 32 * u + 8 * quarter;
          if (as_float) {
            float4 *dst = reinterpret_cast<float4 *>(fdst + dim0);
            dst[0] = make_float4(ot[0], ot[1], ot[2], ot[3]);
            dst[1] = make_float4(ot[4], ot[5], ot[6], ot[7]);
          } else {
            half2_t h0 = {(_Float16)ot[0], (_Float16)ot[1]};
            half2_t h1 = {(_Float16)ot[2], (_Float16)ot[3]};
            half2_t h2 = {(_Float16)ot[4], (_Float16)ot[5]};
            half2_t h3 = {(_Float16)ot[6], (_Float16)ot[7]};
            *reinterpret_cast<uint4 *>(hdst + dim0) = make_uint4(__builtin_bit_cast(uint32_t, h0), __builtin_bit_cast(uint32_t, h1),
                                                                 __builtin_bit_cast(uint32_t, h2), __builtin_bit_cast(uint32_t, h3));
          }
        }
        if (!seq_whole && quarter == 0)
          *reinterpret_cast<float2 *>(a.part_ml + ((size_t)C.it * H + h) * 2) = make_float2(m, lt);
      }
      // The item that ends at the sequence's last key also stores this step's K/V rows (paper §II-A: keys
      // and values of every processed token are kept): row 0 of the load layout stores the K row, row 1 the V row.
      const int pos = C.hi - 1;
      if (a.k_new != nullptr && (C.flags & kItemLast) && row < 2) {
        const int blk = blk_of(C.b, pos >> 4);
        const int64_t in_slab = (row == 0 ? ta.head_k : ta.head_v) + (int64_t)(pos & 15) * D + col * 8;
        const uint4 val = row == 0 ? k_row : v_row;
        *reinterpret_cast<uint4 *>(a.pool_store + slab_base<PAGED>(ta, blk, pos >> 4) + in_slab) = val;
        if (a.pool_mirror) {
          const int mblk = PAGED && a.mirror_is_tail ? 2 * C.b + ((pos >> a.log2_T) & 1) : blk + (PAGED ? a.mirror_shift : 0);
          *reinterpret_cast<uint4 *>(a.pool_mirror + slab_base<PAGED>(ta, mblk, pos >> 4) + in_slab) = val;
        }
      }
    }
    if (!has_next) break;

    // [C] N becomes the unit being reduced; the unit after it is looked up now, a whole item before its
    // first tile is asked for: the next item of the pair, else the first item of the wavefront's next pair
    C = N;
    ta = ta_next;
    live = true;
    if (item + 1 < item_end) {
      ++item;
    } else {
      pair += n_waves;
      has_next = !by_head && pair < n_pairs;             // by head: the wavefront's own stretch is all it has
      if (has_next) {
        item = (int)(pair / (uint32_t)G), item_end = item + 1;
      }
    }
    if (has_next) {
      N.g = by_head ? C.g : (int)(pair % (uint32_t)G);
      N.it = a.item_first + item;
      const const_i32_ptr dp = (const_i32_ptr)(uintptr_t)(a.item_desc + N.it);
      N.b = dp[0], N.lo = dp[1], N.hi = dp[2], N.flags = dp[3];
#pragma unroll
      for (int i = 0; i < PIPE; ++i) N.blk0[i] = blk_of(N.b, min((N.lo >> 4) + i, (N.hi - 1) >> 4));
    }
    const int b = C.b, lo = C.lo, hi = C.hi;
    // The rows to append are patched into the tile in registers, so the attention does not depend on
    // reading its own store back; the store itself is issued with the results ([B]).
    const int pos = hi - 1;
    const bool appending = a.k_new != nullptr && (C.flags & kItemLast) != 0;
    if (appending) {
      const size_t at = ((size_t)b * G + C.g) * LPR + col;
      k_row = reinterpret_cast<const uint4 *>(a.k_new)[at];
      v_row = reinterpret_cast<const uint4 *>(a.v_new)[at];
    }
    half8_t qb[D / 32];
#pragma unroll
    for (int c = 0; c < D / 32; ++c) qb[c] = __builtin_bit_cast(half8_t, rho < R ? q_next[c] : make_uint4(0u, 0u, 0u, 0u));
    m = kNegBig, l = 0.f;
#pragma unroll
    for (int i = 0; i < D / 16; ++i) o[i] = floatx4_t{0.f, 0.f, 0.f, 0.f};

    // Tiles go through the buffers in groups of PIPE (tile t0 + k sits in buffer k % PIPE).  Every group
    // but the last holds full tiles only (an item starts on a tile boundary, so only its last tile can
    // stick out of [lo, hi) or hold the appended row) and refills its buffers from the item itself: each
    // wait covers exactly the tile it needs and the younger loads stay in flight; block ids are fetched
    // one refill ahead through the scalar cache, which has its own counter.  A refill past the item's
    // last tile (only when the tile count is not a multiple of PIPE) asks for the last tile again.  The
    // last group's buffers are refilled at [A], from the next item.
    const int t1 = (hi + 15) >> 4, last_tile = t1 - 1;
    int next_blk[PIPE];
#pragma unroll
    for (int i = 0; i < PIPE; ++i) next_blk[i] = blk_of(b, min((lo >> 4) + PIPE + i, last_tile));
    for (int t = lo >> 4; t < t1; t += PIPE) {
      const bool last = t + PIPE >= t1;
#pragma unroll
      for (int i = 0; i < PIPE; ++i) {
        // at d = 64 two tiles are reduced together: buffer i (even) is staged and waits for buffer i + 1
        constexpr int PAIR = lds_tiles<D>();
        char *const ks_i = ks + (i % PAIR) * lds_tile_bytes<D>(), *const vs_i = vs + (i % PAIR) * lds_tile_bytes<D>();
        if (i - i % PAIR == 0 || t + (i - i % PAIR) < t1) {   // else a second request for the last tile: skipped
          if (last && appending && t + i == (pos >> 4)) {
#pragma unroll
            for (int j = 0; j < LPT; ++j)
              if (((t + i) << 4) + row + j * RPL == pos) {
                buf[i].k[j] = k_row;
                buf[i].v[j] = v_row;
              }
          }
          tile_stage<D>(buf[i], ks_i, vs_i, lane, (t + i) << 4, lo, hi, last);
          if constexpr (PAIR == 1) {
            tile_update_mfma<D>(qb, m, l, o, ks, vs, lane, (t + i) << 4, lo, hi, a.scale_log2e, last);
          } else if (i % PAIR == PAIR - 1) {
            tile_update_pair(qb, m, l, o, ks, vs, lane, (t + i - 1) << 4, t + i < t1, lo, hi, a.scale_log2e, last);
          }
        }
        __builtin_amdgcn_sched_barrier(0);    // keep the refill behind the reduce that frees it,
        if (!last) {
          load_tile(buf[i], ta, min(t + i + PIPE, last_tile), next_blk[i]);
          next_blk[i] = blk_of(b, min(t + i + 2 * PIPE, last_tile));
        }
        __builtin_amdgcn_sched_barrier(0);    // and ahead of the next tile's reduce
      }
    }
  }
}

// out[b][h] = sum_c o_c 2^(m_c - M) / sum_c l_c 2^(m_c - M) over the items c of sequence b.
// One wavefront per (b, h).  The items of a sequence are one contiguous range of the list per
// block class.  Lane c first fetches (m_c, l_c) of item c, so the maxima and weights of up to
// 64 items are formed by wavefront reductions instead of a chain of dependent loads; the
// weighted sums then stream the partial rows four items at a time.
template <int D>
__global__ __launch_bounds__(64) void attn_merge_kernel(const int32_t *chunk_prefix, const float *part_ml, const int32_t B,
                                                         const int32_t n_cls, const int32_t H, const AttnArgs a) {
  // (leading parameters: in scalar registers when the wavefront starts, so the first look-ups need no round trip
  // to the argument segment; most wavefronts of a launch find a sequence in one piece and leave at once)
  constexpr int EPT = D / 64;
  const int b = blockIdx.y, h = blockIdx.x, lane = threadIdx.x;
  float M = kNegBig;
  int total = 0;
  for (int cls = 0; cls < n_cls; ++cls) {
    const int first = chunk_prefix[cls * B + b];
    const int n_chunks = chunk_prefix[cls * B + b + 1] - first;
    total += n_chunks;
    for (int c0 = 0; c0 < n_chunks; c0 += 64) {
      const int c = c0 + lane;
      float mc = c < n_chunks ? part_ml[((size_t)(first + c) * H + h) * 2] : kNegBig;
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) mc = fmaxf(mc, __shfl_xor(mc, off));
      M = fmaxf(M, mc);
    }
  }
  if (total <= 1) return;                              // written by the split kernel
  float L = 0.f, acc[EPT];
#pragma unroll
  for (int e = 0; e < EPT; ++e) acc[e] = 0.f;
  for (int cls = 0; cls < n_cls; ++cls) {
    const int first = chunk_prefix[cls * B + b];
    const int n_chunks = chunk_prefix[cls * B + b + 1] - first;
    for (int c0 = 0; c0 < n_chunks; c0 += 64) {
      const int c = c0 + lane;
      float w = 0.f, lw = 0.f;
      if (c < n_chunks) {
        const float2 ml = *reinterpret_cast<const float2 *>(part_ml + ((size_t)(first + c) * H + h) * 2);
        w = __builtin_amdgcn_exp2f(ml.x - M);
        lw = ml.y * w;
      }
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) lw += __shfl_xor(lw, off);
      L += lw;
      const int cnt = min(64, n_chunks - c0);
      int i = 0;
      for (; i + 4 <= cnt; i += 4) {                     // four independent rows in flight
        float x[4][EPT];
#pragma unroll
        for (int k = 0; k < 4; ++k)
#pragma unroll
          for (int e = 0; e < EPT; ++e)
            x[k][e] = a.part_o[((size_t)(first + c0 + i + k) * H + h) * D + lane * EPT + e];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const float wk = __shfl(w, i + k);
#pragma unroll
          for (int e = 0; e < EPT; ++e) acc[e] += x[k][e] * wk;
        }
      }
      for (; i < cnt; ++i) {
        const float wk = __shfl(w, i);
#pragma unroll
        for (int e = 0; e < EPT; ++e)
          acc[e] += a.part_o[((size_t)(first + c0 + i) * H + h) * D + lane * EPT + e] * wk;
      }
    }
  }
  const float inv = 1.0f / L;
  const size_t at = ((size_t)b * H + h) * D + lane * EPT;
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    if (a.out_fp32)
      reinterpret_cast<float *>(a.out)[at + e] = acc[e] * inv;
    else
      reinterpret_cast<_Float16 *>(a.out)[at + e] = (_Float16)(acc[e] * inv);
  }
}

// Tiles in flight per wavefront.  At d = 128 what counts is bytes: about 8 KiB per wavefront (one tile) times
// a thousand wavefronts is where the memory system runs best (6.4-6.7 TB/s); twice that measured 5.9-6.1.  At
// d = 64 a tile is half the bytes for the same chain of waits (LDS round trip, scores, softmax, weighted sum),
// and that chain, not the memory system, sets the pace: with every tile reduced on its own, two tiles in
// flight (8 KiB) ran at 5.3-5.4 TB/s (32 x 64 heads, batch 64, context 2048), four at 5.9, six at 6.1, eight
// at 6.2; launches of a few dozen microseconds gained less and the shortest lost to the longer loop body from
// six on (11.3 us with two, 11.7 with four, 12.6 with six, 13.9 with eight): four, which tile_update_pair
// reduces two at a time (6.25 TB/s).
#ifndef OKV_PIPE_MULT
#define OKV_PIPE_MULT 1
#endif
template <int D>
constexpr int base_depth() {
  return (D == 64 ? 4 : 1) * OKV_PIPE_MULT;
}

template <int D, bool PAGED, bool HEADS>
void launch_split_as(const AttnArgs &args, dim3 grid, hipStream_t stream) {
  hipLaunchKernelGGL((attn_split_mfma_kernel<D, PAGED, base_depth<D>(), HEADS>), grid, dim3(kWavesPerBlock * 64), 0, stream,
                     args.pair_head, args.pool, args.q, args.n_groups_dev, args.n_groups, args.G, args.H, args.R,
                     args.gg << args.st_log2, args);
}

template <int D>
hipError_t launch_split(const AttnArgs &args, bool paged, dim3 grid, hipStream_t stream) {
  const bool heads = args.pair_head != nullptr;
  if (paged)
    heads ? launch_split_as<D, true, true>(args, grid, stream) : launch_split_as<D, true, false>(args, grid, stream);
  else
    heads ? launch_split_as<D, false, true>(args, grid, stream) : launch_split_as<D, false, false>(args, grid, stream);
  return hipGetLastError();
}

}  // namespace

namespace {

AttnArgs make_args(const AttnLaunch &a) {
  const PoolShape &s = a.shape;
  AttnArgs args;
  args.q = static_cast<const uint16_t *>(a.q);
  args.pool = static_cast<const uint16_t *>(a.pool);
  args.k_new = static_cast<const uint16_t *>(a.k_new);
  args.v_new = static_cast<const uint16_t *>(a.v_new);
  args.pool_store = static_cast<uint16_t *>(a.pool);
  args.pool_mirror = static_cast<uint16_t *>(a.pool_mirror);
  args.out = a.out;
  args.part_o = a.part_o;
  args.part_ml = a.part_ml;
  args.block_table = a.batch.block_table;
  args.chunk_prefix = a.batch.chunk_prefix;
  args.item_desc = a.batch.item_desc;
  args.n_groups_dev = a.n_groups_dev;
  args.pair_head = static_cast<const PairHead *>(a.pair_head);
  args.n_groups = a.pair_head ? a.n_groups : a.item_count;
  args.H = s.H;
  args.G = s.G;
  args.R = s.H / s.G;
  args.log2_T = s.log2_T;
  args.tcap = s.tcap;
  args.gg = s.gg;
  args.st_log2 = s.st_log2;
  args.max_blocks = s.max_blocks;
  args.out_fp32 = a.out_fp32;
  args.item_first = a.item_first;
  args.id_base = a.id_base;
  args.mirror_shift = a.id_base - a.mirror_base;
  args.mirror_is_tail = a.mirror_is_tail;
  args.B = a.batch.B;
  args.n_cls = a.batch.n_cls;
  // exp(x) = 2^(x log2 e): the 1/sqrt(d) scale and log2 e are folded into one factor
  args.scale_log2e = 1.4426950408889634f / sqrtf((float)s.D);
  return args;
}

}  // namespace

hipError_t launch_decode_attn(const AttnLaunch &a, hipStream_t stream, hipEvent_t ev_begin,
                              hipEvent_t ev_end) {
  const PoolShape &s = a.shape;
  if (a.item_count <= 0 || a.item_first < 0 || a.item_first + a.item_count > a.batch.n_items)
    return hipErrorInvalidValue;
  AttnArgs args = make_args(a);
  const int R = s.H / s.G;
  // persistent launch: no more wavefronts than there are (group, KV head) pairs, no more than a.max_waves
  const int64_t want = ((int64_t)args.n_groups * s.G + kWavesPerBlock - 1) / kWavesPerBlock;
  const int64_t cap = std::max<int64_t>(1, a.max_waves / kWavesPerBlock);
  dim3 grid((unsigned)(a.n_groups_dev ? cap : std::min(want, cap)));
  // (stretches come with a table of heads, which needs a wavefront per (stretch, KV head) pair and a pool that
  // holds the blocks as the table numbers them)
  if (a.pair_head && (want > cap || a.id_base != 0 || a.item_first != 0)) return hipErrorInvalidValue;
  hipError_t e;
  if (ev_begin && (e = hipEventRecord(ev_begin, stream)) != hipSuccess) return e;
  if (R < 1 || R > 16 || R * s.G != s.H)
    e = hipErrorInvalidValue;
  else if (s.D == 128)
    e = launch_split<128>(args, s.paged != 0, grid, stream);
  else if (s.D == 64)
    e = launch_split<64>(args, s.paged != 0, grid, stream);
  else
    e = hipErrorInvalidValue;
  if (e != hipSuccess) return e;
  if (ev_end && (e = hipEventRecord(ev_end, stream)) != hipSuccess) return e;
  return hipSuccess;
}

hipError_t launch_merge(const AttnLaunch &a, hipStream_t stream) {
  const PoolShape &s = a.shape;
  const AttnArgs args = make_args(a);
  dim3 mgrid(s.H, a.batch.B);
  if (s.D == 128)
    hipLaunchKernelGGL(attn_merge_kernel<128>, mgrid, dim3(64), 0, stream, args.chunk_prefix, args.part_ml, args.B, args.n_cls, args.H, args);
  else if (s.D == 64)
    hipLaunchKernelGGL(attn_merge_kernel<64>, mgrid, dim3(64), 0, stream, args.chunk_prefix, args.part_ml, args.B, args.n_cls, args.H, args);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

// ---- step bookkeeping ------------------------------------------------------------

namespace {

constexpr int kStepThreads = 256;

// Inclusive scan of one value per thread over the workgroup's kStepThreads threads, and the sum of all of them:
// a shuffle scan inside every wavefront and one hand-over of the wavefronts' sums through LDS (two barriers,
// where a scan through shared memory needs two per doubling: the kernel runs once per step, in front of every
// layer's attention, and a single-sequence step is short enough to see the difference).
__device__ __forceinline__ int64_t block_scan(int64_t v, int64_t *wave_sums, int64_t *total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int64_t up = __shfl_up(v, off);
    if (lane >= off) v += up;
  }
  if (lane == 63) wave_sums[wave] = v;
  __syncthreads();
  int64_t before = 0, all = 0;
#pragma unroll
  for (int w = 0; w < kStepThreads / 64; ++w) {
    const int64_t sw = wave_sums[w];
    before += w < wave ? sw : 0;
    all += sw;
  }
  __syncthreads();                                       // wave_sums may be written again
  *total = all;
  return v + before;
}

__global__ __launch_bounds__(kStepThreads) void step_advance_kernel(int32_t *ctx_lens,
                                                                   int32_t *chunk_prefix,
                                                                   int4 *item_desc, int32_t B,
                                                                   int32_t S, int32_t inc) {
  __shared__ int64_t wave_sums[kStepThreads / 64];
  const int tid = threadIdx.x;
  const int per = (B + kStepThreads - 1) / kStepThreads;     // consecutive sequences per thread
  const int b0 = tid * per, b1 = min(B, b0 + per);
  int32_t mine = 0;
  for (int b = b0; b < b1; ++b) {
    const int32_t n = ctx_lens[b] + inc;
    ctx_lens[b] = n;
    int32_t cnt, sz;
    seq_chunks(n, S, &cnt, &sz);
    mine += cnt;
  }
  int64_t total_items;
  int32_t at = (int32_t)(block_scan(mine, wave_sums, &total_items) - mine);   // exclusive prefix of this thread
  for (int b = b0; b < b1; ++b) {
    chunk_prefix[b] = at;
    const int32_t n = ctx_lens[b];
    int32_t cnt, sz;
    seq_chunks(n, S, &cnt, &sz);
    for (int32_t c = 0; c < cnt; ++c) {
      const ItemRange r = chunk_range(b, c, sz, n);
      const int32_t flags = (c == cnt - 1 ? kItemLast : 0) | (cnt == 1 ? kItemWhole : 0);
      item_desc[at + c] = make_int4(r.b, r.lo, r.hi, flags);
    }
    at += cnt;
  }
  if (tid == kStepThreads - 1) chunk_prefix[B] = (int32_t)total_items;
}

// The bookkeeping for equal stretches: lengths advance, the tiles of all sequences are counted and
// laid end to end, cut into stretches (span_plan), every sequence into the pieces the cuts leave
// (span_pieces), and the first item of every stretch is noted in group_first.  plan_out receives
// (number of stretches in use, number of items, tiles per stretch as two halves).
__global__ __launch_bounds__(kStepThreads) void step_advance_spans_kernel(int32_t *ctx_lens, int32_t *chunk_prefix,
                                                                         int4 *item_desc, int32_t *group_first,
                                                                         int32_t *plan_out, int32_t B,
                                                                         int32_t max_groups, int32_t min_span,
                                                                         int32_t inc, PairHead *pair_head,
                                                                         const HeadGeom hg) {
  __shared__ int64_t wave_sums[kStepThreads / 64];
  // what opens each stretch, for the per-pair records: its first item, that item's descriptor and the block
  // ids of the item's first two tiles (the second clamped to the item's last tile)
  __shared__ int32_t open_item[kHeadGroupsMax + 1];
  __shared__ int4 open_desc[kHeadGroupsMax];
  __shared__ int2 open_blk[kHeadGroupsMax];
  const int tid = threadIdx.x;
  if (pair_head)
    for (int j = tid; j <= kHeadGroupsMax; j += kStepThreads) open_item[j] = -1;
  const int per = (B + kStepThreads - 1) / kStepThreads;     // consecutive sequences per thread
  const int b0 = min(B, tid * per), b1 = min(B, b0 + per);
  int64_t mine = 0;
  for (int b = b0; b < b1; ++b) {
    const int32_t n = ctx_lens[b] + inc;
    if (inc) ctx_lens[b] = n;                                  // inc == 0: the lengths are only read
    mine += (n + 15) >> 4;
  }
  int64_t total_tiles;
  const int64_t tile_first = block_scan(mine, wave_sums, &total_tiles) - mine;   // tiles before this thread's sequences
  const SpanPlan plan = span_plan(total_tiles, max_groups, min_span);
  int64_t items_mine = 0, first = tile_first;
  for (int b = b0; b < b1; ++b) {
    const int64_t tiles = (ctx_lens[b] + 15) >> 4;
    int64_t k0;
    items_mine += span_pieces(first, tiles, plan.span, &k0);
    first += tiles;
  }
  int64_t total_items;
  int32_t at = (int32_t)(block_scan(items_mine, wave_sums, &total_items) - items_mine);
  first = tile_first;
  for (int b = b0; b < b1; ++b) {
    chunk_prefix[b] = at;
    const int32_t n = ctx_lens[b];
    const int64_t tiles = (n + 15) >> 4;
    int64_t k0;
    const int32_t cnt = span_pieces(first, tiles, plan.span, &k0);
    for (int32_t c = 0; c < cnt; ++c) {
      int64_t group;
      const ItemRange r = span_piece(b, c, n, first, tiles, plan.span, k0, &group);
      const int32_t flags = (c == cnt - 1 ? kItemLast : 0) | (cnt == 1 ? kItemWhole : 0);
      item_desc[at + c] = make_int4(r.b, r.lo, r.hi, flags);
      if (c > 0 || first % plan.span == 0) {                               // the item opens its stretch
        group_first[group] = at + c;
        if (pair_head && group < kHeadGroupsMax) {
          open_item[group] = at + c;
          open_desc[group] = make_int4(r.b, r.lo, r.hi, flags);
          int2 blk = make_int2(b, b);
          if (hg.block_table) {
            const int32_t t0 = r.lo >> 4, t1 = min(t0 + 1, (r.hi - 1) >> 4);
            const int32_t *row = hg.block_table + (size_t)b * hg.max_blocks;
            blk.x = row[min((t0 << 4) >> hg.log2_T, hg.max_blocks - 1)];
            blk.y = row[min((t1 << 4) >> hg.log2_T, hg.max_blocks - 1)];
          }
          open_blk[group] = blk;
        }
      }
    }
    at += cnt;
    first += tiles;
  }
  if (tid == kStepThreads - 1) {
    group_first[plan.n_groups] = (int32_t)total_items;
    if (pair_head && plan.n_groups <= kHeadGroupsMax) open_item[plan.n_groups] = (int32_t)total_items;
  }
  if (pair_head) {
    // One record per (stretch, KV head) pair: the stretch's first item and where that head's rows of the
    // item's first two tiles lie.  Nothing is written for pairs past the last stretch: the attention kernel
    // knows how many stretches there are.
    __syncthreads();
    const int32_t St_mask = (1 << hg.st_log2) - 1;
    const int32_t n_pairs = (int32_t)min((int64_t)plan.n_groups * hg.G, (int64_t)hg.max_pairs);
    for (int p = tid; p < n_pairs; p += kStepThreads) {
      const int32_t group = p / hg.G, g = p - group * hg.G;
      PairHead h = {};
      const int32_t it = group < plan.n_groups && group < kHeadGroupsMax ? open_item[group] : -1;
      const int32_t n = it >= 0 ? open_item[group + 1] - it : 0;
      if (n > 0) {                                       // (a batch with no keys at all has one stretch and no item)
        h.item = it, h.count = n;
        const int4 d = open_desc[group];
        h.b = d.x, h.lo = d.y, h.hi = d.z, h.flags_g = d.w | (g << 8);
        const int32_t grp = g / hg.gg;
        const int32_t head_k = ((grp * 2 * hg.gg) << hg.st_log2) + (g - grp * hg.gg);
        const int32_t t0 = d.y >> 4, t_last = (d.z - 1) >> 4;
        for (int i = 0; i < 2; ++i) {
          const int32_t t = min(t0 + i, t_last);
          const int32_t blk = i ? open_blk[group].y : open_blk[group].x;
          const int64_t lin = (int64_t)blk * hg.tiles + (hg.block_table ? t & (hg.tiles - 1) : t);
          const int64_t base = (lin >> hg.st_log2) * ((int64_t)(2 * hg.G) << hg.st_log2) + (lin & St_mask) * hg.gg + head_k;
          (i ? h.base1 : h.base0) = (int32_t)base;
        }
      }
      pair_head[p] = h;
    }
  }
  if (tid == kStepThreads - 1) {
    const int32_t n_items = (int32_t)total_items;
    chunk_prefix[B] = n_items;
    plan_out[0] = plan.n_groups;
    plan_out[1] = n_items;
    plan_out[2] = (int32_t)(plan.span & 0x7fffffff);
    plan_out[3] = (int32_t)(plan.span >> 31);
  }
}

// The same bookkeeping when a sequence is cut into runs of one block class each.  Pairs
// (class, sequence) take the place of sequences: thread t owns a stretch of consecutive
// pairs, counts their items, the counts are scanned, and the items are written class by
// class.  chunk_prefix doubles as the store of the per-pair counts between the passes.
__global__ __launch_bounds__(kStepThreads) void step_advance_classes_kernel(
    int32_t *ctx_lens, const int4 *runs, const int32_t *pair_first, int32_t *chunk_prefix, int4 *item_desc,
    int32_t *seq_total, int32_t B, int32_t n_cls, int32_t S, int32_t inc) {
  __shared__ int32_t part[kStepThreads];
  const int tid = threadIdx.x;
  for (int b = tid; b < B; b += kStepThreads) ctx_lens[b] += inc;
  __syncthreads();
  const int P = n_cls * B;
  const int per = (P + kStepThreads - 1) / kStepThreads;
  const int p0 = min(P, tid * per), p1 = min(P, p0 + per);
  int32_t mine = 0;
  for (int p = p0; p < p1; ++p) {
    const int32_t n = ctx_lens[p % B];
    int32_t cnt = 0;
    for (int r = pair_first[p]; r < pair_first[p + 1]; ++r) {
      const int4 run = runs[r];
      int32_t sz;
      cnt += run_items(run.y, run.z, n, S, &sz);
    }
    chunk_prefix[p] = cnt;
    mine += cnt;
  }
  part[tid] = mine;
  __syncthreads();
  for (int b = tid; b < B; b += kStepThreads) {
    int32_t total = 0;
    for (int cls = 0; cls < n_cls; ++cls) total += chunk_prefix[cls * B + b];
    seq_total[b] = total;
  }
  for (int off = 1; off < kStepThreads; off <<= 1) {
    int32_t add = tid >= off ? part[tid - off] : 0;
    __syncthreads();
    part[tid] += add;
    __syncthreads();
  }
  int32_t at = part[tid] - mine;
  for (int p = p0; p < p1; ++p) {
    const int b = p % B;
    const int32_t n = ctx_lens[b];
    const int32_t whole = seq_total[b] == 1 ? kItemWhole : 0;
    chunk_prefix[p] = at;
    for (int r = pair_first[p]; r < pair_first[p + 1]; ++r) {
      const int4 run = runs[r];
      int32_t sz;
      const int32_t cnt = run_items(run.y, run.z, n, S, &sz);
      const int32_t end = run.z < n ? run.z : n;
      for (int32_t c = 0; c < cnt; ++c) {
        const int32_t lo = run.y + c * sz;
        const int32_t hi = lo + sz < end ? lo + sz : end;
        item_desc[at + c] = make_int4(b, lo, hi, (hi == n ? kItemLast : 0) | whole);
      }
      at += cnt;
    }
  }
  if (tid == kStepThreads - 1) chunk_prefix[P] = part[tid];
}

// Bulk store of new rows: one wavefront per (tile, K or V, KV head).  A tile's destination is
// one contiguous run of 16 * D * 2 bytes of the pool (the head's K or V rows in the tile's slab); its source rows are D * 2 bytes each,
// G * D * 2 bytes apart (token-major input, as a projection writes it).  Every lane moves 16
// bytes per load; rows outside [first, last) of the tile are left alone.
struct BulkArgs {
  const uint16_t *k_rows, *v_rows;
  uint16_t *pool;
  const int4 *tiles;
  const int32_t *row_base;
  int32_t G, gg, tcap, st_log2, n_units;
  int32_t drain_each_tile;   // wait for a tile's stores before starting the next one
};

template <int D, bool PAGED>
__global__ __launch_bounds__(256) void bulk_append_kernel(const BulkArgs a) {
  constexpr int LPR = D / 8, RPL = 64 / LPR, LPT = D / 32;
  const int lane = threadIdx.x & 63;
  const int row = lane / LPR, col = lane % LPR;
  const int n_waves = gridDim.x * 4;
  for (int unit = blockIdx.x * 4 + (threadIdx.x >> 6); unit < a.n_units; unit += n_waves) {
    const int t = unit / (2 * a.G);
    const int rest = unit - t * 2 * a.G;
    const int kv = rest / a.G, g = rest - kv * a.G;
    const int4 tile = a.tiles[t];
    const int b = tile.x, pos0 = tile.y << 4;
    const int first = tile.z & 0xff, last = tile.z >> 8;      // slots of the tile to store: [first, last)
    const int blk = tile.w;
    const TileAddr ta = tile_addr<D>(a.G, a.gg, a.tcap, a.st_log2, g);
    const uint16_t *src = (kv ? a.v_rows : a.k_rows) + (size_t)g * D + col * 8;
    uint16_t *dst = a.pool + slab_base<PAGED>(ta, blk, tile.y) + (kv ? ta.head_v : ta.head_k) + col * 8;
    const int64_t base_row = (int64_t)a.row_base[b] + pos0;
    uint4 v[LPT];
    bool ok[LPT];
#pragma unroll
    for (int j = 0; j < LPT; ++j) {
      const int r = row + j * RPL;
      ok[j] = r >= first && r < last;
      if (ok[j]) v[j] = *reinterpret_cast<const uint4 *>(src + (base_row + r) * a.G * D);
    }
#pragma unroll
    for (int j = 0; j < LPT; ++j) {
      const int r = row + j * RPL;
      if (ok[j]) *reinterpret_cast<uint4 *>(dst + (int64_t)r * D) = v[j];
    }
    // Stores into host memory leave at the link's pace.  Left alone, every wavefront queues
    // dozens of them and anything else on the GPU that has to drain the memory pipeline (each
    // kernel boundary does) waits behind that backlog; holding a wavefront to one tile in
    // flight keeps the backlog to a few KiB per wavefront at no cost in link rate.
    if (a.drain_each_tile) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }
}

// ---- the newest blocks of the sequences, kept in HBM (block-granular offload) ------------------
//
// Rows that a decode step appends to a block of the host pool are not stored across the link one by
// one: they go into a slot in HBM (two per sequence and layer, block j of a sequence uses slot j & 1)
// and the block is written to the host pool once, when it is full.  Until a copy of the host pool that
// was started after that write arrives, the staged chunk lacks those rows; this kernel puts them there
// (mode 0, before the chunk is attended) or writes them out (modes 1 and 2).  A block is
// tiles x [G / Gg][K|V][Gg][16 slots][D]; thread p moves the 16-byte piece p of the block if the
// piece's position lies in the range of rows wanted.
struct TailArgs {
  uint16_t *staged;                  // mode 0: the staged chunk (blocks id_lo .. id_hi - 1)
  uint16_t *const *host_pools;       // modes 1, 2: [layers] device-visible pointers to the host pools (block id_lo first)
  const uint16_t *tail;              // slots of the layer (mode 0) or of layer 0 (modes 1, 2)
  const int32_t *block_table, *ctx_lens, *tail_from;
  int64_t block_elems, layer_stride; // numbers per block; numbers between two layers' slots
  int32_t max_blocks, log2_T, d8;    // d8 = 16-byte pieces per row
  int32_t gg, st_log2;               // KV heads per group and log2 of the tiles per slab (see TileAddr)
  int32_t id_lo, id_hi;
  int32_t mode;                      // 0: blocks j and j - 1 of the newest position, rows before it, into the staged chunk
                                     // 1: the block that this step filled, to the host pool
                                     // 2: the newest block as far as it is filled, to the host pool
};

__global__ __launch_bounds__(256) void tail_rows_kernel(TailArgs a) {
  const int b = blockIdx.y;
  const int n = a.ctx_lens[b];
  const int T = 1 << a.log2_T;
  int j, hi;
  if (a.mode == 0) {
    j = ((n - 1) >> a.log2_T) - (int)blockIdx.z;
    hi = min((j + 1) << a.log2_T, n - 1);
  } else if (a.mode == 1) {
    if (n & (T - 1)) return;
    j = (n >> a.log2_T) - 1;
    hi = n;
  } else {
    j = (n - 1) >> a.log2_T;
    hi = n;
  }
  if (j < 0) return;
  const int lo = max(j << a.log2_T, a.tail_from[b]);
  if (lo >= hi) return;
  const int id = a.block_table[(size_t)b * a.max_blocks + j];
  if (id < a.id_lo || id >= a.id_hi) return;
  const int layer = a.mode == 0 ? 0 : (int)blockIdx.z;
  const uint4 *src = reinterpret_cast<const uint4 *>(a.tail + layer * a.layer_stride + (int64_t)(2 * b + (j & 1)) * a.block_elems);
  uint16_t *dst_pool = a.mode == 0 ? a.staged : a.host_pools[layer];
  uint4 *dst = reinterpret_cast<uint4 *>(dst_pool + (int64_t)(id - a.id_lo) * a.block_elems);
  const int lo_in = lo - (j << a.log2_T), hi_in = hi - (j << a.log2_T);
  const int pieces = (int)(a.block_elems >> 3);
  const int slab_pieces = pieces >> (a.log2_T - 4 - a.st_log2);
  for (int p = blockIdx.x * blockDim.x + threadIdx.x; p < pieces; p += gridDim.x * blockDim.x) {
    const int slab = p / slab_pieces;
    const int row = (p - slab * slab_pieces) / a.d8;                  // ((group, kv), tile in slab, head in group, slot)
    const int pos = (((slab << a.st_log2) + ((row / (16 * a.gg)) & ((1 << a.st_log2) - 1))) << 4) + (row & 15);
    if (pos >= lo_in && pos < hi_in) dst[p] = src[p];
  }
}

__global__ void worklist_dump_kernel(BatchState bs, int32_t *items) {
  const int it = blockIdx.x * blockDim.x + threadIdx.x;
  if (it >= bs.n_items) return;
  const int4 d = bs.item_desc[it];
  items[it * 3 + 0] = d.x;
  items[it * 3 + 1] = d.y;
  items[it * 3 + 2] = d.z;
}

__global__ __launch_bounds__(256) void probe_copy_kernel(uint4 *dst, const uint4 *src, int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void probe_read_kernel(const uint4 *src, int64_t n, uint32_t *sink) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  uint32_t acc = 0;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
    const uint4 v = src[i];
    acc ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  if (acc == 0x9E3779B9u) *sink = acc;    // practically never true; keeps the loads alive
}

}  // namespace

hipError_t launch_step_advance(int32_t *ctx_lens, int32_t *chunk_prefix, int4 *item_desc, int32_t B, int32_t S,
                               int32_t inc, hipStream_t stream) {
  hipLaunchKernelGGL(step_advance_kernel, dim3(1), dim3(kStepThreads), 0, stream, ctx_lens, chunk_prefix, item_desc,
                     B, S, inc);
  return hipGetLastError();
}

hipError_t launch_step_advance_spans(int32_t *ctx_lens, int32_t *chunk_prefix, int4 *item_desc, int32_t *group_first,
                                     int32_t *plan_out, int32_t B, int32_t max_groups, int32_t min_span, int32_t inc,
                                     void *pair_head, const HeadGeom &geom, hipStream_t stream) {
  hipLaunchKernelGGL(step_advance_spans_kernel, dim3(1), dim3(kStepThreads), 0, stream, ctx_lens, chunk_prefix,
                     item_desc, group_first, plan_out, B, max_groups, min_span, inc, static_cast<PairHead *>(pair_head),
                     geom);
  return hipGetLastError();
}

hipError_t launch_step_advance_classes(int32_t *ctx_lens, const int4 *runs, const int32_t *pair_first,
                                       int32_t *chunk_prefix, int4 *item_desc, int32_t *seq_total, int32_t B,
                                       int32_t n_cls, int32_t S, int32_t inc, hipStream_t stream) {
  hipLaunchKernelGGL(step_advance_classes_kernel, dim3(1), dim3(kStepThreads), 0, stream, ctx_lens, runs,
                     pair_first, chunk_prefix, item_desc, seq_total, B, n_cls, S, inc);
  return hipGetLastError();
}

hipError_t launch_bulk_append(const BulkLaunch &a, hipStream_t stream) {
  if (a.n_tiles <= 0) return hipSuccess;
  const PoolShape &s = a.shape;
  BulkArgs args;
  args.k_rows = static_cast<const uint16_t *>(a.k_rows);
  args.v_rows = static_cast<const uint16_t *>(a.v_rows);
  args.pool = static_cast<uint16_t *>(a.pool);
  args.tiles = a.tiles;
  args.row_base = a.row_base;
  args.G = s.G;
  args.gg = s.gg;
  args.st_log2 = s.st_log2;
  args.tcap = s.tcap;
  const int64_t units = (int64_t)a.n_tiles * 2 * s.G;
  if (units > 0x7fffffff) return hipErrorInvalidValue;
  args.n_units = (int32_t)units;
  args.drain_each_tile = a.throttle;
  int64_t blocks = (units + 3) / 4;
  if (a.max_workgroups > 0) blocks = std::min<int64_t>(blocks, a.max_workgroups);
  blocks = std::min<int64_t>(blocks, 1 << 20);
  dim3 grid((unsigned)blocks);
  if (s.D == 128) {
    if (s.paged) hipLaunchKernelGGL((bulk_append_kernel<128, true>), grid, dim3(256), 0, stream, args);
    else hipLaunchKernelGGL((bulk_append_kernel<128, false>), grid, dim3(256), 0, stream, args);
  } else if (s.D == 64) {
    if (s.paged) hipLaunchKernelGGL((bulk_append_kernel<64, true>), grid, dim3(256), 0, stream, args);
    else hipLaunchKernelGGL((bulk_append_kernel<64, false>), grid, dim3(256), 0, stream, args);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_tail_rows(const TailLaunch &t, hipStream_t stream) {
  if (t.B <= 0) return hipSuccess;
  TailArgs a;
  a.staged = static_cast<uint16_t *>(t.staged);
  a.host_pools = reinterpret_cast<uint16_t *const *>(t.host_pools);
  a.tail = static_cast<const uint16_t *>(t.tail);
  a.block_table = t.block_table;
  a.ctx_lens = t.ctx_lens;
  a.tail_from = t.tail_from;
  a.block_elems = t.block_elems;
  a.layer_stride = t.layer_stride;
  a.max_blocks = t.max_blocks;
  a.log2_T = t.log2_T;
  a.d8 = t.D / 8;
  a.gg = t.gg;
  a.st_log2 = t.st_log2;
  a.id_lo = t.id_lo;
  a.id_hi = t.id_hi;
  a.mode = t.mode;
  const int64_t pieces = t.block_elems / 8;
  const unsigned gx = (unsigned)std::max<int64_t>(1, std::min<int64_t>((pieces + 255) / 256, 64));
  hipLaunchKernelGGL(tail_rows_kernel, dim3(gx, t.B, t.mode == 0 ? 2 : t.n_layers), dim3(256), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_worklist_dump(const BatchState &batch, int32_t *items, hipStream_t stream) {
  if (batch.n_items <= 0) return hipSuccess;
  hipLaunchKernelGGL(worklist_dump_kernel, dim3((batch.n_items + 255) / 256), dim3(256), 0, stream,
                     batch, items);
  return hipGetLastError();
}

hipError_t launch_probe_copy(void *dst, const void *src, int64_t bytes, hipStream_t stream) {
  const int64_t n = bytes / 16;
  if (n <= 0) return hipSuccess;
  const int64_t want = (n + 255) / 256;
  const unsigned blocks = (unsigned)(want < 256 * 32 ? want : 256 * 32);
  hipLaunchKernelGGL(probe_copy_kernel, dim3(blocks), dim3(256), 0, stream,
                     static_cast<uint4 *>(dst), static_cast<const uint4 *>(src), n);
  return hipGetLastError();
}

hipError_t launch_probe_read(const void *src, int64_t bytes, void *sink, hipStream_t stream) {
  const int64_t n = bytes / 16;
  if (n <= 0) return hipSuccess;
  const int64_t want = (n + 255) / 256;
  const unsigned blocks = (unsigned)(want < 256 * 32 ? want : 256 * 32);
  hipLaunchKernelGGL(probe_read_kernel, dim3(blocks), dim3(256), 0, stream,
                     static_cast<const uint4 *>(src), n, static_cast<uint32_t *>(sink));
  return hipGetLastError();
}

}  // namespace okv
