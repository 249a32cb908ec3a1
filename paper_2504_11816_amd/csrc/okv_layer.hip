// Linear layers and layer norm of a decoder layer in the decode stage, for gfx950.
//
// out[m][n] = sum_k x[m][k] W[n][k] for a batch of at most 128 rows (paper §IV-D: the
// 8 h1^2 + 4 h1 h2 flops per token of the four projections and the feed-forward block).
// With so few rows every weight is read once and used `m` times: the product is bound by
// streaming W from HBM, so the kernel is built like the attention kernel -- long runs of
// 16-byte-per-lane loads kept many deep in flight -- with the matrix cores doing the
// arithmetic on the side (one fp16 instruction per KiB of weights and 16 rows of x: a few
// percent of the time the loads take).
//
//   * weights are stored pre-arranged (okv_pack_linear_weight) so that one load instruction
//     brings a wavefront the 1 KiB it feeds to one 16x16x32 matrix-core instruction per 16 rows:
//     16 output features x 32 inputs, lane l holding feature l % 16, inputs 8 (l / 16) .. + 7;
//   * beyond a few rows, the rows of x must NOT be fetched per lane in the layout the matrix core
//     wants: such a gather touches 16 half cache lines per instruction, every wavefront needs
//     its own, and the time grows with the rows although x sits in L2 (16384 x 4096, weights
//     from HBM: 25.4 us at 4 rows, 26.6 at 8, 34.3 at 16).  So in the fast kernel a workgroup of
//     4 (or 3) wavefronts takes 64 (48) output features, one 16-feature tile per wavefront, over
//     one stretch of the input dimension, and one more wavefront stages the rows of x for that
//     stretch chunk by chunk in LDS, from where the others read their operands.  The staging
//     wavefront fetches whole rows of a chunk (512 contiguous bytes each), keeps three chunks
//     ahead of the others and meets them at one barrier per 256 inputs; it is a wavefront of
//     its own because the vector memory counter retires loads in order: a wavefront that waited
//     for staged rows would also wait for the weight pieces it issued before them.  16384 x
//     4096 from HBM: 28.4 us at 32 rows, 31.0 at 64, 44.6 at 128; with the staging switched off
//     (timing only) 27.6 and 28.5, of which about 5 us do not depend on the size of the matrix;
//   * the input dimension is cut across workgroups so that the launch has one per compute
//     unit (longer-lived workgroups measured faster than more of them); each writes its fp32
//     share of the tile and a small second kernel adds the shares in a fixed order and applies
//     the epilogue (bias, ReLU, residual, rounding to fp16, scatter into up to three output
//     tensors).  A hand-over inside the kernel (last workgroup adds up) needs device-wide
//     fences, which on this GPU write back and invalidate the L2 caches: 75 us instead of 11.
//     Where three tiles per workgroup fill the compute units without a cut (12288 features on
//     256 units) the workgroups have three streaming wavefronts and there is no second kernel;
//   * up to 8 rows, and shapes the fast kernel does not take (input dimension not a multiple
//     of 256), run the simple kernel: a workgroup per 16 features, its wavefronts split the
//     inputs and add up through LDS, x by gather.
#include "okv_kernels.h"
#include "okv_layer.h"

#include <algorithm>

namespace okv {

namespace {

typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

#ifndef OKV_LIN_DEPTH
#define OKV_LIN_DEPTH 8
#endif
// Up to this many rows the simple kernel is the faster one (its gather of x costs in proportion to the rows, and it
// has more, shorter-lived workgroups and needs no second kernel); measured with the weights coming from HBM, 16384 x
// 4096: 26.6 us against 27.0 at 8 rows, 27.8 against 26.9 at 10, 34.3 against 27.4 at 16.
#ifndef OKV_LIN_SIMPLE_ROWS
#define OKV_LIN_SIMPLE_ROWS 8
#endif
#ifndef OKV_LIN_WAVES
#define OKV_LIN_WAVES 4
#endif
constexpr int kLinWaves = OKV_LIN_WAVES;

template <int MF>
constexpr int lin_depth() {
  return MF <= 2 ? OKV_LIN_DEPTH : MF <= 4 ? OKV_LIN_DEPTH / 2 : OKV_LIN_DEPTH / 4;   // pieces in flight: bounded by the registers x needs beside them
}

struct LinearArgs {
  const uint4 *x;          // [m][n_in] fp16, as 16-byte pieces
  const uint4 *w;          // packed weights
  const _Float16 *bias, *residual;
  _Float16 *out[3];
  int32_t m, n_in, n_kb, relu;
  int32_t seg0_cols, seg_cols;      // width of the first output tensor, of the others (multiples of 16)
  int32_t n_tiles, n_out, splits;   // fast path: 16-feature tiles, cuts of the input dimension
  float *shares;                    // fast path, splits > 1 or a layer norm to follow: [splits][m][n_out] fp32
  int32_t to_shares;                // fast path: write the share even when there is a single cut
  const _Float16 *ln_gamma, *ln_beta;
  _Float16 *ln_out;                 // layer norm of the result, or NULL
  float ln_eps;
};

// Feature n of row mrow lands in output tensor `seg` at element `at` (the tensors are [m][their width]).
__device__ __forceinline__ void seg_of(const LinearArgs &a, int mrow, int n, int &seg, size_t &at) {
  if (n < a.seg0_cols) {
    seg = 0;
    at = (size_t)mrow * a.seg0_cols + n;
  } else {
    const int r = n - a.seg0_cols;
    seg = 1 + r / a.seg_cols;
    at = (size_t)mrow * a.seg_cols + (r - (seg - 1) * a.seg_cols);
  }
}

__device__ __forceinline__ floatx4 mfma16(const uint2 a, const uint2 b, floatx4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(half4, a), __builtin_bit_cast(half4, b), c, 0, 0, 0);
}

// 16 x 16 result tile += [16 rows][32 inputs] . [32 inputs][16 features]; a lane's 16 bytes of either operand are
// inputs 8 (lane / 16) .. + 7 of row (feature) lane % 16
__device__ __forceinline__ floatx4 mfma32(const uint4 a, const uint4 b, floatx4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, b), c, 0, 0, 0);
}

template <int MF>
__global__ __launch_bounds__(kLinWaves * 64) void linear_kernel(const uint4 *w, const uint4 *x, const int32_t n_kb,
                                                                   const int32_t n_in, const int32_t m, const LinearArgs a) {
  // (leading parameters: in scalar registers when the wavefront starts, see linear_lds_kernel)
  constexpr int D = lin_depth<MF>();
  __shared__ floatx4 part[kLinWaves][MF][64];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);      // uniform: the loops below are scalar loops
  const int ntile = blockIdx.x;
  const int kb0 = (int)((int64_t)wave * n_kb / kLinWaves), kb1 = (int)((int64_t)(wave + 1) * n_kb / kLinWaves);
  const int nk = kb1 - kb0;
  const uint4 *wp = w + ((size_t)ntile * n_kb + kb0) * 64 + lane;
  // this lane's piece of x for k-block kb and row fragment f: row 16 f + lane % 16, inputs 32 kb + 8 (lane / 16) .. + 7
  const int row = lane & 15, kq = lane >> 4;
  const int row_pieces = n_in >> 3;
  // Rows past the batch read row 0 instead: a row of x only ever reaches the same row of the
  // result, and those rows are not stored.
  const uint4 *xp[MF];
#pragma unroll
  for (int f = 0; f < MF; ++f)
    xp[f] = x + (size_t)(f * 16 + row < m ? f * 16 + row : 0) * row_pieces + (size_t)kb0 * 4 + kq;
  floatx4 acc[MF];
#pragma unroll
  for (int f = 0; f < MF; ++f) acc[f] = floatx4{0.f, 0.f, 0.f, 0.f};

  uint4 wbuf[D], xbuf[D][MF];
  // Every wavefront walks its blocks from a different starting point (and wraps around).  All
  // ranges have the same length and all wavefronts advance at the same pace, so without the
  // shift every wavefront of the launch would be reading addresses that are equal modulo the
  // range length at any moment, i.e. from a few of the memory channels at a time (the same shift
  // in the staged kernel below is worth up to 10 % on weights that come from HBM).
  const int rot = nk > 0 ? (int)(((unsigned)ntile * 5u + (unsigned)wave * 11u) % (unsigned)nk) : 0;
  auto load = [&](int slot, int k) {                           // k: position in this wavefront's walk
    int kk = k + rot;
    kk = kk >= nk ? kk - nk : kk;                              // block index relative to kb0
    wbuf[slot] = wp[(size_t)kk * 64];
#pragma unroll
    for (int f = 0; f < MF; ++f) xbuf[slot][f] = xp[f][(size_t)kk * 4];
  };
  auto use = [&](int slot) {
    const uint4 w = wbuf[slot];
#pragma unroll
    for (int f = 0; f < MF; ++f) {
      const uint4 x = xbuf[slot][f];
      acc[f] = mfma16(make_uint2(x.x, x.y), make_uint2(w.x, w.y), acc[f]);
      acc[f] = mfma16(make_uint2(x.z, x.w), make_uint2(w.z, w.w), acc[f]);
    }
  };
  int k = 0;
  if (nk >= 2 * D) {
#pragma unroll
    for (int i = 0; i < D; ++i) {
      load(i, i);
      __builtin_amdgcn_sched_barrier(0);    // oldest first: the loop waits for the loads in this order
    }
    for (; k + 2 * D <= nk; k += D) {                          // steady state: no conditional loads
#pragma unroll
      for (int i = 0; i < D; ++i) {
        use(i);
        __builtin_amdgcn_sched_barrier(0);
        load(i, k + D + i);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < D; ++i)
      if (i < nk) load(i, i);
  }
  // drain: at most 2 D - 1 blocks are left, the first D of them in flight
#pragma unroll
  for (int i = 0; i < D; ++i)
    if (k + i < nk) {
      use(i);
      if (k + D + i < nk) load(i, k + D + i);
    }
#pragma unroll
  for (int i = 0; i < D; ++i)
    if (k + D + i < nk) use(i);

  // add the wavefronts' shares and finish: result element (row 16 f + 4 (lane / 16) + r, feature lane % 16)
  // sits in acc[f][r] of that lane
#pragma unroll
  for (int f = 0; f < MF; ++f) part[wave][f][lane] = acc[f];
  __syncthreads();
  for (int o = threadIdx.x; o < MF * 256; o += kLinWaves * 64) {
    const int mrow = o >> 4, j = o & 15;
    if (mrow >= m) continue;
    const int f = mrow >> 4, src_lane = j + 16 * ((mrow & 15) >> 2), r = mrow & 3;
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < kLinWaves; ++w) v += part[w][f][src_lane][r];
    const int n = ntile * 16 + j;
    if (a.bias) v += (float)a.bias[n];
    if (a.relu) v = fmaxf(v, 0.f);
    int seg;
    size_t at;
    seg_of(a, mrow, n, seg, at);
    if (a.residual) v += (float)a.residual[at];
    a.out[seg][at] = (_Float16)v;
  }
}

// Fast path: NW wavefronts x 16 features, x staged in LDS by one or two more wavefronts, input
// dimension cut across workgroups.  NW = 4 or 3 and the number of cuts: whatever linear_plan's model of the
// launch prefers (3 and no cut for 12288 features on 256 compute units, which saves the kernel that adds up
// the shares).
// 32-input blocks per staged chunk of x: 8 (256 inputs), 4 from 112 rows on.  A chunk takes chunk x MF KiB of LDS
// and there are lead + 1 of them: 128 KiB at most up to 128 rows (4 x 32 at 64 and at 128 rows), 144 at 96 rows
// (3 x 48) and from 129 to 192 rows (9 to 12 fragments of 16 rows: 3 x 36 .. 3 x 48).
constexpr int lin_chunk(int mf) { return mf <= 6 ? 8 : 4; }
// How many chunks of x the staging wavefronts are ahead of the others (one LDS buffer more than that).  Bounded by
// LDS and by the counter of loads in flight, which stops at 63: the wait for a chunk leaves the loads of the
// lead - 1 chunks after it outstanding.
constexpr int lin_lead(int mf) { return mf == 5 || mf == 6 || mf > 8 ? 2 : 3; }
// Staging wavefronts per workgroup: two from 64 rows on, each taking every other instruction of a chunk.  (At 128
// rows the rows of x that the workgroups fetch from L2 are twice the bytes of the weights, and that traffic is
// what the time then follows: 16384 x 4096 takes 40 us, 31 with the staging switched off, whether one wavefront
// stages or two, whatever the lead; the second wavefront is worth 1 us.)
constexpr int lin_stagers(int mf) { return mf >= 4 ? 2 : 1; }
// chunks of weights a streaming wavefront has in flight: 8 KiB either way
constexpr int lin_weight_lead(int mf) { return 8 / lin_chunk(mf) > 1 ? 8 / lin_chunk(mf) : 1; }
// s_waitcnt operand that waits until at most n vector memory loads are outstanding and for nothing else
constexpr int vmcnt_only(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }

// waves_per_eu: a workgroup has one or two wavefronts per SIMD and a compute unit holds one workgroup (LDS), so
// up to 128 registers cost nothing (256 with more than 8 row fragments, whose accumulators and operand registers
// need them: a SIMD holds two of the workgroup's six wavefronts at most); without the hint the compiler aimed
// at the occupancy the launch bounds allow and capped the kernel at 64.
template <int MF, int NW>
__global__ __launch_bounds__((NW + lin_stagers(MF)) * 64) __attribute__((amdgpu_waves_per_eu(1, MF > 8 ? 2 : 4))) void linear_lds_kernel(
    const uint4 *w, const uint4 *x, const int32_t n_kb, const int32_t splits, const int32_t n_in, const int32_t m,
    const int32_t n_tiles, const LinearArgs a) {
  // (the parameters in front of `a` are what the first loads need: the build has the leading kernel arguments
  // arrive in scalar registers with the wavefront, so the weight stream starts without a round trip to the
  // argument segment)
  constexpr int NS = lin_stagers(MF);
  constexpr int kFastThreads = (NW + NS) * 64, kTileCols = NW * 16;      // kTileCols: output features of a workgroup
  constexpr int C = lin_chunk(MF), LEAD = lin_lead(MF), NBUF = LEAD + 1, PER = C * MF, MINE = PER / NS;
  static_assert(PER % NS == 0 && (LEAD - 1) * MINE <= 63, "the wait for a staged chunk must fit the load counter");
  // A chunk of x, 16 MF rows of LPR 16-byte pieces (LPR x 8 inputs), as PER staging instructions' worth of 64
  // pieces each.  An operand read takes, for block i of the chunk, piece 4 i + q of row 16 f + rr in lane 16 q + rr.
  // The LDS serves a 16-byte-per-lane read in groups of 16 lanes that are not consecutive (lanes 0-3, 12-15, 20-23,
  // 24-27 and so on: measured, a layout that only spread 16 consecutive lanes over the banks had every read take
  // twice its cycles), so the bank (16-byte unit modulo 16) of a piece is (rr + 2 i + q / 2) mod 16: it does not
  // depend on the low bit of q, and within any such group all 16 rows rr occur once.  The two pieces that share
  // a bank (q even and odd) and the rows of an instruction take the unit's upper bits:
  //   unit = 64 * instruction + 16 * (2 * (rr & 1) + (q & 1)) + bank,
  //   instruction = 8 f + rr / 2 (8 blocks a chunk: rows 2 t and 2 t + 1, 512 bytes each), or
  //                 4 f + (rr % 8) / 2 (4 blocks: rows 2 t, 2 t + 1, 2 t + 8, 2 t + 9, 256 bytes each; of rr and
  //                 rr + 8 exactly one has (bank - rr) mod 16 below 8, which is where 2 i + q / 2 lives then).
  // After the last chunk the same memory holds the fp32 tile [16 MF rows][kTileCols features] for the epilogue.
  static_assert(C == 8 || C == 4, "the LDS layout of x is laid out for chunks of 8 or 4 blocks");
  constexpr int LPR = C * 4, IPF = C;                  // pieces per row; staging instructions per 16 rows
  __shared__ uint4 xs[NBUF][PER][64];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int group = blockIdx.x, cut = blockIdx.y;
  const int nk = n_kb / splits, kb0 = cut * nk, n_chunks = nk / C;
  floatx4 acc[MF];
#pragma unroll
  for (int f = 0; f < MF; ++f) acc[f] = floatx4{0.f, 0.f, 0.f, 0.f};
  // Every workgroup walks its chunks from a different starting point (and wraps around): all stretches have
  // the same length and all workgroups advance at the same pace, so without the shift the whole launch would
  // be reading addresses that are equal modulo the stretch length at any moment, i.e. from a few of the
  // memory channels at a time (16384 x 4096 at 32 rows, weights from HBM: 31.7 us without, 28.8 with).
  const int rot = (int)(((unsigned)group * 5u + (unsigned)cut * 3u) % (unsigned)n_chunks);
  auto rotc = [&](int c) { int cc = c + rot; return cc >= n_chunks ? cc - n_chunks : cc; };

  if (wave >= NW) {
    // The staging wavefront.  Its loads have a counter of their own, so waiting for them never
    // holds up the weight stream of the others.  A load instruction writes straight into LDS, 16 bytes per
    // lane, lane l landing in unit l of the instruction's 1 KiB; every lane fetches the piece that belongs
    // there.  An instruction brings whole rows of the chunk (2 x 512 or 4 x 256 contiguous bytes).  (Fetched in
    // the order the matrix core reads -- 16 rows x 64 bytes per instruction -- the same bytes took twice as
    // many half-used cache lines.)
    const int row_pieces = n_in >> 3;
    const int bank = lane & 15, ql = (lane >> 4) & 1, odd = lane >> 5;
    const int first = wave - NW;                   // this staging wavefront takes instructions first, first + NS, ...
    const uint4 *xg[MINE];
#pragma unroll
    for (int k = 0; k < MINE; ++k) {
      const int j = first + NS * k;
      const int f = j / IPF, t = j % IPF;
      int rr = 2 * t + odd;
      const int d = (bank - rr) & 15;
      if (C == 4 && d >= 8) rr += 8;
      const int v = C == 4 ? (d & 7) : d;                            // 2 i + q / 2
      const int piece = 4 * (v >> 1) + 2 * (v & 1) + ql;
      const int row = 16 * f + rr;                 // rows past the batch read row 0: they only reach result rows that are not stored
      xg[k] = x + (size_t)(row < m ? row : 0) * row_pieces + (size_t)kb0 * 4 + piece;
    }
    auto stage = [&](int chunk, int buf) {
#pragma unroll
      for (int k = 0; k < MINE; ++k)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(xg[k] + (size_t)chunk * LPR),
                                         (__attribute__((address_space(3))) void *)&xs[buf][first + NS * k][0], 16, 0, 0);
    };
    // LEAD chunks ahead of the others, so that a chunk has LEAD of their chunk times to arrive, not one (with one:
    // 3 us of 30 at 32 rows and 16 of 44 at 64 rows went into waiting for it, 16384 x 4096).  Before barrier c
    // chunk c must have landed: the loads of the chunks issued after it, LEAD - 1 of them except at the end, may
    // still be on their way.
    auto landed = [&](int c) {
      if (n_chunks - 1 - c >= LEAD - 1) __builtin_amdgcn_s_waitcnt(vmcnt_only((LEAD - 1) * MINE));
      else __builtin_amdgcn_s_waitcnt(vmcnt_only(0));
    };
#pragma unroll
    for (int j = 0; j < LEAD; ++j)
      if (j < n_chunks) stage(rotc(j), j);
    landed(0);
    __builtin_amdgcn_s_barrier();
    int buf = LEAD;
    for (int c = 0; c < n_chunks; ++c) {
      // the buffer of chunk c - 1: the others finished with it before the barrier this wavefront just passed
      if (c + LEAD < n_chunks) stage(rotc(c + LEAD), buf);
      buf = buf + 1 == NBUF ? 0 : buf + 1;
      if (c + 1 < n_chunks) landed(c + 1);
      __builtin_amdgcn_s_barrier();
    }
  } else {
    const int ntile = group * NW + wave;
    // a wavefront past the last tile streams tile 0 (valid memory) and never stores
    const uint4 *wp = w + ((size_t)(ntile < n_tiles ? ntile : 0) * n_kb + kb0) * 64 + lane;
    // where this lane's operand pieces sit in a chunk (see the layout above): rr = lane % 16, q = lane / 16
    const int rr = lane & 15, q = lane >> 4;
    const int xbase = 64 * (C == 8 ? rr >> 1 : (rr & 7) >> 1) + 16 * (2 * (rr & 1) + (q & 1));
    const int xrq = rr + (q >> 1);
    auto xat = [&](int buf, int i, int f) -> uint4 {
      return (&xs[buf][0][0])[64 * IPF * f + xbase + ((xrq + 2 * i) & 15)];
    };
    // Weights are fetched WD chunks ahead: with more than 64 rows a chunk is only 4 blocks (LDS), and 4 KiB in
    // flight, each refill waiting behind eight matrix instructions, did not keep the stream going (16384 x 4096
    // at 128 rows: 43 us; without the staging and the LDS reads still 36).
    constexpr int WD = lin_weight_lead(MF);
    uint4 wbuf[WD][C];
    auto ahead = [&](int c) { return rotc(c < n_chunks ? c : n_chunks - 1); };   // past the end: the last chunk again
#pragma unroll
    for (int u = 0; u < WD; ++u)
#pragma unroll
      for (int i = 0; i < C; ++i) {                          // oldest first: the loop waits for them in this order
        wbuf[u][i] = wp[((size_t)ahead(u) * C + i) * 64];
        __builtin_amdgcn_sched_barrier(0);
      }
    __syncthreads();
    int buf = 0;
    for (int c0 = 0; c0 < n_chunks; c0 += WD) {
#pragma unroll
      for (int u = 0; u < WD; ++u) {
        const int c = c0 + u;                    // the host only cuts the inputs into stretches of a multiple of WD chunks
        // the chunk WD after this one (past the end the last chunk is fetched once more instead of branching:
        // loads in this loop stay unconditional, so the waits stay exact)
        const int cn = ahead(c + WD);
        // the rows of x for a block are asked from LDS before the matrix instructions of the block before it are
        // issued (two sets of registers), so that they arrive while those run and while this wavefront waits for
        // the block's weights
        uint4 xr[2][MF];
#pragma unroll
        for (int f = 0; f < MF; ++f) xr[0][f] = xat(buf, 0, f);
#pragma unroll
        for (int i = 0; i < C; ++i) {
          if (i + 1 < C) {
#pragma unroll
            for (int f = 0; f < MF; ++f) xr[(i + 1) & 1][f] = xat(buf, i + 1, f);
          }
          const uint4 w = wbuf[u][i];
#pragma unroll
          for (int f = 0; f < MF; ++f) acc[f] = mfma32(xr[i & 1][f], w, acc[f]);
          __builtin_amdgcn_sched_barrier(0);
          wbuf[u][i] = wp[((size_t)cn * C + i) * 64];
          __builtin_amdgcn_sched_barrier(0);
        }
        buf = buf + 1 == NBUF ? 0 : buf + 1;
        __syncthreads();
      }
    }
  }

  // this workgroup's share of the tile [16 MF][128] in LDS (all reads of xs are behind the barrier above):
  // result element (row 16 f + 4 (lane / 16) + r, feature 16 wave + lane % 16) sits in acc[f][r]
  float *tile = reinterpret_cast<float *>(&xs[0][0][0]);
  if (wave < NW) {
#pragma unroll
    for (int f = 0; f < MF; ++f)
#pragma unroll
      for (int r = 0; r < 4; ++r) tile[(f * 16 + 4 * (lane >> 4) + r) * kTileCols + wave * 16 + (lane & 15)] = acc[f][r];
  }
  __syncthreads();
  // eight neighbouring features of a row per thread (feature counts and segment widths are multiples of 16, so
  // a group of eight never straddles a segment and every access below is one aligned 16-byte piece)
  const int n0 = group * kTileCols;
  constexpr int VPR = kTileCols / 8;
  if (splits > 1 || a.to_shares) {                   // this cut's share; a second kernel adds them up
    float *mine = a.shares + (size_t)cut * m * a.n_out;
    for (int o = tid; o < m * VPR; o += kFastThreads) {
      const int mrow = o / VPR, n = n0 + 8 * (o % VPR);
      if (n >= a.n_out) continue;
      const float4 *t = reinterpret_cast<const float4 *>(tile + mrow * kTileCols + 8 * (o % VPR));
      float4 *dst = reinterpret_cast<float4 *>(mine + (size_t)mrow * a.n_out + n);
      dst[0] = t[0];
      dst[1] = t[1];
    }
    return;
  }
  for (int o = tid; o < m * VPR; o += kFastThreads) {
    const int mrow = o / VPR, n = n0 + 8 * (o % VPR);
    if (n >= a.n_out) continue;
    const float4 *t = reinterpret_cast<const float4 *>(tile + mrow * kTileCols + 8 * (o % VPR));
    const float4 t0 = t[0], t1 = t[1];
    float v[8] = {t0.x, t0.y, t0.z, t0.w, t1.x, t1.y, t1.z, t1.w};
    int seg;
    size_t at;
    seg_of(a, mrow, n, seg, at);
    uint4 bb = make_uint4(0u, 0u, 0u, 0u), rb = bb;
    if (a.bias) bb = *reinterpret_cast<const uint4 *>(a.bias + n);
    if (a.residual) rb = *reinterpret_cast<const uint4 *>(a.residual + at);
    const _Float16 *bp = reinterpret_cast<const _Float16 *>(&bb), *rp = reinterpret_cast<const _Float16 *>(&rb);
    uint4 yo;
    _Float16 *yp = reinterpret_cast<_Float16 *>(&yo);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float y = v[e] + (float)bp[e];
      if (a.relu) y = fmaxf(y, 0.f);
      y += (float)rp[e];
      yp[e] = (_Float16)y;
    }
    *reinterpret_cast<uint4 *>(a.out[seg] + at) = yo;
  }
}

// Adds the cuts' shares in a fixed order and applies the epilogue; one thread per output element, a
// workgroup per 256 consecutive features of a row.  A launch of its own rather than a hand-over inside
// the product kernel: a workgroup that reads what other workgroups wrote needs device-wide fences, and on
// this GPU those write back and invalidate the L2 caches (measured: 75 us instead of 11 for a 32 MiB matrix).
__global__ __launch_bounds__(256) void reduce_epilogue_kernel(const float *shares, const int32_t n_out, const int32_t splits,
                                                                 const int32_t m, const LinearArgs a) {
  // four neighbouring features per thread; the shares are fetched four cuts at a time with loads that do not
  // depend on one another (a cut past the last one re-reads the last with weight 0), so a thread waits for
  // one round trip, not for one per cut
  const int n = (blockIdx.x * 256 + threadIdx.x) * 4, mrow = blockIdx.y;
  if (n >= n_out) return;
  float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int s2 = 0; s2 < splits; s2 += 4) {
    float4 part[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int sj = s2 + j < splits ? s2 + j : splits - 1;
      part[j] = *reinterpret_cast<const float4 *>(shares + ((size_t)sj * m + mrow) * n_out + n);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float w = s2 + j < splits ? 1.f : 0.f;
      v.x += w * part[j].x, v.y += w * part[j].y, v.z += w * part[j].z, v.w += w * part[j].w;
    }
  }
  int seg;                                                             // a segment is a multiple of 16 features wide
  size_t at;
  seg_of(a, mrow, n, seg, at);
  float y[4] = {v.x, v.y, v.z, v.w};
  if (a.bias) {
    const uint2 b = *reinterpret_cast<const uint2 *>(a.bias + n);
    const _Float16 *bp = reinterpret_cast<const _Float16 *>(&b);
#pragma unroll
    for (int e = 0; e < 4; ++e) y[e] += (float)bp[e];
  }
  if (a.relu) {
#pragma unroll
    for (int e = 0; e < 4; ++e) y[e] = fmaxf(y[e], 0.f);
  }
  if (a.residual) {
    const uint2 r = *reinterpret_cast<const uint2 *>(a.residual + at);
    const _Float16 *rp = reinterpret_cast<const _Float16 *>(&r);
#pragma unroll
    for (int e = 0; e < 4; ++e) y[e] += (float)rp[e];
  }
  uint2 o;
  _Float16 *op = reinterpret_cast<_Float16 *>(&o);
#pragma unroll
  for (int e = 0; e < 4; ++e) op[e] = (_Float16)y[e];
  *reinterpret_cast<uint2 *>(a.out[seg] + at) = o;
}

// dst piece (block (nt, kb), lane) = src[16 nt + lane % 16][32 kb + 8 (lane / 16) .. + 7]
__global__ __launch_bounds__(256) void pack_weight_kernel(uint4 *dst, const uint4 *src, int32_t n_out, int32_t n_in) {
  const int64_t total = (int64_t)n_out * n_in / 8;
  const int n_kb = n_in / 32, row_pieces = n_in / 8;
  for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < total; p += (int64_t)gridDim.x * blockDim.x) {
    const int lane = (int)(p & 63);
    const int64_t blk = p >> 6;
    const int kb = (int)(blk % n_kb), nt = (int)(blk / n_kb);
    dst[p] = src[(size_t)(nt * 16 + (lane & 15)) * row_pieces + kb * 4 + (lane >> 4)];
  }
}

// One workgroup per row; every thread keeps its (one or two) 16-byte pieces in registers, so the row
// is read once: mean, then variance around it, then the output.  As many threads as the row has pieces, up
// to 1024: with so few rows the kernel takes as long as its chain of dependent loads, and a thread with one
// piece has one round of them.
constexpr int kLnMaxThreads = 1024, kLnMaxPieces = 2;
constexpr int kLnMaxWidth = kLnMaxThreads * kLnMaxPieces * 8;
inline int ln_threads(int h) { return std::min(kLnMaxThreads, ((h >> 3) + 63) / 64 * 64); }

__device__ __forceinline__ float block_sum(float v, float *scratch) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  __syncthreads();                                             // scratch may still be read from the previous call
  if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
  __syncthreads();
  float t = 0.f;
  for (int w = 0; w < (int)(blockDim.x >> 6); ++w) t += scratch[w];
  return t;
}

template <int PPT>
__global__ __launch_bounds__(kLnMaxThreads) void layernorm_kernel(const uint4 *x, const uint4 *gamma, const uint4 *beta, uint4 *out,
                                                                int32_t h, float eps) {
  __shared__ float scratch[kLnMaxThreads / 64];
  const int pieces = h >> 3;
  const uint4 *xr = x + (size_t)blockIdx.x * pieces;
  float v[PPT][8];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < PPT; ++i) {
    const int p = threadIdx.x + i * blockDim.x;
    if (p < pieces) {
      const uint4 u = xr[p];
      const _Float16 *hp = reinterpret_cast<const _Float16 *>(&u);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        v[i][e] = (float)hp[e];
        s += v[i][e];
      }
    }
  }
  const float mean = block_sum(s, scratch) / (float)h;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < PPT; ++i)
    if ((int)(threadIdx.x + i * blockDim.x) < pieces) {
#pragma unroll
      for (int e = 0; e < 8; ++e) q += (v[i][e] - mean) * (v[i][e] - mean);
    }
  const float rstd = 1.0f / sqrtf(block_sum(q, scratch) / (float)h + eps);
  uint4 *orow = out + (size_t)blockIdx.x * pieces;
#pragma unroll
  for (int i = 0; i < PPT; ++i) {
    const int p = threadIdx.x + i * blockDim.x;
    if (p < pieces) {
      const uint4 g = gamma[p], b = beta[p];
      const _Float16 *gp = reinterpret_cast<const _Float16 *>(&g), *bp = reinterpret_cast<const _Float16 *>(&b);
      uint4 o;
      _Float16 *op = reinterpret_cast<_Float16 *>(&o);
#pragma unroll
      for (int e = 0; e < 8; ++e) op[e] = (_Float16)((v[i][e] - mean) * rstd * (float)gp[e] + (float)bp[e]);
      orow[p] = o;
    }
  }
}

// The share reduction and epilogue for whole rows, followed by the layer norm of the result: one
// workgroup per row, the row in registers as in layernorm_kernel.  Saves a launch and a pass over
// the row whenever a product feeds a layer norm (output projection -> second norm, feed-forward
// -> the next layer's first norm).
template <int PPT>
__global__ __launch_bounds__(kLnMaxThreads) void reduce_layernorm_kernel(const float *shares, const int32_t n_out, const int32_t splits,
                                                                           const int32_t m, const LinearArgs a) {
  // (leading parameters: in scalar registers when the wavefront starts, so the shares are asked for at once)
  __shared__ float scratch[kLnMaxThreads / 64];
  const int h = n_out, pieces = h >> 3, mrow = blockIdx.x;
  float v[PPT][8];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < PPT; ++i) {
    const int p = threadIdx.x + i * blockDim.x;
    if (p < pieces) {
      float acc[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = 0.f;
      for (int s2 = 0; s2 < splits; s2 += 4) {             // four cuts at a time, loads independent of one another
        float4 lo[4], hi[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int sj = s2 + j < splits ? s2 + j : splits - 1;      // past the last cut: the last again, weight 0
          const float4 *sp = reinterpret_cast<const float4 *>(shares + ((size_t)sj * m + mrow) * h + p * 8);
          lo[j] = sp[0], hi[j] = sp[1];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float w = s2 + j < splits ? 1.f : 0.f;
          acc[0] += w * lo[j].x, acc[1] += w * lo[j].y, acc[2] += w * lo[j].z, acc[3] += w * lo[j].w;
          acc[4] += w * hi[j].x, acc[5] += w * hi[j].y, acc[6] += w * hi[j].z, acc[7] += w * hi[j].w;
        }
      }
      uint4 rb = make_uint4(0u, 0u, 0u, 0u), bb = rb;
      if (a.bias) bb = reinterpret_cast<const uint4 *>(a.bias)[p];
      if (a.residual) rb = reinterpret_cast<const uint4 *>(a.residual + (size_t)mrow * h)[p];
      const _Float16 *bp = reinterpret_cast<const _Float16 *>(&bb), *rp = reinterpret_cast<const _Float16 *>(&rb);
      uint4 yo;
      _Float16 *yp = reinterpret_cast<_Float16 *>(&yo);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float y = acc[e] + (float)bp[e];
        if (a.relu) y = fmaxf(y, 0.f);
        y += (float)rp[e];
        yp[e] = (_Float16)y;                               // the norm sees the row as it is stored
        v[i][e] = (float)yp[e];
        s += v[i][e];
      }
      reinterpret_cast<uint4 *>(a.out[0] + (size_t)mrow * h)[p] = yo;
    }
  }
  // gamma and beta are fetched before the reductions, whose barriers would otherwise stand between these
  // loads and the statistics they do not depend on
  uint4 gam[PPT], bet[PPT];
#pragma unroll
  for (int i = 0; i < PPT; ++i) {
    const int p = threadIdx.x + i * blockDim.x;
    if (p < pieces) gam[i] = reinterpret_cast<const uint4 *>(a.ln_gamma)[p], bet[i] = reinterpret_cast<const uint4 *>(a.ln_beta)[p];
  }
  const float mean = block_sum(s, scratch) / (float)h;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < PPT; ++i)
    if ((int)(threadIdx.x + i * blockDim.x) < pieces) {
#pragma unroll
      for (int e = 0; e < 8; ++e) q += (v[i][e] - mean) * (v[i][e] - mean);
    }
  const float rstd = 1.0f / sqrtf(block_sum(q, scratch) / (float)h + a.ln_eps);
#pragma unroll
  for (int i = 0; i < PPT; ++i) {
    const int p = threadIdx.x + i * blockDim.x;
    if (p < pieces) {
      const _Float16 *gp = reinterpret_cast<const _Float16 *>(&gam[i]), *bp = reinterpret_cast<const _Float16 *>(&bet[i]);
      uint4 o;
      _Float16 *op = reinterpret_cast<_Float16 *>(&o);
#pragma unroll
      for (int e = 0; e < 8; ++e) op[e] = (_Float16)((v[i][e] - mean) * rstd * (float)gp[e] + (float)bp[e]);
      reinterpret_cast<uint4 *>(a.ln_out + (size_t)mrow * h)[p] = o;
    }
  }
}

template <int MF>
hipError_t launch_linear_mf(const LinearArgs &args, int n_tiles, bool fast, int fast_waves, hipStream_t stream) {
  if (fast) {
    dim3 grid((n_tiles + fast_waves - 1) / fast_waves, args.splits);
    if (fast_waves == 3) hipLaunchKernelGGL((linear_lds_kernel<MF, 3>), grid, dim3((3 + lin_stagers(MF)) * 64), 0, stream, args.w, args.x, args.n_kb,
                                           args.splits, args.n_in, args.m, args.n_tiles, args);
    else hipLaunchKernelGGL((linear_lds_kernel<MF, 4>), grid, dim3((4 + lin_stagers(MF)) * 64), 0, stream, args.w, args.x, args.n_kb,
                            args.splits, args.n_in, args.m, args.n_tiles, args);
    if (args.splits > 1 || args.to_shares) {
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
      if (args.ln_out && (args.n_out >> 3) <= kLnMaxThreads)
        hipLaunchKernelGGL(reduce_layernorm_kernel<1>, dim3(args.m), dim3(ln_threads(args.n_out)), 0, stream, args.shares, args.n_out,
                           args.splits, args.m, args);
      else if (args.ln_out)
        hipLaunchKernelGGL(reduce_layernorm_kernel<2>, dim3(args.m), dim3(ln_threads(args.n_out)), 0, stream, args.shares, args.n_out,
                           args.splits, args.m, args);
      else
        hipLaunchKernelGGL(reduce_epilogue_kernel, dim3((args.n_out + 1023) / 1024, args.m), dim3(256), 0, stream, args.shares,
                           args.n_out, args.splits, args.m, args);
    }
  } else if constexpr (MF <= OKV_LINEAR_MAX_ROWS / 16) {
    hipLaunchKernelGGL(linear_kernel<MF>, dim3(n_tiles), dim3(kLinWaves * 64), 0, stream, args.w, args.x, args.n_kb, args.n_in,
                       args.m, args);
  } else {
    return hipErrorInvalidValue;                       // more than OKV_LINEAR_MAX_ROWS rows: the staged kernel only
  }
  return hipGetLastError();
}

}  // namespace

// Streaming wavefronts per workgroup (4 or 3) and cuts of the input dimension for the fast kernel, by a small
// model of the launch, in microseconds:
//   max(weights / 6.0 MB/us, (weights + rows of x fetched) / 10 MB/us) / fill + second kernel
// -- the weights come from HBM, they and the rows of x (every workgroup fetches the rows of its stretch:
// m x n_in x 2 bytes per group of 64 or 48 features) come through the L2s, `fill` is the share of
// workgroup slots in use when the workgroups are dealt to the compute units in rounds, and a cut costs the
// kernel that adds the shares up (a dependent launch and the shares written and read).  The rates are
// measured on MI355X (16384 x 4096: 27 us at 32 rows, 41 at 128).  Cuts divide the chunks evenly, leave every
// cut at least two chunks, and the kernel takes the chunks `pace` at a time.  A launch with more than two
// workgroups per compute unit is not considered (longer-lived workgroups measured faster than more of them).
// Examples on 256 compute units: 12288 x 4096 -> 3 wavefronts, no cut (256 workgroups); 6144 x 4096 -> 3
// wavefronts, 2 cuts; 4096 x 4096 and 4096 x 16384 -> 4 wavefronts, 4 cuts; 16384 x 4096 -> 4, none.
// Cuts 0: not a shape for the fast kernel.
void linear_plan(int32_t m, int32_t n_out, int32_t n_in, int32_t n_cus, int *waves, int *cuts) {
  *waves = 4;
  *cuts = 0;
  const int chunk = lin_chunk((m + 15) / 16), pace = lin_weight_lead((m + 15) / 16);
  if (n_in % (32 * chunk * pace)) return;
  const int chunks = n_in / (32 * chunk);
  const double weight_mb = (double)n_out * n_in * 2 / 1e6;
  double best = 0;
  for (int w : {4, 3}) {
    const int groups = (n_out / 16 + w - 1) / w;
    const double x_mb = (double)groups * m * n_in * 2 / 1e6;
    for (int s = 1; s <= chunks; ++s) {
      if (chunks % (s * pace)) continue;
      if (s > 1 && chunks / s < 2) break;
      const int64_t wgs = (int64_t)groups * s;
      if (s > 1 && wgs > 2 * (int64_t)n_cus) break;
      const int64_t rounds = (wgs + n_cus - 1) / n_cus;
      const double fill = (double)wgs / (double)(rounds * n_cus);
      double t = std::max(weight_mb / 6.0, (weight_mb + x_mb) / 10.0) / fill;
      if (s > 1) t += 4.5 + 2.0 * s * m * n_out * 4 / 1e6 / 3.0;
      if (*cuts == 0 || t < best * 0.98) {                      // on a near tie the first one found: 4 wavefronts, fewer cuts
        best = t;
        *waves = w;
        *cuts = s;
      }
    }
  }
}

int64_t linear_workspace_bytes(int32_t m, int32_t n_out, int32_t n_in, int32_t n_cus) {
  int waves = 4, s = 0;
  if (m > OKV_LIN_SIMPLE_ROWS) linear_plan(m, n_out, n_in, n_cus, &waves, &s);
  return s < 1 ? 0 : (int64_t)s * m * n_out * 4;        // a single cut still goes through a share when a layer norm follows
}

// Whether one launch of the staged kernel takes m rows of this product with the workspace at hand (the only
// kernel there is for more than OKV_LINEAR_MAX_ROWS rows).
bool linear_staged_takes(int32_t m, int32_t n_out, int32_t n_in, int32_t n_cus, bool have_workspace, int64_t workspace_bytes) {
  if (m <= OKV_LIN_SIMPLE_ROWS || m > OKV_LINEAR_MAX_ROWS_STAGED) return false;
  int waves = 4, s = 0;
  linear_plan(m, n_out, n_in, n_cus, &waves, &s);
  if (s < 1) return false;
  return s == 1 || (have_workspace && workspace_bytes >= (int64_t)s * m * n_out * 4);
}

hipError_t launch_linear(const LinearLaunch &l, hipStream_t stream) {
  LinearArgs a;
  a.x = static_cast<const uint4 *>(l.x);
  a.w = static_cast<const uint4 *>(l.w_packed);
  a.bias = static_cast<const _Float16 *>(l.bias);
  a.residual = static_cast<const _Float16 *>(l.residual);
  for (int s = 0; s < 3; ++s) a.out[s] = static_cast<_Float16 *>(s < l.n_seg ? l.out[s] : l.out[0]);
  a.m = l.m;
  a.n_in = l.n_in;
  a.n_kb = l.n_in / 32;
  a.seg0_cols = l.first_cols ? l.first_cols : l.n_out / l.n_seg;
  a.seg_cols = l.n_seg > 1 ? (l.n_out - a.seg0_cols) / (l.n_seg - 1) : l.n_out;
  a.relu = l.relu;
  const int n_tiles = l.n_out / 16;
  a.n_tiles = n_tiles;
  a.n_out = l.n_out;
  a.splits = 1;
  a.shares = nullptr;
  a.to_shares = 0;
  a.ln_gamma = static_cast<const _Float16 *>(l.ln_gamma);
  a.ln_beta = static_cast<const _Float16 *>(l.ln_beta);
  a.ln_out = nullptr;
  a.ln_eps = l.ln_eps;
  bool fast = false;
  int fast_waves = 4, s = 0;
  linear_plan(l.m, l.n_out, l.n_in, l.n_cus, &fast_waves, &s);
  if (l.m > OKV_LIN_SIMPLE_ROWS && (s == 1 || (s > 1 && l.workspace && l.workspace_bytes >= linear_workspace_bytes(l.m, l.n_out, l.n_in, l.n_cus)))) {
    fast = true;
    a.splits = s;
    a.shares = static_cast<float *>(l.workspace);
  }
  // a layer norm of the result rides on the share reduction when there is one to ride on
  const bool fuse_ln = l.ln_out && fast && l.n_seg == 1 && l.n_out <= kLnMaxWidth && l.workspace &&
                       l.workspace_bytes >= (int64_t)a.splits * l.m * l.n_out * 4;
  if (fuse_ln) {
    a.to_shares = 1;
    a.ln_out = static_cast<_Float16 *>(l.ln_out);
  }
  hipError_t e = hipErrorInvalidValue;
  switch ((l.m + 15) / 16) {
    case 1: e = launch_linear_mf<1>(a, n_tiles, fast, fast_waves, stream); break;
    case 2: e = launch_linear_mf<2>(a, n_tiles, fast, fast_waves, stream); break;
    case 3: e = launch_linear_mf<3>(a, n_tiles, fast, fast_waves, stream); break;
    case 4: e = launch_linear_mf<4>(a, n_tiles, fast, fast_waves, stream); break;
    case 5: e = launch_linear_mf<5>(a, n_tiles, fast, fast_waves, stream); break;
    case 6: e = launch_linear_mf<6>(a, n_tiles, fast, fast_waves, stream); break;
    case 7: e = launch_linear_mf<7>(a, n_tiles, fast, fast_waves, stream); break;
    case 8: e = launch_linear_mf<8>(a, n_tiles, fast, fast_waves, stream); break;
    case 9: e = launch_linear_mf<9>(a, n_tiles, fast, fast_waves, stream); break;
    case 10: e = launch_linear_mf<10>(a, n_tiles, fast, fast_waves, stream); break;
    case 11: e = launch_linear_mf<11>(a, n_tiles, fast, fast_waves, stream); break;
    case 12: e = launch_linear_mf<12>(a, n_tiles, fast, fast_waves, stream); break;
  }
  if (e != hipSuccess || !l.ln_out || fuse_ln) return e;
  return launch_layernorm(l.out[0], l.ln_gamma, l.ln_beta, l.ln_out, l.m, l.n_out, l.ln_eps, stream);   // the same in two steps
}

hipError_t launch_pack_weight(void *dst, const void *src, int32_t n_out, int32_t n_in, hipStream_t stream) {
  const int64_t total = (int64_t)n_out * n_in / 8;
  const unsigned blocks = (unsigned)std::min<int64_t>((total + 255) / 256, 1 << 16);
  hipLaunchKernelGGL(pack_weight_kernel, dim3(blocks), dim3(256), 0, stream, static_cast<uint4 *>(dst),
                     static_cast<const uint4 *>(src), n_out, n_in);
  return hipGetLastError();
}

hipError_t launch_layernorm(const void *x, const void *gamma, const void *beta, void *out, int32_t m, int32_t h, float eps,
                            hipStream_t stream) {
  if ((h >> 3) > kLnMaxThreads)
    hipLaunchKernelGGL(layernorm_kernel<2>, dim3(m), dim3(ln_threads(h)), 0, stream, static_cast<const uint4 *>(x),
                       static_cast<const uint4 *>(gamma), static_cast<const uint4 *>(beta), static_cast<uint4 *>(out), h, eps);
  else
  hipLaunchKernelGGL(layernorm_kernel<1>, dim3(m), dim3(ln_threads(h)), 0, stream, static_cast<const uint4 *>(x),
                     static_cast<const uint4 *>(gamma), static_cast<const uint4 *>(beta), static_cast<uint4 *>(out), h, eps);
  return hipGetLastError();
}

}  // namespace okv
