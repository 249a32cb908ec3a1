// Linear layers and layer norm of a decoder layer in the decode stage, for gfx950.
//
// out[m][n] = sum_k x[m][k] W[n][k] for a batch of at most 128 rows (paper §IV-D: the
// 8 h1^2 + 4 h1 h2 flops per token of the four projections and the feed-forward block).
// With so few rows every weight is read once and used `m` times: the product is bound by
// streaming W from HBM, so the kernel is built like the attention kernel -- long runs of
// 16-byte-per-lane loads kept many deep in flight -- with the matrix cores doing the
// arithmetic on the side (a 16x16x16 fp16 instruction per 512 bytes of weights and 16
// rows of x: a few percent of the time the loads take).
//
//   * weights are stored pre-arranged (okv_pack_linear_weight) so that one load instruction
//     brings a wavefront the 1 KiB it feeds to two matrix-core instructions: 16 output
//     features x 32 inputs, lane l holding feature l % 16, inputs 8 (l / 16) .. + 7;
//   * a workgroup owns 16 output features; its 8 wavefronts split the input dimension, each
//     streaming its share of the weights kDepth pieces ahead, and add up through LDS, so no
//     partial sums ever go to HBM and the epilogue (bias, ReLU, residual, rounding to fp16,
//     scatter into up to three output tensors) runs in the same kernel;
//   * the rows of x (a few hundred KiB, resident in L2) are fetched per lane in the layout
//     the matrix core wants, the same distance ahead as the weights: the vector memory
//     counter retires loads in order, so a shorter distance for x would drain the weights'
//     queue every iteration.
#include "okv_kernels.h"

#include <algorithm>

namespace okv {

namespace {

typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kLinWaves = 8;

template <int MF>
constexpr int lin_depth() {
  return MF <= 2 ? 8 : MF <= 4 ? 4 : 2;       // pieces in flight: bounded by the registers x needs beside them
}

struct LinearArgs {
  const uint4 *x;          // [m][n_in] fp16, as 16-byte pieces
  const uint4 *w;          // packed weights
  const _Float16 *bias, *residual;
  _Float16 *out[3];
  int32_t m, n_in, n_kb, seg_cols, relu;
};

__device__ __forceinline__ floatx4 mfma16(const uint2 a, const uint2 b, floatx4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(half4, a), __builtin_bit_cast(half4, b), c, 0, 0, 0);
}

template <int MF>
__global__ __launch_bounds__(kLinWaves * 64) void linear_kernel(const LinearArgs a) {
  constexpr int D = lin_depth<MF>();
  __shared__ floatx4 part[kLinWaves][MF][64];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);      // uniform: the loops below are scalar loops
  const int ntile = blockIdx.x;
  const int kb0 = (int)((int64_t)wave * a.n_kb / kLinWaves), kb1 = (int)((int64_t)(wave + 1) * a.n_kb / kLinWaves);
  const int nk = kb1 - kb0;
  const uint4 *wp = a.w + ((size_t)ntile * a.n_kb + kb0) * 64 + lane;
  // this lane's piece of x for k-block kb and row fragment f: row 16 f + lane % 16, inputs 32 kb + 8 (lane / 16) .. + 7
  const int row = lane & 15, kq = lane >> 4;
  const int row_pieces = a.n_in >> 3;
  // Rows past the batch read row 0 instead: a row of x only ever reaches the same row of the
  // result, and those rows are not stored.
  const uint4 *xp[MF];
#pragma unroll
  for (int f = 0; f < MF; ++f)
    xp[f] = a.x + (size_t)(f * 16 + row < a.m ? f * 16 + row : 0) * row_pieces + (size_t)kb0 * 4 + kq;
  floatx4 acc[MF];
#pragma unroll
  for (int f = 0; f < MF; ++f) acc[f] = floatx4{0.f, 0.f, 0.f, 0.f};

  uint4 wbuf[D], xbuf[D][MF];
  auto load = [&](int slot, int k) {                           // k: block index relative to kb0
    wbuf[slot] = wp[(size_t)k * 64];
#pragma unroll
    for (int f = 0; f < MF; ++f) xbuf[slot][f] = xp[f][(size_t)k * 4];
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
    if (mrow >= a.m) continue;
    const int f = mrow >> 4, src_lane = j + 16 * ((mrow & 15) >> 2), r = mrow & 3;
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < kLinWaves; ++w) v += part[w][f][src_lane][r];
    const int n = ntile * 16 + j;
    if (a.bias) v += (float)a.bias[n];
    if (a.relu) v = fmaxf(v, 0.f);
    const int seg = n / a.seg_cols, col = n - seg * a.seg_cols;
    const size_t at = (size_t)mrow * a.seg_cols + col;
    if (a.residual) v += (float)a.residual[at];
    a.out[seg][at] = (_Float16)v;
  }
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

// One workgroup per row; every thread keeps its (at most 8) 16-byte pieces in registers, so the row
// is read once: mean, then variance around it, then the output.
constexpr int kLnThreads = 256, kLnPieces = 8;

__device__ __forceinline__ float block_sum(float v, float *scratch) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  __syncthreads();                                             // scratch may still be read from the previous call
  if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
  __syncthreads();
  float t = 0.f;
#pragma unroll
  for (int w = 0; w < kLnThreads / 64; ++w) t += scratch[w];
  return t;
}

__global__ __launch_bounds__(kLnThreads) void layernorm_kernel(const uint4 *x, const uint4 *gamma, const uint4 *beta, uint4 *out,
                                                                int32_t h, float eps) {
  __shared__ float scratch[kLnThreads / 64];
  const int pieces = h >> 3;
  const uint4 *xr = x + (size_t)blockIdx.x * pieces;
  float v[kLnPieces][8];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < kLnPieces; ++i) {
    const int p = threadIdx.x + i * kLnThreads;
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
  for (int i = 0; i < kLnPieces; ++i)
    if (threadIdx.x + i * kLnThreads < pieces) {
#pragma unroll
      for (int e = 0; e < 8; ++e) q += (v[i][e] - mean) * (v[i][e] - mean);
    }
  const float rstd = 1.0f / sqrtf(block_sum(q, scratch) / (float)h + eps);
  uint4 *orow = out + (size_t)blockIdx.x * pieces;
#pragma unroll
  for (int i = 0; i < kLnPieces; ++i) {
    const int p = threadIdx.x + i * kLnThreads;
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

template <int MF>
hipError_t launch_linear_mf(const LinearArgs &args, int n_tiles, hipStream_t stream) {
  hipLaunchKernelGGL(linear_kernel<MF>, dim3(n_tiles), dim3(kLinWaves * 64), 0, stream, args);
  return hipGetLastError();
}

}  // namespace

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
  a.seg_cols = l.n_out / l.n_seg;
  a.relu = l.relu;
  const int n_tiles = l.n_out / 16;
  switch ((l.m + 15) / 16) {
    case 1: return launch_linear_mf<1>(a, n_tiles, stream);
    case 2: return launch_linear_mf<2>(a, n_tiles, stream);
    case 3: return launch_linear_mf<3>(a, n_tiles, stream);
    case 4: return launch_linear_mf<4>(a, n_tiles, stream);
    case 5: return launch_linear_mf<5>(a, n_tiles, stream);
    case 6: return launch_linear_mf<6>(a, n_tiles, stream);
    case 7: return launch_linear_mf<7>(a, n_tiles, stream);
    case 8: return launch_linear_mf<8>(a, n_tiles, stream);
  }
  return hipErrorInvalidValue;
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
  hipLaunchKernelGGL(layernorm_kernel, dim3(m), dim3(kLnThreads), 0, stream, static_cast<const uint4 *>(x),
                     static_cast<const uint4 *>(gamma), static_cast<const uint4 *>(beta), static_cast<uint4 *>(out), h, eps);
  return hipGetLastError();
}

}  // namespace okv
