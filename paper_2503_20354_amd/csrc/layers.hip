// Other layer types whose weight gradients come from the packed activation:
//   * normalisation layers (batch norm over NCHW, layer norm over [tokens, features]): gradients of the scale and the
//     shift from the pruned normalised activation -- the variant of Section 5 that adapts BN layers only.  With
//     y = gamma[c] * x_hat + beta[c] this is Eq. 2's second line for an element-wise layer:
//     dgamma[c] = sum dY * x_hat_pruned, dbeta[c] = sum dY over the elements of channel c.  HBM-bound.
//   * convolutions with channel groups (grouped and depthwise convolutions of the ResNeXt / Segformer networks of
//     Section 5.1): dW[co][cig][u][v] = sum_{b,oh,ow} dY[b][co][oh][ow] * A_pruned[b][g(co)*Cig + cig][ih][iw].
//     Per output channel only Ci/groups (1 - 16) input channels contribute, far too few rows for a matrix-core
//     tile, so the sum runs on the vector ALU.
#include "dw_impl.hpp"

namespace surgeon {

// ---------------------------------------------------------------------------------------------------------
// scale / shift gradients
// ---------------------------------------------------------------------------------------------------------
// Element (o, c, i) of the [outer, C, inner] tensor is at (o*C + c)*inner + i.  Three partial kernels write
// (dgamma, dbeta) partial sums as float2 part[slice][c]; the finishing kernel adds the slices per channel in fp64 in
// a fixed order (deterministic).

// inner % 64 == 0 (batch norm on maps of 8x8 and larger): one wavefront per (o, c) row, lane = element of a mask word
template <typename T, int kAffineBatch>
__global__ __launch_bounds__(256) void affine_rows_kernel(Packed<T> pk, const T* __restrict__ dY, int64_t outer, int C,
                                                          int inner, float2* __restrict__ part) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);  // = o*C + c
  if (row >= outer * C) return;
  const int64_t e0 = row * inner;
  float g = 0.0f, b = 0.0f;
  // kAffineBatch words at a time, level by level (mask words and ranks, then positions, then values), so that a
  // wavefront keeps kAffineBatch independent chains of dependent loads in flight instead of one
  for (int j0 = 0; j0 < inner; j0 += 64 * kAffineBatch) {
    uint64_t word[kAffineBatch];
    uint32_t rank[kAffineBatch];
    float dy[kAffineBatch];
#pragma unroll
    for (int q = 0; q < kAffineBatch; ++q) {
      const int j = min(j0 + 64 * q, inner - 64);  // past the row's end: its last word again, weighted 0 below
      const int64_t w = (e0 + j) >> 6;
      word[q] = pk.mask[w];
      rank[q] = pk.word_rank[w];
      dy[q] = j0 + 64 * q < inner ? widen<T>(dY[e0 + j + lane]) : 0.0f;
    }
    float x[kAffineBatch];
#pragma unroll
    for (int q = 0; q < kAffineBatch; ++q) {
      const uint32_t lo = (uint32_t)word[q], hi = (uint32_t)(word[q] >> 32);
      int64_t pos = (int64_t)rank[q] + __builtin_amdgcn_mbcnt_hi(hi, __builtin_amdgcn_mbcnt_lo(lo, 0u));
      pos = pos > pk.k_last ? pk.k_last : pos;
      const bool kept = (word[q] >> lane) & 1ull;
      x[q] = kept ? widen<T>(pk.vals[pos]) : 0.0f;  // vals is read only where a bit is set (it may be empty otherwise)
    }
#pragma unroll
    for (int q = 0; q < kAffineBatch; ++q) {
      g = __builtin_fmaf(dy[q], x[q], g);
      b += dy[q];
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    g += __shfl_down(g, off, 64);
    b += __shfl_down(b, off, 64);
  }
  const int64_t o = row / C;
  const int c = (int)(row - o * C);
  if (lane == 0) part[o * C + c] = make_float2(g, b);
}

// inner == 1 and C % 64 == 0 (layer norm): a wavefront owns one 64-feature mask word of kLnRows consecutive tokens
constexpr int kLnRows = 16;
constexpr int kAffineBatch = 16;  // = kLnRows: a slice is one batch
template <typename T>
__global__ __launch_bounds__(256) void affine_cols_kernel(Packed<T> pk, const T* __restrict__ dY, int64_t outer, int C,
                                                          float2* __restrict__ part) {
  const int lane = threadIdx.x & 63;
  const int words = C >> 6;
  const int wq = blockIdx.x * 4 + (threadIdx.x >> 6);  // word inside the token row
  if (wq >= words) return;
  const int64_t m0 = (int64_t)blockIdx.y * kLnRows, m1 = min(m0 + kLnRows, outer);
  float g = 0.0f, b = 0.0f;
  for (int64_t mb = m0; mb < m1; mb += kAffineBatch) {  // levels of dependent loads batched as in the row kernel
    uint64_t word[kAffineBatch];
    uint32_t rank[kAffineBatch];
    float dy[kAffineBatch];
#pragma unroll
    for (int q = 0; q < kAffineBatch; ++q) {
      const int64_t m = min(mb + q, m1 - 1);  // past the slice's end: its last token again, weighted 0 below
      const int64_t w = m * words + wq;
      word[q] = pk.mask[w];
      rank[q] = pk.word_rank[w];
      dy[q] = mb + q < m1 ? widen<T>(dY[m * C + wq * 64 + lane]) : 0.0f;
    }
    float x[kAffineBatch];
#pragma unroll
    for (int q = 0; q < kAffineBatch; ++q) {
      const uint32_t lo = (uint32_t)word[q], hi = (uint32_t)(word[q] >> 32);
      int64_t pos = (int64_t)rank[q] + __builtin_amdgcn_mbcnt_hi(hi, __builtin_amdgcn_mbcnt_lo(lo, 0u));
      pos = pos > pk.k_last ? pk.k_last : pos;
      const bool kept = (word[q] >> lane) & 1ull;
      x[q] = kept ? widen<T>(pk.vals[pos]) : 0.0f;  // vals is read only where a bit is set (it may be empty otherwise)
    }
#pragma unroll
    for (int q = 0; q < kAffineBatch; ++q) {
      g = __builtin_fmaf(dy[q], x[q], g);
      b += dy[q];
    }
  }
  part[(int64_t)blockIdx.y * C + wq * 64 + lane] = make_float2(g, b);
}

// any shape: one thread per channel and slice of `outer`
template <typename T>
__global__ __launch_bounds__(256) void affine_generic_kernel(Packed<T> pk, const T* __restrict__ dY, int64_t outer, int C,
                                                             int inner, int64_t o_per_slice, float2* __restrict__ part) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= C) return;
  const int64_t o0 = (int64_t)blockIdx.y * o_per_slice, o1 = min(o0 + o_per_slice, outer);
  float g = 0.0f, b = 0.0f;
  for (int64_t o = o0; o < o1; ++o)
    for (int i = 0; i < inner; ++i) {
      const int64_t e = (o * C + c) * inner + i;
      const float dy = widen<T>(dY[e]);
      g = __builtin_fmaf(dy, unpack_at<T>(pk, e), g);
      b += dy;
    }
  part[(int64_t)blockIdx.y * C + c] = make_float2(g, b);
}

// Adds the slices per channel in fp64, in a fixed order: a workgroup owns 64 channels, its 16 wavefronts take the
// slices s = w, w + 16, ... (eight loads in flight each), and the 16 partial sums are added in wavefront order.
static __global__ __launch_bounds__(1024) void affine_final_kernel(const float2* __restrict__ part, int64_t n_slices, int C,
                                                                   float* __restrict__ dgamma, float* __restrict__ dbeta) {
  __shared__ double sg[16][64], sb[16][64];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + lane;
  double g = 0.0, b = 0.0;
  if (c < C) {
    for (int64_t s0 = w; s0 < n_slices; s0 += 16 * 8) {
      float2 v[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const int64_t s = s0 + 16 * q;
        v[q] = s < n_slices ? part[s * C + c] : make_float2(0.0f, 0.0f);
      }
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        g += (double)v[q].x;
        b += (double)v[q].y;
      }
    }
  }
  sg[w][lane] = g;
  sb[w][lane] = b;
  __syncthreads();
  if (w == 0 && c < C) {
    double tg = 0.0, tb = 0.0;
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      tg += sg[q][lane];
      tb += sb[q][lane];
    }
    dgamma[c] = (float)tg;
    dbeta[c] = (float)tb;
  }
}

struct AffinePlan {
  int mode;  // 0 rows (inner % 64 == 0), 1 columns (inner == 1, C % 64 == 0), 2 generic
  int64_t n, n_words, n_rank_blocks, n_slices, o_per_slice;
  size_t off_rank, off_blocks, off_part, ws_bytes;
};

static int plan_affine(int64_t outer, int64_t C, int64_t inner, AffinePlan* p) {
  if (outer < 0 || C < 1 || inner < 1) return fail(SURGEON_EINVAL, "affine_grad: bad shape");
  if (C > (1 << 24) || inner > (1 << 24) || outer * C * inner > ((int64_t)1 << 31))
    return fail(SURGEON_EUNSUPPORTED, "affine_grad: tensor too large");
  p->n = outer * C * inner;
  p->n_words = ceil_div(p->n, 64);
  p->n_rank_blocks = ceil_div(p->n_words, kRankWordsPerBlock);
  if (inner % 64 == 0) {
    p->mode = 0;
    p->n_slices = outer;
    p->o_per_slice = 1;
  } else if (inner == 1 && C % 64 == 0) {
    p->mode = 1;
    p->n_slices = ceil_div(outer, kLnRows);
    p->o_per_slice = kLnRows;
    if (p->n_slices > 65535) return fail(SURGEON_EUNSUPPORTED, "affine_grad: more than %d rows", 65535 * kLnRows);
  } else {
    p->mode = 2;
    p->n_slices = std::max<int64_t>(1, std::min<int64_t>(outer, 4096 / ceil_div(C, 256)));
    p->o_per_slice = ceil_div(std::max<int64_t>(outer, 1), p->n_slices);
    p->n_slices = ceil_div(std::max<int64_t>(outer, 1), p->o_per_slice);
  }
  size_t off = 0;
  p->off_rank = off;
  off += align_up((size_t)std::max<int64_t>(p->n_words, 1) * 4, 256);
  p->off_blocks = off;
  off += align_up((size_t)std::max<int64_t>(p->n_rank_blocks, 1) * 4, 256);
  p->off_part = off;
  off += align_up((size_t)std::max<int64_t>(p->n_slices, 1) * (size_t)C * sizeof(float2), 256);
  p->ws_bytes = off;
  return SURGEON_OK;
}

template <typename T>
static int run_affine(const AffinePlan& p, const void* vals, const uint64_t* mask, const void* dY, int64_t outer, int C,
                      int inner, int64_t k_total, float* dgamma, float* dbeta, void* ws, hipStream_t st) {
  char* w = (char*)ws;
  uint32_t* word_rank = (uint32_t*)(w + p.off_rank);
  uint32_t* block_sum = (uint32_t*)(w + p.off_blocks);
  float2* part = (float2*)(w + p.off_part);
  ProfScope prof(SURGEON_PROF_AFFINE, st);
  if (p.n > 0) {
    const int rc_rank = launch_rank_table(mask, p.n_words, p.n_rank_blocks, block_sum, word_rank, st);
    if (rc_rank != SURGEON_OK) return rc_rank;
  }
  Packed<T> pk;
  pk.vals = (const T*)vals;
  pk.mask = mask;
  pk.word_rank = word_rank;
  pk.k_last = std::max<int64_t>(k_total - 1, 0);  // vals is only read where a mask bit is set: never when nothing is kept
  pk.n_words = p.n_words;
  int64_t n_slices = p.n_slices;
  if (p.n == 0) {
    n_slices = 0;
  } else if (p.mode == 0) {
    // words of a row requested together: as many as the row has, up to 16 (a shorter batch re-reads nothing)
    const dim3 grid((unsigned)ceil_div(outer * C, 4));
    const int words = inner / 64;
    if (words >= 16) SURGEON_LAUNCH((affine_rows_kernel<T, 16>), grid, dim3(256), 0, st, pk, (const T*)dY, outer, C, inner, part);
    else if (words >= 8) SURGEON_LAUNCH((affine_rows_kernel<T, 8>), grid, dim3(256), 0, st, pk, (const T*)dY, outer, C, inner, part);
    else if (words >= 4) SURGEON_LAUNCH((affine_rows_kernel<T, 4>), grid, dim3(256), 0, st, pk, (const T*)dY, outer, C, inner, part);
    else if (words >= 2) SURGEON_LAUNCH((affine_rows_kernel<T, 2>), grid, dim3(256), 0, st, pk, (const T*)dY, outer, C, inner, part);
    else SURGEON_LAUNCH((affine_rows_kernel<T, 1>), grid, dim3(256), 0, st, pk, (const T*)dY, outer, C, inner, part);
    SURGEON_LAUNCH_CHECK();
  } else if (p.mode == 1) {
    SURGEON_LAUNCH(affine_cols_kernel<T>, dim3((unsigned)ceil_div(C / 64, 4), (unsigned)p.n_slices), dim3(256), 0, st, pk,
                   (const T*)dY, outer, C, part);
    SURGEON_LAUNCH_CHECK();
  } else {
    SURGEON_LAUNCH(affine_generic_kernel<T>, dim3((unsigned)ceil_div(C, 256), (unsigned)p.n_slices), dim3(256), 0, st, pk,
                   (const T*)dY, outer, C, inner, p.o_per_slice, part);
    SURGEON_LAUNCH_CHECK();
  }
  SURGEON_LAUNCH(affine_final_kernel, dim3((unsigned)ceil_div(C, 64)), dim3(1024), 0, st, (const float2*)part, n_slices, C,
                 dgamma, dbeta);
  SURGEON_LAUNCH_CHECK();
  return SURGEON_OK;
}

// ---------------------------------------------------------------------------------------------------------
// convolutions with channel groups
// ---------------------------------------------------------------------------------------------------------
struct GroupedGeom {
  int Nb, Ci, H, W, Co, OH, OW, KH, KW, stride, pad, groups, Cig, Cog;
  int64_t pos_per_split;  // (b, oh, ow) positions per workgroup along the contraction
  int64_t n_pos, n_w;
};

constexpr int kGroupedMaxTaps = 49;

// One workgroup per (co, cig, split): its threads walk the split's output positions, each keeping the kh*kw taps of
// its positions in registers; a workgroup-wide sum in a fixed order writes the split's partial filter.
template <typename T, int TAPS_MAX>
__global__ __launch_bounds__(256) void dw_grouped_kernel(GroupedGeom g, Packed<T> pk, const T* __restrict__ dY,
                                                         float* __restrict__ out) {
  __shared__ float red[4][TAPS_MAX];
  const int pair = blockIdx.x;  // co * Cig + cig
  const int co = pair / g.Cig, cig = pair - co * g.Cig;
  const int ci = (co / g.Cog) * g.Cig + cig;
  const int taps = g.KH * g.KW;
  const int64_t p_begin = (int64_t)blockIdx.y * g.pos_per_split, p_end = min(p_begin + g.pos_per_split, g.n_pos);
  float acc[TAPS_MAX];
#pragma unroll
  for (int t = 0; t < TAPS_MAX; ++t) acc[t] = 0.0f;
  const int ohw = g.OH * g.OW;
  for (int64_t p = p_begin + threadIdx.x; p < p_end; p += 256) {
    const int b = (int)(p / ohw);
    const int rem = (int)(p - (int64_t)b * ohw);
    const int oh = rem / g.OW, ow = rem - oh * g.OW;
    const float dy = widen<T>(dY[((int64_t)b * g.Co + co) * ohw + rem]);
    const int64_t a_base = ((int64_t)b * g.Ci + ci) * g.H;
#pragma unroll
    for (int t = 0; t < TAPS_MAX; ++t) {
      if (t < taps) {
        const int u = t / g.KW, v = t - u * g.KW;
        const int ih = oh * g.stride + u - g.pad, iw = ow * g.stride + v - g.pad;
        if (ih >= 0 && ih < g.H && iw >= 0 && iw < g.W)
          acc[t] = __builtin_fmaf(dy, unpack_at<T>(pk, (a_base + ih) * g.W + iw), acc[t]);
      }
    }
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int t = 0; t < TAPS_MAX; ++t) {
    float v = acc[t];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    if (lane == 0) red[wave][t] = v;
  }
  __syncthreads();
  if (threadIdx.x < taps)
    out[(int64_t)blockIdx.y * g.n_w + (int64_t)pair * taps + threadIdx.x] =
        (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
}

// 3x3, stride 1, pad 1 and 4 to 64 (output channel, input channel) pairs per group (the grouped convolutions of
// ResNeXt): a workgroup owns `gpw` consecutive groups -- 64 pairs, one per lane -- and walks a range of (image, band of
// R rows) tiles.  Per tile the band's dY rows of the groups' output channels and the un-packed input rows with halo of
// their input channels sit in LDS (each element is un-packed once, not once per tap and output channel); the four
// wavefronts split the band's positions, a lane reads its dY value and the nine inputs around it and keeps nine
// accumulators; the wavefronts' sums are added in a fixed order at the end.
struct Grouped3x3Geom {
  int Nb, Ci, Co, H, W, Cig, Cog, groups;
  int gpw;              // groups per workgroup (64 / pairs per group)
  int R, bands;         // rows per band, bands per image
  int SY, SA;           // LDS strides of a channel's dY band and input band (odd: channels spread over the banks)
  int tiles_per_split, n_tiles;
  int64_t n_w;
};

template <typename T>
__global__ __launch_bounds__(256) void dw_grouped3x3_kernel(Grouped3x3Geom g, Packed<T> pk, const T* __restrict__ dY,
                                                            float* __restrict__ out) {
  extern __shared__ float g3_lds[];
  float* ys = g3_lds;                              // [gpw * Cog][SY]
  float* as = g3_lds + g.gpw * g.Cog * g.SY;       // [gpw * Cig][SA]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int group0 = blockIdx.x * g.gpw;
  const int pairs = g.Cog * g.Cig;
  const int gl = lane / pairs, pr = lane - gl * pairs;
  const int co_l = pr / g.Cig, ci_l = pr - co_l * g.Cig;
  const bool lane_ok = group0 + gl < g.groups;     // the last workgroup may own fewer groups
  const int PW = g.W + 2;
  const int n_y = g.gpw * g.Cog * g.R * g.W, n_a = g.gpw * g.Cig * (g.R + 2) * PW;
  const int t_begin = blockIdx.y * g.tiles_per_split, t_end = min(t_begin + g.tiles_per_split, g.n_tiles);
  float acc[9];
#pragma unroll
  for (int t = 0; t < 9; ++t) acc[t] = 0.0f;

  for (int tile = t_begin; tile < t_end; ++tile) {
    const int b = tile / g.bands, r0 = (tile - b * g.bands) * g.R;
    __syncthreads();  // the previous tile's readers are done
    for (int i = tid; i < n_y; i += 256) {
      const int ch = i / (g.R * g.W), p = i - ch * (g.R * g.W);
      const int oh = r0 + p / g.W, ow = p % g.W;
      const int co = group0 * g.Cog + ch;
      float v = 0.0f;
      if (oh < g.H && co < g.Co) v = widen<T>(dY[(((int64_t)b * g.Co + co) * g.H + oh) * g.W + ow]);
      ys[ch * g.SY + p] = v;
    }
    for (int i = tid; i < n_a; i += 256) {
      const int ch = i / ((g.R + 2) * PW), q = i - ch * ((g.R + 2) * PW);
      const int rr = q / PW, cc = q - rr * PW;
      const int ih = r0 - 1 + rr, iw = cc - 1;
      const int ci = group0 * g.Cig + ch;
      float v = 0.0f;
      if (ih >= 0 && ih < g.H && iw >= 0 && iw < g.W && ci < g.Ci)
        v = unpack_at<T>(pk, (((int64_t)b * g.Ci + ci) * g.H + ih) * g.W + iw);
      as[ch * g.SA + q] = v;
    }
    __syncthreads();
    if (lane_ok) {
      const float* yrow = ys + (gl * g.Cog + co_l) * g.SY;
      const float* arow = as + (gl * g.Cig + ci_l) * g.SA;
      // positions of the band in four contiguous parts, one per wavefront
      const int n_pos = g.R * g.W, per = (n_pos + 3) >> 2;
      const int p_begin = wave * per, p_end = min(p_begin + per, n_pos);
      int oh_l = p_begin / g.W, ow = p_begin - oh_l * g.W;
      for (int p = p_begin; p < p_end; ++p) {
        const float dy = yrow[p];
        const float* win = arow + oh_l * PW + ow;  // input (oh + u - 1, ow + v - 1) = staged (oh_l + u, ow + v)
#pragma unroll
        for (int u = 0; u < 3; ++u)
#pragma unroll
          for (int v = 0; v < 3; ++v) acc[u * 3 + v] = __builtin_fmaf(dy, win[u * PW + v], acc[u * 3 + v]);
        if (++ow == g.W) {
          ow = 0;
          ++oh_l;
        }
      }
    }
  }
  // the four wavefronts' partial sums, added in wavefront order
  __syncthreads();
  float* red = g3_lds;  // [4][64][9]
#pragma unroll
  for (int t = 0; t < 9; ++t) red[(wave * 64 + lane) * 9 + t] = acc[t];
  __syncthreads();
  if (wave == 0 && lane_ok) {
    const int co = (group0 + gl) * g.Cog + co_l;
    float* dst = out + (int64_t)blockIdx.y * g.n_w + ((int64_t)co * g.Cig + ci_l) * 9;
#pragma unroll
    for (int t = 0; t < 9; ++t)
      dst[t] = (red[lane * 9 + t] + red[(64 + lane) * 9 + t]) + (red[(128 + lane) * 9 + t] + red[(192 + lane) * 9 + t]);
  }
}

// ---- depthwise 3x3, stride 1, pad 1 (one filter per channel) -----------------------------------------------------------
// dW[c][u][v] = sum_{b,oh,ow} dY[b][c][oh][ow] * A_pruned[b][c][oh+u-1][ow+v-1]: nine multiply-adds per pixel and two
// elements read, an HBM-bound sum.  A workgroup owns one channel (and one split of the (image, band of R rows) units);
// each of its four wavefronts takes units in turn: it un-packs the band's R + 2 input rows -- a contiguous run of the
// flat tensor -- into its own zero-haloed LDS plane (eight elements per lane in flight: mask words and ranks first,
// then the values), then walks the band's pixels with the lanes along the row: one coalesced dY load, nine LDS reads at
// fixed offsets, nine multiply-adds into per-lane sums.  The lanes' sums are added in a fixed tree at the end, the
// splits by the reduction kernel: deterministic.
struct DepthwiseGeom {
  int Nb, C, H, W, R, bands, n_units, units_per_split;
  int w_shift;  // log2(W) when W is a power of two, else -1
};
constexpr int kDepthwiseBatch = 8;

template <typename T>
__global__ __launch_bounds__(256) void dw_depthwise3x3_kernel(DepthwiseGeom g, Packed<T> pk, const T* __restrict__ dY,
                                                              float* __restrict__ out) {
  extern __shared__ float dwl[];  // four planes of (R + 2) x (W + 2)
  __shared__ float red[4][9];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c = blockIdx.x;
  const int PW = g.W + 2, region = (g.R + 2) * PW;
  float* a = dwl + wave * region;
  for (int i = lane; i < region; i += 64) a[i] = 0.0f;  // the halo columns stay zero from here on
  float acc[9];
#pragma unroll
  for (int t = 0; t < 9; ++t) acc[t] = 0.0f;
  const int u_begin = (int)blockIdx.y * g.units_per_split, u_end = min(u_begin + g.units_per_split, g.n_units);
  for (int unit = u_begin + wave; unit < u_end; unit += 4) {
    const int b = unit / g.bands, r0 = (unit - b * g.bands) * g.R;
    const int64_t plane = ((int64_t)b * g.C + c) * g.H;  // row index of the plane's first row
    const int rows_here = min(g.R, g.H - r0);
    // staged row rr <-> input row r0 - 1 + rr; rows 0 .. rows_here + 1 are read.  Those outside the map are zero.
    const int ih_lo = max(r0 - 1, 0), ih_hi = min(r0 + rows_here + 1, g.H);
    if (r0 == 0)
      for (int i = lane; i < g.W; i += 64) a[i + 1] = 0.0f;
    if (r0 + rows_here == g.H)
      for (int i = lane; i < g.W; i += 64) a[(rows_here + 1) * PW + i + 1] = 0.0f;
    const int64_t e_lo = (plane + ih_lo) * g.W;
    const int count = (ih_hi - ih_lo) * g.W;
    float* a_rows = a + (ih_lo - (r0 - 1)) * PW + 1;
    for (int i0 = 0; i0 < count; i0 += 64 * kDepthwiseBatch) {
      uint64_t word[kDepthwiseBatch];
      uint32_t rank[kDepthwiseBatch];
#pragma unroll
      for (int q = 0; q < kDepthwiseBatch; ++q) {
        const int i = min(i0 + 64 * q + lane, count - 1);
        const int64_t w = (e_lo + i) >> 6;
        word[q] = pk.mask[w];
        rank[q] = pk.word_rank[w];
      }
      float x[kDepthwiseBatch];
#pragma unroll
      for (int q = 0; q < kDepthwiseBatch; ++q) {
        const int i = min(i0 + 64 * q + lane, count - 1);
        const int bit = (int)((e_lo + i) & 63);
        const bool kept = (word[q] >> bit) & 1ull;
        int64_t pos = (int64_t)rank[q] + __popcll(word[q] & ((1ull << bit) - 1ull));
        pos = pos > pk.k_last ? pk.k_last : pos;
        x[q] = widen<T>(pk.vals[pos]);  // k_total >= 1 here: position k_last exists
        x[q] = kept ? x[q] : 0.0f;
      }
#pragma unroll
      for (int q = 0; q < kDepthwiseBatch; ++q) {
        const int i = i0 + 64 * q + lane;
        if (i < count) {
          const int row = g.w_shift >= 0 ? i >> g.w_shift : i / g.W;
          a_rows[row * PW + (i - row * g.W)] = x[q];
        }
      }
    }
    // the band's pixels, lanes along the rows
    const int npix = rows_here * g.W;
    const T* __restrict__ y = dY + (plane + r0) * g.W;
    for (int q = lane; q < npix; q += 64) {
      const int oh = g.w_shift >= 0 ? q >> g.w_shift : q / g.W;
      const int ow = q - oh * g.W;
      const float dy = widen<T>(y[q]);
      const float* t = a + oh * PW + ow;  // tap (u, v) reads input (oh + u - 1, ow + v - 1) = staged (oh + u, ow + v)
#pragma unroll
      for (int u = 0; u < 3; ++u)
#pragma unroll
        for (int v = 0; v < 3; ++v) acc[u * 3 + v] = fmaf(dy, t[u * PW + v], acc[u * 3 + v]);
    }
  }
#pragma unroll
  for (int t = 0; t < 9; ++t) {
    float v = acc[t];
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    if (lane == 0) red[wave][t] = v;
  }
  __syncthreads();
  if (threadIdx.x < 9)
    out[((int64_t)blockIdx.y * g.C + c) * 9 + threadIdx.x] =
        (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
}

struct GroupedPlan {
  GroupedGeom g;
  bool tiled;          // the 3x3 stride-1 pad-1 kernel with LDS tiles
  Grouped3x3Geom t;
  bool depthwise;      // the depthwise 3x3 stride-1 pad-1 kernel
  DepthwiseGeom dwg;
  size_t lds_bytes;
  int splits;
  int64_t n, n_words, n_rank_blocks;
  int rank_words_per_group;  // > 0: closed-form group positions (rank_grouped_kernel), as in the plain layers' plan
  int64_t rank_groups, rank_k_full;
  size_t off_rank, off_blocks, off_part, ws_bytes;
};

int plan_grouped(const surgeon_layer_desc* d, GroupedPlan* p) {
  if (d->Nb < 1 || d->Ci < 1 || d->H < 1 || d->W < 1 || d->Co < 1 || d->kh < 1 || d->kw < 1 || d->stride < 1 || d->pad < 0)
    return fail(SURGEON_EINVAL, "dw_from_packed: bad conv shape");
  if (d->groups < 1 || d->Ci % d->groups || d->Co % d->groups)
    return fail(SURGEON_EINVAL, "dw_from_packed: groups = %lld does not divide the channel counts", (long long)d->groups);
  if (d->H + 2 * d->pad < d->kh || d->W + 2 * d->pad < d->kw)
    return fail(SURGEON_EINVAL, "dw_from_packed: filter larger than the padded input");
  if (d->kh * d->kw > kGroupedMaxTaps)
    return fail(SURGEON_EUNSUPPORTED, "dw_from_packed: grouped filters larger than %d taps are not implemented", kGroupedMaxTaps);
  const int64_t big = (int64_t)1 << 31;
  if (d->Nb * d->Ci * d->H * d->W > big || d->Nb * d->Co * d->H * d->W > big)
    return fail(SURGEON_EUNSUPPORTED, "dw_from_packed: conv tensor too large");
  GroupedGeom& g = p->g;
  g.Nb = (int)d->Nb; g.Ci = (int)d->Ci; g.H = (int)d->H; g.W = (int)d->W; g.Co = (int)d->Co;
  g.KH = (int)d->kh; g.KW = (int)d->kw; g.stride = (int)d->stride; g.pad = (int)d->pad;
  g.groups = (int)d->groups;
  g.Cig = g.Ci / g.groups;
  g.Cog = g.Co / g.groups;
  g.OH = (g.H + 2 * g.pad - g.KH) / g.stride + 1;
  g.OW = (g.W + 2 * g.pad - g.KW) / g.stride + 1;
  g.n_pos = (int64_t)g.Nb * g.OH * g.OW;
  g.n_w = (int64_t)g.Co * g.Cig * g.KH * g.KW;
  // Depthwise layers (one pair per group) do not take the tiled kernel: their tile would be 64 channels wide, a band of
  // one or two rows with as much halo again, and the un-pack of the halo costs more than the tile saves (measured on a
  // 1280-channel 64x64 layer: 290-360 us tiled, 200 us generic).  They have a kernel of their own, below.
  const int pairs_per_group = g.Cog * g.Cig;
  p->tiled = g.KH == 3 && g.KW == 3 && g.stride == 1 && g.pad == 1 && pairs_per_group >= 4 && pairs_per_group <= 64 &&
             64 % pairs_per_group == 0;
  p->lds_bytes = 0;
  p->depthwise = false;
  if (g.KH == 3 && g.KW == 3 && g.stride == 1 && g.pad == 1 && g.Cig == 1 && g.Cog == 1 && 3 * (g.W + 2) <= 2048) {
    // bands of at most 2048 / (W + 2) - 2 rows (8 KB of LDS per wavefront), of about equal height
    DepthwiseGeom& q = p->dwg;
    const int r_max = std::min(g.H, 2048 / (g.W + 2) - 2);
    q.Nb = g.Nb; q.C = g.Ci; q.H = g.H; q.W = g.W;
    q.bands = (int)ceil_div(g.H, r_max);
    q.R = (int)ceil_div(g.H, q.bands);
    q.bands = (int)ceil_div(g.H, q.R);
    q.w_shift = (g.W & (g.W - 1)) == 0 ? __builtin_ctz((unsigned)g.W) : -1;
    const int64_t units = (int64_t)g.Nb * q.bands;
    if (units <= 0x7fffffff) {
      p->depthwise = true;
      q.n_units = (int)units;
      // about 1024 workgroups, at least one unit per wavefront
      int64_t splits = std::max<int64_t>(1, std::min<int64_t>(ceil_div(1024, g.Ci), ceil_div(units, 4)));
      splits = std::min<int64_t>(splits, 256);
      q.units_per_split = (int)ceil_div(units, splits);
      p->splits = (int)ceil_div(units, q.units_per_split);
      p->lds_bytes = (size_t)4 * (q.R + 2) * (g.W + 2) * sizeof(float);
      g.pos_per_split = 0;
    }
  }
  if (p->tiled) {
    Grouped3x3Geom& t = p->t;
    t.Nb = g.Nb; t.Ci = g.Ci; t.Co = g.Co; t.H = g.H; t.W = g.W; t.Cig = g.Cig; t.Cog = g.Cog; t.groups = g.groups;
    t.gpw = 64 / pairs_per_group;
    t.n_w = g.n_w;
    // the tallest band whose two tiles fit 64 KB of LDS (two workgroups per compute unit); failing that, the whole LDS
    t.R = 0;
    for (int64_t limit : {(int64_t)64 * 1024, (int64_t)kMaxLds}) {
      for (int R = g.H; R >= 1 && t.R == 0; R = R == 1 ? 0 : (R + 1) / 2) {
        const int64_t SY = (int64_t)R * g.W | 1, SA = (int64_t)(R + 2) * (g.W + 2) | 1;
        const int64_t bytes = std::max<int64_t>(4 * ((int64_t)t.gpw * g.Cog * SY + (int64_t)t.gpw * g.Cig * SA), 4 * 64 * 9 * 4);
        if (bytes <= limit) {
          t.R = R; t.SY = (int)SY; t.SA = (int)SA;
          p->lds_bytes = (size_t)bytes;
        }
      }
      if (t.R) break;
    }
    if (t.R == 0) p->tiled = false;  // a single row does not fit: very wide maps keep the generic kernel
  }
  if (p->depthwise) {
    // planned above
  } else if (p->tiled) {
    Grouped3x3Geom& t = p->t;
    t.bands = (int)ceil_div(g.H, t.R);
    t.n_tiles = g.Nb * t.bands;
    const int64_t wgs = ceil_div(g.groups, t.gpw);
    // about four workgroups per compute unit, at least two tiles each
    int64_t splits = std::max<int64_t>(1, std::min<int64_t>(ceil_div(1024, wgs), ceil_div(t.n_tiles, 2)));
    splits = std::min<int64_t>(splits, 256);
    t.tiles_per_split = (int)ceil_div(t.n_tiles, splits);
    p->splits = (int)ceil_div(t.n_tiles, t.tiles_per_split);
    g.pos_per_split = 0;
  } else {
    // enough workgroups to fill the chip, at least 2048 positions each
    const int64_t pairs = (int64_t)g.Co * g.Cig;
    int64_t splits = std::max<int64_t>(1, std::min<int64_t>(ceil_div(g.n_pos, 2048), ceil_div(4096, pairs)));
    splits = std::min<int64_t>(splits, 256);
    g.pos_per_split = ceil_div(g.n_pos, splits);
    p->splits = (int)ceil_div(g.n_pos, g.pos_per_split);
  }
  p->n = (int64_t)g.Nb * g.Ci * g.H * g.W;
  p->n_words = ceil_div(p->n, 64);
  p->rank_words_per_group = 0;
  if (d->group_len > 0 && d->group_len % 64 == 0 && d->group_len <= kWaveRegMaxGroup && p->n > 0) {
    GroupPlan gp;
    if (make_group_plan(p->n, d->group_len, d->r, &gp) && gp.g % 64 == 0 && gp.k_total == d->k_total &&
        gp.n_groups * gp.k_full < ((int64_t)1 << 32)) {  // gp.g: the group length after clamping to n
      p->rank_words_per_group = (int)(gp.g / 64);
      p->rank_groups = gp.n_groups;
      p->rank_k_full = gp.k_full;
    }
  }
  p->n_rank_blocks = ceil_div(p->n_words, kRankWordsPerBlock);
  size_t off = 0;
  p->off_rank = off;
  off += align_up((size_t)p->n_words * 4, 256);
  p->off_blocks = off;
  off += align_up((size_t)p->n_rank_blocks * 4, 256);
  p->off_part = off;
  if (p->splits > 1) off += align_up((size_t)p->splits * (size_t)g.n_w * 4, 256);
  p->ws_bytes = off;
  return SURGEON_OK;
}

template <typename T>
static int run_grouped_t(const GroupedPlan& p, const surgeon_layer_desc* d, const void* vals, const uint64_t* mask,
                         const void* dY, float* dW, void* ws, hipStream_t st, float* G_out, double* sq_partial) {
  char* w = (char*)ws;
  uint32_t* word_rank = (uint32_t*)(w + p.off_rank);
  uint32_t* block_sum = (uint32_t*)(w + p.off_blocks);
  float* part = (float*)(w + p.off_part);
  const GroupedGeom& g = p.g;
  if (d->k_total == 0) {
    ProfScope prof(SURGEON_PROF_DW_AUX, st);
    SURGEON_LAUNCH(fill_zero_f32_kernel, dim3((unsigned)std::min<int64_t>(ceil_div(g.n_w, 256), 4096)), dim3(256), 0, st, dW,
                   g.n_w, G_out);
    SURGEON_LAUNCH_CHECK();
    return SURGEON_OK;
  }
  if (p.rank_words_per_group > 0) {
    ProfScope prof(SURGEON_PROF_DW_AUX, st);
    SURGEON_LAUNCH(rank_grouped_kernel, dim3((unsigned)ceil_div(p.rank_groups, kRankBlock / 64)), dim3(kRankBlock), 0, st, mask,
                   p.n_words, p.rank_words_per_group, p.rank_groups, (uint32_t)p.rank_k_full, word_rank);
    SURGEON_LAUNCH_CHECK();
  } else {
    ProfScope prof(SURGEON_PROF_DW_AUX, st);
    const int rc_rank = launch_rank_table(mask, p.n_words, p.n_rank_blocks, block_sum, word_rank, st);
    if (rc_rank != SURGEON_OK) return rc_rank;
  }
  Packed<T> pk;
  pk.vals = (const T*)vals;
  pk.mask = mask;
  pk.word_rank = word_rank;
  pk.k_last = d->k_total - 1;
  pk.n_words = p.n_words;
  float* out = p.splits > 1 ? part : dW;
  const dim3 grid((unsigned)(g.Co * g.Cig), (unsigned)p.splits);
  if (p.depthwise) {
    ProfScope prof(SURGEON_PROF_DW_GROUPED, st);
    SURGEON_LAUNCH((dw_depthwise3x3_kernel<T>), dim3((unsigned)g.Ci, (unsigned)p.splits), dim3(256), p.lds_bytes, st, p.dwg, pk,
                   (const T*)dY, out);
    SURGEON_LAUNCH_CHECK();
  } else if (p.tiled) {
    ProfScope prof(SURGEON_PROF_DW_GROUPED, st);
    static std::atomic<uint64_t> lds_set{0};  // this function is instantiated per element type = per kernel
    if (p.lds_bytes > 48 * 1024) {
      const int rc_lds = ensure_dynamic_lds((const void*)dw_grouped3x3_kernel<T>, kMaxLds, lds_set);
      if (rc_lds != SURGEON_OK) return rc_lds;
    }
    SURGEON_LAUNCH((dw_grouped3x3_kernel<T>), dim3((unsigned)ceil_div(g.groups, p.t.gpw), (unsigned)p.splits), dim3(256),
                   p.lds_bytes, st, p.t, pk, (const T*)dY, out);
    SURGEON_LAUNCH_CHECK();
  } else {
    ProfScope prof(SURGEON_PROF_DW_GROUPED, st);
    if (g.KH * g.KW <= 9)
      SURGEON_LAUNCH((dw_grouped_kernel<T, 9>), grid, dim3(256), 0, st, g, pk, (const T*)dY, out);
    else if (g.KH * g.KW <= 25)
      SURGEON_LAUNCH((dw_grouped_kernel<T, 25>), grid, dim3(256), 0, st, g, pk, (const T*)dY, out);
    else
      SURGEON_LAUNCH((dw_grouped_kernel<T, kGroupedMaxTaps>), grid, dim3(256), 0, st, g, pk, (const T*)dY, out);
    SURGEON_LAUNCH_CHECK();
  }
  if (p.splits > 1) {
    const int blocks = (int)std::min<int64_t>(ceil_div(g.n_w, 256), kGiPartials);
    ProfScope prof(SURGEON_PROF_DW_AUX, st);
    if (G_out) {
      SURGEON_LAUNCH((dw_reduce_splits_kernel<true, false>), dim3(blocks), dim3(256), 0, st, (const float*)part, p.splits, g.n_w, dW,
                     sq_partial);
      SURGEON_LAUNCH_CHECK();
      return launch_sumsq_final(sq_partial, blocks, g.n_w, G_out, st);
    }
    SURGEON_LAUNCH((dw_reduce_splits_kernel<false, false>), dim3(blocks), dim3(256), 0, st, (const float*)part, p.splits, g.n_w, dW,
                   (double*)nullptr);
    SURGEON_LAUNCH_CHECK();
  } else if (G_out) {
    return launch_sumsq(dW, g.n_w, sq_partial, G_out, st);
  }
  return SURGEON_OK;
}

int grouped_ws_bytes(const surgeon_layer_desc* d, size_t* bytes) {
  GroupedPlan p;
  const int rc = plan_grouped(d, &p);
  if (rc == SURGEON_OK) *bytes = p.ws_bytes;
  return rc;
}

int run_grouped(const surgeon_layer_desc* d, const void* vals, const uint64_t* mask, const void* dY, float* dW, void* ws,
                size_t ws_bytes, hipStream_t st, float* G_out, size_t* off_gi_out, bool plan_only) {
  GroupedPlan p;
  const int rc = plan_grouped(d, &p);
  if (rc != SURGEON_OK) return rc;
  if (d->k_total < 0 || d->k_total > p.n) return fail(SURGEON_EINVAL, "dw_from_packed: bad k_total");
  const size_t off_gi = align_up(p.ws_bytes, 256);
  if (off_gi_out) *off_gi_out = off_gi;
  if (plan_only) return SURGEON_OK;
  const size_t need = G_out ? off_gi + (size_t)kGiPartials * sizeof(double) : p.ws_bytes;
  if (!ws || ws_bytes < need)
    return fail(SURGEON_ESIZE, "dw_from_packed: workspace of %zu bytes needed, %zu given", need, ws_bytes);
  double* sq_partial = G_out ? (double*)((char*)ws + off_gi) : nullptr;
  if (d->dtype == SURGEON_F32) return run_grouped_t<float>(p, d, vals, mask, dY, dW, ws, st, G_out, sq_partial);
  return run_grouped_t<uint16_t>(p, d, vals, mask, dY, dW, ws, st, G_out, sq_partial);
}

}  // namespace surgeon

using namespace surgeon;

extern "C" int surgeon_affine_grad_ws_bytes(int64_t outer, int64_t C, int64_t inner, size_t* ws_bytes) {
  if (!ws_bytes) return fail(SURGEON_EINVAL, "affine_grad_ws_bytes: null pointer");
  AffinePlan p;
  const int rc = plan_affine(outer, C, inner, &p);
  if (rc == SURGEON_OK) *ws_bytes = p.ws_bytes;
  return rc;
}

extern "C" int surgeon_affine_grad(const void* vals, const uint64_t* mask, const void* dY, int64_t outer, int64_t C,
                                   int64_t inner, int dt, int64_t k_total, float* dgamma, float* dbeta, void* ws,
                                   size_t ws_bytes, void* stream) {
  if (dt != SURGEON_F32 && dt != SURGEON_BF16) return fail(SURGEON_EINVAL, "affine_grad: bad dtype %d", dt);
  AffinePlan p;
  const int rc = plan_affine(outer, C, inner, &p);
  if (rc != SURGEON_OK) return rc;
  if (k_total < 0 || k_total > p.n) return fail(SURGEON_EINVAL, "affine_grad: bad k_total");
  if (!dgamma || !dbeta) return fail(SURGEON_EINVAL, "affine_grad: null output");
  if (p.n > 0 && (!mask || !dY || (k_total > 0 && !vals))) return fail(SURGEON_EINVAL, "affine_grad: null pointer");
  if (!ws || ws_bytes < p.ws_bytes)
    return fail(SURGEON_ESIZE, "affine_grad: workspace of %zu bytes needed, %zu given", p.ws_bytes, ws_bytes);
  if (((uintptr_t)ws % 16) || ((uintptr_t)mask % 8) || ((uintptr_t)dY % (dt == SURGEON_F32 ? 4 : 2)) ||
      ((uintptr_t)vals % (dt == SURGEON_F32 ? 4 : 2)) || ((uintptr_t)dgamma % 4) || ((uintptr_t)dbeta % 4))
    return fail(SURGEON_EINVAL, "affine_grad: misaligned pointer");
  hipStream_t st = (hipStream_t)stream;
  if (dt == SURGEON_F32)
    return run_affine<float>(p, vals, mask, dY, outer, (int)C, (int)inner, k_total, dgamma, dbeta, ws, st);
  return run_affine<uint16_t>(p, vals, mask, dY, outer, (int)C, (int)inner, k_total, dgamma, dbeta, ws, st);
}
