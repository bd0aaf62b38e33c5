#pragma once
// Weight gradient from the packed activation (Alg. 1 lines 11-12, Eq. 2): dW = dY^T . A_pruned.
//
// The dense pruned activation is never written to memory: every workgroup rebuilds the tile it needs from
// (vals, mask) straight into LDS -- element e is vals[rank(e)] if bit e of the mask is set, else 0, where
// rank(e) = (set bits before e) comes from a per-64-element prefix table built by a small pre-pass over the
// mask -- and feeds MFMA from there.  This is the only dense contraction of the path, hence the only MFMA user.
//
//   conv2d : implicit GEMM with the output positions (b, oh, ow) as the contraction dimension.  A workgroup
//            owns a [co x ci] tile for ALL taps (u, v) of the filter (or one filter row for large filters): a
//            K-tile is R output rows of one image; its dY rows and the matching input patch (with halo) sit in
//            LDS, and the taps are just shifted LDS reads of the same patch, so every un-packed activation
//            element is reused kh*kw*tile_co times.
//   linear : dW[o][i] = sum_m dY[m][o] * A[m][i]; K-tiles of TM tokens.
// Long contractions are split over workgroups; each split writes its partial tile to the workspace and a last
// kernel adds the splits in index order (no floating-point atomics: results are reproducible bit for bit).
// bf16 inputs: convolutions with taps widen to fp32 while staging (exact) and feed either the fp32 MFMA or, where the
// patch layout allows, the bf16 MFMA after re-narrowing (the original bits); linear layers and 1x1 stride-1
// convolutions un-pack once to a dense transient copy and run a dense bf16 contraction (dw_bf16.hip).
// Accumulation is always fp32.
#include <algorithm>
#include <type_traits>

#include "common.hpp"

namespace surgeon {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx4_a4 __attribute__((ext_vector_type(4), aligned(4)));  // LDS vector read at 4-byte alignment
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// the high halves (= the bf16 values) of 8 floats that hold exactly widened bf16 numbers, as one MFMA operand
__device__ __forceinline__ bf16x8 pack_bf16x8(floatx4 lo, floatx4 hi) {
  u32x4 d;
  d[0] = __builtin_amdgcn_perm(__float_as_uint(lo[1]), __float_as_uint(lo[0]), 0x07060302u);
  d[1] = __builtin_amdgcn_perm(__float_as_uint(lo[3]), __float_as_uint(lo[2]), 0x07060302u);
  d[2] = __builtin_amdgcn_perm(__float_as_uint(hi[1]), __float_as_uint(hi[0]), 0x07060302u);
  d[3] = __builtin_amdgcn_perm(__float_as_uint(hi[3]), __float_as_uint(hi[2]), 0x07060302u);
  return __builtin_bit_cast(bf16x8, d);
}

template <typename InT>
__device__ __forceinline__ float widen(InT v);
template <>
__device__ __forceinline__ float widen<float>(float v) {
  return v;
}
template <>
__device__ __forceinline__ float widen<uint16_t>(uint16_t v) {
  return __uint_as_float((uint32_t)v << 16);
}

// ---------------------------------------------------------------------------------------------------------
// rank table: word_rank[w] = number of set mask bits before word w
// ---------------------------------------------------------------------------------------------------------
constexpr int kRankBlock = 256;
constexpr int kRankWordsPerBlock = 1024;  // 4 words per thread

__device__ __forceinline__ uint32_t wave_incl_scan_u32(uint32_t v, int lane) {
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t t = (uint32_t)__shfl_up((int)v, off, 64);
    if (lane >= off) v += t;
  }
  return v;
}

// exclusive prefix of `v` over the 256 threads of the block (and the block total in *total)
__device__ __forceinline__ uint32_t block_excl_scan_u32(uint32_t v, uint32_t* lds4, uint32_t* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t incl = wave_incl_scan_u32(v, lane);
  if (lane == 63) lds4[wave] = incl;
  __syncthreads();
  uint32_t base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kRankBlock / 64; ++w) {
    const uint32_t s = lds4[w];
    if (w < wave) base += s;
    tot += s;
  }
  *total = tot;
  return base + incl - v;
}

static __global__ __launch_bounds__(kRankBlock) void rank_block_sum_kernel(const uint64_t* __restrict__ mask, int64_t n_words,
                                                                    uint32_t* __restrict__ block_sum) {
  __shared__ uint32_t lds4[kRankBlock / 64];
  const int64_t w0 = (int64_t)blockIdx.x * kRankWordsPerBlock + threadIdx.x * 4;
  uint32_t s = 0;
#pragma unroll
  for (int q = 0; q < 4; ++q)
    if (w0 + q < n_words) s += (uint32_t)__popcll(mask[w0 + q]);
  uint32_t total;
  block_excl_scan_u32(s, lds4, &total);
  if (threadIdx.x == 0) block_sum[blockIdx.x] = total;
}

// single block: in-place exclusive scan of the block sums
static __global__ __launch_bounds__(1024) void rank_scan_kernel(uint32_t* __restrict__ block_sum, int n_blocks) {
  __shared__ uint32_t part[1024];
  const int tid = threadIdx.x;
  const int per = (n_blocks + 1023) / 1024;
  const int begin = min(tid * per, n_blocks), end = min(begin + per, n_blocks);
  uint32_t s = 0;
  for (int i = begin; i < end; ++i) s += block_sum[i];
  part[tid] = s;
  __syncthreads();
  if (tid == 0) {
    uint32_t acc = 0;
    for (int t = 0; t < 1024; ++t) {
      const uint32_t v = part[t];
      part[t] = acc;
      acc += v;
    }
  }
  __syncthreads();
  uint32_t acc = part[tid];
  for (int i = begin; i < end; ++i) {
    const uint32_t v = block_sum[i];
    block_sum[i] = acc;
    acc += v;
  }
}

// SUM_BASE: block_base holds the blocks' plain sums and each block adds up the ones in front of it itself (for tables of
// at most kRankFusedBlocks blocks -- tensors of up to 33.5 M elements -- this costs less than the single-block scan
// launch in between)
constexpr int kRankFusedBlocks = 512;
template <bool SUM_BASE>
static __global__ __launch_bounds__(kRankBlock) void rank_write_kernel(const uint64_t* __restrict__ mask, int64_t n_words,
                                                                const uint32_t* __restrict__ block_base,
                                                                uint32_t* __restrict__ word_rank) {
  __shared__ uint32_t lds4[kRankBlock / 64];
  uint32_t first = 0;
  if constexpr (SUM_BASE) {
    uint32_t pre = 0;
    for (int i = threadIdx.x; i < (int)blockIdx.x; i += kRankBlock) pre += block_base[i];
    block_excl_scan_u32(pre, lds4, &first);
    __syncthreads();  // lds4 is used again below
  } else {
    first = block_base[blockIdx.x];
  }
  const int64_t w0 = (int64_t)blockIdx.x * kRankWordsPerBlock + threadIdx.x * 4;
  uint32_t c[4];
  uint32_t s = 0;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    c[q] = (w0 + q < n_words) ? (uint32_t)__popcll(mask[w0 + q]) : 0u;
    s += c[q];
  }
  uint32_t total;
  uint32_t base = first + block_excl_scan_u32(s, lds4, &total);
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    if (w0 + q < n_words) word_rank[w0 + q] = base;
    base += c[q];
  }
}

// the general rank table (kept elements in front of every mask word): two launches for tables of moderate size, three
// (with a single-block scan of the block sums) beyond
static inline int launch_rank_table(const uint64_t* mask, int64_t n_words, int64_t n_rank_blocks, uint32_t* block_sum,
                                    uint32_t* word_rank, hipStream_t st) {
  SURGEON_LAUNCH(rank_block_sum_kernel, dim3((unsigned)n_rank_blocks), dim3(kRankBlock), 0, st, mask, n_words, block_sum);
  SURGEON_LAUNCH_CHECK();
  if (n_rank_blocks <= kRankFusedBlocks) {
    SURGEON_LAUNCH(rank_write_kernel<true>, dim3((unsigned)n_rank_blocks), dim3(kRankBlock), 0, st, mask, n_words,
                   (const uint32_t*)block_sum, word_rank);
    SURGEON_LAUNCH_CHECK();
    return SURGEON_OK;
  }
  SURGEON_LAUNCH(rank_scan_kernel, dim3(1), dim3(1024), 0, st, block_sum, (int)n_rank_blocks);
  SURGEON_LAUNCH_CHECK();
  SURGEON_LAUNCH(rank_write_kernel<false>, dim3((unsigned)n_rank_blocks), dim3(kRankBlock), 0, st, mask, n_words,
                 (const uint32_t*)block_sum, word_rank);
  SURGEON_LAUNCH_CHECK();
  return SURGEON_OK;
}

// Rank table when every group of `words_per_group` mask words is known to hold exactly k_full kept elements
// (the packing's group length is a multiple of 64, at most 4096): one wavefront per group, no cross-group pass.
static __global__ __launch_bounds__(kRankBlock) void rank_grouped_kernel(const uint64_t* __restrict__ mask, int64_t n_words,
                                                                         int words_per_group, int64_t n_groups,
                                                                         uint32_t k_full, uint32_t* __restrict__ word_rank) {
  const int lane = threadIdx.x & 63;
  const int64_t grp = (int64_t)blockIdx.x * (kRankBlock / 64) + (threadIdx.x >> 6);
  if (grp >= n_groups) return;
  const int64_t w = grp * words_per_group + lane;
  const bool ok = lane < words_per_group && w < n_words;
  const uint32_t c = ok ? (uint32_t)__popcll(mask[w]) : 0u;
  const uint32_t incl = wave_incl_scan_u32(c, lane);
  if (ok) word_rank[w] = (uint32_t)grp * k_full + incl - c;
}

// ---------------------------------------------------------------------------------------------------------
// un-pack of one element (Alg. 1 line 11)
// ---------------------------------------------------------------------------------------------------------
template <typename InT>
struct Packed {
  const InT* __restrict__ vals;
  const uint64_t* __restrict__ mask;
  const uint32_t* __restrict__ word_rank;
  int64_t k_last;   // k_total - 1: every read of vals is clamped to it
  int64_t n_words;  // mask words
};

template <typename InT>
__device__ __forceinline__ float unpack_at(const Packed<InT>& p, int64_t e) {
  const int64_t w = e >> 6;
  const int bit = (int)(e & 63);
  const uint64_t word = p.mask[w];
  if (!((word >> bit) & 1ull)) return 0.0f;
  int64_t r = (int64_t)p.word_rank[w] + __popcll(word & ((1ull << bit) - 1ull));
  r = r > p.k_last ? p.k_last : r;
  return widen<InT>(p.vals[r]);
}

// ---------------------------------------------------------------------------------------------------------
// conv2d
// ---------------------------------------------------------------------------------------------------------
struct ConvGeom {
  int Nb, Ci, H, W, Co, OH, OW, KH, KW, stride, pad;
  int R;                // output rows per K-tile (divides OH)
  int tiles_per_img;    // OH / R
  int n_ktiles;         // Nb * tiles_per_img
  int tiles_per_split;  // K-tiles per workgroup along the contraction
  int PR, PW, PS;       // patch rows / cols kept in LDS per input channel, and the per-channel stride (floats)
  int lds_step;         // LDS distance between horizontally adjacent output positions (1 for 1x1 filters: only
                        // the pixels a strided 1x1 filter touches are staged), fill_step = stride / lds_step
  int fill_step;
  int ci_tiles;         // output tiles along ci (blockIdx.x = co_tile * ci_tiles + ci_tile)
  int n_patch;          // tile_ci * PR * PW: patch elements staged per K-tile
  uint32_t magic_pw, magic_pr;  // ceil(2^32 / PW), ceil(2^32 / PR) (0 when the divisor is 1)
  int dy_vec;           // dY rows of a K-tile start 4-element aligned and hold a multiple of 4 positions
  int bf16_mfma;        // 1: bf16 inputs go through v_mfma_f32_16x16x32_bf16 (stride-1 LDS patch, OW % 8 == 0)
  int run_mode;         // 1: the patch is staged as runs of 16 consecutive elements with metadata prefetch
  int Wv;               // input columns of a row that fall inside the patch
  int runs_per_row, n_runs;
  uint32_t magic_rpr;   // ceil(2^32 / runs_per_row)
  int n_buf;            // 2: staging overlaps the MFMA work of the previous K-tile; 1: LDS holds one K-tile only
  int64_t n_w;          // Co*Ci*KH*KW
  // Filter rows folded into the channel dimension (layers with few input channels, e.g. a network's first conv):
  // Ci and KH above are then the VIRTUAL sizes (Ci_in * fold channels, one filter row); virtual channel cv reads
  // input channel cv / fold shifted down by cv % fold rows, and [Co][cv][kw] is the same memory as
  // [Co][ci][kh][kw].  fold == 0: no folding, Ci_in == Ci.
  int Ci_in, fold;
  uint32_t magic_fold;  // ceil(2^32 / fold)
};

// n / d for n*d < 2^32 with magic = ceil(2^32 / d); magic == 0 encodes d == 1
__device__ __forceinline__ uint32_t fast_div(uint32_t n, uint32_t magic) { return magic ? __umulhi(n, magic) : n; }

template <typename InT>
struct Vec4;
template <>
struct Vec4<float> {
  typedef float type __attribute__((ext_vector_type(4)));
};
template <>
struct Vec4<uint16_t> {
  typedef uint16_t type __attribute__((ext_vector_type(4)));
};

constexpr int kConvLoaders = 256;  // threads of the four staging wavefronts
constexpr int kConvChunk = 20;     // patch elements a staging thread has in flight at once

// Stages K-tile `tile` (dY rows + un-packed input patch) into one LDS buffer.  Called by the 256 staging
// threads only.  All loads of a chunk are issued before the first dependent use: per chunk there are two
// memory round trips (mask word + rank, then the value), not two per element.
template <typename InT, int KHC, int MT, int NT, int P>
__device__ __forceinline__ void conv_stage_tile(const ConvGeom& gm, const Packed<InT>& pk, const InT* __restrict__ dY,
                                                float* __restrict__ buf, int tile, int ltid, int co0, int ci0, int u0) {
  constexpr int TCO = 2 * MT * 16, SY = P + 4, NY = TCO * P / 4 / kConvLoaders;
  typedef typename Vec4<InT>::type vec_t;
  float* __restrict__ dYs = buf;
  float* __restrict__ As = buf + TCO * SY;
  const int b = tile / gm.tiles_per_img;
  const int oh0 = (tile - b * gm.tiles_per_img) * gm.R;
  const int valid_pos = gm.R * gm.OW;
  const int PW = gm.PW, PS = gm.PS;

  // ---- dY[b, co0.., oh0..oh0+R, :]: R*OW contiguous elements per output channel
  vec_t y[NY];
  if (gm.dy_vec) {
#pragma unroll
    for (int j = 0; j < NY; ++j) {
      const int q = ltid + kConvLoaders * j;
      const int c = q / (P / 4), k4 = q % (P / 4);
      const bool ok = co0 + c < gm.Co && 4 * k4 < valid_pos;
      const int64_t off = ok ? (((int64_t)b * gm.Co + co0 + c) * gm.OH + oh0) * gm.OW + 4 * k4 : 0;
      y[j] = *reinterpret_cast<const vec_t*>(dY + off);
      if (!ok) y[j] = vec_t{0, 0, 0, 0};
    }
  } else {
    for (int idx = ltid; idx < TCO * P; idx += kConvLoaders) {
      const int c = idx / P, k = idx - c * P;
      float v = 0.0f;
      if (co0 + c < gm.Co && k < valid_pos)
        v = widen<InT>(dY[(((int64_t)b * gm.Co + co0 + c) * gm.OH + oh0) * gm.OW + k]);
      dYs[c * SY + k] = v;
    }
  }

  // ---- un-packed input patch: PR rows from ih0 and PW columns from -pad, every fill_step-th pixel
  const int ih0 = oh0 * gm.stride + u0 - gm.pad;
  for (int base = 0; base < gm.n_patch; base += kConvLoaders * kConvChunk) {
    uint64_t word[kConvChunk];
    uint32_t rank0[kConvChunk];
    int where[kConvChunk];  // LDS offset, or -1 past the end of the patch; bit position in the top 6 bits
#pragma unroll
    for (int j = 0; j < kConvChunk; ++j) {
      const uint32_t idx = (uint32_t)(base + j * kConvLoaders + ltid);
      const bool in_patch = idx < (uint32_t)gm.n_patch;
      const uint32_t row = fast_div(idx, gm.magic_pw), col = idx - row * PW;
      const uint32_t c = fast_div(row, gm.magic_pr), pr = row - c * gm.PR;
      const int cv = ci0 + (int)c;
      const int ci = gm.fold ? (int)fast_div((uint32_t)cv, gm.magic_fold) : cv;
      const int kh = gm.fold ? cv - ci * gm.fold : 0;  // filter row folded into this virtual channel
      const int ih = ih0 + (int)pr * gm.fill_step + kh, iw = (int)col * gm.fill_step - gm.pad;
      const bool ok = in_patch && cv < gm.Ci && ih >= 0 && ih < gm.H && iw >= 0 && iw < gm.W;
      const int64_t e = ok ? (((int64_t)b * gm.Ci_in + ci) * gm.H + ih) * gm.W + iw : 0;
      const uint64_t m = pk.mask[e >> 6];
      rank0[j] = pk.word_rank[e >> 6];
      word[j] = ok ? m : 0ull;
      where[j] = in_patch ? (int)((c * PS + pr * PW + col) | ((uint32_t)(e & 63) << 26)) : -1;
    }
    InT raw[kConvChunk];
#pragma unroll
    for (int j = 0; j < kConvChunk; ++j) {
      const int bit = (int)((uint32_t)where[j] >> 26);
      const bool has = (word[j] >> bit) & 1ull;
      int64_t r = (int64_t)rank0[j] + __popcll(word[j] & ((1ull << bit) - 1ull));
      r = r > pk.k_last ? pk.k_last : r;
      raw[j] = pk.vals[has ? r : 0];
    }
#pragma unroll
    for (int j = 0; j < kConvChunk; ++j) {
      if (where[j] != -1) {
        const int bit = (int)((uint32_t)where[j] >> 26);
        const bool has = (word[j] >> bit) & 1ull;
        As[where[j] & 0x3ffffff] = has ? widen<InT>(raw[j]) : 0.0f;
      }
    }
  }
  if (gm.dy_vec) {
#pragma unroll
    for (int j = 0; j < NY; ++j) {
      const int q = ltid + kConvLoaders * j;
      const int c = q / (P / 4), k4 = q % (P / 4);
      typedef float f4 __attribute__((ext_vector_type(4)));
      f4 v = {widen<InT>(y[j][0]), widen<InT>(y[j][1]), widen<InT>(y[j][2]), widen<InT>(y[j][3])};
      *reinterpret_cast<f4*>(&dYs[c * SY + 4 * k4]) = v;
    }
  }
}

// ---- run-based staging: each staging thread un-packs runs of 16 consecutive elements of a patch row --------
// All global reads of this path are buffer loads: 32-bit byte offsets (no 64-bit address arithmetic on the vector
// ALU, which the staging wavefronts share with the matrix instructions of the wavefront on the same SIMD), a
// per-K-tile scalar offset for everything that is uniform, and the hardware range check instead of clamps and
// selects: an offset at or beyond the buffer size returns 0.  The host enables the path only when every buffer is
// smaller than 2 GiB, so kOutOfRange is out of range for all of them.
constexpr int kRunLen = 16;
constexpr int kRunsPerThread = 4;
constexpr uint32_t kOutOfRange = 0x80000000u;
constexpr int kRawBufferWord3 = 0x00020000;  // raw buffer, 32-bit data format (gfx9 family)

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Raw loads describing one run of a K-tile: the mask word holding the run's first element (d0, d1), the low half
// of the next word (d2), and the rank of the first word.  They are issued one K-tile ahead, so that per K-tile only
// one memory round trip (the values and dY) sits on the staging wavefronts' critical path.  A run outside the image
// (padding rows, channels past Ci) loads from kOutOfRange and sees an empty mask.
struct RunLoad {
  uint32_t d0, d1, d2, r0, sh;  // sh: bit offset of the run in (d1:d0), 0..63
};

template <typename InT>
struct DyVec;
template <>
struct DyVec<float> {
  typedef u32x4 raw_t;
  static __device__ __forceinline__ raw_t load(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0);
  }
  static __device__ __forceinline__ floatx4 widen4(raw_t v) { return __builtin_bit_cast(floatx4, v); }
};
template <>
struct DyVec<uint16_t> {
  typedef u32x2 raw_t;
  static __device__ __forceinline__ raw_t load(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
    return __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0);
  }
  static __device__ __forceinline__ floatx4 widen4(raw_t v) {
    u32x4 w = {v.x << 16, v.x & 0xffff0000u, v.y << 16, v.y & 0xffff0000u};
    return __builtin_bit_cast(floatx4, w);
  }
};
__device__ __forceinline__ uint32_t load_val_bits(__amdgpu_buffer_rsrc_t r, uint32_t voff, float, uint32_t soff = 0) {
  return __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0);
}
__device__ __forceinline__ uint32_t load_val_bits(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint16_t, uint32_t soff = 0) {
  return (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(r, voff, soff, 0) << 16;  // bf16 -> the fp32 with the same value
}

// Per-thread state of the run-based staging: everything that does not change from K-tile to K-tile is computed once.
template <typename InT, int MT, int P>
struct RunStager {
  static constexpr int TCO = 2 * MT * 16, SY = P + 4, NY = TCO * P / 4 / kConvLoaders;
  static constexpr uint32_t ES = sizeof(InT);
  __amdgpu_buffer_rsrc_t r_mask, r_rank, r_vals, r_dy;
  uint32_t e_const[kRunsPerThread];  // flat element index of the run minus the K-tile's uniform part (mod 2^32)
  int ih_const[kRunsPerThread];      // input row of the run minus the K-tile's first row; hugely negative: no run
  uint32_t nv_mask[kRunsPerThread];  // low `elements of the run inside the row` bits
  int lds_dst[kRunsPerThread];       // float offset of the run inside the patch area
  uint32_t y_voff[NY];               // byte offset of this thread's j-th dY vector inside the K-tile's dY block
  int y_lds;                         // float offset of the first of them in the dY area (the j-th is 16*SY*j... further)
  // dY rows that are not vector-aligned (e.g. 7x7 maps) are staged element by element: a thread keeps its position
  // k = ltid % P and walks over the output channels ltid / P + j * (256 / P)
  static constexpr int NE = TCO * P / kConvLoaders;
  uint32_t ys_voff;                  // byte offset of the first of them, or kOutOfRange past the valid positions
  int ys_lds;
  const InT* dy_ptr;

  __device__ __forceinline__ void init(const ConvGeom& gm, const Packed<InT>& pk, const InT* __restrict__ dY, int ltid,
                                       int co0, int ci0, int u0) {
    r_mask = __builtin_amdgcn_make_buffer_rsrc((void*)pk.mask, 0, (int)(pk.n_words * 8), kRawBufferWord3);
    r_rank = __builtin_amdgcn_make_buffer_rsrc((void*)pk.word_rank, 0, (int)(pk.n_words * 4), kRawBufferWord3);
    r_vals = __builtin_amdgcn_make_buffer_rsrc((void*)pk.vals, 0, (int)((pk.k_last + 1) * (int64_t)ES), kRawBufferWord3);
    r_dy = __builtin_amdgcn_make_buffer_rsrc((void*)dY, 0, (int)((int64_t)gm.Nb * gm.Co * gm.OH * gm.OW * ES),
                                             kRawBufferWord3);
    dy_ptr = dY;
#pragma unroll
    for (int r = 0; r < kRunsPerThread; ++r) {
      const int q = ltid + kConvLoaders * r;
      const uint32_t row = fast_div((uint32_t)q, gm.magic_rpr), rr = (uint32_t)q - row * gm.runs_per_row;
      const uint32_t c = fast_div(row, gm.magic_pr), pr = row - c * gm.PR;
      // a run is kRunLen LDS columns = kRunLen * fill_step input pixels (fill_step 2: a strided 1x1 filter, pad 0)
      const int fs = gm.fill_step;
      const int cv = ci0 + (int)c;
      const int ci = gm.fold ? (int)fast_div((uint32_t)cv, gm.magic_fold) : cv;
      const int kh = gm.fold ? cv - ci * gm.fold : 0;  // filter row folded into this virtual channel
      const int dih = u0 - gm.pad + (int)pr * fs + kh, col0 = (int)rr * kRunLen, iw0 = col0 * fs;
      const bool has_run = q < gm.n_runs && cv < gm.Ci;
      e_const[r] = (uint32_t)((ci * gm.H + dih) * gm.W + iw0);
      ih_const[r] = has_run ? dih : -(1 << 30);
      // input pixels of the run that exist in the row and whose LDS column exists in the patch row (1..32)
      const int in_valid = min(min(kRunLen, gm.Wv - col0) * fs, gm.W - iw0);
      nv_mask[r] = (q < gm.n_runs) ? (0xffffffffu >> (32 - in_valid)) : 0u;
      lds_dst[r] = (int)(c * gm.PS + pr * gm.PW) + col0 + gm.pad;
    }
    const int valid_pos = gm.R * gm.OW;
#pragma unroll
    for (int j = 0; j < NY; ++j) {
      const int q = ltid + kConvLoaders * j;
      const int c = q / (P / 4), k4 = q % (P / 4);
      const bool ok = co0 + c < gm.Co && 4 * k4 < valid_pos;
      y_voff[j] = ok ? (uint32_t)(c * gm.OH * gm.OW + 4 * k4) * ES : kOutOfRange;
    }
    y_lds = (ltid / (P / 4)) * SY + 4 * (ltid % (P / 4));
    const int ks = ltid % P, cs = ltid / P;
    ys_voff = ks < valid_pos ? (uint32_t)(cs * gm.OH * gm.OW + ks) * ES : kOutOfRange;
    ys_lds = cs * SY + ks;
  }

  // the metadata loads of K-tile `tile`
  __device__ __forceinline__ void issue(const ConvGeom& gm, int tile, RunLoad (&m)[kRunsPerThread]) const {
    const int b = tile / gm.tiles_per_img;
    const int ih_base = (tile - b * gm.tiles_per_img) * gm.R * gm.stride;
    const uint32_t e_base = (uint32_t)(b * gm.Ci_in * gm.H + ih_base) * (uint32_t)gm.W;
#pragma unroll
    for (int r = 0; r < kRunsPerThread; ++r) {
      if (kConvLoaders * r >= gm.n_runs) continue;  // uniform: no thread has an r-th run in this geometry
      const bool ok = (uint32_t)(ih_base + ih_const[r]) < (uint32_t)gm.H;
      const uint32_t e0 = e_base + e_const[r];
      const uint32_t off8 = ok ? (e0 >> 6) * 8u : kOutOfRange;
      const u32x2 w = __builtin_amdgcn_raw_buffer_load_b64(r_mask, off8, 0, 0);
      m[r].d0 = w.x;
      m[r].d1 = w.y;
      m[r].d2 = __builtin_amdgcn_raw_buffer_load_b32(r_mask, off8 + 8u, 0, 0);
      m[r].r0 = __builtin_amdgcn_raw_buffer_load_b32(r_rank, off8 >> 1, 0, 0);
      m[r].sh = e0 & 63u;
    }
  }

  // Stages K-tile `tile` from the metadata in `cur`; replaces `cur` by the metadata of K-tile tile + 1 when
  // prefetch_next is set.  LEN = 16 / 8: LDS columns a run can have in this geometry; FULL: every run has exactly
  // LEN; FS = fill_step (1 or 2): LDS column t of a run is input pixel t * FS of it; DYV: dY rows are vector-aligned.
  template <int LEN, bool FULL, int FS, bool DYV>
  __device__ __forceinline__ void stage(const ConvGeom& gm, float* __restrict__ buf, int tile, int co0,
                                        RunLoad (&cur)[kRunsPerThread], bool prefetch_next) const {
    float* __restrict__ dYs = buf;
    float* __restrict__ As = buf + TCO * SY;
    const int b = tile / gm.tiles_per_img;
    const int oh0 = (tile - b * gm.tiles_per_img) * gm.R;
    const uint32_t y_soff = (uint32_t)(((b * gm.Co + co0) * gm.OH + oh0) * gm.OW) * ES;
    typename DyVec<InT>::raw_t y[DYV ? NY : 1];
    uint32_t ys[DYV ? 1 : NE];
    if constexpr (DYV) {
#pragma unroll
      for (int j = 0; j < NY; ++j) y[j] = DyVec<InT>::load(r_dy, y_voff[j], y_soff);
    } else {
      // The range check is documented for the VGPR offset only (the compiler's buffer intrinsics exclude the scalar
      // offset from it; gfx950 was measured to include it, which this code does not rely on), so the whole offset goes
      // there, and the resource of this K-tile ends with the last channel of image b: output channels past Co (last co
      // tile) are then out of range and read 0 instead of the next image or memory behind dY.
      const uint32_t step = (uint32_t)((kConvLoaders / P) * gm.OH * gm.OW) * ES;
      const __amdgpu_buffer_rsrc_t r_img = __builtin_amdgcn_make_buffer_rsrc(
          (void*)dy_ptr, 0, (int)((uint32_t)((b + 1) * gm.Co * gm.OH * gm.OW) * ES), kRawBufferWord3);
      uint32_t voff = ys_voff + y_soff;  // kOutOfRange + y_soff stays out of range: every buffer is below 2 GiB
#pragma unroll
      for (int j = 0; j < NE; ++j) {
        ys[j] = load_val_bits(r_img, voff, InT());
        voff += step;
      }
    }

    uint32_t bits[kRunsPerThread], raw[kRunsPerThread][LEN];
#pragma unroll
    for (int r = 0; r < kRunsPerThread; ++r) {
      if (kConvLoaders * r >= gm.n_runs) continue;
      const uint32_t sh = cur[r].sh, s5 = sh & 31u;
      const bool upper = sh >= 32u;
      const uint32_t below5 = (1u << s5) - 1u;
      // the run's bits: 32 bits of (d2:d1:d0) starting at sh, cut to the run's length
      bits[r] = __builtin_amdgcn_alignbit(upper ? cur[r].d2 : cur[r].d1, upper ? cur[r].d1 : cur[r].d0, s5) & nv_mask[r];
      // kept elements of the word before the run
      const uint32_t before = (uint32_t)__builtin_popcount(upper ? cur[r].d0 : (cur[r].d0 & below5)) +
                              (uint32_t)__builtin_popcount(upper ? (cur[r].d1 & below5) : 0u);
      uint32_t off = (cur[r].r0 + before) * ES;  // byte offset in vals of the run's first kept element
#pragma unroll
      for (int t = 0; t < LEN; ++t) {
        // a dropped element reads the next kept value (or 0 past the end) and is masked when it is stored
        if (FS == 1) {
          raw[r][t] = load_val_bits(r_vals, off, InT());
          off += ((bits[r] >> t) & 1u) * ES;
        } else {
          const uint32_t kept_before = (uint32_t)__builtin_popcount(bits[r] & ((1u << (t * FS)) - 1u));
          raw[r][t] = load_val_bits(r_vals, off + kept_before * ES, InT());
        }
      }
    }
    if (prefetch_next) issue(gm, tile + 1, cur);
#pragma unroll
    for (int r = 0; r < kRunsPerThread; ++r) {
      if (kConvLoaders * r >= gm.n_runs) continue;
      if (nv_mask[r]) {
        float* __restrict__ dst = As + lds_dst[r];
#pragma unroll
        for (int t = 0; t < LEN; ++t) {
          const uint32_t keep = (uint32_t)(((int32_t)(bits[r] << (31 - t * FS))) >> 31);  // all ones if the pixel's bit is set
          if (FULL || ((nv_mask[r] >> (t * FS)) & 1u)) dst[t] = __uint_as_float(raw[r][t] & keep);
        }
      }
    }
    if constexpr (DYV) {
#pragma unroll
      for (int j = 0; j < NY; ++j)
        *reinterpret_cast<floatx4*>(&dYs[y_lds + j * (kConvLoaders / (P / 4)) * SY]) = DyVec<InT>::widen4(y[j]);
    } else {
#pragma unroll
      for (int j = 0; j < NE; ++j) dYs[ys_lds + j * (kConvLoaders / P) * SY] = __uint_as_float(ys[j]);
    }
  }
};

// Workgroup = 8 wavefronts.  Wavefronts 0-3 are the MFMA wavefronts, arranged 2 (co) x 2 (ci), each owning
// MT x NT MFMA 16x16 tiles for KHC*KW taps.  Wavefronts 4-7 stage the next K-tile into the other LDS buffer
// while the MFMA wavefronts work on the current one; one barrier per K-tile hands the buffers over.
// blockIdx.y = split along the contraction, blockIdx.z = first filter row handled (u0 = z * KHC).
template <typename InT, bool BF, int KHC, int KW, int MT, int NT, int P>
__global__ __attribute__((amdgpu_flat_work_group_size(512, 512))) void dw_conv_kernel(ConvGeom gm, Packed<InT> pk,
                                                                                      const InT* __restrict__ dY,
                                                                                      float* __restrict__ out) {
  constexpr int TCO = 2 * MT * 16, TCI = 2 * NT * 16, SY = P + 4, TAPS = KHC * KW, STEPS = P / 4;
  extern __shared__ float smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  int tile_id, split_id;  // the tiles of a split share its positions (dY rows, input patches): whole splits per XCD
  xcd_ordered_work_item(&tile_id, &split_id);
  const int co_tile = tile_id / gm.ci_tiles, ci_tile = tile_id % gm.ci_tiles;
  const int co0 = co_tile * TCO, ci0 = ci_tile * TCI;
  const int u0 = blockIdx.z * KHC;
  const int PW = gm.PW, PS = gm.PS;
  const int buf_floats = TCO * SY + TCI * PS;
  const int t_begin = split_id * gm.tiles_per_split;
  const int t_end = min(t_begin + gm.tiles_per_split, gm.n_ktiles);

  // A zero area after every channel's patch in both buffers (written once): contraction positions past R*OW point
  // at its start, and their dY is zero as well.  Reads of such a position reach KHC - 1 rows and KW - 1 columns
  // further, the bf16 path 7 more floats.
  const int zero_len = (KHC - 1) * PW + KW + 7;
  for (int t = tid; t < gm.n_buf * TCI * zero_len; t += 512) {
    const int bsel = t / (TCI * zero_len), rem = t - bsel * (TCI * zero_len);
    const int c = rem / zero_len, x = rem - c * zero_len;
    smem[bsel * buf_floats + TCO * SY + c * PS + gm.PR * PW + x] = 0.0f;
  }
  if (gm.run_mode) {  // halo columns are never written by the run-based staging: clear both patches once
    for (int t = tid; t < gm.n_buf * TCI * PS; t += 512) {
      const int bsel = t / (TCI * PS);
      smem[bsel * buf_floats + TCO * SY + (t - bsel * (TCI * PS))] = 0.0f;
    }
  }

  if (wave >= 4) {
    // ------------------------------ staging wavefronts ------------------------------
    // their few vector instructions win arbitration against the MFMA wavefront sharing the SIMD, so that a tile is
    // staged promptly instead of in whatever issue slots the matrix pipeline leaves free
    __builtin_amdgcn_s_setprio(3);
    const int ltid = tid - 256;
    if (gm.n_buf == 1) {
      for (int tile = t_begin; tile < t_end; ++tile) {
        conv_stage_tile<InT, KHC, MT, NT, P>(gm, pk, dY, smem, tile, ltid, co0, ci0, u0);
        __syncthreads();  // the tile is staged
        __syncthreads();  // the MFMA wavefronts are done with it
      }
      return;
    }
    if (gm.run_mode) {
      RunStager<InT, MT, P> rs;
      rs.init(gm, pk, dY, ltid, co0, ci0, u0);
      RunLoad meta[kRunsPerThread];
      if (t_begin < t_end) rs.issue(gm, t_begin, meta);
      __syncthreads();  // the patches are cleared before the first run is written
      // uniform choice of the variant: runs of up to 16 or up to 8 columns, all runs full or not, every pixel or every
      // second one, dY rows vector-aligned or not
      const int fs = gm.fill_step;
      const bool len8 = gm.Wv <= 8;
      const bool full = len8 ? (gm.Wv == 8 && gm.W == 8 * fs) : (gm.Wv % kRunLen == 0 && gm.W % (kRunLen * fs) == 0);
      for (int tile = t_begin; tile < t_end; ++tile) {
        float* __restrict__ buf = smem + ((tile - t_begin) & 1) * buf_floats;
        const bool more = tile + 1 < t_end;
#define SURGEON_STAGE(LEN, FULL, FS) \
  do { \
    if (gm.dy_vec) rs.template stage<LEN, FULL, FS, true>(gm, buf, tile, co0, meta, more); \
    else rs.template stage<LEN, FULL, FS, false>(gm, buf, tile, co0, meta, more); \
  } while (0)
        bool staged = false;
        if constexpr (KHC == 1 && KW == 1) {  // only a strided 1x1 filter skips pixels inside a run
          if (fs == 2) {
            staged = true;
            if (len8 && full) SURGEON_STAGE(8, true, 2);
            else if (len8) SURGEON_STAGE(8, false, 2);
            else if (full) SURGEON_STAGE(16, true, 2);
            else SURGEON_STAGE(16, false, 2);
          }
        }
        if (!staged) {
          if (len8 && full) SURGEON_STAGE(8, true, 1);
          else if (len8) SURGEON_STAGE(8, false, 1);
          else if (full) SURGEON_STAGE(16, true, 1);
          else SURGEON_STAGE(16, false, 1);
        }
#undef SURGEON_STAGE
        __syncthreads();  // this buffer is complete; the other one is no longer being read
      }
      return;
    }
    if (t_begin < t_end) conv_stage_tile<InT, KHC, MT, NT, P>(gm, pk, dY, smem, t_begin, ltid, co0, ci0, u0);
    for (int tile = t_begin; tile < t_end; ++tile) {
      __syncthreads();  // buffer (tile - t_begin) & 1 is complete; the other one is no longer being read
      if (tile + 1 < t_end)
        conv_stage_tile<InT, KHC, MT, NT, P>(gm, pk, dY, smem + ((tile + 1 - t_begin) & 1) * buf_floats, tile + 1, ltid,
                                             co0, ci0, u0);
    }
    return;
  }

  // ------------------------------ MFMA wavefronts ------------------------------
  const int wm = wave >> 1, wn = wave & 1;
  const int i16 = lane & 15, kk = lane >> 4;
  // LDS offset of the input pixel under tap (0,0) for each contraction position this lane feeds
  int aoff[STEPS];
#pragma unroll
  for (int s = 0; s < STEPS; ++s) {
    const int k = 4 * s + kk;
    const int r = k / gm.OW, ow = k - r * gm.OW;
    aoff[s] = (r < gm.R) ? (r * gm.lds_step) * PW + ow * gm.lds_step : gm.PR * PW;
  }
  // bf16 matrix-core path: each lane feeds 8 consecutive positions (32*s + 8*kk ...), which never straddle an
  // output row because OW is a multiple of 8 there
  static_assert(!BF || std::is_same<InT, uint16_t>::value, "the bf16 matrix-core loop needs bf16 inputs");
  constexpr int STEPS_B = BF ? P / 32 : 1;
  int aoff_b[STEPS_B];
#pragma unroll
  for (int s = 0; s < STEPS_B; ++s) {
    const int k = 32 * s + 8 * kk;
    const int r = k / gm.OW, ow = k - r * gm.OW;
    aoff_b[s] = (r < gm.R) ? r * PW + ow : gm.PR * PW;
  }
  floatx4 acc[MT][NT][TAPS];
#pragma unroll
  for (int a = 0; a < MT; ++a)
#pragma unroll
    for (int b = 0; b < NT; ++b)
#pragma unroll
      for (int t = 0; t < TAPS; ++t) acc[a][b][t] = floatx4{0.f, 0.f, 0.f, 0.f};

  if (gm.run_mode) __syncthreads();  // pairs with the staging wavefronts' barrier after the patches are cleared
  for (int tile = t_begin; tile < t_end; ++tile) {
    __syncthreads();
    const float* __restrict__ dYs = smem + ((tile - t_begin) & (gm.n_buf - 1)) * buf_floats;
    const float* __restrict__ As = dYs + TCO * SY;
    const float* __restrict__ a_base = dYs + (wm * MT * 16 + i16) * SY + kk;
    const float* __restrict__ b_base = As + (wn * NT * 16 + i16) * PS;
    if constexpr (BF) {
      const float* __restrict__ ya = dYs + (wm * MT * 16 + i16) * SY + 8 * kk;
#pragma unroll
      for (int s = 0; s < STEPS_B; ++s) {
        bf16x8 av[MT];
#pragma unroll
        for (int a = 0; a < MT; ++a) {
          const float* y = ya + a * 16 * SY + 32 * s;
          av[a] = pack_bf16x8(*reinterpret_cast<const floatx4*>(y), *reinterpret_cast<const floatx4*>(y + 4));
        }
#pragma unroll
        for (int du = 0; du < KHC; ++du) {
#pragma unroll
          for (int v = 0; v < KW; ++v) {
#pragma unroll
            for (int bn = 0; bn < NT; ++bn) {
              const float* q = b_base + bn * 16 * PS + aoff_b[s] + du * PW + v;
              const bf16x8 bv = pack_bf16x8(*reinterpret_cast<const floatx4_a4*>(q), *reinterpret_cast<const floatx4_a4*>(q + 4));
#pragma unroll
              for (int a = 0; a < MT; ++a)
                acc[a][bn][du * KW + v] =
                    __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[a], bv, acc[a][bn][du * KW + v], 0, 0, 0);
            }
          }
        }
      }
    } else {
    // taps are shifted reads of the same patch
#pragma unroll
    for (int s = 0; s < STEPS; ++s) {
      float av[MT];
#pragma unroll
      for (int a = 0; a < MT; ++a) av[a] = a_base[a * 16 * SY + 4 * s];
#pragma unroll
      for (int du = 0; du < KHC; ++du) {
#pragma unroll
        for (int v = 0; v < KW; ++v) {
#pragma unroll
          for (int bn = 0; bn < NT; ++bn) {
            const float bv = b_base[bn * 16 * PS + aoff[s] + du * PW + v];
#pragma unroll
            for (int a = 0; a < MT; ++a)
              acc[a][bn][du * KW + v] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[a], bv, acc[a][bn][du * KW + v], 0, 0, 0);
          }
        }
      }
    }
    }
    if (gm.n_buf == 1) __syncthreads();
  }

  // ---- write this split's partial tile: lane holds rows 4*kk..4*kk+3 (co), column i16 (ci) of each 16x16 tile
  float* __restrict__ dst = out + (int64_t)split_id * gm.n_w;
#pragma unroll
  for (int a = 0; a < MT; ++a) {
#pragma unroll
    for (int bn = 0; bn < NT; ++bn) {
      const int ci = ci0 + wn * NT * 16 + bn * 16 + i16;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int co = co0 + wm * MT * 16 + a * 16 + 4 * kk + r;
        if (co < gm.Co && ci < gm.Ci) {
          const int64_t base = (((int64_t)co * gm.Ci + ci) * gm.KH + u0) * gm.KW;
#pragma unroll
          for (int du = 0; du < KHC; ++du)
#pragma unroll
            for (int v = 0; v < KW; ++v) dst[base + du * gm.KW + v] = acc[a][bn][du * KW + v][r];
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------------------
// linear
// ---------------------------------------------------------------------------------------------------------
struct LinGeom {
  int64_t M, K, N;
  int i_tiles;            // tiles along in-features (blockIdx.x = o_tile * i_tiles + i_tile)
  int64_t rows_per_split; // tokens per workgroup along the contraction (multiple of TM)
  int64_t n_w;
};

template <typename InT, int MT, int NT, int TM>
__global__ __attribute__((amdgpu_flat_work_group_size(256, 256))) void dw_linear_kernel(LinGeom gm, Packed<InT> pk,
                                                                                        const InT* __restrict__ dY,
                                                                                        float* __restrict__ out) {
  constexpr int TO = 2 * MT * 16, TI = 2 * NT * 16, SO = TO + 16, SI = TI + 16, STEPS = TM / 4;
  __shared__ float dYs[TM * SO];
  __shared__ float As[TM * SI];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int i16 = lane & 15, kk = lane >> 4;
  const int o_tile = blockIdx.x / gm.i_tiles, i_tile = blockIdx.x % gm.i_tiles;
  const int64_t o0 = (int64_t)o_tile * TO, i0 = (int64_t)i_tile * TI;

  floatx4 acc[MT][NT];
#pragma unroll
  for (int a = 0; a < MT; ++a)
#pragma unroll
    for (int b = 0; b < NT; ++b) acc[a][b] = floatx4{0.f, 0.f, 0.f, 0.f};

  const int64_t m_begin = (int64_t)blockIdx.y * gm.rows_per_split;
  const int64_t m_end = min(m_begin + gm.rows_per_split, gm.M);
  for (int64_t m0 = m_begin; m0 < m_end; m0 += TM) {
    __syncthreads();
    for (int idx = tid; idx < TM * TO; idx += 256) {
      const int r = idx / TO, c = idx - r * TO;
      const int64_t m = m0 + r, o = o0 + c;
      dYs[r * SO + c] = (m < m_end && o < gm.N) ? widen<InT>(dY[m * gm.N + o]) : 0.0f;
    }
    for (int idx = tid; idx < TM * TI; idx += 256) {
      const int r = idx / TI, c = idx - r * TI;
      const int64_t m = m0 + r, i = i0 + c;
      As[r * SI + c] = (m < m_end && i < gm.K) ? unpack_at<InT>(pk, m * gm.K + i) : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int s = 0; s < STEPS; ++s) {
      float av[MT], bv[NT];
#pragma unroll
      for (int a = 0; a < MT; ++a) av[a] = dYs[(4 * s + kk) * SO + wm * MT * 16 + a * 16 + i16];
#pragma unroll
      for (int b = 0; b < NT; ++b) bv[b] = As[(4 * s + kk) * SI + wn * NT * 16 + b * 16 + i16];
#pragma unroll
      for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int b = 0; b < NT; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[a], bv[b], acc[a][b], 0, 0, 0);
    }
  }
  float* __restrict__ dst = out + (int64_t)blockIdx.y * gm.n_w;
#pragma unroll
  for (int a = 0; a < MT; ++a)
#pragma unroll
    for (int b = 0; b < NT; ++b) {
      const int64_t i = i0 + wn * NT * 16 + b * 16 + i16;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int64_t o = o0 + wm * MT * 16 + a * 16 + 4 * kk + r;
        if (o < gm.N && i < gm.K) dst[o * gm.K + i] = acc[a][b][r];
      }
    }
}

// adds the split partials in index order.  GI: also the sum of squares of what this workgroup wrote (Eq. 4's sum folded
// into the pass that produces dW, so that the gradient is not read again): fp64, fixed order, one partial per workgroup.
// VEC: four consecutive weights per thread with 16-byte accesses (n_w a multiple of 4, dW 16-byte aligned; the partials
// start on a 256-byte boundary of the workspace).  Each weight's additions run in split order either way.
template <bool GI, bool VEC>
static __global__ __launch_bounds__(256) void dw_reduce_splits_kernel(const float* __restrict__ part, int n_splits, int64_t n_w,
                                                               float* __restrict__ dW, double* __restrict__ sq_partial) {
  double sq = 0.0;
  if constexpr (VEC) {
    const int64_t n4 = n_w >> 2;
    const float4* __restrict__ part4 = reinterpret_cast<const float4*>(part);
    float4* __restrict__ dW4 = reinterpret_cast<float4*>(dW);
    for (int64_t x = (int64_t)blockIdx.x * 256 + threadIdx.x; x < n4; x += (int64_t)gridDim.x * 256) {
      float4 s = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
      int k = 0;
      for (; k + 4 <= n_splits; k += 4) {  // four 16-byte loads in flight; the additions stay in split order
        float4 v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = part4[(int64_t)(k + q) * n4 + x];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          s.x += v[q].x; s.y += v[q].y; s.z += v[q].z; s.w += v[q].w;
        }
      }
      for (; k < n_splits; ++k) {
        const float4 v = part4[(int64_t)k * n4 + x];
        s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
      }
      dW4[x] = s;
      if (GI) sq += ((double)s.x * (double)s.x + (double)s.y * (double)s.y) + ((double)s.z * (double)s.z + (double)s.w * (double)s.w);
    }
  } else {
    for (int64_t x = (int64_t)blockIdx.x * 256 + threadIdx.x; x < n_w; x += (int64_t)gridDim.x * 256) {
      // eight loads in flight at a time; the additions stay in split order, so the result does not depend on the batching
      float s = 0.0f;
      int k = 0;
      for (; k + 8 <= n_splits; k += 8) {
        float v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) v[q] = part[(int64_t)(k + q) * n_w + x];
#pragma unroll
        for (int q = 0; q < 8; ++q) s += v[q];
      }
      for (; k < n_splits; ++k) s += part[(int64_t)k * n_w + x];
      dW[x] = s;
      if (GI) sq += (double)s * (double)s;
    }
  }
  if (GI) {
    __shared__ double wave_sq[4];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sq += __shfl_down(sq, off, 64);
    if ((threadIdx.x & 63) == 0) wave_sq[threadIdx.x >> 6] = sq;
    __syncthreads();
    if (threadIdx.x == 0) sq_partial[blockIdx.x] = (wave_sq[0] + wave_sq[1]) + (wave_sq[2] + wave_sq[3]);
  }
}

static __global__ void fill_zero_f32_kernel(float* __restrict__ p, int64_t n, float* __restrict__ also_zero) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = 0.0f;
  if (also_zero && blockIdx.x == 0 && threadIdx.x == 0) also_zero[0] = 0.0f;  // Gradient Importance of a zero gradient
}

// ---------------------------------------------------------------------------------------------------------
// host planning
// ---------------------------------------------------------------------------------------------------------
constexpr int kConvSlots = 256;    // the conv kernel keeps one 8-wavefront workgroup per compute unit
constexpr int kLinSlots = 512;     // the linear kernel fits two workgroups per compute unit
constexpr int kMaxSplits = 256;
constexpr double kBf16FlopsPerCuPerUs = 9.8e6;  // bf16 MFMA rate of one compute unit (2.5 PFLOP/s / 256)
constexpr double kFlopsPerCuPerUs = 0.6e6;  // fp32 MFMA rate of one compute unit (157.3 TFLOP/s / 256), per microsecond
constexpr size_t kMaxLds = 160 * 1024;

struct ConvPlan {
  ConvGeom g;
  int gemm1x1;               // 1: bf16 1x1 stride-1 layer handled as a dense contraction over the pixels
  int64_t gemm_ktiles_per_split;
  int sparse;                // 1: fp32 3x3 stride-1 layer with few kept elements, gradient from the kept elements alone
  int sparse_tiles_per_split;
  int khc, kw_t, mt, nt, p;  // kernel variant
  int co_tiles, z, splits;
  size_t lds_bytes;
};

// which weight-gradient kernel a convolution may use
enum SparseChoice { SPARSE_BY_DENSITY = -1, SPARSE_NEVER = 0, SPARSE_IF_SHAPE_ALLOWS = 1 };
// kept percentage up to which the kernel that skips the dropped elements beats the dense matrix-core kernel: its time
// grows linearly with the kept count and crosses the dense kernel's at 18.5 % with 32-channel workgroups and at 24 %
// with 64-channel ones on the layers measured
static inline int64_t sparse_max_kept_percent(int Ci) { return sparse_conv_waves(Ci) == 16 ? 22 : 17; }

struct LinPlan {
  LinGeom g;
  int mt, nt, tm;
  int o_tiles, splits;
  bool bf16_mfma;  // dense bf16-MFMA path: un-pack to the workspace, then contract
  int bf16_wide;   // 1: the 128 x 256 tile of the bf16 path
  bool bf16_big;   // the dense bf16 path with the 256 x 128 tile of eight wavefronts
};

struct DwPlan {
  bool conv;
  ConvPlan c;
  LinPlan l;
  int64_t n, n_words, n_rank_blocks, n_w;
  int rank_words_per_group;  // > 0: closed-form group positions (rank_grouped_kernel)
  int64_t rank_groups, rank_k_full;
  int splits;
  size_t off_rank, off_blocks, off_part, off_dense, ws_bytes;
};

// Splits along the contraction.  Modelled time of a launch with s splits:
//   rounds(s) * (tiles_per_split * tile_us + fixed_us)  +  time to write and re-read s partial copies of dW,
// rounds = ceil(out_tiles * s / slots).  The smallest s with the least modelled time wins.
static int choose_splits(int64_t k_tiles, int64_t out_tiles, int slots, double tile_us, int64_t n_w,
                         int64_t* tiles_per_split) {
  const double fixed_us = 15.0, partial_us_per_split = (double)n_w * 8.0 / 4.0e6;  // 8 bytes per element at 4 TB/s
  int64_t best_s = 1;
  double best_cost = -1.0;
  const int64_t s_max = std::min<int64_t>(k_tiles, kMaxSplits);
  for (int64_t s = 1; s <= s_max; ++s) {
    const int64_t per = ceil_div(k_tiles, s);
    const int64_t s_eff = ceil_div(k_tiles, per);
    const double rounds = (double)ceil_div(out_tiles * s_eff, slots);
    const double cost = rounds * ((double)per * tile_us + fixed_us) + (s_eff > 1 ? s_eff * partial_us_per_split : 0.0);
    if (best_cost < 0.0 || cost < best_cost) {
      best_cost = cost;
      best_s = s_eff;
    }
  }
  const int64_t per = ceil_div(k_tiles, best_s);
  *tiles_per_split = per;
  return (int)ceil_div(k_tiles, per);
}

static int plan_conv(const surgeon_layer_desc* d, ConvPlan* cp, int sparse_choice) {
  if (d->Nb < 1 || d->Ci < 1 || d->H < 1 || d->W < 1 || d->Co < 1 || d->kh < 1 || d->kw < 1 || d->stride < 1 ||
      d->pad < 0)
    return fail(SURGEON_EINVAL, "dw_from_packed: bad conv shape");
  if (d->H + 2 * d->pad < d->kh || d->W + 2 * d->pad < d->kw)
    return fail(SURGEON_EINVAL, "dw_from_packed: filter larger than the padded input");
  const int64_t big = (int64_t)1 << 31;
  if (d->Nb * d->Ci * d->H * d->W > big || d->Nb >= (1 << 24) || d->Co * d->Ci * d->kh * d->kw > big)
    return fail(SURGEON_EUNSUPPORTED, "dw_from_packed: conv tensor too large");
  ConvGeom& g = cp->g;
  g.Nb = (int)d->Nb; g.Ci = (int)d->Ci; g.H = (int)d->H; g.W = (int)d->W; g.Co = (int)d->Co;
  g.KH = (int)d->kh; g.KW = (int)d->kw; g.stride = (int)d->stride; g.pad = (int)d->pad;
  g.OH = (g.H + 2 * g.pad - g.KH) / g.stride + 1;
  g.OW = (g.W + 2 * g.pad - g.KW) / g.stride + 1;
  g.n_w = (int64_t)g.Co * g.Ci * g.KH * g.KW;
  cp->gemm1x1 = 0;
  cp->sparse = 0;
  if (sparse_choice != SPARSE_NEVER && d->dtype == SURGEON_F32 && g.KH == 3 && g.KW == 3 && g.stride == 1 && g.pad == 1 &&
      (g.W == 8 || g.W == 16 || g.W == 32) && g.H % sparse_conv_band_rows(g.W) == 0 && g.Co >= kSparseCo / 2 &&
      d->k_total < ((int64_t)1 << 32) && (int64_t)g.Nb * g.H < ((int64_t)1 << 30) &&
      (sparse_choice == SPARSE_IF_SHAPE_ALLOWS ||
       d->k_total * 100 <= sparse_max_kept_percent(g.Ci) * (int64_t)g.Nb * g.Ci * g.H * g.W)) {
    cp->sparse = 1;
    cp->khc = 3; cp->kw_t = 3; cp->mt = cp->nt = 0; cp->p = 0; cp->z = 1; cp->lds_bytes = 0;
    cp->co_tiles = (int)ceil_div(g.Co, kSparseCo);
    const int sp_waves = sparse_conv_waves(g.Ci);
    g.ci_tiles = (int)ceil_div(g.Ci, sp_waves * kSparseCiPerWave);
    g.Ci_in = g.Ci; g.fold = 0; g.magic_fold = 0;
    // all workgroups resident at once and none left for a second round; every split walks whole (image, band) tiles
    const int64_t n_tiles = (int64_t)g.Nb * (g.H / sparse_conv_band_rows(g.W));
    const int64_t want = std::min<int64_t>(std::min<int64_t>(n_tiles, kMaxSplits),
                                           std::max<int64_t>(1, sparse_conv_slots(sp_waves) / ((int64_t)cp->co_tiles * g.ci_tiles)));
    cp->sparse_tiles_per_split = (int)ceil_div(n_tiles, want);
    cp->splits = (int)ceil_div(n_tiles, cp->sparse_tiles_per_split);
    return SURGEON_OK;
  }
  if (d->dtype == SURGEON_BF16 && g.KH == 1 && g.KW == 1 && g.stride == 1 && g.pad == 0 && (g.H * g.W) % 4 == 0) {
    // a 1x1 stride-1 convolution has no tap reuse to pay for un-packing inside the tile loads: un-pack once to a
    // dense transient copy and contract over the pixels on the bf16 matrix cores (as the bf16 linear path does)
    cp->gemm1x1 = 1;
    cp->khc = 1; cp->kw_t = 1; cp->mt = cp->nt = 0; cp->p = 0; cp->z = 1; cp->lds_bytes = 0;
    cp->co_tiles = (int)ceil_div(g.Co, kBf16LinearTile);
    g.ci_tiles = (int)ceil_div(g.Ci, kBf16LinearTile);
    g.Ci_in = g.Ci; g.fold = 0; g.magic_fold = 0;
    const int64_t k_tiles = (int64_t)g.Nb * ceil_div((int64_t)g.H * g.W, kBf16LinearTokens);
    const double tile_us = 2.0 * kBf16LinearTile * kBf16LinearTile * kBf16LinearTokens / (0.35 * kBf16FlopsPerCuPerUs);
    int64_t per;
    cp->splits = choose_splits(k_tiles, (int64_t)cp->co_tiles * g.ci_tiles, kLinSlots, tile_us, g.n_w, &per);
    cp->gemm_ktiles_per_split = per;
    return SURGEON_OK;
  }
  if (g.KH == 3 && g.KW == 3) {
    cp->khc = 3; cp->kw_t = 3;
  } else if (g.KW == 1 || g.KW == 3 || g.KW == 5 || g.KW == 7) {
    cp->khc = 1; cp->kw_t = g.KW;
  } else {
    return fail(SURGEON_EUNSUPPORTED, "dw_from_packed: filter width %d not implemented (1, 3, 5, 7)", g.KW);
  }
  cp->z = g.KH / cp->khc;
  if (g.OW > 128) return fail(SURGEON_EUNSUPPORTED, "dw_from_packed: output width %d > 128 not implemented", g.OW);
  g.lds_step = (g.KH == 1 && g.KW == 1) ? 1 : g.stride;
  g.fill_step = g.stride / g.lds_step;
  g.Ci_in = g.Ci;
  g.fold = 0;
  g.magic_fold = 0;
  if (g.KH > 1) {
    // Folding the filter rows into the channels pays when the channel tile (32) is mostly padding: compare the
    // matrix work (padded tile sizes x taps x filter-row slices) of both forms.
    auto padded = [](int64_t x, int64_t t) { return ceil_div(x, t) * t; };
    const int mt_plain = cp->khc == 3 ? ((g.Co % 160 == 0) ? 5 : (g.Co > 64 ? 4 : 2)) : (g.Co > 64 ? 4 : 2);
    const int mt_fold = g.Co > 64 ? 4 : 2;
    const int64_t work_plain = padded(g.Co, 32 * mt_plain) * padded(g.Ci, 32) * cp->khc * g.KW * cp->z;
    const int64_t work_fold = padded(g.Co, 32 * mt_fold) * padded((int64_t)g.Ci * g.KH, 32) * g.KW;
    if (work_fold < work_plain) {
      g.fold = g.KH;
      g.magic_fold = (uint32_t)(0xffffffffu / (uint32_t)g.fold) + 1u;
      g.Ci = g.Ci_in * g.KH;
      g.KH = 1;
      cp->khc = 1;
      cp->kw_t = g.KW;
      cp->z = 1;
    }
  }
  // tile shape
  if (cp->kw_t == 1 && cp->khc == 1) {
    cp->mt = (g.Co > 64 || g.Ci > 64) ? 4 : 2;  // implemented pairs: (4,4), (2,2) and, for few input channels, (4,1), (2,1)
    cp->nt = g.Ci <= 32 ? 1 : cp->mt;
  } else if (cp->khc == 3) {
    cp->nt = 1;
    cp->mt = (g.Co % 160 == 0) ? 5 : (g.Co > 64 ? 4 : 2);
  } else {
    cp->nt = 1;
    cp->mt = g.Co > 64 ? 4 : 2;
  }
  const int tco = 2 * cp->mt * 16, tci = 2 * cp->nt * 16;
  cp->co_tiles = (int)ceil_div(g.Co, tco);
  g.ci_tiles = (int)ceil_div(g.Ci, tci);
  // K-tile: P contraction positions = R whole output rows of one image (R divides OH).  Among the implemented
  // P, take the one whose rows fill it best and whose two LDS buffers fit; 64 is preferred on a near tie.
  double best_score = -1.0;
  const int p_options[3] = {64, 32, 128};
  for (int n_buf = 2; n_buf >= 1 && best_score < 0.0; --n_buf) {
    for (int pi = 0; pi < 3; ++pi) {
      const int p = p_options[pi];
      for (int r = g.OH; r >= 1; --r) {
        if (g.OH % r != 0 || r * g.OW > p) continue;
        const int pr = (r - 1) * g.lds_step + cp->khc;
        const int pw = (g.OW - 1) * g.lds_step + g.KW;
        int ps = (pr + cp->khc - 1) * pw + cp->kw_t + 7;  // patch + the zero area behind it
        ps += (4 - ps % 32 + 32) % 32;  // per-channel stride = 4 (mod 32) floats: spreads channels over LDS banks
        const size_t lds = n_buf * ((size_t)tco * (p + 4) + (size_t)tci * ps) * sizeof(float);
        if (lds > kMaxLds) continue;
        // the run-based staging (far cheaper per element) needs at most kRunsPerThread runs per staging thread
        const int wv = g.fill_step == 1 ? std::min(g.W, pw - g.pad) : std::min(pw, (g.W + g.fill_step - 1) / g.fill_step);
        const bool runs_fit = (int64_t)tci * pr * ceil_div(std::max(wv, 1), kRunLen) <= kRunsPerThread * kConvLoaders &&
                              n_buf == 2;
        const double score = (double)(r * g.OW) / p - (p == 64 ? 0.0 : 0.05) + (runs_fit ? 0.5 : 0.0);
        if (score > best_score) {
          best_score = score;
          cp->p = p;
          g.R = r;
          g.PR = pr;
          g.PW = pw;
          g.PS = ps;
          g.n_buf = n_buf;
          cp->lds_bytes = lds;
        }
        break;  // smaller r only lowers the fill of this P
      }
    }
  }
  if (best_score < 0.0) return fail(SURGEON_EUNSUPPORTED, "dw_from_packed: conv tile does not fit LDS (OW = %d)", g.OW);
  g.tiles_per_img = g.OH / g.R;
  g.n_ktiles = g.Nb * g.tiles_per_img;
  g.n_patch = tci * g.PR * g.PW;
  g.magic_pw = g.PW > 1 ? (uint32_t)(0xffffffffu / (uint32_t)g.PW) + 1u : 0u;
  g.magic_pr = g.PR > 1 ? (uint32_t)(0xffffffffu / (uint32_t)g.PR) + 1u : 0u;
  if ((int64_t)g.n_patch * std::max(g.PW, g.PR) >= ((int64_t)1 << 32) || g.n_patch >= (1 << 26))
    return fail(SURGEON_EUNSUPPORTED, "dw_from_packed: conv patch too large");
  g.dy_vec = ((g.R * g.OW) % 4 == 0 && ((int64_t)g.OH * g.OW) % 4 == 0) ? 1 : 0;
  g.bf16_mfma = (d->dtype == SURGEON_BF16 && g.lds_step == 1 && g.OW % 8 == 0) ? 1 : 0;
  // LDS columns of a patch row that hold an input pixel: column c is pixel c * fill_step - pad
  g.Wv = g.fill_step == 1 ? std::min(g.W, g.PW - g.pad) : std::min(g.PW, (g.W + g.fill_step - 1) / g.fill_step);
  g.runs_per_row = (int)ceil_div(std::max(g.Wv, 1), kRunLen);
  g.n_runs = tci * g.PR * g.runs_per_row;
  g.magic_rpr = g.runs_per_row > 1 ? (uint32_t)(0xffffffffu / (uint32_t)g.runs_per_row) + 1u : 0u;
  // the run-based staging addresses vals and dY with 32-bit byte offsets whose top bit marks "no access"
  const int64_t es = d->dtype == SURGEON_F32 ? 4 : 2;
  const bool small_buffers = d->k_total * es < big && (int64_t)g.Nb * g.Co * g.OH * g.OW * es < big;
  g.run_mode = ((g.fill_step == 1 || (g.fill_step == 2 && g.pad == 0)) && g.n_buf == 2 && g.Wv >= 1 && small_buffers &&
                g.n_runs <= kRunsPerThread * kConvLoaders) ? 1 : 0;
  int64_t per;
  const double tile_us = 2.0 * tco * tci * cp->khc * cp->kw_t * cp->p / kFlopsPerCuPerUs;
  cp->splits = choose_splits(g.n_ktiles, (int64_t)cp->co_tiles * g.ci_tiles * cp->z, kConvSlots, tile_us, g.n_w, &per);
  g.tiles_per_split = (int)per;
  return SURGEON_OK;
}

static int plan_linear(const surgeon_layer_desc* d, LinPlan* lp) {
  if (d->M < 0 || d->K < 1 || d->N < 1) return fail(SURGEON_EINVAL, "dw_from_packed: bad linear shape");
  const int64_t big = (int64_t)1 << 31;
  if (d->M * d->K > big || d->N * d->K > big || d->M * d->N > ((int64_t)1 << 40))
    return fail(SURGEON_EUNSUPPORTED, "dw_from_packed: linear tensor too large");
  LinGeom& g = lp->g;
  g.M = d->M; g.K = d->K; g.N = d->N;
  g.n_w = d->N * d->K;
  lp->bf16_mfma = d->dtype == SURGEON_BF16 && d->K % 8 == 0 && d->M > 0;
  lp->bf16_wide = 0;
  lp->bf16_big = false;
  if (lp->bf16_mfma && d->N % 8 == 0 && d->M * d->N * 2 < big && d->M * d->K * 2 < big) {
    // the 256 x 128 tile of eight wavefronts against the 128 x 128 one: it is taken when padding the layer to it costs at
    // most a third more matrix work (its loads are buffer loads with 32-bit offsets: operands below 2 GiB)
    auto padded = [](int64_t x, int64_t t) { return ceil_div(x, t) * t; };
    const int64_t work_big = padded(d->N, kBf16BigTileO) * padded(d->K, kBf16BigTileI);
    const int64_t work_dense = padded(d->N, kBf16LinearTile) * padded(d->K, kBf16LinearTile);
    if (3 * work_big <= 4 * work_dense) {
      lp->bf16_big = true;
      lp->mt = lp->nt = 0;
      lp->tm = kBf16BigTokens;
      lp->o_tiles = (int)ceil_div(d->N, kBf16BigTileO);
      g.i_tiles = (int)ceil_div(d->K, kBf16BigTileI);
      int64_t per;
      const int64_t k_tiles = ceil_div(d->M, lp->tm);
      const double tile_us = 2.0 * kBf16BigTileO * kBf16BigTileI * lp->tm / (0.3 * kBf16FlopsPerCuPerUs);
      lp->splits = choose_splits(k_tiles, (int64_t)lp->o_tiles * g.i_tiles, kConvSlots, tile_us, g.n_w, &per);
      g.rows_per_split = per * lp->tm;
      return SURGEON_OK;
    }
  }
  if (lp->bf16_mfma) {
    lp->mt = lp->nt = 0;
    // the wide tile when the in-feature dimension fills it and the layer is large enough to keep the chip busy with it
    lp->bf16_wide = (d->K % kBf16LinearTileWide == 0 && d->N % 8 == 0 &&
                     ceil_div(d->N, kBf16LinearTile) * (d->K / kBf16LinearTileWide) >= 36) ? 1 : 0;
    const int tile_i = lp->bf16_wide ? kBf16LinearTileWide : kBf16LinearTile;
    lp->tm = lp->bf16_wide ? kBf16LinearTokensWide : kBf16LinearTokens;
    lp->o_tiles = (int)ceil_div(d->N, kBf16LinearTile);
    g.i_tiles = (int)ceil_div(d->K, tile_i);
    int64_t per;
    const int64_t k_tiles = ceil_div(d->M, lp->tm);
    const double tile_us = 2.0 * kBf16LinearTile * tile_i * lp->tm / (0.35 * kBf16FlopsPerCuPerUs);
    lp->splits = choose_splits(k_tiles, (int64_t)lp->o_tiles * g.i_tiles, kLinSlots, tile_us, g.n_w, &per);
    g.rows_per_split = per * lp->tm;
    return SURGEON_OK;
  }
  const bool small = d->N <= 64 && d->K <= 64;
  lp->mt = small ? 2 : 4;
  lp->nt = small ? 2 : 4;
  lp->tm = 32;
  const int to = 2 * lp->mt * 16, ti = 2 * lp->nt * 16;
  lp->o_tiles = (int)ceil_div(d->N, to);
  g.i_tiles = (int)ceil_div(d->K, ti);
  int64_t per;
  const int64_t k_tiles = std::max<int64_t>(1, ceil_div(d->M, lp->tm));
  const double tile_us = 2.0 * to * ti * lp->tm / kFlopsPerCuPerUs;
  lp->splits = choose_splits(k_tiles, (int64_t)lp->o_tiles * g.i_tiles, kLinSlots, tile_us, g.n_w, &per);
  g.rows_per_split = per * lp->tm;
  return SURGEON_OK;
}

static int plan_dw(const surgeon_layer_desc* d, DwPlan* p, int sparse_choice = SPARSE_BY_DENSITY) {
  if (!d) return fail(SURGEON_EINVAL, "dw_from_packed: null descriptor");
  if (d->dtype != SURGEON_F32 && d->dtype != SURGEON_BF16) return fail(SURGEON_EINVAL, "dw_from_packed: bad dtype");
  if (d->k_total < 0) return fail(SURGEON_EINVAL, "dw_from_packed: k_total < 0");
  int rc;
  if (d->kind == SURGEON_CONV2D) {
    p->conv = true;
    if ((rc = plan_conv(d, &p->c, sparse_choice)) != SURGEON_OK) return rc;
    p->n = d->Nb * d->Ci * d->H * d->W;
    p->n_w = p->c.g.n_w;
    p->splits = p->c.splits;
  } else if (d->kind == SURGEON_LINEAR) {
    p->conv = false;
    if ((rc = plan_linear(d, &p->l)) != SURGEON_OK) return rc;
    p->n = d->M * d->K;
    p->n_w = p->l.g.n_w;
    p->splits = p->l.splits;
  } else {
    return fail(SURGEON_EINVAL, "dw_from_packed: bad layer kind %d", d->kind);
  }
  if (d->k_total > p->n) return fail(SURGEON_EINVAL, "dw_from_packed: k_total exceeds the activation size");
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
  if (p->splits > 1) off += align_up((size_t)p->splits * (size_t)p->n_w * 4, 256);
  p->off_dense = off;
  if ((!p->conv && p->l.bf16_mfma) || (p->conv && p->c.gemm1x1)) off += align_up((size_t)p->n * 2, 256);  // transient dense activation
  p->ws_bytes = off;
  return SURGEON_OK;
}



template <typename InT, bool BF, int KHC, int KW, int MT, int NT, int P>
static int launch_conv_variant(const ConvPlan& cp, const Packed<InT>& pk, const void* dY, float* out, hipStream_t st) {
  auto kernel = dw_conv_kernel<InT, BF, KHC, KW, MT, NT, P>;
  // the dynamic-LDS limit is raised to the whole LDS once per kernel (this function is instantiated per kernel) and
  // device; what a launch occupies is its own lds_bytes
  static std::atomic<uint64_t> lds_set{0};
  if (cp.lds_bytes > 48 * 1024) {
    const int rc = ensure_dynamic_lds((const void*)kernel, kMaxLds, lds_set);
    if (rc != SURGEON_OK) return rc;
  }
  const dim3 grid((unsigned)(cp.co_tiles * cp.g.ci_tiles), (unsigned)cp.splits, (unsigned)cp.z);
  ProfScope prof(SURGEON_PROF_DW, st);
  SURGEON_LAUNCH(kernel, grid, dim3(512), cp.lds_bytes, st, cp.g, pk, (const InT*)dY, out);
  SURGEON_LAUNCH_CHECK();
  return SURGEON_OK;
}

template <typename InT, int KHC, int KW, int MT, int NT>
static int launch_conv_p(const ConvPlan& cp, const Packed<InT>& pk, const void* dY, float* out, hipStream_t st) {
  if constexpr (std::is_same<InT, uint16_t>::value) {
    if (cp.g.bf16_mfma) {
      if (cp.p == 32) return launch_conv_variant<InT, true, KHC, KW, MT, NT, 32>(cp, pk, dY, out, st);
      if (cp.p == 64) return launch_conv_variant<InT, true, KHC, KW, MT, NT, 64>(cp, pk, dY, out, st);
      return launch_conv_variant<InT, true, KHC, KW, MT, NT, 128>(cp, pk, dY, out, st);
    }
  }
  if (cp.p == 32) return launch_conv_variant<InT, false, KHC, KW, MT, NT, 32>(cp, pk, dY, out, st);
  if (cp.p == 64) return launch_conv_variant<InT, false, KHC, KW, MT, NT, 64>(cp, pk, dY, out, st);
  return launch_conv_variant<InT, false, KHC, KW, MT, NT, 128>(cp, pk, dY, out, st);
}

template <typename InT>
static int launch_conv(const ConvPlan& cp, const Packed<InT>& pk, const void* dY, float* out, hipStream_t st) {
  if (cp.khc == 3) {
    if (cp.mt == 5) return launch_conv_p<InT, 3, 3, 5, 1>(cp, pk, dY, out, st);
    if (cp.mt == 4) return launch_conv_p<InT, 3, 3, 4, 1>(cp, pk, dY, out, st);
    return launch_conv_p<InT, 3, 3, 2, 1>(cp, pk, dY, out, st);
  }
  if (cp.kw_t == 1) {
    if (cp.nt == 1) {
      if (cp.mt == 4) return launch_conv_p<InT, 1, 1, 4, 1>(cp, pk, dY, out, st);
      return launch_conv_p<InT, 1, 1, 2, 1>(cp, pk, dY, out, st);
    }
    if (cp.mt == 4) return launch_conv_p<InT, 1, 1, 4, 4>(cp, pk, dY, out, st);
    return launch_conv_p<InT, 1, 1, 2, 2>(cp, pk, dY, out, st);
  }
  if (cp.kw_t == 3) {
    if (cp.mt == 4) return launch_conv_p<InT, 1, 3, 4, 1>(cp, pk, dY, out, st);
    return launch_conv_p<InT, 1, 3, 2, 1>(cp, pk, dY, out, st);
  }
  if (cp.kw_t == 5) {
    if (cp.mt == 4) return launch_conv_p<InT, 1, 5, 4, 1>(cp, pk, dY, out, st);
    return launch_conv_p<InT, 1, 5, 2, 1>(cp, pk, dY, out, st);
  }
  if (cp.mt == 4) return launch_conv_p<InT, 1, 7, 4, 1>(cp, pk, dY, out, st);
  return launch_conv_p<InT, 1, 7, 2, 1>(cp, pk, dY, out, st);
}

template <typename InT>
static int launch_linear(const LinPlan& lp, const Packed<InT>& pk, const void* dY, float* out, hipStream_t st) {
  const dim3 grid((unsigned)(lp.o_tiles * lp.g.i_tiles), (unsigned)lp.splits);
  ProfScope prof(SURGEON_PROF_DW, st);
  if (lp.mt == 4)
    SURGEON_LAUNCH((dw_linear_kernel<InT, 4, 4, 32>), grid, dim3(256), 0, st, lp.g, pk, (const InT*)dY, out);
  else
    SURGEON_LAUNCH((dw_linear_kernel<InT, 2, 2, 32>), grid, dim3(256), 0, st, lp.g, pk, (const InT*)dY, out);
  SURGEON_LAUNCH_CHECK();
  return SURGEON_OK;
}

// G_out != nullptr: also Eq. 4 of the gradient just computed; sq_partial then holds kGiPartials doubles of scratch
template <typename InT>
int run_dw(const DwPlan& p, const surgeon_layer_desc* d, const void* vals, const uint64_t* mask, const void* dY,
                  float* dW, void* ws, hipStream_t st, float* G_out, double* sq_partial) {
  char* w = (char*)ws;
  uint32_t* word_rank = (uint32_t*)(w + p.off_rank);
  uint32_t* block_sum = (uint32_t*)(w + p.off_blocks);
  float* part = (float*)(w + p.off_part);

  // nothing kept (or no tokens): the gradient is exactly zero
  if (d->k_total == 0 || p.n == 0) {
    ProfScope prof(SURGEON_PROF_DW_AUX, st);
    const int blocks = (int)std::min<int64_t>(ceil_div(p.n_w, 256), 4096);
    SURGEON_LAUNCH(fill_zero_f32_kernel, dim3(blocks), dim3(256), 0, st, dW, p.n_w, G_out);
    SURGEON_LAUNCH_CHECK();
    return SURGEON_OK;
  }
  // the bf16 linear path un-packs whole groups when their positions are known in closed form: no rank table at all
  const bool dense_path = (!p.conv && p.l.bf16_mfma) || (p.conv && p.c.gemm1x1);
  const bool grouped_unpack = dense_path && p.rank_words_per_group > 0;
  const int aux_class = (p.conv && p.c.sparse) ? SURGEON_PROF_DW_SPARSE_AUX : SURGEON_PROF_DW_AUX;
  // rank table
  if (!grouped_unpack) {
  ProfScope prof(aux_class, st);
  if (p.rank_words_per_group > 0) {
    SURGEON_LAUNCH(rank_grouped_kernel, dim3((unsigned)ceil_div(p.rank_groups, kRankBlock / 64)), dim3(kRankBlock), 0, st,
                       mask, p.n_words, p.rank_words_per_group, p.rank_groups, (uint32_t)p.rank_k_full, word_rank);
    SURGEON_LAUNCH_CHECK();
  } else {
  const int rc_rank = launch_rank_table(mask, p.n_words, p.n_rank_blocks, block_sum, word_rank, st);
  if (rc_rank != SURGEON_OK) return rc_rank;
  }
  }

  Packed<InT> pk;
  pk.vals = (const InT*)vals;
  pk.mask = mask;
  pk.word_rank = word_rank;
  pk.k_last = d->k_total - 1;
  pk.n_words = p.n_words;
  float* out = p.splits > 1 ? part : dW;
  int rc;
  if (dense_path) {
    void* dense = w + p.off_dense;
    rc = grouped_unpack ? launch_unpack_grouped(vals, mask, p.n_words, p.rank_words_per_group, p.rank_groups, p.rank_k_full,
                                                p.n, d->k_total, dense, st)
                        : launch_unpack_dense(SURGEON_BF16, vals, mask, word_rank, p.n, d->k_total, dense, st);
    if (rc == SURGEON_OK) {
      if (p.conv)
        rc = launch_conv1x1_bf16(p.c.g.Nb, p.c.g.Ci, p.c.g.Co, p.c.g.H * p.c.g.W, dense, dY, out, p.c.splits,
                                 p.c.gemm_ktiles_per_split, st);
      else if (p.l.bf16_big)
        rc = launch_linear_bf16_big(p.l.g.M, p.l.g.K, p.l.g.N, dense, dY, out, p.l.splits, p.l.g.rows_per_split, st);
      else
        rc = launch_linear_bf16(p.l.g.M, p.l.g.K, p.l.g.N, dense, dY, out, p.l.splits, p.l.g.rows_per_split, p.l.bf16_wide, st);
    }
  } else if (p.conv && p.c.sparse) {
    rc = launch_conv3x3_sparse_f32(p.c.g.Nb, p.c.g.Ci, p.c.g.Co, p.c.g.H, p.c.g.W, d->k_total, p.c.splits,
                                   p.c.sparse_tiles_per_split, vals, mask, word_rank, dY, out, st);
  } else {
    rc = p.conv ? launch_conv<InT>(p.c, pk, dY, out, st) : launch_linear<InT>(p.l, pk, dY, out, st);
  }
  if (rc != SURGEON_OK) return rc;
  if (p.splits > 1) {
    // with Gradient Importance: at most 1024 workgroups, so that the finishing launch adds 4 partials per thread
    // 16-byte accesses pay once there are enough weights to fill the chip with a quarter of the threads
    const bool vec = p.n_w % 4 == 0 && p.n_w >= (1 << 19) && ((uintptr_t)dW % 16) == 0 && ((uintptr_t)part % 16) == 0;
    const int blocks = (int)std::min<int64_t>(ceil_div(vec ? p.n_w / 4 : p.n_w, 256), G_out ? 1024 : kGiPartials);
    ProfScope prof(aux_class, st);
    if (G_out) {
      if (vec)
        SURGEON_LAUNCH((dw_reduce_splits_kernel<true, true>), dim3(blocks), dim3(256), 0, st, (const float*)part, p.splits,
                       p.n_w, dW, sq_partial);
      else
        SURGEON_LAUNCH((dw_reduce_splits_kernel<true, false>), dim3(blocks), dim3(256), 0, st, (const float*)part, p.splits,
                       p.n_w, dW, sq_partial);
      SURGEON_LAUNCH_CHECK();
      return launch_sumsq_final(sq_partial, blocks, p.n_w, G_out, st);
    }
    if (vec)
      SURGEON_LAUNCH((dw_reduce_splits_kernel<false, true>), dim3(blocks), dim3(256), 0, st, (const float*)part, p.splits,
                     p.n_w, dW, (double*)nullptr);
    else
      SURGEON_LAUNCH((dw_reduce_splits_kernel<false, false>), dim3(blocks), dim3(256), 0, st, (const float*)part, p.splits,
                     p.n_w, dW, (double*)nullptr);
    SURGEON_LAUNCH_CHECK();
  } else if (G_out) {
    // the matrix-core kernel wrote dW itself: one read of it (small, mostly still in cache) for the sum of squares
    return launch_sumsq(dW, p.n_w, sq_partial, G_out, st);
  }
  return SURGEON_OK;
}

}  // namespace surgeon
