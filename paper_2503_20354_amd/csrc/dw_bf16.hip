// bf16 weight gradient of linear layers and of 1x1 stride-1 convolutions (Eq. 2, Alg. 1 lines 11-12) on the bf16
// matrix cores.
//
// At bf16 MFMA rates (16x the fp32 rate) un-packing inside the GEMM's tile loads would cost more vector-ALU time
// than the contraction itself, so this path does what Alg. 1 line 11 says literally: un-pack the cached activation
// to a dense, transient bf16 copy in the workspace (an HBM-bound kernel: reads k*2 + n/8 bytes, writes 2n), then
// run a dense contraction  dW[o][i] = sum_m dY[m][o] * A[m][i]  with v_mfma_f32_32x32x16_bf16, fp32 accumulation.
//
// Both operands have the contraction index m (tokens) as their slow index.  The MFMA wants, per lane, 8 consecutive
// contraction values of one row.  Tiles are staged into LDS exactly as they sit in memory ([token][feature]) and read
// back with ds_read_b64_tr_b16, gfx950's transposing LDS read: within a block of 16 lanes, lane i receives in element
// r the value source lane 4r + i/4 pointed at, element i%4.  Pointing source lane s at [token t0 + s/4][feature
// f0 + 4*(s%4)] therefore gives lane i the 4 consecutive tokens t0..t0+3 of feature f0 + i.
// (A 1x1 convolution in NCHW has the contraction index, the pixels, as the FAST index of both operands: no transpose.)
#include "common.hpp"

namespace surgeon {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------------------------------------
// Alg. 1 line 11: dense pruned activation from (vals, mask); 8 elements per thread
// ---------------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void unpack_dense_kernel(const T* __restrict__ vals, const uint64_t* __restrict__ mask,
                                                           const uint32_t* __restrict__ word_rank, int64_t n,
                                                           int64_t k_last, T* __restrict__ dense) {
  const int64_t n8 = (n + 7) >> 3;
  for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < n8; t += (int64_t)gridDim.x * 256) {
    const int64_t e0 = t << 3;
    const int sh = (int)(e0 & 63);
    const uint64_t word = mask[e0 >> 6];
    const uint32_t bits = (uint32_t)(word >> sh) & 0xffu;
    const int64_t rank = (int64_t)word_rank[e0 >> 6] + __popcll(word & ((1ull << sh) - 1ull));
    T v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      int64_t i = rank + __builtin_popcount(bits & ((1u << j) - 1u));
      i = i > k_last ? k_last : i;
      v[j] = vals[i];
    }
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (!((bits >> j) & 1u)) v[j] = (T)0;
    if (e0 + 8 <= n) {
#pragma unroll
      for (int j = 0; j < 8; ++j) dense[e0 + j] = v[j];  // contiguous: merged into 16-byte stores by the compiler
    } else {
      for (int j = 0; j < 8 && e0 + j < n; ++j) dense[e0 + j] = v[j];
    }
  }
}

// The same un-pack when every group of `words_per_group` mask words is known to hold exactly k_full kept elements (the
// packing's group length is a multiple of 64, at most 4096): one wavefront per group finds its words' positions with
// a popcount and a prefix sum over the lanes, so no rank table is needed.  The group's kept values are contiguous in
// `vals`: the wavefront copies them into its part of LDS with coalesced loads and expands from there (lane l builds 8
// consecutive elements, one 16-byte store), so the per-element gathers run on the LDS instead of as 64-address
// 2-byte loads through the texture path, with 32-bit positions and no clamps.  `lds_per_wave` >= k_full + 1 elements.
template <typename T>
__global__ __launch_bounds__(256) void unpack_grouped_kernel(const T* __restrict__ vals, const uint64_t* __restrict__ mask,
                                                             int64_t n_words, int words_per_group, int64_t n_groups,
                                                             uint32_t k_full, int64_t k_last, int64_t n, int lds_per_wave,
                                                             T* __restrict__ dense) {
  extern __shared__ __attribute__((aligned(16))) unsigned char unpack_lds[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t grp = (int64_t)blockIdx.x * 4 + wave;
  if (grp >= n_groups) return;
  T* lv = reinterpret_cast<T*>(unpack_lds) + (size_t)wave * lds_per_wave;
  const int64_t w0 = grp * words_per_group;
  const bool has_word = lane < words_per_group && w0 + lane < n_words;
  const uint64_t word = has_word ? mask[w0 + lane] : 0ull;
  const uint32_t c = (uint32_t)__popcll(word);
  uint32_t incl = c;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t up = (uint32_t)__shfl_up((int)incl, off, 64);
    if (lane >= off) incl += up;
  }
  const uint32_t rank = incl - c;  // position of the word's first kept value inside the group
  // the group's kept values -> LDS (a mask that disagrees with the hint cannot carry the copy past the group's part
  // of LDS or past the end of vals)
  const int64_t v0 = grp * (int64_t)k_full;
  const uint32_t v_left = (uint32_t)max(min(k_last + 1 - v0, (int64_t)k_full), (int64_t)0);  // values from v0 to the end
  const uint32_t k_here = min((uint32_t)__builtin_amdgcn_readlane((int)incl, 63), v_left);
  const T* __restrict__ gv = vals + v0;
  for (uint32_t i0 = 0; i0 < k_here; i0 += 256) {  // wave-uniform trip count; four loads in flight per lane
    uint32_t idx[4];
    T t[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      idx[q] = min(i0 + 64u * q + (uint32_t)lane, k_here - 1u);  // past the end: the last value again (same address)
      t[q] = gv[idx[q]];
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) lv[idx[q]] = t[q];
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  const int n_here = (int)min((int64_t)words_per_group, n_words - w0);
  const int sh = 8 * (lane & 7);
  // 8 words = 512 elements per step: lane l expands byte l % 8 of word l / 8
  for (int j0 = 0; j0 < n_here; j0 += 8) {
    const int src = j0 + (lane >> 3);
    const bool has = src < n_here;
    const uint32_t w_lo = (uint32_t)__shfl((int)(uint32_t)word, src & 63, 64);
    const uint32_t w_hi = (uint32_t)__shfl((int)(uint32_t)(word >> 32), src & 63, 64);
    const uint32_t r0 = (uint32_t)__shfl((int)rank, src & 63, 64);
    const uint64_t w = has ? (((uint64_t)w_hi << 32) | w_lo) : 0ull;
    const uint32_t bits = (uint32_t)(w >> sh) & 0xffu;
    const uint32_t first = min(r0 + (uint32_t)__popcll(w & ((1ull << sh) - 1ull)), k_here);
    T v[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      // at most k_here for a dropped element behind the last kept one: inside the wavefront's part of LDS
      const uint32_t pos = min(first + (uint32_t)__builtin_popcount(bits & ((1u << t) - 1u)), k_here);
      const T x = lv[pos];
      v[t] = ((bits >> t) & 1u) ? x : (T)0;
    }
    const int64_t e0 = (w0 + src) * 64 + sh;
    if (has && e0 + 8 <= n) {
#pragma unroll
      for (int t = 0; t < 8; ++t) dense[e0 + t] = v[t];  // contiguous: merged into one 16-byte store by the compiler
    } else if (has) {
      for (int t = 0; t < 8 && e0 + t < n; ++t) dense[e0 + t] = v[t];
    }
  }
}

// Variant for short groups (a few mask words, e.g. token rows of 64-256 features): the wavefront expands one word per
// step with all 64 lanes on its 64 elements, which keeps every lane busy where the 8-elements-per-lane form above
// would use only 8 lanes per word.
template <typename T>
__global__ __launch_bounds__(256) void unpack_grouped_short_kernel(const T* __restrict__ vals,
                                                                   const uint64_t* __restrict__ mask, int64_t n_words,
                                                                   int words_per_group, int64_t n_groups, uint32_t k_full,
                                                                   int64_t k_last, int64_t n, T* __restrict__ dense) {
  const int lane = threadIdx.x & 63;
  const int64_t grp = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (grp >= n_groups) return;
  const int64_t w0 = grp * words_per_group;
  const bool has_word = lane < words_per_group && w0 + lane < n_words;
  const uint64_t word = has_word ? mask[w0 + lane] : 0ull;
  const uint32_t c = (uint32_t)__popcll(word);
  uint32_t incl = c;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t up = (uint32_t)__shfl_up((int)incl, off, 64);
    if (lane >= off) incl += up;
  }
  const uint32_t rank = (uint32_t)grp * k_full + incl - c;
  const int n_here = (int)min((int64_t)words_per_group, n_words - w0);
  for (int j = 0; j < n_here; ++j) {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)word, j);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(word >> 32), j);
    const uint32_t r0 = (uint32_t)__builtin_amdgcn_readlane((int)rank, j);
    const bool kept = (lane < 32 ? (lo >> lane) : (hi >> (lane - 32))) & 1u;
    int64_t pos = (int64_t)__builtin_amdgcn_mbcnt_hi(hi, __builtin_amdgcn_mbcnt_lo(lo, r0));
    pos = pos > k_last ? k_last : pos;
    const T v = kept ? vals[pos] : (T)0;
    const int64_t e = (w0 + j) * 64 + lane;
    if (e < n) dense[e] = v;
  }
}

int launch_unpack_grouped(const void* vals, const uint64_t* mask, int64_t n_words, int words_per_group, int64_t n_groups,
                          int64_t k_full, int64_t n, int64_t k_total, void* dense, hipStream_t st) {
  if (n == 0) return SURGEON_OK;
  ProfScope prof(SURGEON_PROF_DW_AUX, st);
  if (words_per_group <= 4 && 64 % words_per_group == 0) {
    // groups of one, two or four mask words: 64 words' worth of consecutive groups are one wavefront's unit.  Every
    // group but the tensor's last holds exactly k_full values, so the unit is a group of 64 words with that many times
    // k_full values as far as the kernel is concerned (a sixteenth to a quarter of the wavefronts, 16-byte stores).
    const int per = 64 / words_per_group;
    const int64_t k_unit = k_full * per;
    const int lds_per_wave = (int)align_up((size_t)k_unit + 1, 8);
    SURGEON_LAUNCH(unpack_grouped_kernel<uint16_t>, dim3((unsigned)ceil_div(ceil_div(n_groups, per), 4)), dim3(256),
                   (size_t)4 * lds_per_wave * sizeof(uint16_t), st, (const uint16_t*)vals, mask, n_words, 64,
                   ceil_div(n_groups, per), (uint32_t)k_unit, k_total - 1, n, lds_per_wave, (uint16_t*)dense);
  } else if (words_per_group <= 4)
    SURGEON_LAUNCH(unpack_grouped_short_kernel<uint16_t>, dim3((unsigned)ceil_div(n_groups, 4)), dim3(256), 0, st,
                   (const uint16_t*)vals, mask, n_words, words_per_group, n_groups, (uint32_t)k_full, k_total - 1, n,
                   (uint16_t*)dense);
  else {
    // LDS: each of the four wavefronts holds its group's kept values (and one element of slack)
    const int lds_per_wave = (int)align_up((size_t)k_full + 1, 8);
    SURGEON_LAUNCH(unpack_grouped_kernel<uint16_t>, dim3((unsigned)ceil_div(n_groups, 4)), dim3(256),
                   (size_t)4 * lds_per_wave * sizeof(uint16_t), st, (const uint16_t*)vals, mask, n_words, words_per_group,
                   n_groups, (uint32_t)k_full, k_total - 1, n, lds_per_wave, (uint16_t*)dense);
  }
  SURGEON_LAUNCH_CHECK();
  return SURGEON_OK;
}

int launch_unpack_dense(int dtype, const void* vals, const uint64_t* mask, const uint32_t* word_rank, int64_t n,
                        int64_t k_total, void* dense, hipStream_t st) {
  if (n == 0) return SURGEON_OK;
  const int blocks = (int)std::min<int64_t>(ceil_div(ceil_div(n, 8), 256), 65536);
  ProfScope prof(SURGEON_PROF_DW_AUX, st);
  if (dtype == SURGEON_F32)
    SURGEON_LAUNCH(unpack_dense_kernel<uint32_t>, dim3(blocks), dim3(256), 0, st, (const uint32_t*)vals, mask, word_rank,
                       n, k_total - 1, (uint32_t*)dense);
  else
    SURGEON_LAUNCH(unpack_dense_kernel<uint16_t>, dim3(blocks), dim3(256), 0, st, (const uint16_t*)vals, mask, word_rank,
                       n, k_total - 1, (uint16_t*)dense);
  SURGEON_LAUNCH_CHECK();
  return SURGEON_OK;
}

// ---------------------------------------------------------------------------------------------------------
// dense TN contraction on bf16 MFMA
// ---------------------------------------------------------------------------------------------------------
// Workgroup = 4 wavefronts as 2 (out) x 2 (in); a wavefront owns PO x PI MFMA 32x32 tiles, so the workgroup tile is
// 64*PO out-features x 64*PI in-features; TOK tokens per K-tile.  Two shapes are built: 128 x 128 with 64 tokens, and
// 128 x 256 with 32 tokens, which issues 8 matrix instructions per 12 transposing LDS reads instead of 4 per 8 (the LDS
// port is the limit of this kernel) and needs a quarter less L2 traffic per flop.
constexpr int kBfPad = 16;  // LDS row padding in elements: 4 consecutive rows hit distinct banks

// one 16-byte chunk (8 bf16) of row `row`, columns col0..col0+7, zero outside the matrix.  ALIGN = 8: the row pitch
// is a multiple of 8 elements (and the base 16-byte aligned), so a chunk is inside or outside as a whole and is one
// 16-byte load; ALIGN = 4: the same with halves of a chunk and two 8-byte loads; ALIGN = 1: the chunk is gathered from
// eight 2-byte loads, each with its own column check.
template <int ALIGN>
__device__ __forceinline__ u32x4 load_chunk(const uint16_t* __restrict__ src, int64_t row, int64_t row_end, int64_t col0,
                                            int64_t n_cols, int64_t ld) {
  if constexpr (ALIGN == 8) {
    const bool ok = row < row_end && col0 < n_cols;
    const int64_t off = ok ? row * ld + col0 : 0;
    u32x4 v = *reinterpret_cast<const u32x4*>(src + off);
    if (!ok) v = u32x4{0, 0, 0, 0};
    return v;
  } else if constexpr (ALIGN == 4) {
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    const bool ok0 = row < row_end && col0 < n_cols, ok1 = row < row_end && col0 + 4 < n_cols;
    const u32x2 lo = *reinterpret_cast<const u32x2*>(src + (ok0 ? row * ld + col0 : 0));
    const u32x2 hi = *reinterpret_cast<const u32x2*>(src + (ok1 ? row * ld + col0 + 4 : 0));
    return u32x4{ok0 ? lo[0] : 0u, ok0 ? lo[1] : 0u, ok1 ? hi[0] : 0u, ok1 ? hi[1] : 0u};
  } else {
    u32x4 v = {0, 0, 0, 0};
    if (row < row_end && col0 < n_cols) {
      const uint16_t* __restrict__ p = src + row * ld + col0;
      const int left = (int)min((int64_t)8, n_cols - col0);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint32_t e0 = 2 * q < left ? (uint32_t)p[2 * q] : 0u;
        const uint32_t e1 = 2 * q + 1 < left ? (uint32_t)p[2 * q + 1] : 0u;
        v[q] = e0 | (e1 << 16);
      }
    }
    return v;
  }
}

// 8 consecutive tokens (t0..t0+7) of feature (f0 + lane%16) as one MFMA operand register set
template <int STRIDE>
__device__ __forceinline__ bf16x8 read_operand(const uint16_t* tile, int t0, int f0, int lane) {
  const int s = lane & 15;
  const uint16_t* p = tile + (t0 + (s >> 2)) * STRIDE + f0 + 4 * (s & 3);
  typedef shortx4 __attribute__((address_space(3))) * lds_ptr;
  const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)p);
  const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 4 * STRIDE));
  typedef short shortx8 __attribute__((ext_vector_type(8)));
  const shortx8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, both);
}

// How a result leaves the kernel.  kOutSplitsF32: fp32, out[split][o][i] (the weight gradient's partial sums).  The other
// two serve the activation gradient of 1x1 convolutions, where a batch entry is an image, o an input channel and i an
// output pixel: kOutBf16 stores bf16 at out[o][i]; kOutBf16Stride2 stores pixel i = (oh, ow) at (2 oh, 2 ow) of a map
// out_w wide and out_h high and zeros at the three other pixels of its 2 x 2 block (what a stride-2 layer's input
// gradient holds there).
enum { kOutSplitsF32 = 0, kOutBf16 = 1, kOutBf16Stride2 = 2 };
struct BatchedOperands {
  int64_t a_batch = 0, y_batch = 0, out_batch = 0;  // element strides of blockIdx.z
  int out_w = 0, out_h = 0, in_w = 0;               // kOutBf16Stride2: dA's map, and the width of dY's map
};

__device__ __forceinline__ uint32_t bf16_bits_rne(float f) {  // round to nearest even; NaN stays NaN
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x0040u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

// blockIdx.x = o_tile * i_tiles + i_tile, blockIdx.y = split along the tokens, blockIdx.z = batch entry.
// YROWS: the dY operand is given with the contraction index fast -- dY[o][t], row pitch M -- as the activation
// gradient of a linear layer has it (its "tokens" are the layer's out-features): the tile is then staged [o][t] and an
// operand register set is a plain 16-byte LDS read, as in the 1x1 convolution kernel below; rows 144 bytes apart, so
// eight rows cover all banks.  Needs M % 8 == 0 and 16-byte aligned rows (YALIGNED).
template <int PO, int PI, int TOK, bool YALIGNED, int AALIGN = 8, int OUT = kOutSplitsF32, bool YROWS = false>
__global__ __launch_bounds__(256) void dw_linear_bf16_kernel(int64_t M, int64_t K, int64_t N, int i_tiles,
                                                             int64_t rows_per_split, const uint16_t* __restrict__ A,
                                                             const uint16_t* __restrict__ dY, float* __restrict__ out,
                                                             BatchedOperands bo) {
  A += (int64_t)blockIdx.z * bo.a_batch;
  dY += (int64_t)blockIdx.z * bo.y_batch;
  constexpr int TO = 64 * PO, TI = 64 * PI, SO = TO + kBfPad, SI = TI + kBfPad;
  constexpr int ST = TOK + 8;  // YROWS: row pitch of the [o][t] tile
  constexpr int CY = TOK * TO / 8 / 256, CA = TOK * TI / 8 / 256;  // 16-byte chunks per thread and K-tile
  static_assert(TOK * TO / 8 % 256 == 0 && TOK * TI / 8 % 256 == 0 && TOK % 16 == 0, "tile shape");
  static_assert(!YROWS || YALIGNED, "row-major dY tiles are loaded 16 bytes at a time");
  __shared__ __attribute__((aligned(16))) uint16_t Ys[2][YROWS ? TO * ST : TOK * SO];
  __shared__ __attribute__((aligned(16))) uint16_t As[2][TOK * SI];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int64_t o0 = (int64_t)(blockIdx.x / i_tiles) * TO, i0 = (int64_t)(blockIdx.x % i_tiles) * TI;
  const int64_t m_begin = (int64_t)blockIdx.y * rows_per_split;
  const int64_t m_end = min(m_begin + rows_per_split, M);

  floatx16 acc[PO][PI];
#pragma unroll
  for (int a = 0; a < PO; ++a)
#pragma unroll
    for (int b = 0; b < PI; ++b)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[a][b][q] = 0.0f;

  // staging: thread t moves chunks t, t+256, ... of each operand tile (TOK rows x T/8 chunks of 8 elements)
  u32x4 ry[CY], ra[CA];
  auto load_tile = [&](int64_t m0) {
#pragma unroll
    for (int j = 0; j < CY; ++j) {
      if constexpr (YROWS) {
        const int c = tid + 256 * j, row = c / (TOK / 8), col = (c % (TOK / 8)) * 8;  // row: out-feature, col: token
        ry[j] = load_chunk<8>(dY, o0 + row, N, m0 + col, m_end, M);
      } else {
        const int c = tid + 256 * j, row = c / (TO / 8), col = (c % (TO / 8)) * 8;
        ry[j] = load_chunk<(YALIGNED ? 8 : 1)>(dY, m0 + row, m_end, o0 + col, N, N);
      }
    }
#pragma unroll
    for (int j = 0; j < CA; ++j) {
      const int c = tid + 256 * j, row = c / (TI / 8), col = (c % (TI / 8)) * 8;
      ra[j] = load_chunk<AALIGN>(A, m0 + row, m_end, i0 + col, K, K);
    }
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int j = 0; j < CY; ++j) {
      if constexpr (YROWS) {
        const int c = tid + 256 * j, row = c / (TOK / 8), col = (c % (TOK / 8)) * 8;
        *reinterpret_cast<u32x4*>(&Ys[buf][row * ST + col]) = ry[j];
      } else {
        const int c = tid + 256 * j, row = c / (TO / 8), col = (c % (TO / 8)) * 8;
        *reinterpret_cast<u32x4*>(&Ys[buf][row * SO + col]) = ry[j];
      }
    }
#pragma unroll
    for (int j = 0; j < CA; ++j) {
      const int c = tid + 256 * j, row = c / (TI / 8), col = (c % (TI / 8)) * 8;
      *reinterpret_cast<u32x4*>(&As[buf][row * SI + col]) = ra[j];
    }
  };

  if (m_begin < m_end) {
    load_tile(m_begin);
    store_tile(0);
  }
  __syncthreads();
  int buf = 0;
  for (int64_t m0 = m_begin; m0 < m_end; m0 += TOK) {
    const bool more = m0 + TOK < m_end;
    if (more) load_tile(m0 + TOK);  // in flight while the matrix cores work on the current tile
    const uint16_t* ys = Ys[buf];
    const uint16_t* as = As[buf];
    const int blk = lane >> 4;  // 16-lane block: rows 16*(blk&1).., contraction half blk>>1
#pragma unroll
    for (int ks = 0; ks < TOK; ks += 16) {
      const int t0 = ks + 8 * (blk >> 1);
      bf16x8 a[PO], b[PI];
#pragma unroll
      for (int q = 0; q < PO; ++q) {
        if constexpr (YROWS)  // row = out-feature lane % 32 of the block, eight tokens from t0 on
          a[q] = *reinterpret_cast<const bf16x8*>(&ys[(wm * 32 * PO + q * 32 + (lane & 31)) * ST + t0]);
        else
          a[q] = read_operand<SO>(ys, t0, wm * 32 * PO + q * 32 + 16 * (blk & 1), lane);
      }
#pragma unroll
      for (int q = 0; q < PI; ++q) b[q] = read_operand<SI>(as, t0, wn * 32 * PI + q * 32 + 16 * (blk & 1), lane);
#pragma unroll
      for (int p = 0; p < PO; ++p)
#pragma unroll
        for (int q = 0; q < PI; ++q) acc[p][q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[p], b[q], acc[p][q], 0, 0, 0);
    }
    if (more) store_tile(buf ^ 1);
    __syncthreads();
    buf ^= 1;
  }

  // 32x32 result tile: lane holds column lane%32 and rows 8*(v/4) + 4*(lane/32) + v%4, v = 0..15
  const int col = lane & 31, half = lane >> 5;
#pragma unroll
  for (int p = 0; p < PO; ++p)
#pragma unroll
    for (int q = 0; q < PI; ++q) {
      const int64_t i = i0 + wn * 32 * PI + q * 32 + col;
      int64_t at = i;  // where column i goes inside a row of the result
      int map = 0;     // kOutBf16Stride2: bit 0 = the pixel right of (2 oh, 2 ow) exists, bit 1 = the row below exists
      if constexpr (OUT == kOutBf16Stride2) {
        const int oh = (int)(i / bo.in_w), ow = (int)(i - (int64_t)oh * bo.in_w);
        at = (int64_t)2 * oh * bo.out_w + 2 * ow;
        map = (2 * ow + 1 < bo.out_w ? 1 : 0) | (2 * oh + 1 < bo.out_h ? 2 : 0);
      }
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int64_t o = o0 + wm * 32 * PO + p * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
        if (o < N && i < K) {
          if constexpr (OUT == kOutSplitsF32) {
            out[(int64_t)blockIdx.y * N * K + o * K + i] = acc[p][q][v];
          } else if constexpr (OUT == kOutBf16) {
            uint16_t* __restrict__ img = reinterpret_cast<uint16_t*>(out) + (int64_t)blockIdx.z * bo.out_batch;
            img[o * K + i] = (uint16_t)bf16_bits_rne(acc[p][q][v]);
          } else {
            uint16_t* __restrict__ px = reinterpret_cast<uint16_t*>(out) + (int64_t)blockIdx.z * bo.out_batch +
                                        o * ((int64_t)bo.out_w * bo.out_h) + at;
            px[0] = (uint16_t)bf16_bits_rne(acc[p][q][v]);
            if (map & 1) px[1] = 0;
            if (map & 2) {
              px[bo.out_w] = 0;
              if (map & 1) px[bo.out_w + 1] = 0;
            }
          }
        }
      }
    }
}

// ---------------------------------------------------------------------------------------------------------
// The same contraction for layers that fill a 256 x 128 tile: eight wavefronts (two per SIMD) as 4 (out) x 2 (in), each
// owning 2 x 2 matrix tiles of 32 x 32; 64 tokens per K-tile; one workgroup per compute unit.
//
// K-tiles go from memory straight into LDS (buffer loads with the `lds` bit: lane l of a wavefront delivers its 16
// bytes at M0 + 16 l), so no registers and no LDS store instructions are spent on staging, and three unpadded K-tile
// buffers of 48 KB fit: two K-tiles are in flight behind the one being multiplied.  A load instruction covers 1024
// contiguous LDS bytes (two token rows of the dY tile, four of the input tile), so rows cannot be padded against bank
// conflicts; instead the four 64-byte segments that the transposing reads of four consecutive tokens touch are spread
// over the banks by storing segment s of token t at position s ^ (t & 3) (the lanes of a load fetch the permuted
// source chunk; the reads apply the same permutation).
// The loads are inline asm (the compiler would otherwise wait for every outstanding LDS-direct load before any LDS
// read): this kernel counts its own vmcnt.  Nothing else in the loop uses vmcnt.
//
// What was measured on the chip and shapes this kernel (ViT-B/16 layers, 12 608 tokens):
//   * two wavefronts per SIMD drive the matrix pipeline at 2.4 PFLOP/s (one reaches 1.95), and one operand read of
//     16 bytes per lane and matrix instruction still leaves 2.0 as long as a read is requested one K-step before it
//     is used: the LDS port is not the bound, so the operands of K-step s+1 are read before the matrix work of step s;
//   * a K-tile's trip from memory takes about as long as four K-tiles of matrix work.  The first version staged
//     K-tiles through two register sets (global -> registers -> LDS stores, rows padded by 32 elements) and ran at
//     590-700 TFLOP/s; the LDS-direct loads, which free the registers and remove the store phase, reach 870-890;
//   * whole splits per XCD (xcd_ordered_work_item): 627 -> 697 TFLOP/s on the register-staged version, L2 misses per
//     launch halved (373 -> 167 MB);
//   * more K-tiles in flight do not help further: 32-token K-tiles in six buffers (five in flight) run at the speed of
//     64-token K-tiles in three; one extra load per wavefront that touches the lines of a K-tile several tiles ahead
//     (an L2 prefetch) is slower (loads return in order, so the LDS-direct loads queue behind it);
//   * a 256 x 256 tile (32 tokens, four buffers; a third fewer operand bytes per flop) reaches 965 TFLOP/s as a
//     kernel, but a split contraction writes and re-reads partial tiles whose total size is the accumulator capacity in
//     use on the chip, twice as much with this tile: the layer as a whole is no faster, so it is not built in.
// ---------------------------------------------------------------------------------------------------------
constexpr int kBigTO = 256;

template <int TI>
struct BigShape {
  static constexpr int TOK = kBf16BigTokens;                 // tokens per K-tile
  static constexpr int NBUF = (144 * 1024) / (TOK * (kBigTO + TI) * 2) > 6 ? 6 : (144 * 1024) / (TOK * (kBigTO + TI) * 2);  // K-tile buffers in LDS
  static constexpr int YROW = kBigTO * 2, AROW = TI * 2;     // row bytes
  static constexpr int YBYTES = TOK * YROW, ABYTES = TOK * AROW;
  static constexpr int BUF = YBYTES + ABYTES;                // 48 KB / 32 KB
  static constexpr int YI = YBYTES / 1024 / 8, AI = ABYTES / 1024 / 8;  // load instructions per wavefront and K-tile
  static constexpr int LOADS = YI + AI;
  static constexpr size_t LDS = (size_t)NBUF * BUF;          // 144 KB / 128 KB
};

__device__ __forceinline__ void lds_direct_load16(uint32_t lds_byte, uint32_t voff, u32x4 rsrc) {
  // One wait state between the scalar write of M0 and the LDS-direct load that reads it.  M0 is a register the compiler
  // reserves and writes itself right before the few instructions that read it; the kernel below contains none of those,
  // so nothing else depends on its value.
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
               :: "s"(lds_byte), "v"(voff), "s"(rsrc) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt");
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// BF16OUT: one split, and the result goes out as bf16 at out[o][i] (the activation gradient's use of this kernel)
template <int TI, bool BF16OUT = false>
__global__ __launch_bounds__(512) void dw_linear_bf16_big_kernel(int64_t M, int64_t K, int64_t N, int i_tiles,
                                                                 int64_t rows_per_split, const uint16_t* __restrict__ A,
                                                                 const uint16_t* __restrict__ dY, float* __restrict__ out) {
  using S = BigShape<TI>;
  constexpr int NB = TI / 64, TOK = S::TOK, NBUF = S::NBUF, YROW = S::YROW, AROW = S::AROW, YBYTES = S::YBYTES;
  constexpr int ACH = AROW / 16;  // 16-byte chunks per input row
  extern __shared__ __attribute__((aligned(16))) uint16_t big_lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wo = wave & 3, wi = wave >> 2;
  int tile_id, split_id;  // the tiles of a split share its token rows: whole splits per XCD
  xcd_ordered_work_item(&tile_id, &split_id);
  const int64_t o0 = (int64_t)(tile_id / i_tiles) * kBigTO, i0 = (int64_t)(tile_id % i_tiles) * TI;
  const int64_t m_begin = (int64_t)split_id * rows_per_split;
  const int64_t m_end = min(m_begin + rows_per_split, M);

  floatx16 acc[2][NB];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[a][b][q] = 0.0f;

  // Resources end at the split's last row.  The whole byte offset travels in the vector offset, which the hardware
  // checks against that size: rows past the split's end (the last K-tile, and the loads issued past it) read zeros.
  const uint64_t p_dy = (uint64_t)dY, p_a = (uint64_t)A;
  const u32x4 r_dy = {(uint32_t)p_dy, (uint32_t)(p_dy >> 32) & 0xffffu, (uint32_t)(m_end * N * 2), 0x00020000u};
  const u32x4 r_a = {(uint32_t)p_a, (uint32_t)(p_a >> 32) & 0xffffu, (uint32_t)(m_end * K * 2), 0x00020000u};
  // this wavefront's loads of a K-tile: dY instructions YI wave .. (two tokens each), input instructions AI wave ..
  // (1024 / AROW tokens each); per lane the source byte offset inside the K-tile's rows, 0x80000000 = no access
  uint32_t vy[S::YI], va[S::AI];
#pragma unroll
  for (int j = 0; j < S::YI; ++j) {
    const int tok = 2 * (S::YI * wave + j) + (lane >> 5), c = lane & 31;
    const int lc = (((c >> 2) ^ (tok & 3)) << 2) | (c & 3);  // source chunk that belongs at chunk position c of this token
    vy[j] = o0 + lc * 8 < N ? (uint32_t)((tok * N + o0 + lc * 8) * 2) : 0x80000000u;
  }
#pragma unroll
  for (int j = 0; j < S::AI; ++j) {
    const int tok = (64 / ACH) * (S::AI * wave + j) + lane / ACH, c = lane % ACH;
    const int lc = (((c >> 2) ^ (tok & 3)) << 2) | (c & 3);
    va[j] = i0 + lc * 8 < K ? (uint32_t)((tok * K + i0 + lc * 8) * 2) : 0x80000000u;
  }
  auto load_tile = [&](int buf, int64_t m0) {
    // past 2 GiB the sum wraps into "no access" or stays above every resource size: the operands are below 2 GiB
    const uint32_t sy = (uint32_t)min(m0 * N * 2, (int64_t)0x7fffffff), sa = (uint32_t)min(m0 * K * 2, (int64_t)0x7fffffff);
    const uint32_t base = (uint32_t)(buf * S::BUF);
#pragma unroll
    for (int j = 0; j < S::YI; ++j) lds_direct_load16(base + (uint32_t)((S::YI * wave + j) * 1024), vy[j] >= 0x80000000u ? vy[j] : vy[j] + sy, r_dy);
#pragma unroll
    for (int j = 0; j < S::AI; ++j) lds_direct_load16(base + (uint32_t)(YBYTES + (S::AI * wave + j) * 1024), va[j] >= 0x80000000u ? va[j] : va[j] + sa, r_a);
  };

  // LDS byte offsets of a lane's transposing reads inside a K-tile buffer, per matrix tile q of the wavefront
  typedef shortx4 __attribute__((address_space(3))) * lds_ptr;
  const int blk = lane >> 4, s16 = lane & 15;
  const int lane_tok = 8 * (blk >> 1) + (s16 >> 2), lane_col = 16 * (blk & 1) + 4 * (s16 & 3);
  const int tl = lane_tok & 3;  // (token & 3) of every read of this lane: K-steps and the +4 rows keep it
  uint32_t yoff[2], aoff[NB];
#pragma unroll
  for (int q = 0; q < 2; ++q) yoff[q] = (uint32_t)(lane_tok * YROW + (((wo * 2 + q) ^ tl) << 6) + lane_col * 2);
#pragma unroll
  for (int q = 0; q < NB; ++q) aoff[q] = (uint32_t)(YBYTES + lane_tok * AROW + (((wi * NB + q) ^ tl) << 6) + lane_col * 2);
  char __attribute__((address_space(3))) * const lds_base = (char __attribute__((address_space(3))) *)big_lds;

  auto mfma_tile = [&](int buf) {
    bf16x8 a[2][2], b[2][NB];
    auto read8 = [&](uint32_t byte_off, int row_bytes) {
      const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(lds_base + byte_off));
      const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(lds_base + byte_off + 4 * row_bytes));
      typedef short shortx8 __attribute__((ext_vector_type(8)));
      const shortx8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      return __builtin_bit_cast(bf16x8, both);
    };
    auto read_step = [&](int set, int ks) {
#pragma unroll
      for (int q = 0; q < 2; ++q) a[set][q] = read8(yoff[q] + (uint32_t)(buf * S::BUF + ks * YROW), YROW);
#pragma unroll
      for (int q = 0; q < NB; ++q) b[set][q] = read8(aoff[q] + (uint32_t)(buf * S::BUF + ks * AROW), AROW);
    };
    read_step(0, 0);
#pragma unroll
    for (int s = 0; s < TOK / 16; ++s) {
      if (s + 1 < TOK / 16) read_step((s + 1) & 1, 16 * (s + 1));
#pragma unroll
      for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int q = 0; q < NB; ++q)
          acc[p][q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[s & 1][p], b[s & 1][q], acc[p][q], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  const int64_t n_kt = m_begin < m_end ? (m_end - m_begin + TOK - 1) / TOK : 0;
  // Every step issues the same number of loads (tiles past the split's end read zeros into a buffer nobody reads
  // again), so one constant tells when a tile has landed: loads return in order, and the LOADS of the tile wanted next
  // are followed by the (NBUF - 2) * LOADS of the younger tiles.
  if (n_kt > 0) {
#pragma unroll
    for (int u = 0; u < NBUF - 1; ++u) load_tile(u, m_begin + (int64_t)u * TOK);
    wait_vmcnt<(NBUF - 2) * S::LOADS>();  // tile 0
  }
  __syncthreads();
  // tile t sits in buffer t % NBUF; tiles t + 1 .. t + NBUF - 1 are on their way into the others
  for (int64_t t = 0; t < n_kt; t += NBUF) {
#pragma unroll
    for (int u = 0; u < NBUF; ++u) {
      if (t + u >= n_kt) break;
      // buffer (u + NBUF - 1) % NBUF was last read for tile t + u - 1, and every wavefront has passed the barrier since
      load_tile((u + NBUF - 1) % NBUF, m_begin + (t + u + NBUF - 1) * TOK);
      mfma_tile(u);
      wait_vmcnt<(NBUF - 2) * S::LOADS>();  // tile t + u + 1 has landed
      __syncthreads();
    }
  }
  wait_vmcnt<0>();  // the loads past the end have written their zeros before the LDS is given up

  float* __restrict__ dst = out + (int64_t)split_id * N * K;
  const int col = lane & 31, half = lane >> 5;
#pragma unroll
  for (int p = 0; p < 2; ++p)
#pragma unroll
    for (int q = 0; q < NB; ++q) {
      const int64_t i = i0 + wi * (TI / 2) + q * 32 + col;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int64_t o = o0 + wo * 64 + p * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
        if (o < N && i < K) {
          if constexpr (BF16OUT)
            reinterpret_cast<uint16_t*>(out)[o * K + i] = (uint16_t)bf16_bits_rne(acc[p][q][v]);
          else
            dst[o * K + i] = acc[p][q][v];
        }
      }
    }
}

int launch_linear_bf16_big(int64_t M, int64_t K, int64_t N, const void* A_dense, const void* dY, float* out, int splits,
                           int64_t rows_per_split, hipStream_t st, bool bf16_out) {
  constexpr int TI = kBf16BigTileI;
  static_assert(BigShape<TI>::TOK == kBf16BigTokens, "the planner sizes splits in K-tiles of this many tokens");
  const int i_tiles = (int)ceil_div(K, TI), o_tiles = (int)ceil_div(N, kBigTO);
  const dim3 grid((unsigned)(o_tiles * i_tiles), (unsigned)splits);
  ProfScope prof(SURGEON_PROF_DW, st);
  if (bf16_out) {
    if (splits != 1) return fail(SURGEON_EINVAL, "bf16 contraction: a bf16 result needs a single split");
    static std::atomic<uint64_t> lds_set_bf16{0};
    const int rc_lds = ensure_dynamic_lds((const void*)dw_linear_bf16_big_kernel<TI, true>, BigShape<TI>::LDS, lds_set_bf16);
    if (rc_lds != SURGEON_OK) return rc_lds;
    SURGEON_LAUNCH((dw_linear_bf16_big_kernel<TI, true>), grid, dim3(512), BigShape<TI>::LDS, st, M, K, N, i_tiles,
                   rows_per_split, (const uint16_t*)A_dense, (const uint16_t*)dY, out);
    SURGEON_LAUNCH_CHECK();
    return SURGEON_OK;
  }
  static std::atomic<uint64_t> lds_set{0};
  const int rc_lds = ensure_dynamic_lds((const void*)dw_linear_bf16_big_kernel<TI>, BigShape<TI>::LDS, lds_set);
  if (rc_lds != SURGEON_OK) return rc_lds;
  SURGEON_LAUNCH(dw_linear_bf16_big_kernel<TI>, grid, dim3(512), BigShape<TI>::LDS, st, M, K, N, i_tiles, rows_per_split,
                 (const uint16_t*)A_dense, (const uint16_t*)dY, out);
  SURGEON_LAUNCH_CHECK();
  return SURGEON_OK;
}

// ---------------------------------------------------------------------------------------------------------
// 1x1 stride-1 convolution in NCHW = per image a contraction over the pixels, which are the contiguous index of
// both operands: dW[co][ci] = sum_b sum_p dY[b][co][p] * A[b][ci][p].  Tiles are staged [channel][pixel] and read
// back with plain 16-byte LDS reads (8 consecutive pixels of one channel are exactly one MFMA operand register set).
// Same shape as the linear kernel: 128 x 128 tile, 4 wavefronts, 64 pixels per K-tile; a K-tile never spans images.
// ---------------------------------------------------------------------------------------------------------
constexpr int kPxTile = 128, kPxTok = 64, kPxStride = kPxTok + 8;  // row stride 144 bytes: 8 rows cover all banks
constexpr size_t kPxLdsBytes = (size_t)2 * 2 * kPxTile * kPxStride * sizeof(uint16_t);

// CE = elements per staged chunk: 8 (16 bytes; HW a multiple of 8) or 4 (8 bytes; HW a multiple of 4, e.g. 14 x 14 maps)
template <int CE>
__global__ __launch_bounds__(256) void dw_conv1x1_bf16_kernel(int Nb, int Ci, int Co, int HW, int i_tiles, int tiles_per_img,
                                                              int64_t ktiles_per_split, const uint16_t* __restrict__ A,
                                                              const uint16_t* __restrict__ dY, float* __restrict__ out) {
  extern __shared__ __attribute__((aligned(16))) uint16_t px_lds[];
  constexpr int TILE_ELEMS = kPxTile * kPxStride;
  constexpr int CPR = kPxTok / CE;                // chunks per tile row
  constexpr int CH = kPxTile * CPR / 256;         // chunks per thread, operand and K-tile
  typedef uint32_t chunk_t __attribute__((ext_vector_type(CE / 2)));
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  int tile_id, split_id;  // the tiles of a split share its pixels: whole splits per XCD
  xcd_ordered_work_item(&tile_id, &split_id);
  const int o0 = (tile_id / i_tiles) * kPxTile, i0 = (tile_id % i_tiles) * kPxTile;
  const int64_t n_ktiles = (int64_t)Nb * tiles_per_img;
  const int64_t t_begin = (int64_t)split_id * ktiles_per_split;
  const int64_t t_end = min(t_begin + ktiles_per_split, n_ktiles);

  floatx16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[a][b][q] = 0.0f;

  // one chunk = CE consecutive pixels of one channel; zero past the channel count or the image
  auto chunk = [&](const uint16_t* __restrict__ src, int C, int c0, int64_t t, int c) {
    const int b = (int)(t / tiles_per_img), p0 = (int)(t - (int64_t)b * tiles_per_img) * kPxTok;
    const int row = c / CPR, px = p0 + (c % CPR) * CE;
    const bool ok = c0 + row < C && px < HW;  // HW is a multiple of CE
    const int64_t off = ok ? ((int64_t)b * C + c0 + row) * HW + px : 0;
    chunk_t v = *reinterpret_cast<const chunk_t*>(src + off);
    if (!ok) v = chunk_t(0);
    return v;
  };
  chunk_t ry[CH], ra[CH];
  auto load_tile = [&](int64_t t) {
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      ry[j] = chunk(dY, Co, o0, t, tid + 256 * j);
      ra[j] = chunk(A, Ci, i0, t, tid + 256 * j);
    }
  };
  auto store_tile = [&](int buf) {
    uint16_t* ys = px_lds + (2 * buf) * TILE_ELEMS;
    uint16_t* as = ys + TILE_ELEMS;
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      const int c = tid + 256 * j, row = c / CPR, col = (c % CPR) * CE;
      *reinterpret_cast<chunk_t*>(&ys[row * kPxStride + col]) = ry[j];
      *reinterpret_cast<chunk_t*>(&as[row * kPxStride + col]) = ra[j];
    }
  };

  if (t_begin < t_end) {
    load_tile(t_begin);
    store_tile(0);
  }
  __syncthreads();
  int buf = 0;
  const int row32 = lane & 31, khalf = 8 * (lane >> 5);
  for (int64_t t = t_begin; t < t_end; ++t) {
    const bool more = t + 1 < t_end;
    if (more) load_tile(t + 1);
    const uint16_t* ys = px_lds + (2 * buf) * TILE_ELEMS;
    const uint16_t* as = ys + TILE_ELEMS;
#pragma unroll
    for (int ks = 0; ks < kPxTok; ks += 16) {
      bf16x8 a[2], b[2];
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        a[q] = *reinterpret_cast<const bf16x8*>(&ys[(wm * 64 + q * 32 + row32) * kPxStride + ks + khalf]);
        b[q] = *reinterpret_cast<const bf16x8*>(&as[(wn * 64 + q * 32 + row32) * kPxStride + ks + khalf]);
      }
#pragma unroll
      for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int q = 0; q < 2; ++q) acc[p][q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[p], b[q], acc[p][q], 0, 0, 0);
    }
    if (more) store_tile(buf ^ 1);
    __syncthreads();
    buf ^= 1;
  }

  // 32x32 result tile: lane holds column lane%32 and rows 8*(v/4) + 4*(lane/32) + v%4, v = 0..15
  float* __restrict__ dst = out + (int64_t)split_id * Co * Ci;
  const int col = lane & 31, half = lane >> 5;
#pragma unroll
  for (int p = 0; p < 2; ++p)
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const int i = i0 + wn * 64 + q * 32 + col;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int o = o0 + wm * 64 + p * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
        if (o < Co && i < Ci) dst[(int64_t)o * Ci + i] = acc[p][q][v];
      }
    }
}

template <int CE>
static int launch_conv1x1_bf16_ce(int Nb, int Ci, int Co, int HW, const void* A_dense, const void* dY, float* out,
                                  int splits, int64_t ktiles_per_split, hipStream_t st) {
  const int i_tiles = (int)ceil_div(Ci, kPxTile), o_tiles = (int)ceil_div(Co, kPxTile);
  const int tiles_per_img = (int)ceil_div(HW, kPxTok);
  const dim3 grid((unsigned)(o_tiles * i_tiles), (unsigned)splits);
  static std::atomic<uint64_t> lds_set{0};
  const int rc_lds = ensure_dynamic_lds((const void*)dw_conv1x1_bf16_kernel<CE>, kPxLdsBytes, lds_set);
  if (rc_lds != SURGEON_OK) return rc_lds;
  ProfScope prof(SURGEON_PROF_DW, st);
  SURGEON_LAUNCH(dw_conv1x1_bf16_kernel<CE>, grid, dim3(256), kPxLdsBytes, st, Nb, Ci, Co, HW, i_tiles, tiles_per_img,
                 ktiles_per_split, (const uint16_t*)A_dense, (const uint16_t*)dY, out);
  SURGEON_LAUNCH_CHECK();
  return SURGEON_OK;
}

int launch_conv1x1_bf16(int Nb, int Ci, int Co, int HW, const void* A_dense, const void* dY, float* out, int splits,
                        int64_t ktiles_per_split, hipStream_t st) {
  if (HW % 8 == 0) return launch_conv1x1_bf16_ce<8>(Nb, Ci, Co, HW, A_dense, dY, out, splits, ktiles_per_split, st);
  return launch_conv1x1_bf16_ce<4>(Nb, Ci, Co, HW, A_dense, dY, out, splits, ktiles_per_split, st);
}

int launch_linear_bf16(int64_t M, int64_t K, int64_t N, const void* A_dense, const void* dY, float* out, int splits,
                       int64_t rows_per_split, int wide, hipStream_t st) {
  const int tile_i = wide ? kBf16LinearTileWide : kBf16LinearTile;
  const int i_tiles = (int)ceil_div(K, tile_i), o_tiles = (int)ceil_div(N, kBf16LinearTile);
  const dim3 grid((unsigned)(o_tiles * i_tiles), (unsigned)splits);
  ProfScope prof(SURGEON_PROF_DW, st);
  if (N % 8 != 0)  // dY rows are not 16-byte aligned: element-wise dY loads (never chosen together with the wide tile)
    SURGEON_LAUNCH((dw_linear_bf16_kernel<2, 2, kBf16LinearTokens, false>), grid, dim3(256), 0, st, M, K, N, i_tiles,
                   rows_per_split, (const uint16_t*)A_dense, (const uint16_t*)dY, out, BatchedOperands{});
  else if (wide)
    SURGEON_LAUNCH((dw_linear_bf16_kernel<2, 4, kBf16LinearTokensWide, true>), grid, dim3(256), 0, st, M, K, N, i_tiles,
                   rows_per_split, (const uint16_t*)A_dense, (const uint16_t*)dY, out, BatchedOperands{});
  else
    SURGEON_LAUNCH((dw_linear_bf16_kernel<2, 2, kBf16LinearTokens, true>), grid, dim3(256), 0, st, M, K, N, i_tiles,
                   rows_per_split, (const uint16_t*)A_dense, (const uint16_t*)dY, out, BatchedOperands{});
  SURGEON_LAUNCH_CHECK();
  return SURGEON_OK;
}

// Activation gradient of a bf16 1x1 convolution without padding, stride 1 or 2 (Eq. 2, first line), image by image on
// the contraction above: the "tokens" are the Co output channels, the filter W [co][ci] is the operand whose rows become
// the result's rows, the image's dY [co][OH * OW] the one whose rows become its columns, and the result [ci][pixels] is
// the image's NCHW slice of dA, stored as bf16 by the kernel itself (one split: a workgroup walks all of Co).
int launch_da_conv1x1_bf16(int Nb, int Ci, int Co, int H, int W, int stride, const void* Wt, const void* dY, void* dA,
                           hipStream_t st) {
  const int OH = (H - 1) / stride + 1, OW = (W - 1) / stride + 1;
  const int64_t px = (int64_t)OH * OW;
  BatchedOperands bo;
  bo.a_batch = (int64_t)Co * px;
  bo.y_batch = 0;
  bo.out_batch = (int64_t)Ci * H * W;
  bo.out_w = W; bo.out_h = H; bo.in_w = OW;
  // 64-pixel tiles where they leave fewer columns empty than 128-pixel tiles (7 x 7 maps: 49 of 64 instead of 128)
  const bool narrow = ceil_div(px, 64) * 64 < ceil_div(px, 128) * 128;
  const int tile_i = narrow ? 64 : 128;
  const int i_tiles = (int)ceil_div(px, tile_i), o_tiles = (int)ceil_div(Ci, kBf16LinearTile);
  const dim3 grid((unsigned)(o_tiles * i_tiles), 1, (unsigned)Nb);
  const bool ya = Ci % 8 == 0 && ((uintptr_t)Wt % 16) == 0;
  // dY's rows (one per output channel, px elements): 16-byte chunks, 8-byte halves (14 x 14 maps) or single elements
  const int aa = (px % 8 == 0 && ((uintptr_t)dY % 16) == 0) ? 8 : (px % 4 == 0 && ((uintptr_t)dY % 8) == 0) ? 4 : 1;
  const int64_t M = Co, K = px, N = Ci;
  ProfScope prof(SURGEON_PROF_DA, st);
#define SURGEON_DA1X1(PI, YA, AA, OUT)                                                                                 \
  SURGEON_LAUNCH((dw_linear_bf16_kernel<2, PI, kBf16LinearTokens, YA, AA, OUT>), grid, dim3(256), 0, st, M, K, N, i_tiles, \
                 M, (const uint16_t*)dY, (const uint16_t*)Wt, (float*)dA, bo)
#define SURGEON_DA1X1_ALIGN(PI, OUT)            \
  do {                                          \
    if (ya && aa == 8) SURGEON_DA1X1(PI, true, 8, OUT);      \
    else if (ya && aa == 4) SURGEON_DA1X1(PI, true, 4, OUT); \
    else if (ya) SURGEON_DA1X1(PI, true, 1, OUT);            \
    else if (aa == 8) SURGEON_DA1X1(PI, false, 8, OUT);      \
    else SURGEON_DA1X1(PI, false, 1, OUT);                   \
  } while (0)
  if (stride == 1) {
    if (narrow) SURGEON_DA1X1_ALIGN(1, kOutBf16);
    else SURGEON_DA1X1_ALIGN(2, kOutBf16);
  } else {
    if (narrow) SURGEON_DA1X1_ALIGN(1, kOutBf16Stride2);
    else SURGEON_DA1X1_ALIGN(2, kOutBf16Stride2);
  }
#undef SURGEON_DA1X1_ALIGN
#undef SURGEON_DA1X1
  SURGEON_LAUNCH_CHECK();
  return SURGEON_OK;
}

// Activation gradient of a bf16 linear layer (Eq. 2, first line) on the same contraction, dY read where it lies:
// dA[m][k] = sum_n dY[m][n] W[n][k] -- the contraction index n is the fast one of dY (row-major tiles, plain LDS
// reads) and the slow one of W (the kernel's usual operand).  One split; the kernel stores bf16.  Needs N % 8 == 0 and
// 16-byte aligned dY; K % 8 != 0 or an unaligned W take 2-byte loads.
int launch_da_linear_bf16(int64_t M, int64_t K, int64_t N, const void* dY, const void* Wt, void* dA, hipStream_t st) {
  const int i_tiles = (int)ceil_div(K, kBf16LinearTile), o_tiles = (int)ceil_div(M, kBf16LinearTile);
  const dim3 grid((unsigned)(o_tiles * i_tiles), 1, 1);
  const bool wa = K % 8 == 0 && ((uintptr_t)Wt % 16) == 0;
  ProfScope prof(SURGEON_PROF_DA, st);
  // kernel arguments: contraction length ("tokens") = N, in-features = K, out rows = M; A operand = W, dY operand = dY
  if (wa)
    SURGEON_LAUNCH((dw_linear_bf16_kernel<2, 2, kBf16LinearTokens, true, 8, kOutBf16, true>), grid, dim3(256), 0, st, N, K, M,
                   i_tiles, N, (const uint16_t*)Wt, (const uint16_t*)dY, (float*)dA, BatchedOperands{});
  else
    SURGEON_LAUNCH((dw_linear_bf16_kernel<2, 2, kBf16LinearTokens, true, 1, kOutBf16, true>), grid, dim3(256), 0, st, N, K, M,
                   i_tiles, N, (const uint16_t*)Wt, (const uint16_t*)dY, (float*)dA, BatchedOperands{});
  SURGEON_LAUNCH_CHECK();
  return SURGEON_OK;
}

}  // namespace surgeon
