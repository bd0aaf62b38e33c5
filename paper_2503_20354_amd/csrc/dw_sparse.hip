// Weight gradient of a 3x3, stride-1, pad-1 convolution straight from the kept elements (Eq. 2; Alg. 1 lines 11-12
// without building the dense activation): every kept element a at (b, ci, ih, iw) adds a * dY[b, :, ih+1-u, iw+1-v]
// to dW[:, ci, u, v].  With few kept elements (at most 17 - 22 % of the layer) this takes less time than the dense
// contraction on the matrix cores, which spends most of its multiplications on zeros.
//
// One workgroup owns 64 output channels (one per lane) and WAVES * CPW input channels (CPW per wavefront, nine
// accumulators each, in registers), and walks a range of (image, band of R input rows) tiles.  Per tile it stages the
// R + 2 rows of dY that the band touches as [row][column + halo][channel] in LDS (the halo columns and out-of-range
// rows are zero, so the taps need no bounds checks); then each wavefront walks the mask words of its channels: the
// kept values of one 64-bit word are one coalesced load (lane j = j-th kept element), each set bit gives a wave-uniform
// value (v_readlane) and LDS position, nine LDS reads at compile-time offsets and nine multiply-adds.
// The kernel is bound by LDS bandwidth (one 4-byte read per multiply-add).  fp32 accumulation in element order inside a
// split, splits summed in index order afterwards: deterministic.
#include "common.hpp"

namespace surgeon {

namespace {

// floats per staged pixel = the 64 channels of the tile, unpadded: any two taps of an element are then a multiple of
// 64 floats apart, so one ds_read2st64_b32 fetches two of them (an LDS instruction occupies the LDS for four cycles
// whether it moves 256 or 512 bytes)
constexpr int kSpPix = kSparseCo;

struct SparseGeom {
  int Nb, Ci, Co, H;
  int ci_tiles, bands, tiles_per_split, n_tiles;
  int64_t n_w;
  uint32_t k_last;
};

// 16 wavefronts: 64 registers per lane (8 wavefronts per SIMD), so that two such workgroups fit a compute unit;
// 8 wavefronts: three workgroups per compute unit (LDS), 6 wavefronts per SIMD
// SHARE: walk the pixels kept in any of the wavefront's channels and read the taps once per pixel (pays from about
// 15 % kept on, where several channels often keep the same pixel); otherwise walk each channel's kept pixels on its own.
template <int W, int R, int CPW, int WAVES, bool SHARE>
__global__ __launch_bounds__(64 * WAVES) __attribute__((amdgpu_waves_per_eu(WAVES == 16 ? 8 : 6))) void dw_conv3x3_sparse_kernel(SparseGeom g, const float* __restrict__ vals,
                                                                            const uint64_t* __restrict__ mask,
                                                                            const uint32_t* __restrict__ word_rank,
                                                                            const float* __restrict__ dY,
                                                                            float* __restrict__ out) {
  constexpr int kThreads = 64 * WAVES;
  constexpr int PW = W + 2, ROWS = R + 2;
  constexpr int kLdsFloats = ROWS * PW * kSpPix;
  constexpr int kWords = R * W / 64;            // mask words per (image, channel, band)
  constexpr int kLog2W = W == 32 ? 5 : (W == 16 ? 4 : 3);
  constexpr int kChunksPerRow = W / 4;          // 16-byte chunks per dY row
  constexpr int kChunks = ROWS * kSparseCo * kChunksPerRow;
  static_assert((R * W) % 64 == 0 && R * W <= 128 && (W == 8 || W == 16 || W == 32), "band shape");
  extern __shared__ __attribute__((aligned(16))) float ys[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int co0 = (int)(blockIdx.x / (unsigned)g.ci_tiles) * kSparseCo;
  const int ci0 = (int)(blockIdx.x % (unsigned)g.ci_tiles) * (WAVES * CPW) + wave * CPW;
  const int t_begin = (int)blockIdx.y * g.tiles_per_split;
  const int t_end = min(t_begin + g.tiles_per_split, g.n_tiles);

  float acc[CPW][9];
#pragma unroll
  for (int c = 0; c < CPW; ++c)
#pragma unroll
    for (int t = 0; t < 9; ++t) acc[c][t] = 0.0f;

  for (int i = tid; i < kLdsFloats; i += kThreads) ys[i] = 0.0f;  // the halo columns stay zero from here on

  for (int tile = t_begin; tile < t_end; ++tile) {
    const int b = tile / g.bands, r0 = (tile - b * g.bands) * R;
    // ---- this wavefront's mask words, their ranks and kept values for the whole band, requested before the staging so
    // that their latency passes behind it (all wave-uniform except the values: lane j = j-th kept element of a word)
    uint64_t mw[CPW][kWords];
    float kept[CPW][kWords];
#pragma unroll
    for (int c = 0; c < CPW; ++c) {
      const int ci = min(ci0 + c, g.Ci - 1);
      const int64_t w0 = ((((int64_t)b * g.Ci + ci) * g.H + r0) * W) >> 6;
#pragma unroll
      for (int wi = 0; wi < kWords; ++wi) {
        mw[c][wi] = ci0 + c < g.Ci ? mask[w0 + wi] : 0ull;
        const uint32_t base = word_rank[w0 + wi];
        kept[c][wi] = vals[min(base + (uint32_t)lane, g.k_last)];
      }
    }
    __syncthreads();  // the previous tile's readers (first pass: the zero fill) are done
    // ---- stage dY rows r0-1 .. r0+R of 64 output channels.  Lanes run over the channels, so that the LDS writes of a
    // wavefront fall on consecutive banks; a lane reads its channel's row 16 bytes at a time (the other seven chunks of
    // the 128-byte line are read by the neighbouring chunk indices and hit in the vector cache).
    for (int c = tid; c < kChunks; c += kThreads) {
      const int co = c % kSparseCo, c4 = (c / kSparseCo) % kChunksPerRow, rr = c / (kChunksPerRow * kSparseCo);
      const int oh = r0 - 1 + rr;
      float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
      if (oh >= 0 && oh < g.H && co0 + co < g.Co)
        v = *reinterpret_cast<const float4*>(dY + (((int64_t)b * g.Co + co0 + co) * g.H + oh) * W + 4 * c4);
      float* dst = ys + (rr * PW + 1 + 4 * c4) * kSpPix + co;
      dst[0] = v.x;
      dst[kSpPix] = v.y;
      dst[2 * kSpPix] = v.z;
      dst[3 * kSpPix] = v.w;
    }
    __syncthreads();
    // ---- the kept elements of this wavefront's channels inside the band
    if constexpr (SHARE) {
      // The dY neighbourhood of a pixel does not depend on the input channel: the nine taps are read once per pixel kept
      // in ANY of the wavefront's channels and applied to every channel that keeps it (27 % fewer LDS reads at 21 % kept
      // with four channels, for eight more scalar instructions per pixel).
#pragma unroll
      for (int wi = 0; wi < kWords; ++wi) {
        const int word_pos = 64 * wi + 2 * (64 * wi / W);  // staged position of the word's first pixel, as below
        uint64_t any = 0;
#pragma unroll
        for (int c = 0; c < CPW; ++c) any |= mw[c][wi];
        int j[CPW];
#pragma unroll
        for (int c = 0; c < CPW; ++c) j[c] = 0;
        while (any != 0) {
          const int p = __builtin_ctzll(any);
          any &= any - 1;
          const float* src = ys + (p + 2 * (p >> kLog2W)) * kSpPix + lane;
          float d[9];
#pragma unroll
          for (int u = 0; u < 3; ++u)
#pragma unroll
            for (int x = 0; x < 3; ++x) d[u * 3 + x] = src[(word_pos + (2 - u) * PW + (2 - x)) * kSpPix];
#pragma unroll
          for (int c = 0; c < CPW; ++c) {
            if ((mw[c][wi] >> p) & 1ull) {  // wave-uniform
              const float a = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, kept[c][wi]), j[c]));
              ++j[c];
#pragma unroll
              for (int t = 0; t < 9; ++t) acc[c][t] = fmaf(a, d[t], acc[c][t]);
            }
          }
        }
      }
    } else {
#pragma unroll
      for (int c = 0; c < CPW; ++c) {
#pragma unroll
        for (int wi = 0; wi < kWords; ++wi) {
          // pixel q = 64 * wi + p of the band sits at staged position row * PW + col = q + 2 * (q / W); the part that
          // comes from wi is a constant once this loop is unrolled and folds into the LDS offsets
          const int word_pos = 64 * wi + 2 * (64 * wi / W);
          uint64_t m = mw[c][wi];
          int j = 0;
          while (m != 0) {
            const int p = __builtin_ctzll(m);
            m &= m - 1;
            const float a = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, kept[c][wi]), j));
            ++j;
            // tap (u, x) reads dY row (ih + 1 - u), column (iw + 1 - x): staged row (row + 2 - u), column (col + 2 - x)
            const float* src = ys + (p + 2 * (p >> kLog2W)) * kSpPix + lane;
#pragma unroll
            for (int u = 0; u < 3; ++u)
#pragma unroll
              for (int x = 0; x < 3; ++x)
                acc[c][u * 3 + x] = fmaf(a, src[(word_pos + (2 - u) * PW + (2 - x)) * kSpPix], acc[c][u * 3 + x]);
          }
        }
      }
    }
  }

  float* __restrict__ dst = out + (int64_t)blockIdx.y * g.n_w;
  const int co = co0 + lane;
  if (co < g.Co) {
#pragma unroll
    for (int c = 0; c < CPW; ++c) {
      const int ci = ci0 + c;
      if (ci < g.Ci) {
#pragma unroll
        for (int t = 0; t < 9; ++t) dst[((int64_t)co * g.Ci + ci) * 9 + t] = acc[c][t];
      }
    }
  }
}

template <int W, int R, int CPW, int WAVES, bool SHARE>
int launch_variant(const SparseGeom& g, int co_tiles, int splits, const float* vals, const uint64_t* mask,
                   const uint32_t* word_rank, const float* dY, float* out, hipStream_t st) {
  auto kernel = dw_conv3x3_sparse_kernel<W, R, CPW, WAVES, SHARE>;
  const size_t lds = (size_t)(R + 2) * (W + 2) * kSpPix * sizeof(float);
  if (lds > 48 * 1024) {
    static std::atomic<uint64_t> lds_set{0};  // one per instantiation = per kernel; lds is a constant of the instantiation
    const int rc_lds = ensure_dynamic_lds((const void*)kernel, lds, lds_set);
    if (rc_lds != SURGEON_OK) return rc_lds;
  }
  const dim3 grid((unsigned)(co_tiles * g.ci_tiles), (unsigned)splits);
  ProfScope prof(SURGEON_PROF_DW_SPARSE, st);
  SURGEON_LAUNCH(kernel, grid, dim3(64 * WAVES), lds, st, g, vals, mask, word_rank, dY, out);
  SURGEON_LAUNCH_CHECK();
  return SURGEON_OK;
}

}  // namespace

int sparse_conv_band_rows(int W) { return W == 32 ? 4 : 8; }

int sparse_conv_waves(int Ci) {
  int best = 8;
  const int64_t best_padded = ceil_div(Ci, 8 * kSparseCiPerWave) * 8 * kSparseCiPerWave;
  const int64_t padded16 = ceil_div(Ci, 16 * kSparseCiPerWave) * 16 * kSparseCiPerWave;
  if (padded16 <= best_padded) best = 16;
  return best;
}

template <int W, int R>
static int launch_waves(int waves, bool share, const SparseGeom& g, int co_tiles, int splits, const float* v, const uint64_t* mask,
                        const uint32_t* word_rank, const float* y, float* out, hipStream_t st) {
  // 8-wavefront workgroups are only used below the kept fraction at which sharing the tap reads pays
  if (waves == 16 && share)
    return launch_variant<W, R, kSparseCiPerWave, 16, true>(g, co_tiles, splits, v, mask, word_rank, y, out, st);
  if (waves == 16) return launch_variant<W, R, kSparseCiPerWave, 16, false>(g, co_tiles, splits, v, mask, word_rank, y, out, st);
  return launch_variant<W, R, kSparseCiPerWave, 8, false>(g, co_tiles, splits, v, mask, word_rank, y, out, st);
}

int launch_conv3x3_sparse_f32(int Nb, int Ci, int Co, int H, int W, int64_t k_total, int splits, int tiles_per_split,
                              const void* vals, const uint64_t* mask, const uint32_t* word_rank, const void* dY, float* out,
                              hipStream_t st) {
  const int R = sparse_conv_band_rows(W);
  SparseGeom g;
  g.Nb = Nb; g.Ci = Ci; g.Co = Co; g.H = H;
  const int waves = sparse_conv_waves(Ci);
  const bool share = k_total * 100 > (int64_t)15 * Nb * Ci * H * W;  // more than 15 % kept
  g.ci_tiles = (int)ceil_div(Ci, waves * kSparseCiPerWave);
  g.bands = H / R;
  g.n_tiles = Nb * g.bands;
  g.tiles_per_split = tiles_per_split;
  g.n_w = (int64_t)Co * Ci * 9;
  g.k_last = (uint32_t)(k_total - 1);
  const int co_tiles = (int)ceil_div(Co, kSparseCo);
  const float* v = (const float*)vals;
  const float* y = (const float*)dY;
  if (W == 32) return launch_waves<32, 4>(waves, share, g, co_tiles, splits, v, mask, word_rank, y, out, st);
  if (W == 16) return launch_waves<16, 8>(waves, share, g, co_tiles, splits, v, mask, word_rank, y, out, st);
  if (W == 8) return launch_waves<8, 8>(waves, share, g, co_tiles, splits, v, mask, word_rank, y, out, st);
  return fail(SURGEON_EUNSUPPORTED, "sparse conv: width %d", W);
}

}  // namespace surgeon
