// Activation gradient dA = dY . W (Eq. 2, first line) and the gradient step of Alg. 1 line 14.
//
// Together with surgeon_dw_from_packed this completes one layer's backward step of Alg. 1 (line 12 computes both
// gradients); dA does not involve the pruned activation at all, so it is an ordinary dense contraction:
//   linear : dA[m][k]         = sum_n        dY[m][n]        * W[n][k]
//   conv2d : dA[b][ci][ih][iw] = sum_{co,u,v} dY[b][co][oh][ow] * W[co][ci][u][v]   with oh*stride + u - pad == ih (same for w)
// Implicit GEMM on the fp32 matrix cores (v_mfma_f32_16x16x4_f32): one operand is gathered from dY (rows = the
// positions of dA, i.e. tokens or pixels), the other from W (rows = the channels of dA), the contraction runs over
// q = (co, u, v).  bf16 inputs are widened exactly while staging; accumulation is fp32; the result is rounded once
// (to nearest even) when dA is stored as bf16.
#include "common.hpp"

namespace surgeon {

typedef float floatx4 __attribute__((ext_vector_type(4)));

struct DaGeom {
  int Nb, Ci, H, W, Co, OH, OW, KH, KW, stride, pad;  // linear: Nb = M, Ci = K, Co = N, every spatial size 1
  int64_t P;  // positions of dA: Nb * H * W
  int Q;      // contraction length: Co * KH * KW
  int HW;
  // 1x1 layers with a stride (no padding) run on dY's own grid (H, W = dY's map, stride 1): position (oh, ow) is pixel
  // (spread oh, spread ow) of a dA map spread_h x spread_w, and it also writes the zeros of the spread x spread block
  // that starts there (no output pixel reaches those).  spread = 0: off.
  int spread, spread_h, spread_w;
};

template <typename T>
__device__ __forceinline__ float da_widen(T v);
template <>
__device__ __forceinline__ float da_widen<float>(float v) {
  return v;
}
template <>
__device__ __forceinline__ float da_widen<uint16_t>(uint16_t v) {
  return __uint_as_float((uint32_t)v << 16);
}

// fp32 -> bf16 bits, round to nearest even; NaN stays NaN
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

template <typename T>
__device__ __forceinline__ void da_store(T* p, float v);
template <>
__device__ __forceinline__ void da_store<float>(float* p, float v) {
  *p = v;
}
template <>
__device__ __forceinline__ void da_store<uint16_t>(uint16_t* p, float v) {
  *p = f32_to_bf16_rne(v);
}

constexpr int kDaTP = 128;  // positions per workgroup tile
constexpr int kDaTC = 128;  // channels of dA per workgroup tile
constexpr int kDaTQ = 32;   // contraction elements per K-tile
constexpr int kDaSX = kDaTP + 1, kDaSY = kDaTC + 1;  // LDS row strides: odd, so that column-wise staging writes spread over the banks

// blockIdx.x = position tile, blockIdx.y = channel tile.  4 wavefronts as 2 (positions) x 2 (channels), each 64 x 64.
// LINEAR: positions are the rows of the 16x16 result tiles and channels the columns (dA is [m][k], k contiguous);
// otherwise channels are the rows and positions the columns (dA is NCHW, pixels contiguous): either way a wavefront
// stores runs of 16 consecutive elements.
template <typename T, bool LINEAR>
__global__ __launch_bounds__(256) void da_kernel(DaGeom g, const T* __restrict__ dY, const T* __restrict__ Wt,
                                                 T* __restrict__ dA) {
  __shared__ float Xs[kDaTQ * kDaSX];  // [q][position]: gathered dY
  __shared__ float Ys[kDaTQ * kDaSY];  // [q][channel]:  W
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wp = wave >> 1, wc = wave & 1;
  const int i16 = lane & 15, kk = lane >> 4;
  const int64_t p0 = (int64_t)blockIdx.x * kDaTP;
  const int c0 = blockIdx.y * kDaTC;

  floatx4 acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) acc[a][b] = floatx4{0.f, 0.f, 0.f, 0.f};

  // staging roles.  LINEAR: both operands are contiguous along their fast index in memory (dY along n = q, W along k = c).
  // conv: dY is contiguous along the pixels (p), W is small and cached.
  // X: LINEAR thread -> (q = tid % 32, p = tid / 32 + 8 j); conv thread -> (p = tid % 128, q = tid / 128 + 2 j)
  int my_b = 0, my_ih = 0, my_iw = 0;
  bool my_ok = false;
  if (!LINEAR) {
    const int64_t p = p0 + (tid & (kDaTP - 1));
    my_ok = p < g.P;
    if (my_ok) {
      my_b = (int)(p / g.HW);
      const int rem = (int)(p - (int64_t)my_b * g.HW);
      my_ih = rem / g.W;
      my_iw = rem - my_ih * g.W;
    }
  }

  // The values of a K-tile travel global memory -> registers -> LDS; the loads of tile t + 1 are issued before the
  // matrix instructions of tile t, so their latency passes behind them.
  constexpr int kPerThread = kDaTP * kDaTQ / 256;  // 16 values of each operand per thread and K-tile
  static_assert(kDaTP == kDaTC && kPerThread == kDaTQ / 2 && kPerThread == kDaTP / 8, "staging roles");
  float xr[kPerThread], yr[kPerThread];
  auto load_tile = [&](int q0) {
    if (LINEAR) {
      const int q = q0 + (tid & 31);
#pragma unroll
      for (int j = 0; j < kPerThread; ++j) {
        const int64_t m = p0 + (tid >> 5) + 8 * j;
        xr[j] = (m < g.P && q < g.Q) ? da_widen<T>(dY[m * g.Co + q]) : 0.0f;
      }
    } else {
      // q = (co, u, v) advanced incrementally: this thread walks q0 + (tid / 128) + 2 j
      int q = q0 + (tid >> 7);
      const int taps = g.KH * g.KW;
      int co = q / taps;
      int t = q - co * taps;
      int u = t / g.KW, v = t - u * g.KW;
#pragma unroll
      for (int j = 0; j < kPerThread; ++j) {
        float val = 0.0f;
        if (my_ok && q < g.Q) {
          const int top = my_ih + g.pad - u, left = my_iw + g.pad - v;
          if (top >= 0 && left >= 0) {
            int oh = top, ow = left;
            bool hit = true;
            if (g.stride > 1) {
              oh = top / g.stride;
              ow = left / g.stride;
              hit = (oh * g.stride == top) && (ow * g.stride == left);
            }
            if (hit && oh < g.OH && ow < g.OW)
              val = da_widen<T>(dY[(((int64_t)my_b * g.Co + co) * g.OH + oh) * g.OW + ow]);
          }
        }
        xr[j] = val;
        q += 2;
        v += 2;
        while (v >= g.KW) {
          v -= g.KW;
          ++u;
        }
        while (u >= g.KH) {
          u -= g.KH;
          ++co;
        }
      }
    }
    const int c = c0 + (tid & (kDaTC - 1));
#pragma unroll
    for (int j = 0; j < kPerThread; ++j) {
      const int q = q0 + (tid >> 7) + 2 * j;
      float val = 0.0f;
      if (c < g.Ci && q < g.Q) {
        if (LINEAR) {
          val = da_widen<T>(Wt[(int64_t)q * g.Ci + c]);
        } else {
          const int taps = g.KH * g.KW;
          const int co = q / taps, t = q - co * taps;
          val = da_widen<T>(Wt[((int64_t)co * g.Ci + c) * taps + t]);
        }
      }
      yr[j] = val;
    }
  };
  // X: LINEAR thread -> (q = tid % 32, p = tid / 32 + 8 j); conv thread -> (p = tid % 128, q = tid / 128 + 2 j)
  // Y: thread -> (c = tid % 128, q = tid / 128 + 2 j)
  auto store_tile = [&]() {
#pragma unroll
    for (int j = 0; j < kPerThread; ++j) {
      if (LINEAR) Xs[(tid & 31) * kDaSX + (tid >> 5) + 8 * j] = xr[j];
      else Xs[((tid >> 7) + 2 * j) * kDaSX + (tid & (kDaTP - 1))] = xr[j];
      Ys[((tid >> 7) + 2 * j) * kDaSY + (tid & (kDaTC - 1))] = yr[j];
    }
  };

  load_tile(0);
  for (int q0 = 0; q0 < g.Q; q0 += kDaTQ) {
    __syncthreads();  // the previous tile's readers are done
    store_tile();
    __syncthreads();
    if (q0 + kDaTQ < g.Q) load_tile(q0 + kDaTQ);
    const float* rows = LINEAR ? Xs : Ys;  // operand whose index becomes the rows of the result tiles
    const float* cols = LINEAR ? Ys : Xs;
    const int srow = LINEAR ? kDaSX : kDaSY, scol = LINEAR ? kDaSY : kDaSX;
    const int wr = LINEAR ? wp : wc, wcl = LINEAR ? wc : wp;
#pragma unroll
    for (int s = 0; s < kDaTQ / 4; ++s) {
      float av[4], bv[4];
#pragma unroll
      for (int a = 0; a < 4; ++a) av[a] = rows[(4 * s + kk) * srow + wr * 64 + a * 16 + i16];
#pragma unroll
      for (int b = 0; b < 4; ++b) bv[b] = cols[(4 * s + kk) * scol + wcl * 64 + b * 16 + i16];
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[a], bv[b], acc[a][b], 0, 0, 0);
    }
  }

  // result tile: the lane holds rows 4*kk .. 4*kk+3 and column i16
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        if (LINEAR) {
          const int64_t m = p0 + wp * 64 + a * 16 + 4 * kk + r;
          const int c = c0 + wc * 64 + b * 16 + i16;
          if (m < g.P && c < g.Ci) da_store<T>(&dA[m * g.Ci + c], acc[a][b][r]);
        } else {
          const int c = c0 + wc * 64 + a * 16 + 4 * kk + r;
          const int64_t p = p0 + wp * 64 + b * 16 + i16;
          if (p < g.P && c < g.Ci) {
            const int64_t bimg = p / g.HW;
            if (g.spread == 0) {
              da_store<T>(&dA[(bimg * g.Ci + c) * g.HW + (p - bimg * g.HW)], acc[a][b][r]);
            } else {
              const int rem = (int)(p - bimg * g.HW);
              const int oh = rem / g.W, ow = rem - oh * g.W;
              T* __restrict__ px =
                  dA + ((bimg * g.Ci + c) * g.spread_h + (int64_t)oh * g.spread) * g.spread_w + ow * g.spread;
              for (int dh = 0; dh < g.spread && oh * g.spread + dh < g.spread_h; ++dh)
                for (int dw = 0; dw < g.spread && ow * g.spread + dw < g.spread_w; ++dw)
                  da_store<T>(&px[(int64_t)dh * g.spread_w + dw], (dh | dw) == 0 ? acc[a][b][r] : 0.0f);
            }
          }
        }
      }
}

// ---- layers with at most four input channels (a network's first convolution): one thread per pixel of dA --------------
// A 128-channel matrix tile would be almost empty here.  The filter sits in LDS as fp32, four channels wide; a thread
// walks the taps that reach its pixel under the layer's stride and, per tap, the output channels; its reads of dY
// coincide with its neighbours' (the same or the adjacent output pixel).  fp32 accumulation in the order (tap, output
// channel).
constexpr int kDaFewCi = 4;
template <typename T>
__global__ __launch_bounds__(256) void da_conv_fewch_kernel(DaGeom g, const T* __restrict__ dY, const T* __restrict__ Wt,
                                                            T* __restrict__ dA) {
  extern __shared__ floatx4 fw_lds[];  // [tap][co], the (up to) four input channels of a filter tap side by side
  const int taps = g.KH * g.KW, n_w = g.Co * taps;
  for (int i = threadIdx.x; i < n_w; i += 256) {
    const int co = i / taps, t = i - co * taps;
    floatx4 w4 = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int c = 0; c < g.Ci; ++c) w4[c] = da_widen<T>(Wt[((int64_t)co * g.Ci + c) * taps + t]);
    fw_lds[t * g.Co + co] = w4;
  }
  __syncthreads();
  const int64_t pos = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (pos >= g.P) return;
  const int b = (int)(pos / g.HW), rem = (int)(pos - (int64_t)b * g.HW);
  const int ih = rem / g.W, iw = rem - ih * g.W;
  const int64_t ohw = (int64_t)g.OH * g.OW;
  float acc[kDaFewCi] = {0.0f, 0.0f, 0.0f, 0.0f};
  for (int u = 0; u < g.KH; ++u) {
    const int th = ih + g.pad - u;
    if (th < 0 || th % g.stride) continue;
    const int oh = th / g.stride;
    if (oh >= g.OH) continue;
    for (int v = 0; v < g.KW; ++v) {
      const int tw = iw + g.pad - v;
      if (tw < 0 || tw % g.stride) continue;
      const int ow = tw / g.stride;
      if (ow >= g.OW) continue;
      const T* __restrict__ y = dY + (int64_t)b * g.Co * ohw + (int64_t)oh * g.OW + ow;
      const floatx4* __restrict__ w = fw_lds + (u * g.KW + v) * g.Co;
      for (int co = 0; co < g.Co; ++co) {
        const float yv = da_widen<T>(y[co * ohw]);
        const floatx4 w4 = w[co];
#pragma unroll
        for (int c = 0; c < kDaFewCi; ++c) acc[c] = __builtin_fmaf(yv, w4[c], acc[c]);
      }
    }
  }
#pragma unroll
  for (int c = 0; c < kDaFewCi; ++c)
    if (c < g.Ci) da_store<T>(&dA[((int64_t)b * g.Ci + c) * g.HW + rem], acc[c]);
}

// ---- convolutions with channel groups (grouped and depthwise layers): one thread per pixel of dA ----------------------
// Input channel ci receives from the Co / groups output channels of its group only: far too few for a matrix tile.
// A workgroup owns one (image, input channel) plane; that channel's filter taps of the group's output channels sit in
// LDS as fp32; a thread walks the taps that reach its pixel under the layer's stride and, per tap, the group's output
// channels.  fp32 accumulation in the order (tap, output channel).
template <typename T>
__global__ __launch_bounds__(256) void da_conv_grouped_kernel(DaGeom g, int Cig, int Cog, const T* __restrict__ dY,
                                                              const T* __restrict__ Wt, T* __restrict__ dA) {
  extern __shared__ float gw_lds[];  // [output channel of the group][tap]
  const int plane = blockIdx.x;      // b * Ci + ci
  const int b = plane / g.Ci, ci = plane - b * g.Ci;
  const int grp = ci / Cig, cig = ci - grp * Cig;
  const int taps = g.KH * g.KW;
  for (int i = threadIdx.x; i < Cog * taps; i += 256) {
    const int co_l = i / taps, t = i - co_l * taps;
    gw_lds[i] = da_widen<T>(Wt[((int64_t)(grp * Cog + co_l) * Cig + cig) * taps + t]);
  }
  __syncthreads();
  const int64_t ohw = (int64_t)g.OH * g.OW;
  const T* __restrict__ ybase = dY + ((int64_t)b * g.Co + (int64_t)grp * Cog) * ohw;
  for (int pos = (int)blockIdx.y * 256 + (int)threadIdx.x; pos < g.HW; pos += (int)gridDim.y * 256) {
    const int ih = pos / g.W, iw = pos - ih * g.W;
    float acc = 0.0f;
    for (int u = 0; u < g.KH; ++u) {
      const int th = ih + g.pad - u;
      if (th < 0 || th % g.stride) continue;
      const int oh = th / g.stride;
      if (oh >= g.OH) continue;
      for (int v = 0; v < g.KW; ++v) {
        const int tw = iw + g.pad - v;
        if (tw < 0 || tw % g.stride) continue;
        const int ow = tw / g.stride;
        if (ow >= g.OW) continue;
        const T* __restrict__ y = ybase + (int64_t)oh * g.OW + ow;
        const float* __restrict__ w = gw_lds + u * g.KW + v;
        for (int co_l = 0; co_l < Cog; ++co_l) acc = __builtin_fmaf(da_widen<T>(y[co_l * ohw]), w[co_l * taps], acc);
      }
    }
    da_store<T>(&dA[(int64_t)plane * g.HW + pos], acc);
  }
}

// ---- 3x3, stride 1, pad 1 convolutions: the taps as shifted reads of one staged patch ---------------------------------
// dA[b][ci][ih][iw] = sum_{co,u,v} dY[b][co][ih+1-u][iw+1-v] * W[co][ci][u][v].  A workgroup owns up to 128 positions
// -- a band of R rows of one image, or several whole images of a small map -- and a tile of 16 NC input channels, and
// walks the output channels eight at a time.  Per step it stages the eight channels' dY rows with halo once (zero
// outside the map) and the eight filters' (ci, tap) blocks -- contiguous in memory -- as [tap][co][ci]; the
// contraction runs over (tap, co), so a matrix instruction's four contraction elements are four output channels under
// one tap: the dY operand is the same patch read at a per-tap offset, with no index arithmetic per element.  The next
// step's values are loaded into registers before the matrix instructions of the current one.  Four wavefronts split
// the positions.  Measured on the three WideResNet-28-10 stages (200 images): 95 to 99 TFLOP/s, against 42 for the
// gathering kernel above.  Eight wavefronts of 16 positions each (four per SIMD on a compute unit instead of two) were
// slower, 85 to 93: twice the filter-tile reads per matrix instruction, and 128 registers do not hold the 160-channel tile.
constexpr int kDa3Co = 8;         // output channels per step

constexpr int da3_filter_row_stride(int ct) {
  int ws = ct + 16;
  while (ws % 32 != 16 || ws * 9 < ((ct * 9 + 255) / 256) * 256) ws += 1;
  return ws;
}

template <typename T, int NC, int PB>  // NC: 16-channel blocks per tile; PB: 16-position blocks per wavefront (P = 64 PB)
__global__ __launch_bounds__(256) void da_conv3x3_kernel(DaGeom g, int R, int imgs, int PS, const T* __restrict__ dY,
                                                         const T* __restrict__ Wt, T* __restrict__ dA) {
  constexpr int CT = 16 * NC;                   // input channels per tile
  constexpr int WCH = (CT * 9 + 255) / 256;     // filter values per thread and channel
  // LDS stride of a (tap, co) row of the filter tile: 16 banks past a multiple of 32, and wide enough for channel index
  // (256 WCH - 1) / 9, the last one the staging threads write
  constexpr int WS = da3_filter_row_stride(CT);
  constexpr int TS = kDa3Co * WS + 4;           // ... of a tap: four banks on, so staging writes of a channel's taps spread
  extern __shared__ float da3_lds[];
  float* patch = da3_lds;                       // [co 8][PS]: per image of the tile rows r0-1 .. r0+R, columns -1 .. W
  float* wt = da3_lds + kDa3Co * PS;            // [tap 9] x TS, inside a tap [co 8][WS]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int i16 = lane & 15, kk = lane >> 4;
  const int PW = g.W + 2, PP = (R + 2) * PW;
  const int bands = (g.H + R - 1) / R;
  // a tile is a band of R rows of one image (the last band of a map may be shorter), or -- small maps -- `imgs` whole
  // images (bands = 1; the last tile may hold fewer).  Tile positions past imgs * R * W, past the map's last row or
  // past the last image compute on zeros and are not stored.
  const int b = (blockIdx.x / bands) * imgs, r0 = (blockIdx.x - (blockIdx.x / bands) * bands) * R;
  const int RW = R * g.W;  // positions per image of the tile
  const int ci0 = blockIdx.y * CT;
  const int64_t hw = g.HW;

  floatx4 acc[NC][PB];
#pragma unroll
  for (int a = 0; a < NC; ++a)
#pragma unroll
    for (int q = 0; q < PB; ++q) acc[a][q] = floatx4{0.f, 0.f, 0.f, 0.f};

  // Staging walks one output channel at a time, so a thread's addresses are the same in every channel up to a uniform
  // offset: the few per-thread values below are all that stays live across the steps.
  constexpr int XPER = 2;                         // dY values per thread and channel (imgs (R + 2)(W + 2) <= 512)
  int x_src[XPER];                                // offset from the channel's map in the tile's first image, -1: a zero
#pragma unroll
  for (int j = 0; j < XPER; ++j) {
    const int idx = tid + 256 * j;
    const int img = idx / PP, rem = idx - img * PP;
    const int rr = rem / PW, cc = rem - rr * PW;
    const int ih = r0 - 1 + rr, iw = cc - 1;
    const bool in_map = img < imgs && b + img < g.Nb && ih >= 0 && ih < g.H && iw >= 0 && iw < g.W;
    x_src[j] = in_map ? img * g.Co * (int)hw + ih * g.W + iw : -1;
  }
  int w_dst[WCH];                                 // LDS index inside a channel's rows of the filter tile
  bool w_ok[WCH];                                 // the input channel exists
#pragma unroll
  for (int j = 0; j < WCH; ++j) {
    const int rem = tid + 256 * j;
    const int ci = rem / 9, tap = rem - ci * 9;
    w_dst[j] = tap * TS + ci;
    w_ok[j] = rem < CT * 9 && ci0 + ci < g.Ci;
  }
  float xr[kDa3Co][XPER], wr[kDa3Co][WCH];
  // Every load is issued unconditionally from an address inside the tensors (a channel past the end reads the last one,
  // a position outside the map reads the map's first pixel); what must be zero is zeroed when the value goes to LDS,
  // one step later, so nothing waits for a load before the matrix instructions that run in between.  The LDS writes
  // are unconditional too: a thread with nothing to stage writes into the padding of the rows (PS >= 512 + 16 and WS
  // leave room for the threads' whole index range).
  auto load_step = [&](int co0) {
#pragma unroll
    for (int c = 0; c < kDa3Co; ++c) {
      const int cc = min(co0 + c, g.Co - 1);
      const T* __restrict__ yc = dY + ((int64_t)b * g.Co + cc) * hw;
      const T* __restrict__ wc = Wt + ((int64_t)cc * g.Ci + ci0) * 9;
#pragma unroll
      for (int j = 0; j < XPER; ++j) xr[c][j] = da_widen<T>(yc[max(x_src[j], 0)]);
#pragma unroll
      for (int j = 0; j < WCH; ++j) wr[c][j] = da_widen<T>(wc[w_ok[j] ? tid + 256 * j : 0]);
    }
  };
  auto store_step = [&](int co0) {  // co0: the step the registers were loaded for
#pragma unroll
    for (int c = 0; c < kDa3Co; ++c) {
      const bool ch = co0 + c < g.Co;  // false on the last step of a channel count that 8 does not divide
#pragma unroll
      for (int j = 0; j < XPER; ++j) patch[c * PS + tid + 256 * j] = (ch && x_src[j] >= 0) ? xr[c][j] : 0.0f;
#pragma unroll
      for (int j = 0; j < WCH; ++j) wt[w_dst[j] + c * WS] = (ch && w_ok[j]) ? wr[c][j] : 0.0f;
    }
  };

  // this lane's positions: block q of the wavefront, column i16 of the result tiles
  int pos_off[PB];  // where the position's own pixel sits in a channel's patch (tap (1, 1) shifted by one row and column)
  int64_t out_off[PB];  // where its result goes in dA (channel 0), -1: not a position of the layer
#pragma unroll
  for (int q = 0; q < PB; ++q) {
    const int p = (wave * PB + q) * 16 + i16;
    const int img = p / RW, pl = p - img * RW;
    const int ihl = pl / g.W, iw = pl - ihl * g.W;
    const bool valid = img < imgs && b + img < g.Nb && r0 + ihl < g.H;
    pos_off[q] = valid ? img * PP + ihl * PW + iw : 0;
    out_off[q] = valid ? (int64_t)(b + img) * g.Ci * hw + (int64_t)(r0 + ihl) * g.W + iw : -1;
  }

  load_step(0);
  for (int co0 = 0; co0 < g.Co; co0 += kDa3Co) {
    __syncthreads();  // the previous step's readers are done
    store_step(co0);
    __syncthreads();
    if (co0 + kDa3Co < g.Co) load_step(co0 + kDa3Co);
    // 18 contraction steps of four (tap, then half of the eight channels); the operands of step s + 1 are read from LDS
    // before the matrix instructions of step s are issued, and the scheduling barriers keep that order, so that the
    // reads' latency passes under 4 NC PB matrix instructions instead of in front of every few of them
    constexpr int KS = 9 * kDa3Co / 4;
    float av[2][NC], bv[2][PB];
    auto read_operands = [&](int ks, float* a_out, float* b_out) {
      const int tap = ks / (kDa3Co / 4), sstep = ks - tap * (kDa3Co / 4);
      const int u = tap / 3, v = tap - 3 * u;
      const int tap_off = (2 - u) * PW + (2 - v);  // staged row ihl + 2 - u, column iw + 2 - v
#pragma unroll
      for (int a = 0; a < NC; ++a) a_out[a] = wt[tap * TS + (4 * sstep + kk) * WS + a * 16 + i16];
#pragma unroll
      for (int q = 0; q < PB; ++q) b_out[q] = patch[(4 * sstep + kk) * PS + pos_off[q] + tap_off];
    };
    read_operands(0, av[0], bv[0]);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if (ks + 1 < KS) read_operands(ks + 1, av[(ks + 1) & 1], bv[(ks + 1) & 1]);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int a = 0; a < NC; ++a)
#pragma unroll
        for (int q = 0; q < PB; ++q)
          acc[a][q] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[ks & 1][a], bv[ks & 1][q], acc[a][q], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  // result tile: the lane holds channels 4*kk .. 4*kk+3 (rows) of position i16 (column)
#pragma unroll
  for (int a = 0; a < NC; ++a)
#pragma unroll
    for (int q = 0; q < PB; ++q) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int c = ci0 + a * 16 + 4 * kk + r;
        if (c < g.Ci && out_off[q] >= 0) da_store<T>(&dA[out_off[q] + c * hw], acc[a][q][r]);
      }
    }
}

// How the 3x3 kernel tiles a layer: R rows per band and `imgs` images per tile, imgs * R * W <= 128 positions.
struct Da3Plan {
  bool ok = false;
  int R = 0, imgs = 1;
  int64_t tiles = 0;
};
static Da3Plan plan_da3(const DaGeom& g) {
  Da3Plan p;
  if (g.KH != 3 || g.KW != 3 || g.stride != 1 || g.pad != 1 || g.W > 128) return p;
  if ((int64_t)g.Co * g.HW >= ((int64_t)1 << 27)) return p;  // 32-bit offsets inside the dY of a tile's (at most eight) images
  p.R = std::min(g.H, 128 / g.W);
  if (p.R == g.H) p.imgs = std::max(1, std::min(std::min(8, g.Nb), 128 / g.HW));  // small maps: several whole images
  // a channel's patch is staged by two passes of the 256 threads
  while (p.imgs > 1 && p.imgs * (p.R + 2) * (g.W + 2) > 512) --p.imgs;
  if ((p.R + 2) * (g.W + 2) > 512) return p;
  p.tiles = ceil_div(g.Nb, p.imgs) * ceil_div(g.H, p.R);
  p.ok = p.tiles <= 0x7fffffff;
  return p;
}

template <typename T, int NC>
static int launch_da3(const DaGeom& g, const Da3Plan& plan, const void* dY, const void* Wt, void* dA, hipStream_t st) {
  const int PW = g.W + 2, R = plan.R, imgs = plan.imgs;
  int PS = imgs * (R + 2) * PW;
  PS = std::max(PS, 512);     // the staging threads write 512 values per channel, whatever the patch holds
  PS += (48 - PS % 32) % 32;  // channel stride 16 banks past a multiple of 32: the four channels of a read spread over the banks
  const size_t lds = ((size_t)kDa3Co * PS + (size_t)9 * (kDa3Co * da3_filter_row_stride(16 * NC) + 4)) * sizeof(float);
  const dim3 grid((unsigned)plan.tiles, (unsigned)ceil_div(g.Ci, 16 * NC));
  ProfScope prof(SURGEON_PROF_DA, st);
  if (imgs * R * g.W > 64) {
    auto kernel = da_conv3x3_kernel<T, NC, 2>;
    static std::atomic<uint64_t> lds_set{0};
    if (lds > 48 * 1024) {
      const int rc = ensure_dynamic_lds((const void*)kernel, 96 * 1024, lds_set);
      if (rc != SURGEON_OK) return rc;
    }
    SURGEON_LAUNCH(kernel, grid, dim3(256), lds, st, g, R, imgs, PS, (const T*)dY, (const T*)Wt, (T*)dA);
  } else {
    auto kernel = da_conv3x3_kernel<T, NC, 1>;
    static std::atomic<uint64_t> lds_set{0};
    if (lds > 48 * 1024) {
      const int rc = ensure_dynamic_lds((const void*)kernel, 96 * 1024, lds_set);
      if (rc != SURGEON_OK) return rc;
    }
    SURGEON_LAUNCH(kernel, grid, dim3(256), lds, st, g, R, imgs, PS, (const T*)dY, (const T*)Wt, (T*)dA);
  }
  SURGEON_LAUNCH_CHECK();
  return SURGEON_OK;
}

// ---- 3x3, stride 2, pad 1 convolutions --------------------------------------------------------------------------------
// Under stride 2 a pixel of dA receives only the taps whose offset has its parity: pixel (2 jh + ph, 2 jw + pw) takes
// row tap u = 1 for ph = 0 (from dY row jh) and u = 0, 2 for ph = 1 (from rows jh + 1 and jh), and the same along the
// columns, so the four pixels of a 2 x 2 cell split the nine taps 1 + 2 + 2 + 4 among them.  The kernel above is kept
// in shape -- band patch of dY, filter tile as [tap][co][ci], contraction over (tap, co), operands read a step ahead --
// with cells in place of positions: a wavefront owns 16 cells and four result blocks per channel block, one per pixel
// of the cell, and each tap's matrix instructions go to the block of the pixel that tap reaches.  No matrix work is
// spent on the taps that stride 2 rules out (the gathering kernel multiplies zeros there).
template <typename T, int NC>
__global__ __launch_bounds__(256) void da_conv3x3s2_kernel(DaGeom g, int RC, int PS, const T* __restrict__ dY,
                                                           const T* __restrict__ Wt, T* __restrict__ dA) {
  constexpr int CT = 16 * NC;
  constexpr int WCH = (CT * 9 + 255) / 256;
  constexpr int WS = da3_filter_row_stride(CT);
  constexpr int TS = kDa3Co * WS + 4;
  extern __shared__ float da3_lds[];
  float* patch = da3_lds;             // [co 8][PS]: dY rows j0 .. j0+RC, columns 0 .. CW (zero past the map)
  float* wt = da3_lds + kDa3Co * PS;  // [tap 9] x TS, inside a tap [co 8][WS]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int i16 = lane & 15, kk = lane >> 4;
  const int CW = (g.W + 1) / 2, CH = (g.H + 1) / 2;  // cells per row and column of the map
  const int PW = CW + 1, PP = (RC + 1) * PW;
  const int bands = (CH + RC - 1) / RC;
  const int b = blockIdx.x / bands, j0 = (blockIdx.x - b * bands) * RC;
  const int ci0 = blockIdx.y * CT;
  const int64_t hw = g.HW, ohw = (int64_t)g.OH * g.OW;

  floatx4 acc[NC][4];  // [channel block][2 ph + pw]
#pragma unroll
  for (int a = 0; a < NC; ++a)
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[a][q] = floatx4{0.f, 0.f, 0.f, 0.f};

  int x_src;  // this thread's value of a channel's patch: offset in the channel's dY map, -1: a zero
  {
    const int rr = tid / PW, cc = tid - rr * PW;
    const int oh = j0 + rr, ow = cc;
    x_src = (tid < PP && oh < g.OH && ow < g.OW) ? oh * g.OW + ow : -1;
  }
  int w_dst[WCH];
  bool w_ok[WCH];
#pragma unroll
  for (int j = 0; j < WCH; ++j) {
    const int rem = tid + 256 * j;
    const int ci = rem / 9, tap = rem - ci * 9;
    w_dst[j] = tap * TS + ci;
    w_ok[j] = rem < CT * 9 && ci0 + ci < g.Ci;
  }
  float xr[kDa3Co], wr[kDa3Co][WCH];
  // loads from addresses inside the tensors whatever the thread stages; zeros are put in when the values go to LDS
  auto load_step = [&](int co0) {
#pragma unroll
    for (int c = 0; c < kDa3Co; ++c) {
      const int cc = min(co0 + c, g.Co - 1);
      const T* __restrict__ yc = dY + ((int64_t)b * g.Co + cc) * ohw;
      const T* __restrict__ wc = Wt + ((int64_t)cc * g.Ci + ci0) * 9;
      xr[c] = da_widen<T>(yc[max(x_src, 0)]);
#pragma unroll
      for (int j = 0; j < WCH; ++j) wr[c][j] = da_widen<T>(wc[w_ok[j] ? tid + 256 * j : 0]);
    }
  };
  auto store_step = [&](int co0) {
#pragma unroll
    for (int c = 0; c < kDa3Co; ++c) {
      const bool ch = co0 + c < g.Co;
      patch[c * PS + tid] = (ch && x_src >= 0) ? xr[c] : 0.0f;  // PS >= 256: every thread has a slot
#pragma unroll
      for (int j = 0; j < WCH; ++j) wt[w_dst[j] + c * WS] = (ch && w_ok[j]) ? wr[c][j] : 0.0f;
    }
  };

  // this lane's cell
  const int cell = wave * 16 + i16;
  const int jhl = cell / CW, jw = cell - jhl * CW;
  const bool valid = jhl < RC && j0 + jhl < CH;
  const int cell_off = valid ? jhl * PW + jw : 0;

  load_step(0);
  for (int co0 = 0; co0 < g.Co; co0 += kDa3Co) {
    __syncthreads();
    store_step(co0);
    __syncthreads();
    if (co0 + kDa3Co < g.Co) load_step(co0 + kDa3Co);
    constexpr int KS = 9 * kDa3Co / 4;
    float av[2][NC], bv[2];
    auto read_operands = [&](int ks, float* a_out, float* b_out) {
      const int tap = ks / (kDa3Co / 4), sstep = ks - tap * (kDa3Co / 4);
      const int u = tap / 3, v = tap - 3 * u;
      // taps 0 reach the next dY row / column, taps 1 and 2 the cell's own
      const int tap_off = (u == 0 ? PW : 0) + (v == 0 ? 1 : 0);
#pragma unroll
      for (int a = 0; a < NC; ++a) a_out[a] = wt[tap * TS + (4 * sstep + kk) * WS + a * 16 + i16];
      *b_out = patch[(4 * sstep + kk) * PS + cell_off + tap_off];
    };
    read_operands(0, av[0], &bv[0]);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if (ks + 1 < KS) read_operands(ks + 1, av[(ks + 1) & 1], &bv[(ks + 1) & 1]);
      __builtin_amdgcn_sched_barrier(0);
      const int tap = ks / (kDa3Co / 4), u = tap / 3, v = tap - 3 * u;
      const int cls = (u != 1 ? 2 : 0) + (v != 1 ? 1 : 0);  // the pixel of the cell this tap reaches
#pragma unroll
      for (int a = 0; a < NC; ++a)
        acc[a][cls] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[ks & 1][a], bv[ks & 1], acc[a][cls], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  // the lane holds channels 4*kk .. 4*kk+3 of its cell's four pixels
  if (valid) {
    const int ih0 = 2 * (j0 + jhl), iw0 = 2 * jw;
#pragma unroll
    for (int a = 0; a < NC; ++a)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int c = ci0 + a * 16 + 4 * kk + r;
        if (c >= g.Ci) continue;
        T* __restrict__ px = dA + ((int64_t)b * g.Ci + c) * hw + (int64_t)ih0 * g.W + iw0;
#pragma unroll
        for (int ph = 0; ph < 2; ++ph)
          if (ih0 + ph < g.H) {
            da_store<T>(&px[ph * g.W], acc[a][2 * ph][r]);
            if (iw0 + 1 < g.W) da_store<T>(&px[ph * g.W + 1], acc[a][2 * ph + 1][r]);
          }
      }
  }
}

// cell rows per band for the stride-2 kernel, or 0 when the layer does not fit it
static int da3s2_band_rows(const DaGeom& g) {
  if (g.KH != 3 || g.KW != 3 || g.stride != 2 || g.pad != 1) return 0;
  const int CW = (g.W + 1) / 2, CH = (g.H + 1) / 2;
  if (CW > 64 || (int64_t)g.Nb * CH > 0x7fffffff) return 0;
  return std::min(CH, 64 / CW);
}

template <typename T, int NC>
static int launch_da3s2(const DaGeom& g, int RC, const void* dY, const void* Wt, void* dA, hipStream_t st) {
  const int CH = (g.H + 1) / 2;
  int PS = 256;               // one slot per staging thread; (RC + 1)(CW + 1) <= 130 of them hold the patch
  PS += (48 - PS % 32) % 32;  // channel stride 16 banks past a multiple of 32
  const size_t lds = ((size_t)kDa3Co * PS + (size_t)9 * (kDa3Co * da3_filter_row_stride(16 * NC) + 4)) * sizeof(float);
  const dim3 grid((unsigned)(g.Nb * ceil_div(CH, RC)), (unsigned)ceil_div(g.Ci, 16 * NC));
  ProfScope prof(SURGEON_PROF_DA, st);
  SURGEON_LAUNCH((da_conv3x3s2_kernel<T, NC>), grid, dim3(256), lds, st, g, RC, PS, (const T*)dY, (const T*)Wt, (T*)dA);
  SURGEON_LAUNCH_CHECK();
  return SURGEON_OK;
}

// Alg. 1 line 14 as one plain gradient step, in place: W <- W - lr * dW
template <typename T>
__global__ __launch_bounds__(256) void weight_update_kernel(T* __restrict__ Wt, const float* __restrict__ dW, int64_t n,
                                                            float lr) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256)
    da_store<T>(&Wt[i], __builtin_fmaf(-lr, dW[i], da_widen<T>(Wt[i])));
}

// ---- the gradient step for many tensors in one launch: the weights of a layer are small next to the chip (at most a
// few MB), so one launch per layer is mostly launch gap.  Up to kUpdateBatch tensors travel as kernel arguments; a
// workgroup owns one 4096-element chunk of one tensor (workgroup -> tensor by the tensors' first workgroups).
constexpr int kUpdateBatch = 64;
constexpr int kUpdateChunk = 4096;
struct UpdateBatch {
  void* Wt[kUpdateBatch];
  const float* dW[kUpdateBatch];
  int64_t n[kUpdateBatch];
  int first_block[kUpdateBatch + 1];  // entries past the last tensor hold the total
};

template <typename T>
__global__ __launch_bounds__(256) void weight_update_batched_kernel(UpdateBatch bt, float lr) {
  // the tensor of this workgroup: the last boundary at or below its index (branch-free binary search, scalar loads)
  int t = 0;
#pragma unroll
  for (int step = kUpdateBatch / 2; step >= 1; step >>= 1) {
    const int c = t + step;  // <= kUpdateBatch - 1
    t = (int)blockIdx.x >= bt.first_block[c] ? c : t;
  }
  T* __restrict__ Wt = (T*)bt.Wt[t];
  const float* __restrict__ dW = bt.dW[t];
  const int64_t n = bt.n[t];
  const int64_t c0 = (int64_t)((int)blockIdx.x - bt.first_block[t]) * kUpdateChunk;
  // four consecutive elements per thread and round: 16-byte accesses when both pointers allow them
  const bool wide = (((uintptr_t)Wt % (4 * sizeof(T))) | ((uintptr_t)dW % 16)) == 0;
#pragma unroll
  for (int q = 0; q < kUpdateChunk / 1024; ++q) {
    const int64_t i = c0 + q * 1024 + threadIdx.x * 4;
    if (wide && i + 4 <= n) {
      const float4 g = *reinterpret_cast<const float4*>(dW + i);
      if constexpr (sizeof(T) == 4) {
        float4 w = *reinterpret_cast<const float4*>(Wt + i);
        w.x = __builtin_fmaf(-lr, g.x, w.x); w.y = __builtin_fmaf(-lr, g.y, w.y);
        w.z = __builtin_fmaf(-lr, g.z, w.z); w.w = __builtin_fmaf(-lr, g.w, w.w);
        *reinterpret_cast<float4*>(Wt + i) = w;
      } else {
        ushort4 w = *reinterpret_cast<const ushort4*>(Wt + i);
        da_store<T>(&w.x, __builtin_fmaf(-lr, g.x, da_widen<T>(w.x)));
        da_store<T>(&w.y, __builtin_fmaf(-lr, g.y, da_widen<T>(w.y)));
        da_store<T>(&w.z, __builtin_fmaf(-lr, g.z, da_widen<T>(w.z)));
        da_store<T>(&w.w, __builtin_fmaf(-lr, g.w, da_widen<T>(w.w)));
        *reinterpret_cast<ushort4*>(Wt + i) = w;
      }
    } else {
      for (int64_t j = i; j < min(i + 4, n); ++j) da_store<T>(&Wt[j], __builtin_fmaf(-lr, dW[j], da_widen<T>(Wt[j])));
    }
  }
}

// ---- bf16 linear layers on the bf16 matrix cores ---------------------------------------------------------------
// dA[m][k] = sum_n dY[m][n] * W[n][k] is the contraction of the bf16 weight-gradient kernel (out[o][i] = sum_t
// Y[t][o] * X[t][i], the contraction index slow in both operands) with t = n, Y = dY transposed, X = W.  dY is
// transposed once into the workspace (2 bytes read and written per element), the 256 x 128 kernel writes fp32 (partial)
// results, and a finishing kernel adds the splits in index order and rounds once to bf16.

// out[c][r] = in[r][c] for a [R][C] matrix of 2-byte elements: 64 x 64 tiles through LDS
__global__ __launch_bounds__(256) void transpose16_kernel(const uint16_t* __restrict__ in, uint16_t* __restrict__ out,
                                                          int64_t R, int64_t C) {
  __shared__ uint16_t tile[64][66];
  const int64_t r0 = (int64_t)blockIdx.y * 64, c0 = (int64_t)blockIdx.x * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const int64_t r = r0 + ty + 4 * j, c = c0 + tx;
    tile[ty + 4 * j][tx] = (r < R && c < C) ? in[r * C + c] : (uint16_t)0;
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const int64_t c = c0 + ty + 4 * j, r = r0 + tx;
    if (c < C && r < R) out[c * R + r] = tile[tx][ty + 4 * j];
  }
}

__global__ __launch_bounds__(256) void da_finish_bf16_kernel(const float* __restrict__ part, int splits, int64_t n,
                                                             uint16_t* __restrict__ dA) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    float v = part[i];
    for (int s = 1; s < splits; ++s) v += part[(int64_t)s * n + i];
    dA[i] = f32_to_bf16_rne(v);
  }
}

struct DaFastPlan {
  bool ok;
  int splits;
  int64_t rows_per_split;
  size_t off_part, ws_bytes;
};

// the bf16 matrix-core route needs 16-byte rows in both operands and 32-bit byte offsets
static DaFastPlan plan_da_fast(const surgeon_layer_desc* d) {
  DaFastPlan p;
  p.ok = false;
  p.splits = 0;
  p.rows_per_split = 0;
  p.off_part = p.ws_bytes = 0;
  const int64_t big = (int64_t)1 << 31;
  if (d->kind != SURGEON_LINEAR || d->dtype != SURGEON_BF16) return p;
  if (d->M < 256 || d->K < 64 || d->N < 64 || d->M % 8 || d->K % 8) return p;
  if (d->M * d->N * 2 >= big || d->N * d->K * 2 >= big || d->M * d->K * 4 >= big) return p;
  const int64_t tiles = ceil_div(d->M, kBf16BigTileO) * ceil_div(d->K, kBf16BigTileI);
  const int64_t k_tiles = ceil_div(d->N, kBf16BigTokens);
  // one round of workgroups on the chip's 256 compute units; a split is at least four K-tiles long
  int64_t splits = std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(256 / std::max<int64_t>(tiles, 1), k_tiles / 4), 16));
  const int64_t per = ceil_div(k_tiles, splits);
  p.splits = (int)ceil_div(k_tiles, per);
  p.rows_per_split = per * kBf16BigTokens;
  p.off_part = align_up((size_t)d->M * d->N * 2, 256);
  // one split: the contraction kernel stores bf16 itself and there are no partial results
  p.ws_bytes = p.off_part + (p.splits > 1 ? align_up((size_t)p.splits * d->M * d->K * 4, 256) : 0);
  p.ok = true;
  return p;
}

}  // namespace surgeon

using namespace surgeon;

extern "C" int surgeon_weight_update_batched(int l, void* const* Wt, const float* const* dW, const int64_t* n, float lr, int dt,
                                             void* stream) {
  if (dt != SURGEON_F32 && dt != SURGEON_BF16) return fail(SURGEON_EINVAL, "weight_update_batched: bad dtype %d", dt);
  if (l < 0 || !(lr == lr)) return fail(SURGEON_EINVAL, "weight_update_batched: bad arguments");
  if (l == 0) return SURGEON_OK;
  if (!Wt || !dW || !n) return fail(SURGEON_EINVAL, "weight_update_batched: null array");
  for (int i = 0; i < l; ++i) {  // everything is checked before the first launch
    if (n[i] < 0) return fail(SURGEON_EINVAL, "weight_update_batched: tensor %d has n < 0", i);
    if (n[i] > 0 && (!Wt[i] || !dW[i])) return fail(SURGEON_EINVAL, "weight_update_batched: tensor %d: null pointer", i);
    if (((uintptr_t)Wt[i] % (dt == SURGEON_F32 ? 4 : 2)) || ((uintptr_t)dW[i] % 4))
      return fail(SURGEON_EINVAL, "weight_update_batched: tensor %d: misaligned pointer", i);
    if (ceil_div(n[i], kUpdateChunk) > 0x3fffffff) return fail(SURGEON_EUNSUPPORTED, "weight_update_batched: tensor %d too large", i);
  }
  hipStream_t st = (hipStream_t)stream;
  ProfScope prof(SURGEON_PROF_UPDATE, st);
  UpdateBatch bt;
  int count = 0;
  int64_t blocks = 0;
  auto flush = [&]() -> int {
    if (count == 0) return SURGEON_OK;
    for (int i = count; i <= kUpdateBatch; ++i) bt.first_block[i] = (int)blocks;
    for (int i = count; i < kUpdateBatch; ++i) { bt.Wt[i] = nullptr; bt.dW[i] = nullptr; bt.n[i] = 0; }
    if (dt == SURGEON_F32)
      SURGEON_LAUNCH(weight_update_batched_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, st, bt, lr);
    else
      SURGEON_LAUNCH(weight_update_batched_kernel<uint16_t>, dim3((unsigned)blocks), dim3(256), 0, st, bt, lr);
    SURGEON_LAUNCH_CHECK();
    count = 0;
    blocks = 0;
    return SURGEON_OK;
  };
  for (int i = 0; i < l; ++i) {
    if (n[i] == 0) continue;
    const int64_t b = ceil_div(n[i], kUpdateChunk);
    if (count == kUpdateBatch || blocks + b > 0x7fffffff) {
      const int rc = flush();
      if (rc != SURGEON_OK) return rc;
    }
    bt.Wt[count] = Wt[i]; bt.dW[count] = dW[i]; bt.n[count] = n[i];
    bt.first_block[count] = (int)blocks;
    blocks += b;
    ++count;
  }
  return flush();
}

static int da_entry(const surgeon_layer_desc* d, const void* dY, const void* Wt, void* dA, void* ws, size_t ws_bytes,
                    bool use_ws, void* stream) {
  if (!d) return fail(SURGEON_EINVAL, "da: null descriptor");
  if (d->dtype != SURGEON_F32 && d->dtype != SURGEON_BF16) return fail(SURGEON_EINVAL, "da: bad dtype");
  DaGeom g;
  bool linear;
  if (d->kind == SURGEON_LINEAR) {
    if (d->M < 0 || d->K < 1 || d->N < 1) return fail(SURGEON_EINVAL, "da: bad linear shape");
    if (d->K > (1 << 30) || d->N > (1 << 30)) return fail(SURGEON_EUNSUPPORTED, "da: linear layer too wide");
    linear = true;
    g.Nb = 1; g.Ci = (int)d->K; g.Co = (int)d->N;
    g.H = g.W = g.OH = g.OW = g.KH = g.KW = g.stride = 1;
    g.pad = 0;
    g.P = d->M;
    g.Q = (int)d->N;
    g.HW = 1;
    g.spread = g.spread_h = g.spread_w = 0;
  } else if (d->kind == SURGEON_CONV2D) {
    if (d->Nb < 1 || d->Ci < 1 || d->H < 1 || d->W < 1 || d->Co < 1 || d->kh < 1 || d->kw < 1 || d->stride < 1 || d->pad < 0)
      return fail(SURGEON_EINVAL, "da: bad conv shape");
    if (d->H + 2 * d->pad < d->kh || d->W + 2 * d->pad < d->kw)
      return fail(SURGEON_EINVAL, "da: filter larger than the padded input");
    if (d->groups > 1 && (d->Ci % d->groups || d->Co % d->groups))
      return fail(SURGEON_EINVAL, "da: groups = %lld does not divide the channel counts", (long long)d->groups);
    const int64_t big = (int64_t)1 << 31;
    if (d->Co * d->kh * d->kw >= big || d->H * d->W >= big || d->Ci >= big || d->Nb >= big)
      return fail(SURGEON_EUNSUPPORTED, "da: conv tensor too large");
    linear = false;
    g.Nb = (int)d->Nb; g.Ci = (int)d->Ci; g.H = (int)d->H; g.W = (int)d->W; g.Co = (int)d->Co;
    g.KH = (int)d->kh; g.KW = (int)d->kw; g.stride = (int)d->stride; g.pad = (int)d->pad;
    g.OH = (g.H + 2 * g.pad - g.KH) / g.stride + 1;
    g.OW = (g.W + 2 * g.pad - g.KW) / g.stride + 1;
    g.HW = g.H * g.W;
    g.P = (int64_t)g.Nb * g.HW;
    g.Q = g.Co * g.KH * g.KW;
    g.spread = g.spread_h = g.spread_w = 0;
  } else {
    return fail(SURGEON_EINVAL, "da: bad layer kind %d", d->kind);
  }
  if (g.P == 0) return SURGEON_OK;
  if (!dY || !Wt || !dA) return fail(SURGEON_EINVAL, "da: null pointer");
  const size_t es = d->dtype == SURGEON_F32 ? 4 : 2;
  if (((uintptr_t)dY % es) || ((uintptr_t)Wt % es) || ((uintptr_t)dA % es)) return fail(SURGEON_EINVAL, "da: misaligned pointer");
  hipStream_t st = (hipStream_t)stream;
  if (use_ws) {
    const DaFastPlan fp = plan_da_fast(d);
    if (fp.ok) {
      if (!ws || ws_bytes < fp.ws_bytes)
        return fail(SURGEON_ESIZE, "da: workspace of %zu bytes needed, %zu given", fp.ws_bytes, ws_bytes);
      if (((uintptr_t)ws % 16) || ((uintptr_t)Wt % 16)) return fail(SURGEON_EINVAL, "da: workspace / W not 16-byte aligned");
      uint16_t* dYt = (uint16_t*)ws;
      float* part = (float*)((char*)ws + fp.off_part);
      {
        ProfScope prof(SURGEON_PROF_DA, st);
        SURGEON_LAUNCH(transpose16_kernel, dim3((unsigned)ceil_div(d->N, 64), (unsigned)ceil_div(d->M, 64)), dim3(256), 0, st,
                       (const uint16_t*)dY, dYt, d->M, d->N);
        SURGEON_LAUNCH_CHECK();
      }
      {
        // contraction over n: "tokens" = N, out-features = M (from dY^T), in-features = K (from W)
        ProfForce as_da(SURGEON_PROF_DA);
        const bool direct = fp.splits == 1;
        const int rc = launch_linear_bf16_big(d->N, d->K, d->M, Wt, dYt, direct ? (float*)dA : part, fp.splits,
                                              fp.rows_per_split, st, direct);
        if (rc != SURGEON_OK) return rc;
        if (direct) return SURGEON_OK;
      }
      ProfScope prof(SURGEON_PROF_DA, st);
      const int64_t n_out = d->M * d->K;
      SURGEON_LAUNCH(da_finish_bf16_kernel, dim3((unsigned)std::min<int64_t>(ceil_div(n_out, 256), 8192)), dim3(256), 0, st,
                     (const float*)part, fp.splits, n_out, (uint16_t*)dA);
      SURGEON_LAUNCH_CHECK();
      return SURGEON_OK;
    }
  }
  if (!linear && d->groups > 1) {
    const int Cig = (int)(d->Ci / d->groups), Cog = (int)(d->Co / d->groups);
    const size_t lds = (size_t)Cog * g.KH * g.KW * sizeof(float);
    if (lds > 48 * 1024) return fail(SURGEON_EUNSUPPORTED, "da: a group's filters for one input channel exceed 48 KB");
    if ((int64_t)g.Nb * g.Ci > 0x7fffffff) return fail(SURGEON_EUNSUPPORTED, "da: too many (image, channel) planes");
    const dim3 grid((unsigned)(g.Nb * g.Ci), (unsigned)std::min<int64_t>(ceil_div(g.HW, 256), 64));
    ProfScope prof(SURGEON_PROF_DA, st);
    if (d->dtype == SURGEON_F32)
      SURGEON_LAUNCH(da_conv_grouped_kernel<float>, grid, dim3(256), lds, st, g, Cig, Cog, (const float*)dY, (const float*)Wt,
                     (float*)dA);
    else
      SURGEON_LAUNCH(da_conv_grouped_kernel<uint16_t>, grid, dim3(256), lds, st, g, Cig, Cog, (const uint16_t*)dY,
                     (const uint16_t*)Wt, (uint16_t*)dA);
    SURGEON_LAUNCH_CHECK();
    return SURGEON_OK;
  }
  if (linear && d->dtype == SURGEON_BF16 && d->N % 8 == 0 && ((uintptr_t)dY % 16) == 0 && d->M >= 64 && d->K >= 64 &&
      d->N >= 64 && ceil_div(d->M, kBf16LinearTile) * ceil_div(d->K, kBf16LinearTile) <= 0x7fffffff)
    return launch_da_linear_bf16(d->M, d->K, d->N, dY, Wt, dA, st);
  if (!linear && d->dtype == SURGEON_BF16 && g.KH == 1 && g.KW == 1 && g.pad == 0 && (g.stride == 1 || g.stride == 2) &&
      g.Nb <= 65535 && (int64_t)g.Ci * g.HW < ((int64_t)1 << 31))
    return launch_da_conv1x1_bf16(g.Nb, g.Ci, g.Co, g.H, g.W, g.stride, Wt, dY, dA, st);
  if (!linear && g.Ci <= kDaFewCi && (size_t)g.Q * 16 <= 64 * 1024 && ceil_div(g.P, 256) <= 0x7fffffff) {
    const dim3 grid((unsigned)ceil_div(g.P, 256));
    const size_t lds = (size_t)g.Q * 16;
    static std::atomic<uint64_t> lds_f32{0}, lds_bf16{0};
    ProfScope prof(SURGEON_PROF_DA, st);
    if (d->dtype == SURGEON_F32) {
      const int rc = ensure_dynamic_lds((const void*)da_conv_fewch_kernel<float>, 64 * 1024, lds_f32);
      if (rc != SURGEON_OK) return rc;
      SURGEON_LAUNCH(da_conv_fewch_kernel<float>, grid, dim3(256), lds, st, g, (const float*)dY, (const float*)Wt, (float*)dA);
    } else {
      const int rc = ensure_dynamic_lds((const void*)da_conv_fewch_kernel<uint16_t>, 64 * 1024, lds_bf16);
      if (rc != SURGEON_OK) return rc;
      SURGEON_LAUNCH(da_conv_fewch_kernel<uint16_t>, grid, dim3(256), lds, st, g, (const uint16_t*)dY, (const uint16_t*)Wt,
                     (uint16_t*)dA);
    }
    SURGEON_LAUNCH_CHECK();
    return SURGEON_OK;
  }
  if (!linear) {
    const int RC = da3s2_band_rows(g);
    if (RC > 0) {
      const bool five = g.Ci % 80 == 0;  // 80-channel tiles where they divide the channels, else 64
      if (d->dtype == SURGEON_F32)
        return five ? launch_da3s2<float, 5>(g, RC, dY, Wt, dA, st) : launch_da3s2<float, 4>(g, RC, dY, Wt, dA, st);
      return five ? launch_da3s2<uint16_t, 5>(g, RC, dY, Wt, dA, st) : launch_da3s2<uint16_t, 4>(g, RC, dY, Wt, dA, st);
    }
  }
  if (!linear) {
    const Da3Plan plan = plan_da3(g);
    if (plan.ok) {
      // channel tile: 160 where it divides the channels (the widths of WideResNet), else 128, 64, 32 or 16
      const int nc = g.Ci % 160 == 0 ? 10 : g.Ci >= 128 ? 8 : g.Ci > 32 ? 4 : g.Ci > 16 ? 2 : 1;
      if (d->dtype == SURGEON_F32) {
        if (nc == 10) return launch_da3<float, 10>(g, plan, dY, Wt, dA, st);
        if (nc == 8) return launch_da3<float, 8>(g, plan, dY, Wt, dA, st);
        if (nc == 4) return launch_da3<float, 4>(g, plan, dY, Wt, dA, st);
        if (nc == 2) return launch_da3<float, 2>(g, plan, dY, Wt, dA, st);
        return launch_da3<float, 1>(g, plan, dY, Wt, dA, st);
      }
      if (nc == 10) return launch_da3<uint16_t, 10>(g, plan, dY, Wt, dA, st);
      if (nc == 8) return launch_da3<uint16_t, 8>(g, plan, dY, Wt, dA, st);
      if (nc == 4) return launch_da3<uint16_t, 4>(g, plan, dY, Wt, dA, st);
      if (nc == 2) return launch_da3<uint16_t, 2>(g, plan, dY, Wt, dA, st);
      return launch_da3<uint16_t, 1>(g, plan, dY, Wt, dA, st);
    }
  }
  if (!linear && g.KH == 1 && g.KW == 1 && g.pad == 0 && g.stride > 1) {
    // a strided 1x1 layer: contract on dY's grid, a stride^2-th of dA's positions, and spread the result
    g.spread = g.stride; g.spread_h = g.H; g.spread_w = g.W;
    g.H = g.OH; g.W = g.OW; g.stride = 1;
    g.HW = g.H * g.W;
    g.P = (int64_t)g.Nb * g.HW;
  }
  const int64_t p_tiles = ceil_div(g.P, kDaTP), c_tiles = ceil_div(g.Ci, kDaTC);
  if (p_tiles > 0x7fffffff || c_tiles > 65535) return fail(SURGEON_EUNSUPPORTED, "da: too many tiles");
  const dim3 grid((unsigned)p_tiles, (unsigned)c_tiles);
  ProfScope prof(SURGEON_PROF_DA, st);
  if (d->dtype == SURGEON_F32) {
    if (linear)
      SURGEON_LAUNCH((da_kernel<float, true>), grid, dim3(256), 0, st, g, (const float*)dY, (const float*)Wt, (float*)dA);
    else
      SURGEON_LAUNCH((da_kernel<float, false>), grid, dim3(256), 0, st, g, (const float*)dY, (const float*)Wt, (float*)dA);
  } else {
    if (linear)
      SURGEON_LAUNCH((da_kernel<uint16_t, true>), grid, dim3(256), 0, st, g, (const uint16_t*)dY, (const uint16_t*)Wt,
                     (uint16_t*)dA);
    else
      SURGEON_LAUNCH((da_kernel<uint16_t, false>), grid, dim3(256), 0, st, g, (const uint16_t*)dY, (const uint16_t*)Wt,
                     (uint16_t*)dA);
  }
  SURGEON_LAUNCH_CHECK();
  return SURGEON_OK;
}

extern "C" int surgeon_da(const surgeon_layer_desc* d, const void* dY, const void* Wt, void* dA, void* stream) {
  return da_entry(d, dY, Wt, dA, nullptr, 0, false, stream);
}

extern "C" int surgeon_da_ws_bytes(const surgeon_layer_desc* d, size_t* ws_bytes) {
  if (!d || !ws_bytes) return fail(SURGEON_EINVAL, "da_ws_bytes: null pointer");
  if (d->dtype != SURGEON_F32 && d->dtype != SURGEON_BF16) return fail(SURGEON_EINVAL, "da_ws_bytes: bad dtype");
  *ws_bytes = plan_da_fast(d).ws_bytes;
  return SURGEON_OK;
}

extern "C" int surgeon_da_ws(const surgeon_layer_desc* d, const void* dY, const void* Wt, void* dA, void* ws, size_t ws_bytes,
                             void* stream) {
  return da_entry(d, dY, Wt, dA, ws, ws_bytes, true, stream);
}

extern "C" int surgeon_weight_update(void* Wt, const float* dW, int64_t n, float lr, int dt, void* stream) {
  if (dt != SURGEON_F32 && dt != SURGEON_BF16) return fail(SURGEON_EINVAL, "weight_update: bad dtype %d", dt);
  if (n < 0 || !(lr == lr)) return fail(SURGEON_EINVAL, "weight_update: bad arguments");
  if (n == 0) return SURGEON_OK;
  if (!Wt || !dW) return fail(SURGEON_EINVAL, "weight_update: null pointer");
  if (((uintptr_t)Wt % (dt == SURGEON_F32 ? 4 : 2)) || ((uintptr_t)dW % 4)) return fail(SURGEON_EINVAL, "weight_update: misaligned pointer");
  const int blocks = (int)std::min<int64_t>(ceil_div(n, 256), 8192);
  hipStream_t st = (hipStream_t)stream;
  ProfScope prof(SURGEON_PROF_UPDATE, st);
  if (dt == SURGEON_F32)
    SURGEON_LAUNCH(weight_update_kernel<float>, dim3(blocks), dim3(256), 0, st, (float*)Wt, dW, n, lr);
  else
    SURGEON_LAUNCH(weight_update_kernel<uint16_t>, dim3(blocks), dim3(256), 0, st, (uint16_t*)Wt, dW, n, lr);
  SURGEON_LAUNCH_CHECK();
  return SURGEON_OK;
}
