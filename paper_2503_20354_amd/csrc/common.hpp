// Internal helpers shared by the translation units of libsurgeon (gfx950 only; not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <algorithm>
#include <atomic>
#include <stdint.h>
#include <stdio.h>

#include "surgeon.h"

namespace surgeon {

// thread-local error text behind surgeon_last_error()
void set_error(const char* fmt, ...);
int fail(int status, const char* fmt, ...);

#define SURGEON_HIP_CHECK(expr)                                                                   \
  do {                                                                                            \
    hipError_t e_ = (expr);                                                                       \
    if (e_ != hipSuccess)                                                                         \
      return ::surgeon::fail(SURGEON_EHIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), \
                             __FILE__, __LINE__);                                                 \
  } while (0)

// launch check: catches bad launch configurations without synchronising
#define SURGEON_LAUNCH_CHECK() SURGEON_HIP_CHECK(hipGetLastError())

// Kernel timing aid (surgeon_profile_begin/end).  A ProfScope names the kernel class of the launches inside its
// scope; while profiling is on, SURGEON_LAUNCH attaches a start and a stop event to each kernel it launches (the
// events ride on the kernel's own dispatch packet: no extra packets between kernels), else it is a plain launch.
struct ProfScope {
  ProfScope(int kind, hipStream_t stream);
  ~ProfScope();
  int prev_;
};
// While one lives, the launches of this thread are booked under `kind` whatever class their own ProfScope names (a
// kernel shared by two entry points is then timed with the entry point that called it).
struct ProfForce {
  explicit ProfForce(int kind);
  ~ProfForce();
  int prev_;
};
// true while profiling is on and a class is current: hands out the two events of the next kernel
bool prof_next_events(hipEvent_t* start, hipEvent_t* stop);

#define SURGEON_LAUNCH(kernel, grid, block, shmem, st, ...)                                              \
  do {                                                                                                    \
    hipEvent_t prof_e0_, prof_e1_;                                                                        \
    if (surgeon::prof_next_events(&prof_e0_, &prof_e1_))                                                  \
      hipExtLaunchKernelGGL(kernel, grid, block, shmem, st, prof_e0_, prof_e1_, 0, __VA_ARGS__);         \
    else                                                                                                  \
      hipLaunchKernelGGL(kernel, grid, block, shmem, st, __VA_ARGS__);                                    \
  } while (0)

// Work item (x, y) of the calling workgroup for kernels whose grid is (tiles, splits) and whose tiles of one split read
// the same rows of the operands.  Workgroups go to the chip's eight XCDs (each with its own L2) round-robin in dispatch
// order; here work item w = y * gridDim.x + x is handed out so that each XCD gets a run of consecutive w, i.e. whole
// splits: its L2 then fetches a split's rows once for all of its tiles instead of once per XCD.  A bijection of the
// grid onto itself for any grid size.
#if defined(__HIPCC__)
__device__ __forceinline__ void xcd_ordered_work_item(int* x, int* y) {
  const uint32_t nx = gridDim.x, total = gridDim.x * gridDim.y;
  const uint32_t b = blockIdx.y * gridDim.x + blockIdx.x;
  const uint32_t xcd = b & 7u, j = b >> 3, base = total >> 3, rem = total & 7u;
  const uint32_t w = xcd * base + (xcd < rem ? xcd : rem) + j;
  *x = (int)(w % nx);
  *y = (int)(w / nx);
}
#endif

// Raises a kernel's dynamic-LDS limit once per (kernel, device): the attribute belongs to the device, the flag word is
// one bit per device and is only ever OR-ed into, so host threads that race here at worst set the attribute twice.
// `done` is a static of the calling launch function (one per kernel).
inline int ensure_dynamic_lds(const void* kernel, size_t bytes, std::atomic<uint64_t>& done) {
  int dev = 0;
  SURGEON_HIP_CHECK(hipGetDevice(&dev));
  const uint64_t bit = 1ull << (dev & 63);
  if (done.load(std::memory_order_acquire) & bit) return SURGEON_OK;
  SURGEON_HIP_CHECK(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
  done.fetch_or(bit, std::memory_order_release);
  return SURGEON_OK;
}

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---- layout of the packed-sizes arithmetic, shared by host entry points ----
struct GroupPlan {
  int64_t n, g, n_groups, len_last, k_full, k_last, k_total;
};
// returns false when (n, group_len, r) is invalid
bool make_group_plan(int64_t n, int64_t group_len, float r, GroupPlan* p);

// workspace of the large-group (multi-kernel radix select) path of prune_pack; 0 for the in-register path
size_t prune_pack_ws_bytes(const GroupPlan& p);
// copies of a group's digit histogram in the large-group path (spreads the atomics of many workgroups)
int global_hist_replicas(const GroupPlan& p);

// selection paths of prune_pack
enum PrunePath { PATH_WAVE_REG = 0, PATH_WAVE_MEM = 1, PATH_GLOBAL = 2, PATH_TWO_READ = 3 };
PrunePath choose_prune_path(const GroupPlan& p);

// bf16 linear weight gradient: un-pack to a dense transient copy, then a dense bf16-MFMA contraction (dw_bf16.hip)
int launch_unpack_dense(int dtype, const void* vals, const uint64_t* mask, const uint32_t* word_rank, int64_t n,
                        int64_t k_total, void* dense, hipStream_t st);
int launch_unpack_grouped(const void* vals, const uint64_t* mask, int64_t n_words, int words_per_group, int64_t n_groups,
                          int64_t k_full, int64_t n, int64_t k_total, void* dense, hipStream_t st);
int launch_linear_bf16(int64_t M, int64_t K, int64_t N, const void* A_dense, const void* dY, float* out, int splits,
                       int64_t rows_per_split, int wide, hipStream_t st);
int launch_conv1x1_bf16(int Nb, int Ci, int Co, int HW, const void* A_dense, const void* dY, float* out, int splits,
                        int64_t ktiles_per_split, hipStream_t st);
// dense bf16 contraction with a 256 (out) x 128 (in) workgroup tile of eight wavefronts and LDS-direct loads, for layers
// that fill it (dw_bf16.hip)
// bf16_out: `out` is a bf16 matrix [N x K] that the kernel writes itself (needs splits == 1)
int launch_linear_bf16_big(int64_t M, int64_t K, int64_t N, const void* A_dense, const void* dY, float* out, int splits,
                           int64_t rows_per_split, hipStream_t st, bool bf16_out = false);
// activation gradient of a bf16 1x1 convolution (pad 0, stride 1 or 2) on the same matrix-core contraction, one image
// per grid z (dw_bf16.hip); Nb <= 65535
int launch_da_conv1x1_bf16(int Nb, int Ci, int Co, int H, int W, int stride, const void* Wt, const void* dY, void* dA,
                           hipStream_t st);
// activation gradient of a bf16 linear layer with dY read in place (dw_bf16.hip); N % 8 == 0, dY 16-byte aligned
int launch_da_linear_bf16(int64_t M, int64_t K, int64_t N, const void* dY, const void* Wt, void* dA, hipStream_t st);
constexpr int kBf16BigTileO = 256, kBf16BigTileI = 128, kBf16BigTokens = 64;
constexpr int kBf16LinearTile = 128, kBf16LinearTokens = 64;          // 128 x 128 tile, 64 tokens per K-tile
constexpr int kBf16LinearTileWide = 256, kBf16LinearTokensWide = 32;  // 128 (out) x 256 (in) tile, 32 tokens

// 3x3 stride-1 pad-1 fp32 convolutions with few kept elements: weight gradient from the kept elements alone
// (dw_sparse.hip).  One workgroup = 64 output channels x (waves x kSparseCiPerWave) input channels, with 8 or 16
// wavefronts (32 or 64 input channels) chosen per layer.
constexpr int kSparseCo = 64, kSparseCiPerWave = 4;
// wavefronts per workgroup for a layer with Ci input channels: the largest channel tile that pads Ci the least
int sparse_conv_waves(int Ci);
// workgroups of that size resident on the chip at once (LDS: 3 per compute unit; 32 wavefronts per compute unit)
inline int sparse_conv_slots(int waves) { return (waves > 8 ? 2 : 3) * 256; }
int sparse_conv_band_rows(int W);  // input rows per staged band for a map of width W (8, 16 or 32)
int launch_conv3x3_sparse_f32(int Nb, int Ci, int Co, int H, int W, int64_t k_total, int splits, int tiles_per_split,
                              const void* vals, const uint64_t* mask, const uint32_t* word_rank, const void* dY, float* out,
                              hipStream_t st);

// Eq. 4 folded into the weight-gradient call: fp64 partial sums of squares, at most kGiPartials of them (importance.hip)
constexpr int kGiPartials = 8192;
// sqrt(sum of the n_partial partials / n) -> G_out[0]
int launch_sumsq_final(const double* partial, int n_partial, int64_t n, float* G_out, hipStream_t st);
// Eq. 4 of x[0..n): partial sums into `partial` (kGiPartials doubles of scratch), then the finishing kernel
int launch_sumsq(const float* x, int64_t n, double* partial, float* G_out, hipStream_t st);

// weight gradient of convolutions with channel groups (layers.hip).  run_grouped validates, sizes and launches;
// plan_only: validation and *off_gi (offset of the Gradient Importance partials behind its workspace) only.
int grouped_ws_bytes(const surgeon_layer_desc* d, size_t* bytes);
int run_grouped(const surgeon_layer_desc* d, const void* vals, const uint64_t* mask, const void* dY, float* dW, void* ws,
                size_t ws_bytes, hipStream_t st, float* G_out, size_t* off_gi, bool plan_only);

constexpr int kWaveRegMaxGroup = 4096;  // largest group one wavefront keeps in registers (64 lanes x 64)
constexpr int kGlobalHistChunk = 16384;  // elements per block in the histogram passes of the global path
constexpr int kGlobalWaveChunk = 4096;   // elements per wavefront in the count / pack passes of the global path
constexpr int kGlobalDigitBits = 11;     // key bits resolved per histogram pass
constexpr int kGlobalHistBins = 1 << kGlobalDigitBits;
constexpr int kTwoReadMinGroup = 32768;   // shortest group that takes the sampled two-read selection
constexpr int kTwoReadSlotKeys = 1024;    // candidate keys kept per 4096-element chunk on that path

}  // namespace surgeon
