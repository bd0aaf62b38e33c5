// Gradient Importance (Eq. 4): G = sqrt( sum_j dW_j^2 / n_w ), an HBM-bound reduction.
//
// One pass over dW with 16-byte loads; squares are accumulated in fp64 (full-rate on CDNA) so the result
// does not depend on n_w's size; partial sums are combined in a fixed order, so the result is reproducible.
#include <algorithm>
#include <atomic>

#include "common.hpp"

namespace surgeon {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kImpBlock = 256;
constexpr int kImpMaxBlocks = 2048;
constexpr int kImpPerThread = 16;  // floats per thread per grid-stride step (4 x float4)

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
  return v;
}

// block-wide sum in a fixed order; valid in thread 0
__device__ __forceinline__ double block_sum(double v, double* lds) {
  v = wave_sum(v);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) lds[wave] = v;
  __syncthreads();
  double total = 0.0;
  if (threadIdx.x == 0) {
    for (int w = 0; w < kImpBlock / 64; ++w) total += lds[w];
  }
  return total;
}

template <bool VEC4>
__device__ __forceinline__ double thread_sumsq(const float* __restrict__ x, int64_t n) {
  double acc0 = 0.0, acc1 = 0.0, acc2 = 0.0, acc3 = 0.0;
  const int64_t tid = (int64_t)blockIdx.x * kImpBlock + threadIdx.x;
  const int64_t nthreads = (int64_t)gridDim.x * kImpBlock;
  if (VEC4) {
    const f32x4* x4 = reinterpret_cast<const f32x4*>(x);
    const int64_t n4 = n >> 2;
    int64_t i = tid;
    // four independent 16-byte loads in flight per thread
    for (; i + 3 * nthreads < n4; i += 4 * nthreads) {
      const f32x4 a = __builtin_nontemporal_load(&x4[i]);
      const f32x4 b = __builtin_nontemporal_load(&x4[i + nthreads]);
      const f32x4 c = __builtin_nontemporal_load(&x4[i + 2 * nthreads]);
      const f32x4 d = __builtin_nontemporal_load(&x4[i + 3 * nthreads]);
      acc0 += (double)a.x * a.x + (double)a.y * a.y + (double)a.z * a.z + (double)a.w * a.w;
      acc1 += (double)b.x * b.x + (double)b.y * b.y + (double)b.z * b.z + (double)b.w * b.w;
      acc2 += (double)c.x * c.x + (double)c.y * c.y + (double)c.z * c.z + (double)c.w * c.w;
      acc3 += (double)d.x * d.x + (double)d.y * d.y + (double)d.z * d.z + (double)d.w * d.w;
    }
    for (; i < n4; i += nthreads) {
      const f32x4 a = x4[i];
      acc0 += (double)a.x * a.x + (double)a.y * a.y + (double)a.z * a.z + (double)a.w * a.w;
    }
    for (int64_t j = (n4 << 2) + tid; j < n; j += nthreads) acc1 += (double)x[j] * x[j];
  } else {
    for (int64_t j = tid; j < n; j += nthreads) acc0 += (double)x[j] * x[j];
  }
  return (acc0 + acc1) + (acc2 + acc3);
}

template <bool VEC4>
__global__ __launch_bounds__(kImpBlock) void sumsq_partial_kernel(const float* __restrict__ x, int64_t n,
                                                                  double* __restrict__ partial) {
  __shared__ double lds[kImpBlock / 64];
  const double total = block_sum(thread_sumsq<VEC4>(x, n), lds);
  if (threadIdx.x == 0) partial[blockIdx.x] = total;
}

// one block: adds the per-block partials in index order and finishes Eq. 4
__global__ __launch_bounds__(kImpBlock) void sumsq_final_kernel(const double* __restrict__ partial, int n_partial,
                                                                int64_t n, float* __restrict__ out) {
  __shared__ double lds[kImpBlock / 64];
  double acc = 0.0;
  for (int i = threadIdx.x; i < n_partial; i += kImpBlock) acc += partial[i];
  const double total = block_sum(acc, lds);
  if (threadIdx.x == 0) out[0] = (float)sqrt(total / (double)n);
}

// small layers: a single block does both steps
template <bool VEC4>
__global__ __launch_bounds__(kImpBlock) void sumsq_single_kernel(const float* __restrict__ x, int64_t n,
                                                                 float* __restrict__ out) {
  __shared__ double lds[kImpBlock / 64];
  const double total = block_sum(thread_sumsq<VEC4>(x, n), lds);
  if (threadIdx.x == 0) out[0] = n > 0 ? (float)sqrt(total / (double)n) : 0.0f;
}

static int importance_blocks(int64_t n_w) {
  int64_t b = ceil_div(n_w, (int64_t)kImpBlock * kImpPerThread);
  if (b < 1) b = 1;
  if (b > kImpMaxBlocks) b = kImpMaxBlocks;
  return (int)b;
}

// ---- all layers in one launch --------------------------------------------------------------------------
constexpr int kImpBatch = 64;           // layers per launch (their descriptors travel as kernel arguments)
constexpr int kImpChunk = 16384;        // elements per workgroup

struct ImpBatch {
  const float* ptr[kImpBatch];
  int64_t n[kImpBatch];
  int first_block[kImpBatch + 1];  // workgroups [first_block[i], first_block[i+1]) belong to layer i
  int layers;
};

template <bool VEC4>
__global__ __launch_bounds__(kImpBlock) void sumsq_batched_partial_kernel(ImpBatch bt, double* __restrict__ partial) {
  __shared__ double lds[kImpBlock / 64];
  // the layer of this workgroup = the last layer boundary at or below its index (entries past the last layer hold
  // the total, which no index reaches), by a branch-free binary search: six dependent scalar loads.  Counting
  // independent compares over the whole table compiles to a compare, a select and a lane read per entry.
  int layer = 0;
#pragma unroll
  for (int step = kImpBatch / 2; step >= 1; step >>= 1) {
    const int c = layer + step;  // <= kImpBatch - 1
    layer = (int)blockIdx.x >= bt.first_block[c] ? c : layer;
  }
  const float* __restrict__ x = bt.ptr[layer];
  const int64_t begin = (int64_t)((int)blockIdx.x - bt.first_block[layer]) * kImpChunk;
  const int64_t end = min(begin + kImpChunk, bt.n[layer]);
  double acc0 = 0.0, acc1 = 0.0;
  if (VEC4) {
    // begin is a multiple of 4 and x is 16-byte aligned: whole float4s, then the tail
    const f32x4* x4 = reinterpret_cast<const f32x4*>(x + begin);
    const int64_t n4 = (end - begin) >> 2;
    // a full chunk is 16 float4 per thread: all of them are in flight before the first is consumed
    constexpr int kInFlight = kImpChunk / 4 / kImpBlock;
    f32x4 v[kInFlight];
#pragma unroll
    for (int q = 0; q < kInFlight; ++q) {
      const int64_t i = threadIdx.x + (int64_t)q * kImpBlock;
      v[q] = __builtin_nontemporal_load(&x4[i < n4 ? i : 0]);  // unconditional: loads must not serialise
      if (i >= n4) v[q] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int q = 0; q < kInFlight; q += 2) {
      acc0 += (double)v[q].x * v[q].x + (double)v[q].y * v[q].y + (double)v[q].z * v[q].z + (double)v[q].w * v[q].w;
      acc1 += (double)v[q + 1].x * v[q + 1].x + (double)v[q + 1].y * v[q + 1].y + (double)v[q + 1].z * v[q + 1].z +
              (double)v[q + 1].w * v[q + 1].w;
    }
    for (int64_t j = begin + (n4 << 2) + threadIdx.x; j < end; j += kImpBlock) acc0 += (double)x[j] * x[j];
  } else {
    for (int64_t j = begin + threadIdx.x; j < end; j += kImpBlock) acc0 += (double)x[j] * x[j];
  }
  const double total = block_sum(acc0 + acc1, lds);
  if (threadIdx.x == 0) partial[blockIdx.x] = total;
}

// one workgroup per layer: adds that layer's partials in index order and finishes Eq. 4
__global__ __launch_bounds__(kImpBlock) void sumsq_batched_final_kernel(ImpBatch bt, const double* __restrict__ partial,
                                                                        float* __restrict__ out) {
  __shared__ double lds[kImpBlock / 64];
  const int layer = blockIdx.x;
  double acc = 0.0;
  for (int i = bt.first_block[layer] + threadIdx.x; i < bt.first_block[layer + 1]; i += kImpBlock) acc += partial[i];
  const double total = block_sum(acc, lds);
  if (threadIdx.x == 0) out[layer] = bt.n[layer] > 0 ? (float)sqrt(total / (double)bt.n[layer]) : 0.0f;
}

static int64_t batched_blocks(int64_t n_w) { return n_w > 0 ? ceil_div(n_w, kImpChunk) : 0; }

// ---- partial sums of surgeon_grad_importance_static: device memory that belongs to the library image ----------
// One copy per GPU the library runs on (16 KB each, held until the process ends).  In host code the array's name
// is only a handle: its device address comes from hipGetSymbolAddress, once per device, and only that address is
// ever passed to a kernel.
static __device__ __align__(256) double scratch[kImpMaxBlocks];
constexpr int kMaxDevices = 64;
static std::atomic<double*> g_scratch_addr[kMaxDevices];

static int scratch_of_current_device(double** out) {
  int dev = -1;
  SURGEON_HIP_CHECK(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(SURGEON_EUNSUPPORTED, "grad_importance_static: device %d", dev);
  double* p = g_scratch_addr[dev].load(std::memory_order_acquire);
  if (!p) {
    SURGEON_HIP_CHECK(hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(SURGEON_EHIP, "grad_importance_static: no device address for the scratch array");
    g_scratch_addr[dev].store(p, std::memory_order_release);  // every thread resolves the same address: a race is benign
  }
  *out = p;
  return SURGEON_OK;
}

int launch_sumsq_final(const double* partial, int n_partial, int64_t n, float* G_out, hipStream_t st) {
  ProfScope prof(SURGEON_PROF_IMPORTANCE, st);
  SURGEON_LAUNCH(sumsq_final_kernel, dim3(1), dim3(kImpBlock), 0, st, partial, n_partial, n, G_out);
  SURGEON_LAUNCH_CHECK();
  return SURGEON_OK;
}

int launch_sumsq(const float* x, int64_t n, double* partial, float* G_out, hipStream_t st) {
  const bool vec4 = ((uintptr_t)x & 15) == 0;
  const int nb = importance_blocks(n);
  ProfScope prof(SURGEON_PROF_IMPORTANCE, st);
  if (nb == 1) {
    if (vec4)
      SURGEON_LAUNCH(sumsq_single_kernel<true>, dim3(1), dim3(kImpBlock), 0, st, x, n, G_out);
    else
      SURGEON_LAUNCH(sumsq_single_kernel<false>, dim3(1), dim3(kImpBlock), 0, st, x, n, G_out);
    SURGEON_LAUNCH_CHECK();
    return SURGEON_OK;
  }
  if (vec4)
    SURGEON_LAUNCH(sumsq_partial_kernel<true>, dim3(nb), dim3(kImpBlock), 0, st, x, n, partial);
  else
    SURGEON_LAUNCH(sumsq_partial_kernel<false>, dim3(nb), dim3(kImpBlock), 0, st, x, n, partial);
  SURGEON_LAUNCH_CHECK();
  SURGEON_LAUNCH(sumsq_final_kernel, dim3(1), dim3(kImpBlock), 0, st, (const double*)partial, nb, n, G_out);
  SURGEON_LAUNCH_CHECK();
  return SURGEON_OK;
}

}  // namespace surgeon

using namespace surgeon;

extern "C" size_t surgeon_grad_importance_ws_bytes(int64_t n_w) {
  if (n_w < 0) return 0;
  const int nb = importance_blocks(n_w);
  return nb > 1 ? align_up((size_t)nb * sizeof(double), 256) : 0;
}

extern "C" int surgeon_grad_importance(const float* dW, int64_t n_w, float* G_out, void* ws, size_t ws_bytes,
                                       void* stream) {
  if (n_w < 0) return fail(SURGEON_EINVAL, "grad_importance: n_w = %lld", (long long)n_w);
  if (!G_out || (n_w > 0 && !dW)) return fail(SURGEON_EINVAL, "grad_importance: null pointer");
  if (((uintptr_t)dW & 3) != 0) return fail(SURGEON_EINVAL, "grad_importance: dW is not 4-byte aligned");
  const size_t need = surgeon_grad_importance_ws_bytes(n_w);
  if (need > 0 && (!ws || ws_bytes < need))
    return fail(SURGEON_ESIZE, "grad_importance: workspace of %zu bytes needed, %zu given", need, ws_bytes);
  hipStream_t st = (hipStream_t)stream;
  const bool vec4 = ((uintptr_t)dW & 15) == 0;
  const int nb = importance_blocks(n_w);
  ProfScope prof(SURGEON_PROF_IMPORTANCE, st);
  if (nb == 1) {
    if (vec4)
      SURGEON_LAUNCH(sumsq_single_kernel<true>, dim3(1), dim3(kImpBlock), 0, st, dW, n_w, G_out);
    else
      SURGEON_LAUNCH(sumsq_single_kernel<false>, dim3(1), dim3(kImpBlock), 0, st, dW, n_w, G_out);
    SURGEON_LAUNCH_CHECK();
    return SURGEON_OK;
  }
  double* partial = (double*)ws;
  if (vec4)
    SURGEON_LAUNCH(sumsq_partial_kernel<true>, dim3(nb), dim3(kImpBlock), 0, st, dW, n_w, partial);
  else
    SURGEON_LAUNCH(sumsq_partial_kernel<false>, dim3(nb), dim3(kImpBlock), 0, st, dW, n_w, partial);
  SURGEON_LAUNCH_CHECK();
  SURGEON_LAUNCH(sumsq_final_kernel, dim3(1), dim3(kImpBlock), 0, st, (const double*)partial, nb, n_w, G_out);
  SURGEON_LAUNCH_CHECK();
  return SURGEON_OK;
}

extern "C" size_t surgeon_grad_importance_batched_ws_bytes(const int64_t* n_w, int l) {
  if (!n_w || l < 1) return 0;
  int64_t most = 0;
  for (int i0 = 0; i0 < l; i0 += kImpBatch) {
    int64_t blocks = 0;
    for (int i = i0; i < l && i < i0 + kImpBatch; ++i) blocks += batched_blocks(n_w[i]);
    most = std::max(most, blocks);
  }
  return align_up((size_t)std::max<int64_t>(most, 1) * sizeof(double), 256);
}

extern "C" int surgeon_grad_importance_batched(const float* const* dW, const int64_t* n_w, int l, float* G_out, void* ws,
                                               size_t ws_bytes, void* stream) {
  if (!dW || !n_w || !G_out) return fail(SURGEON_EINVAL, "grad_importance_batched: null pointer");
  if (l < 1) return fail(SURGEON_EINVAL, "grad_importance_batched: l = %d", l);
  bool vec4 = true;
  for (int i = 0; i < l; ++i) {
    if (n_w[i] < 0 || (n_w[i] > 0 && !dW[i])) return fail(SURGEON_EINVAL, "grad_importance_batched: bad layer %d", i);
    if ((uintptr_t)dW[i] & 3) return fail(SURGEON_EINVAL, "grad_importance_batched: dW[%d] is not 4-byte aligned", i);
    if ((uintptr_t)dW[i] & 15) vec4 = false;
  }
  const size_t need = surgeon_grad_importance_batched_ws_bytes(n_w, l);
  if (!ws || ws_bytes < need)
    return fail(SURGEON_ESIZE, "grad_importance_batched: workspace of %zu bytes needed, %zu given", need, ws_bytes);
  hipStream_t st = (hipStream_t)stream;
  ProfScope prof(SURGEON_PROF_IMPORTANCE, st);
  for (int i0 = 0; i0 < l; i0 += kImpBatch) {
    ImpBatch bt;
    bt.layers = std::min(kImpBatch, l - i0);
    int64_t blocks = 0;
    for (int i = 0; i < kImpBatch; ++i) {
      bt.first_block[i] = (int)blocks;
      bt.ptr[i] = i < bt.layers ? dW[i0 + i] : nullptr;
      bt.n[i] = i < bt.layers ? n_w[i0 + i] : 0;
      blocks += batched_blocks(bt.n[i]);
      if (blocks > 0x7fffffff) return fail(SURGEON_EUNSUPPORTED, "grad_importance_batched: too many elements");
    }
    bt.first_block[kImpBatch] = (int)blocks;
    for (int i = bt.layers; i <= kImpBatch; ++i) bt.first_block[i] = (int)blocks;
    double* partial = (double*)ws;
    if (blocks > 0) {
      if (vec4)
        SURGEON_LAUNCH(sumsq_batched_partial_kernel<true>, dim3((unsigned)blocks), dim3(kImpBlock), 0, st, bt, partial);
      else
        SURGEON_LAUNCH(sumsq_batched_partial_kernel<false>, dim3((unsigned)blocks), dim3(kImpBlock), 0, st, bt, partial);
      SURGEON_LAUNCH_CHECK();
    }
    SURGEON_LAUNCH(sumsq_batched_final_kernel, dim3((unsigned)bt.layers), dim3(kImpBlock), 0, st, bt,
                       (const double*)partial, G_out + i0);
    SURGEON_LAUNCH_CHECK();
  }
  return SURGEON_OK;
}

extern "C" int surgeon_grad_importance_static(const float* dW, int64_t n_w, float* G_out, void* stream) {
  if (n_w < 0) return fail(SURGEON_EINVAL, "grad_importance_static: n_w = %lld", (long long)n_w);
  if (n_w > ((int64_t)1 << 31))
    return fail(SURGEON_EUNSUPPORTED, "grad_importance_static: n_w = %lld exceeds the limit of 2^31 elements",
                (long long)n_w);
  if (!G_out || (n_w > 0 && !dW)) return fail(SURGEON_EINVAL, "grad_importance_static: null pointer");
  if (((uintptr_t)dW & 3) != 0) return fail(SURGEON_EINVAL, "grad_importance_static: dW is not 4-byte aligned");
  double* partial = nullptr;
  const int rc = scratch_of_current_device(&partial);
  if (rc != SURGEON_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  const bool vec4 = ((uintptr_t)dW & 15) == 0;
  const int nb = importance_blocks(n_w);
  ProfScope prof(SURGEON_PROF_IMPORTANCE, st);
  if (nb == 1) {
    if (vec4)
      SURGEON_LAUNCH(sumsq_single_kernel<true>, dim3(1), dim3(kImpBlock), 0, st, dW, n_w, G_out);
    else
      SURGEON_LAUNCH(sumsq_single_kernel<false>, dim3(1), dim3(kImpBlock), 0, st, dW, n_w, G_out);
    SURGEON_LAUNCH_CHECK();
    return SURGEON_OK;
  }
  // every one of the nb partials is written before the finishing kernel reads exactly nb of them: nothing of the
  // previous call's contents is ever read, so the array needs no clearing
  if (vec4)
    SURGEON_LAUNCH(sumsq_partial_kernel<true>, dim3(nb), dim3(kImpBlock), 0, st, dW, n_w, partial);
  else
    SURGEON_LAUNCH(sumsq_partial_kernel<false>, dim3(nb), dim3(kImpBlock), 0, st, dW, n_w, partial);
  SURGEON_LAUNCH_CHECK();
  SURGEON_LAUNCH(sumsq_final_kernel, dim3(1), dim3(kImpBlock), 0, st, (const double*)partial, nb, n_w, G_out);
  SURGEON_LAUNCH_CHECK();
  return SURGEON_OK;
}
