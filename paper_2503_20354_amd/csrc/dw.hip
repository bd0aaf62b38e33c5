// C entry points of the weight gradient from the packed activation (Eq. 2, Alg. 1 lines 11-12).
// The kernels and the host planning live in dw_impl.hpp; run_dw<float> and run_dw<uint16_t> are instantiated in
// dw_f32.hip and dw_bf16in.hip so that the two sets of kernel variants compile in parallel.
#include "dw_impl.hpp"

namespace surgeon {
extern template int run_dw<float>(const DwPlan&, const surgeon_layer_desc*, const void*, const uint64_t*, const void*, float*,
                                  void*, hipStream_t, float*, double*);
extern template int run_dw<uint16_t>(const DwPlan&, const surgeon_layer_desc*, const void*, const uint64_t*, const void*,
                                     float*, void*, hipStream_t, float*, double*);
}  // namespace surgeon

using namespace surgeon;

static bool is_grouped(const surgeon_layer_desc* desc) {
  return desc && desc->kind == SURGEON_CONV2D && desc->groups > 1;
}

extern "C" int surgeon_dw_ws_bytes(const surgeon_layer_desc* desc, size_t* ws_bytes) {
  if (!ws_bytes) return fail(SURGEON_EINVAL, "dw_ws_bytes: null pointer");
  if (is_grouped(desc)) return grouped_ws_bytes(desc, ws_bytes);
  // the kernel is chosen per call from k_total: size the workspace for either choice, so that one query covers
  // every prune ratio the layer will see
  DwPlan p, q;
  int rc = plan_dw(desc, &p, SPARSE_NEVER);
  if (rc != SURGEON_OK) return rc;
  rc = plan_dw(desc, &q, SPARSE_IF_SHAPE_ALLOWS);
  if (rc != SURGEON_OK) return rc;
  *ws_bytes = std::max(p.ws_bytes, q.ws_bytes);
  return SURGEON_OK;
}

extern "C" int surgeon_dw_kernel_class(const surgeon_layer_desc* desc, int* kernel_class) {
  if (!kernel_class) return fail(SURGEON_EINVAL, "dw_kernel_class: null pointer");
  if (is_grouped(desc)) {
    size_t unused;
    const int rc = grouped_ws_bytes(desc, &unused);
    if (rc == SURGEON_OK) *kernel_class = SURGEON_PROF_DW_GROUPED;
    return rc;
  }
  DwPlan p;
  const int rc = plan_dw(desc, &p);
  if (rc != SURGEON_OK) return rc;
  *kernel_class = (p.conv && p.c.sparse) ? SURGEON_PROF_DW_SPARSE : SURGEON_PROF_DW;
  return SURGEON_OK;
}

// shared body of surgeon_dw_from_packed and surgeon_dw_from_packed_gi (G_out == nullptr: no Gradient Importance)
static int dw_entry(const char* who, const surgeon_layer_desc* desc, const void* vals, const uint64_t* mask, const void* dY,
                    float* dW, float* G_out, void* ws, size_t ws_bytes, void* stream) {
  if (is_grouped(desc)) {
    if (desc->dtype != SURGEON_F32 && desc->dtype != SURGEON_BF16) return fail(SURGEON_EINVAL, "%s: bad dtype", who);
    if (!dW || (desc->k_total > 0 && (!vals || !mask || !dY))) return fail(SURGEON_EINVAL, "%s: null pointer", who);
    if (((uintptr_t)ws % 16) || ((uintptr_t)mask % 8) || ((uintptr_t)dW % 4) || ((uintptr_t)G_out % 4) ||
        ((uintptr_t)dY % (desc->dtype == SURGEON_F32 ? 4 : 2)) || ((uintptr_t)vals % (desc->dtype == SURGEON_F32 ? 4 : 2)))
      return fail(SURGEON_EINVAL, "%s: misaligned pointer", who);
    return run_grouped(desc, vals, mask, dY, dW, ws, ws_bytes, (hipStream_t)stream, G_out, nullptr, false);
  }
  DwPlan p;
  const int rc = plan_dw(desc, &p);
  if (rc != SURGEON_OK) return rc;
  if (!dW) return fail(SURGEON_EINVAL, "%s: null dW", who);
  if (p.n > 0 && desc->k_total > 0 && (!vals || !mask || !dY)) return fail(SURGEON_EINVAL, "%s: null pointer", who);
  // the partial sums of squares follow the weight gradient's own workspace
  const size_t off_gi = align_up(p.ws_bytes, 256);
  const size_t need = G_out ? off_gi + (size_t)kGiPartials * sizeof(double) : p.ws_bytes;
  if (need > 0 && (!ws || ws_bytes < need))
    return fail(SURGEON_ESIZE, "%s: workspace of %zu bytes needed, %zu given", who, need, ws_bytes);
  if (((uintptr_t)ws % 16) || ((uintptr_t)mask % 8) || ((uintptr_t)dW % 4) || ((uintptr_t)dY % 16) ||
      ((uintptr_t)G_out % 4) || ((uintptr_t)vals % (desc->dtype == SURGEON_F32 ? 4 : 2)))
    return fail(SURGEON_EINVAL, "%s: misaligned pointer", who);
  hipStream_t st = (hipStream_t)stream;
  double* sq_partial = G_out ? (double*)((char*)ws + off_gi) : nullptr;
  if (desc->dtype == SURGEON_F32) return run_dw<float>(p, desc, vals, mask, dY, dW, ws, st, G_out, sq_partial);
  return run_dw<uint16_t>(p, desc, vals, mask, dY, dW, ws, st, G_out, sq_partial);
}

extern "C" int surgeon_dw_from_packed(const surgeon_layer_desc* desc, const void* vals, const uint64_t* mask,
                                      const void* dY, float* dW, void* ws, size_t ws_bytes, void* stream) {
  return dw_entry("dw_from_packed", desc, vals, mask, dY, dW, nullptr, ws, ws_bytes, stream);
}

extern "C" int surgeon_dw_gi_ws_bytes(const surgeon_layer_desc* desc, size_t* ws_bytes) {
  const int rc = surgeon_dw_ws_bytes(desc, ws_bytes);
  if (rc != SURGEON_OK) return rc;
  *ws_bytes = align_up(*ws_bytes, 256) + (size_t)kGiPartials * sizeof(double);
  return SURGEON_OK;
}

extern "C" int surgeon_dw_from_packed_gi(const surgeon_layer_desc* desc, const void* vals, const uint64_t* mask,
                                         const void* dY, float* dW, float* G_out, void* ws, size_t ws_bytes,
                                         void* stream) {
  if (!G_out) return fail(SURGEON_EINVAL, "dw_from_packed_gi: null G_out");
  return dw_entry("dw_from_packed_gi", desc, vals, mask, dY, dW, G_out, ws, ws_bytes, stream);
}
