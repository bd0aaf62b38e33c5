// C entry points of the weight gradient from the packed activation (Eq. 2, Alg. 1 lines 11-12).
// The kernels and the host planning live in dw_impl.hpp; run_dw<float> and run_dw<uint16_t> are instantiated in
// dw_f32.hip and dw_bf16in.hip so that the two sets of kernel variants compile in parallel.
#include "dw_impl.hpp"

namespace surgeon {
extern template int run_dw<float>(const DwPlan&, const surgeon_layer_desc*, const void*, const uint64_t*, const void*, float*,
                                  void*, hipStream_t);
extern template int run_dw<uint16_t>(const DwPlan&, const surgeon_layer_desc*, const void*, const uint64_t*, const void*,
                                     float*, void*, hipStream_t);
}  // namespace surgeon

using namespace surgeon;

extern "C" int surgeon_dw_ws_bytes(const surgeon_layer_desc* desc, size_t* ws_bytes) {
  if (!ws_bytes) return fail(SURGEON_EINVAL, "dw_ws_bytes: null pointer");
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
  DwPlan p;
  const int rc = plan_dw(desc, &p);
  if (rc != SURGEON_OK) return rc;
  *kernel_class = (p.conv && p.c.sparse) ? SURGEON_PROF_DW_SPARSE : SURGEON_PROF_DW;
  return SURGEON_OK;
}

extern "C" int surgeon_dw_from_packed(const surgeon_layer_desc* desc, const void* vals, const uint64_t* mask,
                                      const void* dY, float* dW, void* ws, size_t ws_bytes, void* stream) {
  DwPlan p;
  const int rc = plan_dw(desc, &p);
  if (rc != SURGEON_OK) return rc;
  if (!dW) return fail(SURGEON_EINVAL, "dw_from_packed: null dW");
  if (p.n > 0 && desc->k_total > 0 && (!vals || !mask || !dY)) return fail(SURGEON_EINVAL, "dw_from_packed: null pointer");
  if (p.ws_bytes > 0 && (!ws || ws_bytes < p.ws_bytes))
    return fail(SURGEON_ESIZE, "dw_from_packed: workspace of %zu bytes needed, %zu given", p.ws_bytes, ws_bytes);
  if (((uintptr_t)ws % 16) || ((uintptr_t)mask % 8) || ((uintptr_t)dW % 4) || ((uintptr_t)dY % 16) ||
      ((uintptr_t)vals % (desc->dtype == SURGEON_F32 ? 4 : 2)))
    return fail(SURGEON_EINVAL, "dw_from_packed: misaligned pointer");
  hipStream_t st = (hipStream_t)stream;
  if (desc->dtype == SURGEON_F32) return run_dw<float>(p, desc, vals, mask, dY, dW, ws, st);
  return run_dw<uint16_t>(p, desc, vals, mask, dY, dW, ws, st);
}
