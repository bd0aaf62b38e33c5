/*
 * surgeon.h -- C ABI of the MI355X (gfx950) hot path of SURGEON's adaptation step
 * (layer-wise dynamic activation pruning, Section 4 of the paper).
 *
 * The four operations follow Algorithm 1 and Eq. 2, 4-7:
 *   - surgeon_grad_importance : Eq. 4       (RMS of one layer's weight gradient)
 *   - surgeon_layer_ratios    : Eq. 5, 6, 7 (Layer Activation Memory, combined indicator, pruning ratio)
 *   - surgeon_prune_pack      : Alg. 1 lines 6-7 (prune A_i at ratio p_i, cache as non-zero values + 1 bit/element)
 *   - surgeon_dw_from_packed  : Alg. 1 lines 11-12 with Eq. 2 (rebuild the pruned activation, weight gradient)
 *
 * Conventions shared by every entry point
 *   - "device" pointers are HIP device memory the CALLER owns; the library never allocates, frees or
 *     retains device memory.  It keeps no state between calls except: the thread-local text behind
 *     surgeon_last_error(), the event pool and records of the timing aid at the end of this header (process-wide,
 *     touched only between surgeon_profile_begin/end), the per-device address of the static array that
 *     surgeon_grad_importance_static uses, and the value of surgeon_set_select_margin.  "host" pointers are ordinary memory.
 *   - All device work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the default stream)
 *     and the call returns without synchronising.
 *   - The return value is a surgeon_status.  Argument errors are found on the host before any launch and
 *     leave every output untouched.  surgeon_last_error() returns a thread-local description.
 *   - Inputs are read-only; outputs are fully overwritten (never accumulated into).
 *   - Workspaces (`ws`) are scratch device memory whose size comes from the matching *_ws_bytes query;
 *     contents on entry are irrelevant and contents on exit are unspecified.  Pointers must be 16-byte
 *     aligned (any torch / hipMalloc allocation is).
 */
#ifndef SURGEON_H_
#define SURGEON_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SURGEON_F32 = 0,  /* IEEE binary32                                   */
  SURGEON_BF16 = 1  /* bfloat16 storage; every accumulation is in fp32 */
} surgeon_dtype;

typedef enum {
  SURGEON_OK = 0,
  SURGEON_EINVAL = 1,       /* null pointer, negative size, r outside [0,1] or NaN, group_len < 1, bad dtype */
  SURGEON_ESIZE = 2,        /* a caller buffer or workspace is too small                                    */
  SURGEON_EUNSUPPORTED = 3, /* shape / layout outside the implemented set                                   */
  SURGEON_EHIP = 4          /* a HIP runtime call failed; see surgeon_last_error()                          */
} surgeon_status;

typedef enum { SURGEON_LINEAR = 0, SURGEON_CONV2D = 1 } surgeon_layer_kind;

/* kernel classes of the timing aid at the end of this header */
enum { SURGEON_PROF_SELECT_PACK = 0, SURGEON_PROF_DW = 1, SURGEON_PROF_IMPORTANCE = 2, SURGEON_PROF_DW_AUX = 3,
       SURGEON_PROF_SELECT_OTHER = 4, SURGEON_PROF_DW_SPARSE = 5, SURGEON_PROF_DA = 6, SURGEON_PROF_UPDATE = 7,
       SURGEON_PROF_AFFINE = 8, SURGEON_PROF_DW_GROUPED = 9, SURGEON_PROF_DW_SPARSE_AUX = 10, SURGEON_PROF_CLASSES = 11 };

/*
 * Shape of one adapted layer for surgeon_dw_from_packed (Eq. 2, second line).
 *   LINEAR : cached activation A is [M tokens x K in-features] row-major, dY is [M x N out-features]
 *            row-major, dW is [N x K] row-major (the layout of a framework's `weight`; it is the
 *            transpose of Eq. 2's A^T dY).
 *   CONV2D : A is [Nb, Ci, H, W], dY is [Nb, Co, OH, OW], dW is [Co, Ci/groups, kh, kw], all contiguous NCHW
 *            (channels-last layouts are not expressible: there is no layout field),
 *            OH = (H + 2*pad - kh)/stride + 1 (same for OW); cross-correlation, zero padding, no dilation, no bias.
 *            groups (0 and 1 both mean an ordinary convolution) must divide Ci and Co; output channel co then sees
 *            input channels (co / (Co/groups)) * (Ci/groups) + [0, Ci/groups) only; groups == Ci == Co is depthwise.
 * dtype is the element type of vals and dY; dW is always fp32.
 * k_total is the number of values in the packed stream (as returned by surgeon_packed_sizes);
 * it bounds every read of `vals`.
 * group_len / r (optional hint): the arguments surgeon_prune_pack was called with for this (vals, mask); the
 * caller vouches for them.  When group_len is a multiple of 64 and at most 4096, and k_total equals the count
 * those arguments imply, every group's position in `vals` is known in closed form and a cheaper pre-pass is
 * used; the result is the same as without the hint.  A hint that does not describe the packing gives wrong
 * values (never an out-of-bounds access).  group_len = 0 means "unknown".
 */
typedef struct {
  int32_t kind;  /* surgeon_layer_kind */
  int32_t dtype; /* surgeon_dtype      */
  int64_t M, K, N;                                   /* LINEAR */
  int64_t Nb, Ci, H, W, Co, kh, kw, stride, pad;     /* CONV2D */
  int64_t k_total;
  int64_t group_len; /* 0 = unknown */
  float r;
  int64_t groups;    /* CONV2D: channel groups; 0 or 1 = ordinary convolution */
} surgeon_layer_desc;

/*
 * Number of elements kept out of `len` at prune ratio r (Alg. 1 line 6 leaves the rounding open; this
 * is the single formula both the library and its callers use):
 *     clamp( (int64) ceil( (1.0 - (double)r) * (double)len ), 0, len )
 * evaluated in IEEE double from the float32 r, no FMA contraction.  Host only.  Returns -1 if r is NaN
 * or outside [0,1] or len < 0.
 */
int64_t surgeon_keep_count(int64_t len, float r);

/*
 * Sizes of the packed form of an n-element activation pruned in groups of group_len consecutive
 * elements (the last group may be shorter).  Host only.  Any output pointer may be NULL.
 *   k_total    : sum over groups of surgeon_keep_count(len_g, r)
 *   vals_bytes : k_total * sizeof(element)
 *   mask_bytes : 8 * ceil(n / 64)
 *   ws_bytes   : workspace surgeon_prune_pack needs for this call
 */
int surgeon_packed_sizes(int64_t n, int64_t group_len, float r, int dt,
                         int64_t* k_total, size_t* vals_bytes, size_t* mask_bytes, size_t* ws_bytes);

/*
 * Eq. 5-7.  Host only; G, m, r_out are host arrays of length l.
 *   M_i = -log(m_i / sum_j m_j)                              (Eq. 5; m_i = size of A_i, caller's unit)
 *   I_i = (M_i / max_j M_j) * (G_i / max_j G_j)              (Eq. 6, max normalisation; 0/0 := 1)
 *   p_i = 1 - I_i / max_j I_j                                (Eq. 7; max I = 0 gives p = 0)
 *   r_out[i] = r_lo + (r_hi - r_lo) * p_i                    ((r_lo, r_hi) = (0, 1) is Eq. 7 itself)
 * computed in double, rounded once to float.  Errors: l < 1, null pointers, any m_i == 0, G_i negative
 * or non-finite, r_lo/r_hi outside [0,1] or r_lo > r_hi  ->  SURGEON_EINVAL.
 */
int surgeon_layer_ratios(const float* G, const uint64_t* m, int l, float r_lo, float r_hi, float* r_out);

/*
 * Alg. 1 lines 6-7: prune and pack.  A, vals, mask, idx, ws are device pointers.
 * Within every group the k_g = surgeon_keep_count(len_g, r) elements of largest magnitude are kept,
 * under the total order (key descending, index ascending) with key = the element's bit pattern with the
 * sign bit cleared, read as an unsigned integer (so +0 and -0 tie, Inf is above every finite value and
 * NaNs above Inf).  Outputs:
 *   vals : k_total elements of dtype dt, bit-exact copies of the kept elements in ascending flat index
 *          (group j's values start at element sum_{j'<j} k_j').
 *   mask : ceil(n/64) uint64 words; element e <-> bit (e % 64) of word e / 64; padding bits are 0.
 *   idx  : NULL, or k_total uint32 = offset of each kept element inside its group, same order as vals.
 * n == 0 or k_total == 0 is legal.  ws/ws_bytes as reported by surgeon_packed_sizes (ws may be NULL when
 * that size is 0).  Requires n <= 2^31 (larger: SURGEON_EUNSUPPORTED); group_len > n is treated as n.
 */
int surgeon_prune_pack(const void* A, int64_t n, int64_t group_len, float r, int dt,
                       void* vals, uint64_t* mask, uint32_t* idx,
                       void* ws, size_t ws_bytes, void* stream);

/*
 * Tuning knob of surgeon_prune_pack for groups of 32768 elements or more (the whole-tensor scope among them).  There
 * the threshold is first bracketed from a 2048-element sample, `deviations` standard deviations of the sample rank to
 * either side, so that the activation is read twice (once to count and to copy the few per cent of elements inside the
 * bracket, once to pack) instead of five times.  A bracket that misses the threshold is detected on the device and
 * the call then selects over the whole group: the result is bit-identical for every value of the knob, only the time
 * differs.  Default 5 (a miss about once in a million groups); smaller values copy fewer elements and miss more often;
 * negative values make every bracket miss (a test hook for the full-width route).  Process-wide; a call reads the
 * value once when it starts.  Host only.  Outside [-100, 100]: SURGEON_EINVAL.
 */
int surgeon_set_select_margin(float deviations);

/*
 * Benchmark aid (not part of the method): the memory pattern of the fused select+pack kernel without its selection.
 * One wavefront per group of 4096 elements issues the group's loads up front as that kernel does, keeps the elements
 * whose magnitude bits are at least `threshold_bits` (a fixed threshold instead of a search), stores them compacted
 * with the same ballot / prefix-rank walk at vals + group * k_cap (at most k_cap per group; the rest are dropped) and
 * writes the group's 64 mask words.  What this runs at is what the memory system gives that access pattern.
 * A: n elements of dt on the device, n a multiple of 4096; vals: (n / 4096) * k_cap elements; mask: n / 64 words.
 * Timed under kernel class 4 (SURGEON_PROF_SELECT_OTHER).
 */
int surgeon_select_pack_pattern_probe(const void* A, int64_t n, int dt, uint32_t threshold_bits, int64_t k_cap, void* vals,
                                      uint64_t* mask, void* stream);

/*
 * Alg. 1 lines 6-7 for l tensors in one call: the same results, bit for bit, as l calls of surgeon_prune_pack without
 * idx.  The layers of a network are small next to the chip, so per-tensor launches each pay a launch gap and a ragged
 * tail; here tensors whose group lengths share a kernel variant go out in one launch (at most ten launches per 48
 * tensors).  A, n, group_len, r, vals, mask are HOST arrays of l entries (device pointers / sizes / ratios per
 * tensor); all tensors have dtype dt.  Every tensor must take the in-register selection path: group_len (after
 * clamping to n) a multiple of 64 and at most 4096, else SURGEON_EUNSUPPORTED and nothing is launched.  No workspace.
 */
int surgeon_prune_pack_batched(int l, const void* const* A, const int64_t* n, const int64_t* group_len, const float* r,
                               int dt, void* const* vals, uint64_t* const* mask, void* stream);

/* Workspace surgeon_dw_from_packed needs for `desc`, whatever its k_total: one query serves every prune ratio the
 * layer will be called with.  Host only. */
int surgeon_dw_ws_bytes(const surgeon_layer_desc* desc, size_t* ws_bytes);

/*
 * Which kernel surgeon_dw_from_packed will use for `desc` (it depends on the shape and on k_total): writes
 * SURGEON_PROF_DW (dense contraction on the matrix cores; Alg. 1 line 11 read literally) or SURGEON_PROF_DW_SPARSE
 * (fp32 3x3 stride-1 pad-1 layers of width 8, 16 or 32 with at most 17 % of the elements kept, 22 % when the input
 * channels fill 64-channel tiles without padding: the sum of Eq. 2 taken
 * over the kept elements only; same result up to fp32 summation order).  For benchmarks that account flops per
 * kernel.  Host only.
 */
int surgeon_dw_kernel_class(const surgeon_layer_desc* desc, int* kernel_class);

/*
 * Alg. 1 lines 11-12 / Eq. 2 (weight gradient): dW = dY^T . A_pruned, where A_pruned is rebuilt from
 * (vals, mask) with dropped positions +0.  For fp32 layers and for bf16 convolutions with filters larger than 1x1
 * the rebuilding happens while a tile is staged into LDS and A_pruned never exists in memory.  For bf16 linear layers
 * and bf16 1x1 stride-1 convolutions it is first written once, dense and in bf16, into `ws` (n elements; part of the
 * size surgeon_dw_ws_bytes reports) and a dense contraction reads it from there: on these layers un-packing inside the
 * tile load was measured slower than the extra 2 bytes per element written and read.
 * vals, mask, dY, dW, ws are device pointers; desc is a host pointer.  dW (fp32) is overwritten.
 * The result does not depend on the group_len / r the packing used.  Deterministic: the same inputs give
 * the same bits on every call.
 */
int surgeon_dw_from_packed(const surgeon_layer_desc* desc, const void* vals, const uint64_t* mask,
                           const void* dY, float* dW, void* ws, size_t ws_bytes, void* stream);

/*
 * surgeon_dw_from_packed that also returns the layer's Gradient Importance (Eq. 4) of the gradient it has just
 * computed: the sum of squares is taken inside the pass that produces dW (the reduction over the contraction's
 * splits) instead of reading dW again in a separate stage.  G_out: one fp32 on the device.  Same dW bits as
 * surgeon_dw_from_packed; G agrees with surgeon_grad_importance(dW) to fp32 rounding (fp64 accumulation in a fixed
 * order, deterministic).  Workspace from surgeon_dw_gi_ws_bytes (host only; 64 KB more than surgeon_dw_ws_bytes).
 */
int surgeon_dw_gi_ws_bytes(const surgeon_layer_desc* desc, size_t* ws_bytes);
int surgeon_dw_from_packed_gi(const surgeon_layer_desc* desc, const void* vals, const uint64_t* mask, const void* dY,
                              float* dW, float* G_out, void* ws, size_t ws_bytes, void* stream);

/*
 * Eq. 2, first line: the activation gradient dA = dY . W of the layer `desc` describes (k_total, group_len, r and the
 * packed activation play no part: dA does not depend on A).
 *   LINEAR : dY [M x N], W [N x K] (a framework's weight), dA [M x K]:  dA[m][k] = sum_n dY[m][n] * W[n][k]
 *   CONV2D : dY [Nb, Co, OH, OW], W [Co, Ci/groups, kh, kw], dA [Nb, Ci, H, W]; with groups > 1 an input channel
 *            receives from the Co/groups output channels of its own group only:
 *            dA[b][ci][ih][iw] = sum over (co, u, v) with oh*stride + u - pad == ih, ow*stride + v - pad == iw
 * dY, W and dA are device pointers of desc->dtype; products are exact (bf16 inputs widened or multiplied on the bf16
 * matrix cores), accumulation is fp32 (matrix cores; vector ALU for layers with at most four input channels), bf16
 * results are rounded once to nearest even.  Every element of dA is overwritten, also those a strided layer leaves
 * zero.  No workspace.  Deterministic.
 */
int surgeon_da(const surgeon_layer_desc* desc, const void* dY, const void* W, void* dA, void* stream);

/*
 * The same gradient with a workspace, for large bf16 linear layers: for LINEAR, bf16, M >= 256, M and K multiples of
 * 8, N and K >= 64 and every operand below 2 GiB, dY is transposed once into `ws` and the contraction runs as the
 * large-tile bf16 weight-gradient kernel does (fp32 accumulation, one rounding to bf16; the summation order differs
 * from surgeon_da's, the result agrees to within one bf16 rounding), about a tenth faster on transformer-sized layers
 * than surgeon_da, which reads dY where it lies.  Every other layer takes surgeon_da's route and needs no workspace
 * (surgeon_da_ws_bytes reports 0).  W must then be 16-byte aligned.
 * ws_bytes smaller than reported: SURGEON_ESIZE.  Deterministic.
 */
int surgeon_da_ws_bytes(const surgeon_layer_desc* desc, size_t* ws_bytes);
int surgeon_da_ws(const surgeon_layer_desc* desc, const void* dY, const void* W, void* dA, void* ws, size_t ws_bytes,
                  void* stream);

/*
 * Alg. 1 line 14 as one plain gradient step, in place: W[j] <- W[j] - lr * dW[j] (the paper leaves its optimiser to an
 * appendix; anything more elaborate is the caller's).  W: n elements of dtype dt on the device; dW: n fp32 on the
 * device.  Computed as one fused multiply-add in fp32, bf16 weights rounded once to nearest even.
 */
int surgeon_weight_update(void* W, const float* dW, int64_t n, float lr, int dt, void* stream);

/*
 * Alg. 1 line 14 for l tensors in one call: the same results, bit for bit, as l calls of surgeon_weight_update.  The
 * weights of a layer are small next to the chip, so per-layer launches are mostly launch gap; here up to 64 tensors go
 * out in one launch.  W, dW, n are HOST arrays of l entries (device pointers / element counts per tensor); all W have
 * dtype dt, all dW are fp32.  Everything is validated before the first launch.
 */
int surgeon_weight_update_batched(int l, void* const* W, const float* const* dW, const int64_t* n, float lr, int dt,
                                  void* stream);

/*
 * Normalisation layers (the variant of Section 5 that adapts BN layers only): gradients of the scale and the shift
 * of y = gamma[c] * x_hat + beta[c] from the pruned, packed normalised activation x_hat and dY,
 *     dgamma[c] = sum dY * x_hat_pruned,   dbeta[c] = sum dY        over every element of channel c.
 * The tensor is [outer, C, inner] with element (o, c, i) at (o*C + c)*inner + i: batch norm over NCHW is
 * (Nb, C, H*W), layer norm over [tokens, features] is (tokens, features, 1).  vals / mask as written by
 * surgeon_prune_pack for that tensor (any group_len), k_total its value count; dY has the dtype dt of vals.
 * dgamma, dbeta: C fp32 each on the device, overwritten.  fp32 partial sums per slice, added per channel in fp64 in
 * index order (deterministic).  Workspace from surgeon_affine_grad_ws_bytes (host only).
 */
int surgeon_affine_grad_ws_bytes(int64_t outer, int64_t C, int64_t inner, size_t* ws_bytes);
int surgeon_affine_grad(const void* vals, const uint64_t* mask, const void* dY, int64_t outer, int64_t C, int64_t inner,
                        int dt, int64_t k_total, float* dgamma, float* dbeta, void* ws, size_t ws_bytes, void* stream);

/* Workspace surgeon_grad_importance needs for n_w elements.  Host only. */
size_t surgeon_grad_importance_ws_bytes(int64_t n_w);

/*
 * Eq. 4: G = sqrt( sum_j dW_j^2 / n_w ) with N_i read as the number of weight elements of the layer.
 * dW: n_w fp32 on the device; G_out: one fp32 on the device (the caller copies all layers' scalars back
 * in one transfer).  Accumulation is in fp64 in a fixed order (deterministic).  n_w == 0 writes 0.
 */
int surgeon_grad_importance(const float* dW, int64_t n_w, float* G_out,
                            void* ws, size_t ws_bytes, void* stream);

/*
 * surgeon_grad_importance for callers that cannot allocate or carry a workspace (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): same arithmetic, same kernels and the same bits as
 * surgeon_grad_importance, but the per-workgroup partial sums live in a 16 KB array that is part of the library's
 * device image (one copy per GPU, held until the process ends) instead of a caller workspace.  The call allocates
 * nothing and frees nothing.  Limit: n_w <= 2^31, larger sizes return SURGEON_EUNSUPPORTED.  The first call on a
 * device looks the array's address up (make it outside any stream capture); later calls only launch.
 * All calls on one GPU share that array: two calls whose kernels may overlap on the same GPU (different streams, or
 * different host threads) race on it -- serialise them or use surgeon_grad_importance with separate workspaces.
 */
int surgeon_grad_importance_static(const float* dW, int64_t n_w, float* G_out, void* stream);

/*
 * Eq. 4 for l layers in one call (one pair of launches per 64 layers instead of one per layer: the layers of a
 * network are small, so per-layer launches are latency-bound).  dW and n_w are HOST arrays of l device pointers /
 * element counts; G_out is a DEVICE array of l floats, G_out[i] for layer i.  Same arithmetic as
 * surgeon_grad_importance (fp64 accumulation, fixed order, deterministic); the two entry points agree to
 * fp32 rounding but not necessarily bit for bit, because partial sums are grouped differently.
 * ws/ws_bytes as reported by surgeon_grad_importance_batched_ws_bytes (host only).  Consecutive batches of a call
 * reuse the workspace in stream order.
 */
size_t surgeon_grad_importance_batched_ws_bytes(const int64_t* n_w, int l);
int surgeon_grad_importance_batched(const float* const* dW, const int64_t* n_w, int l, float* G_out,
                                    void* ws, size_t ws_bytes, void* stream);

/*
 * Kernel timing aid for benchmarks (not part of the method).  Between surgeon_profile_begin() and
 * surgeon_profile_end() every kernel the library launches carries a start and a stop HIP event on the caller's
 * stream (attached to the kernel's own dispatch, so no extra work is queued between kernels).
 * surgeon_profile_end() waits for the events and returns, per kernel class, the summed kernel time in
 * milliseconds and the number of kernels launched, then discards the events:
 *   class 0 SURGEON_PROF_SELECT_PACK  fused select+pack kernel (group_len % 64 == 0, <= 4096)
 *   class 1 SURGEON_PROF_DW           the MFMA weight-gradient kernel (conv or linear)
 *   class 2 SURGEON_PROF_IMPORTANCE   sum-of-squares kernels of Eq. 4
 *   class 3 SURGEON_PROF_DW_AUX       rank-table pre-pass, dense transient copy and split reduction around classes 1 and 9
 *   class 4 SURGEON_PROF_SELECT_OTHER kernels of the other two selection paths, mask clearing
 *   class 5 SURGEON_PROF_DW_SPARSE    the weight-gradient kernel that works from the kept elements alone
 *   class 6 SURGEON_PROF_DA           activation-gradient kernel (surgeon_da)
 *   class 7 SURGEON_PROF_UPDATE       gradient step (surgeon_weight_update)
 *   class 8 SURGEON_PROF_AFFINE       scale / shift gradients of normalisation layers, with their rank pre-pass
 *   class 9 SURGEON_PROF_DW_GROUPED   weight-gradient kernel of grouped / depthwise convolutions
 *   class 10 SURGEON_PROF_DW_SPARSE_AUX  rank-table pre-pass and split reduction around class 5
 * ms / launches are host arrays of n_classes entries (at most SURGEON_PROF_CLASSES are filled).
 * Not thread-safe; intended for one benchmarking thread.  Event objects are created by the HIP runtime, kept in a
 * pool and reused by later profiling sessions of the process.
 */
int surgeon_profile_begin(void);
int surgeon_profile_end(int n_classes, double* ms, int64_t* launches);

/* Description of the last error on the calling thread (static storage, never NULL). */
const char* surgeon_last_error(void);

/* Library version string, e.g. "surgeon-gfx950 0.1". */
const char* surgeon_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SURGEON_H_ */
