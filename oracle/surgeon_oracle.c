/*
 * surgeon_oracle.c -- plain CPU oracle for SURGEON's activation-pruning hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct definition the GPU library is
 * checked against.  It shares no code, header, table or helper with the HIP path; only tests, the smoke
 * check and the benchmark's cpu_baseline leg may call it.
 *
 * Everything here is the plain definition written out (the method reaches uniquely defined results):
 *   oracle_keep_count      kept count for "prune with ratio p" (Alg. 1 line 6), rounding fixed as ceil((1-r)*len)
 *   oracle_prune_pack      Alg. 1 lines 6-7: per group, sort by (|a| bit pattern descending, index ascending),
 *                          keep the first k; store kept values (ascending index) + 1 bit per element
 *   oracle_unpack          Alg. 1 line 11: rebuild the dense pruned activation (dropped -> +0)
 *   oracle_dw_linear       Eq. 2 (weight gradient), linear layer, returned as [out x in]
 *   oracle_dw_conv2d       the same for a 2-D convolution: textbook 7-loop weight gradient
 *   oracle_dw_*_at         the same definitions evaluated at caller-chosen output entries only
 *   oracle_grad_importance Eq. 4
 *   oracle_layer_scores / oracle_layer_ratios   Eq. 5, 6, 7
 *   oracle_da_linear / oracle_da_conv2d (+ _at) / oracle_da_conv2d_grouped  Eq. 2, first line: the activation gradient dA = dY . W
 *   oracle_weight_update   Alg. 1 line 14 read as one plain gradient step W <- W - lr * dW (the paper defers its
 *                          optimiser settings to an appendix that is not available)
 *   oracle_affine_grad     gradients of a normalisation layer's scale and shift from the pruned normalised
 *                          activation (the variant of Section 5 that updates BN layers only): the same sum as
 *                          Eq. 2's second line for an element-wise layer y = gamma * x_hat + beta
 *   oracle_dw_conv2d_grouped (+ _at)  the convolution weight gradient with channel groups (grouped and depthwise
 *                          convolutions of the ResNeXt / Segformer networks of Section 5.1)
 *
 * Floating point: every accumulation is in double; results are rounded once to float (or once, to nearest even,
 * to bfloat16 where an output is stored in the layer's own dtype).
 * Pins: tests/test_oracle_*.py check each function against brute-force rank counting, numpy float64
 * matmul, torch.nn.grad.conv2d_weight / conv2d_input in float64 (also with groups), the adjoint identity
 * <dY, conv(A, W)> = <dA, A> = <dW, W>, closed forms and hand-derived examples of Eq. 5-7.
 * The paper prints no numeric example for any quantity on this path, so there is no pin against a value
 * printed in the paper ("parity unpinned" with respect to the paper's own tables).
 *
 * The `#pragma omp` lines only spread independent groups / output entries over host threads; they change
 * no arithmetic and no order of accumulation inside an output.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

static size_t elem_size(int dt) { return dt == ORACLE_F32 ? 4u : 2u; }

/* bit pattern of element i, widened to 32 bits in fp32 position (bf16 occupies the high half) */
static uint32_t elem_bits32(const void* p, int dt, int64_t i) {
  if (dt == ORACLE_F32) return ((const uint32_t*)p)[i];
  return ((uint32_t)((const uint16_t*)p)[i]) << 16;
}

static double elem_as_double(const void* p, int dt, int64_t i) {
  uint32_t b = elem_bits32(p, dt, i);
  float f;
  memcpy(&f, &b, 4);
  return (double)f; /* bf16 -> fp32 -> double is exact */
}

/* magnitude key: the stored bit pattern with its sign bit cleared, as an unsigned integer */
static uint32_t elem_key(const void* p, int dt, int64_t i) {
  if (dt == ORACLE_F32) return ((const uint32_t*)p)[i] & 0x7fffffffu;
  return (uint32_t)(((const uint16_t*)p)[i] & 0x7fffu);
}

int64_t oracle_keep_count(int64_t len, float r) {
  if (len < 0 || !(r >= 0.0f && r <= 1.0f)) return -1;
  volatile double keep_frac = 1.0 - (double)r; /* volatile: forbid fusing the subtraction into the product */
  volatile double prod = keep_frac * (double)len;
  int64_t k = (int64_t)ceil(prod);
  if (k < 0) k = 0;
  if (k > len) k = len;
  return k;
}

typedef struct {
  uint32_t key;
  uint32_t pos; /* offset inside the group */
} keyed_t;

static int cmp_key_desc_pos_asc(const void* a, const void* b) {
  const keyed_t* x = (const keyed_t*)a;
  const keyed_t* y = (const keyed_t*)b;
  if (x->key != y->key) return x->key > y->key ? -1 : 1;
  if (x->pos != y->pos) return x->pos < y->pos ? -1 : 1;
  return 0;
}

/*
 * Alg. 1 lines 6-7.  vals must hold k_total elements, mask ceil(n/64) words, idx (nullable) k_total words.
 * Returns 0, or -1 on bad arguments.  *k_total_out (nullable) receives the number of kept elements.
 */
int oracle_prune_pack(const void* A, int64_t n, int64_t group_len, float r, int dt, void* vals,
                      uint64_t* mask, uint32_t* idx, int64_t* k_total_out) {
  if (n < 0 || group_len < 1 || !(r >= 0.0f && r <= 1.0f)) return -1;
  if (dt != ORACLE_F32 && dt != ORACLE_BF16) return -1;
  if (group_len > n && n > 0) group_len = n;
  const int64_t n_words = (n + 63) / 64;
  const int64_t n_groups = n == 0 ? 0 : (n + group_len - 1) / group_len;
  const int64_t k_full = oracle_keep_count(group_len, r);
  const size_t es = elem_size(dt);
  uint8_t* keep = (uint8_t*)calloc((size_t)(n > 0 ? n : 1), 1);
  if (!keep) return -1;

  /* selection: every group on its own */
#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t g = 0; g < n_groups; ++g) {
    const int64_t start = g * group_len;
    const int64_t len = (start + group_len <= n) ? group_len : (n - start);
    const int64_t k = oracle_keep_count(len, r);
    keyed_t* order = (keyed_t*)malloc(sizeof(keyed_t) * (size_t)len);
    for (int64_t t = 0; t < len; ++t) {
      order[t].key = elem_key(A, dt, start + t);
      order[t].pos = (uint32_t)t;
    }
    qsort(order, (size_t)len, sizeof(keyed_t), cmp_key_desc_pos_asc);
    for (int64_t t = 0; t < k; ++t) keep[start + order[t].pos] = 1;
    free(order);
  }

  /* storage: values in ascending flat index, one bit per element */
  for (int64_t w = 0; w < n_words; ++w) mask[w] = 0;
  int64_t out = 0;
  for (int64_t e = 0; e < n; ++e) {
    if (!keep[e]) continue;
    mask[e / 64] |= (uint64_t)1 << (e % 64);
    memcpy((uint8_t*)vals + (size_t)out * es, (const uint8_t*)A + (size_t)e * es, es);
    if (idx) idx[out] = (uint32_t)(e % group_len);
    ++out;
  }
  free(keep);
  /* consistency of the size rule: all groups but the last are full */
  if (n_groups > 0) {
    const int64_t last_len = n - (n_groups - 1) * group_len;
    if (out != (n_groups - 1) * k_full + oracle_keep_count(last_len, r)) return -2;
  }
  if (k_total_out) *k_total_out = out;
  return 0;
}

/* Alg. 1 line 11: dense pruned activation as doubles (dropped positions are +0.0) */
static double* unpack_to_double(const void* vals, const uint64_t* mask, int64_t n, int dt) {
  double* d = (double*)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
  if (!d) return NULL;
  int64_t next = 0;
  for (int64_t e = 0; e < n; ++e) {
    if ((mask[e / 64] >> (e % 64)) & 1u) {
      d[e] = elem_as_double(vals, dt, next);
      ++next;
    } else {
      d[e] = 0.0;
    }
  }
  return d;
}

/* Alg. 1 line 11 in the storage dtype: dense[e] = next packed value if bit e is set, else +0 */
void oracle_unpack(const void* vals, const uint64_t* mask, int64_t n, int dt, void* dense) {
  const size_t es = elem_size(dt);
  int64_t next = 0;
  for (int64_t e = 0; e < n; ++e) {
    uint8_t* dst = (uint8_t*)dense + (size_t)e * es;
    if ((mask[e / 64] >> (e % 64)) & 1u) {
      memcpy(dst, (const uint8_t*)vals + (size_t)next * es, es);
      ++next;
    } else {
      memset(dst, 0, es);
    }
  }
}

/* Eq. 2, linear layer without bias: dW[o][i] = sum_m dY[m][o] * A_pruned[m][i]; A is [M x K], dY [M x N] */
int oracle_dw_linear(const void* vals, const uint64_t* mask, const void* dY, int64_t M, int64_t K,
                     int64_t N, int dt, float* dW) {
  double* Ad = unpack_to_double(vals, mask, M * K, dt);
  if (!Ad) return -1;
#pragma omp parallel for schedule(static)
  for (int64_t o = 0; o < N; ++o) {
    for (int64_t i = 0; i < K; ++i) {
      double acc = 0.0;
      for (int64_t m = 0; m < M; ++m) acc += elem_as_double(dY, dt, m * N + o) * Ad[m * K + i];
      dW[o * K + i] = (float)acc;
    }
  }
  free(Ad);
  return 0;
}

/* the same definition at chosen flat positions of dW ([N x K] row-major) */
int oracle_dw_linear_at(const void* vals, const uint64_t* mask, const void* dY, int64_t M, int64_t K,
                        int64_t N, int dt, const int64_t* where, int64_t n_where, float* out) {
  double* Ad = unpack_to_double(vals, mask, M * K, dt);
  if (!Ad) return -1;
#pragma omp parallel for schedule(static)
  for (int64_t s = 0; s < n_where; ++s) {
    const int64_t o = where[s] / K, i = where[s] % K;
    double acc = 0.0;
    for (int64_t m = 0; m < M; ++m) acc += elem_as_double(dY, dt, m * N + o) * Ad[m * K + i];
    out[s] = (float)acc;
  }
  free(Ad);
  return 0;
}

/* one entry of the convolution weight gradient, from the definition */
static double conv_dw_entry(const double* Ad, const void* dY, int dt, int64_t Nb, int64_t Ci, int64_t H,
                            int64_t W, int64_t Co, int64_t OH, int64_t OW, int64_t stride, int64_t pad,
                            int64_t co, int64_t ci, int64_t u, int64_t v) {
  double acc = 0.0;
  for (int64_t b = 0; b < Nb; ++b) {
    for (int64_t oh = 0; oh < OH; ++oh) {
      const int64_t ih = oh * stride + u - pad;
      if (ih < 0 || ih >= H) continue; /* zero padding */
      for (int64_t ow = 0; ow < OW; ++ow) {
        const int64_t iw = ow * stride + v - pad;
        if (iw < 0 || iw >= W) continue;
        acc += elem_as_double(dY, dt, ((b * Co + co) * OH + oh) * OW + ow) * Ad[((b * Ci + ci) * H + ih) * W + iw];
      }
    }
  }
  return acc;
}

/*
 * Weight gradient of y = conv2d(A, W) (cross-correlation, zero padding, no dilation, groups = 1):
 * dW[co][ci][u][v] = sum_{b,oh,ow} dY[b][co][oh][ow] * A_pruned[b][ci][oh*stride+u-pad][ow*stride+v-pad].
 */
int oracle_dw_conv2d(const void* vals, const uint64_t* mask, const void* dY, int64_t Nb, int64_t Ci,
                     int64_t H, int64_t W, int64_t Co, int64_t kh, int64_t kw, int64_t stride, int64_t pad,
                     int dt, float* dW) {
  const int64_t OH = (H + 2 * pad - kh) / stride + 1, OW = (W + 2 * pad - kw) / stride + 1;
  double* Ad = unpack_to_double(vals, mask, Nb * Ci * H * W, dt);
  if (!Ad) return -1;
#pragma omp parallel for schedule(static) collapse(2)
  for (int64_t co = 0; co < Co; ++co) {
    for (int64_t ci = 0; ci < Ci; ++ci) {
      for (int64_t u = 0; u < kh; ++u) {
        for (int64_t v = 0; v < kw; ++v) {
          dW[((co * Ci + ci) * kh + u) * kw + v] =
              (float)conv_dw_entry(Ad, dY, dt, Nb, Ci, H, W, Co, OH, OW, stride, pad, co, ci, u, v);
        }
      }
    }
  }
  free(Ad);
  return 0;
}

int oracle_dw_conv2d_at(const void* vals, const uint64_t* mask, const void* dY, int64_t Nb, int64_t Ci,
                        int64_t H, int64_t W, int64_t Co, int64_t kh, int64_t kw, int64_t stride,
                        int64_t pad, int dt, const int64_t* where, int64_t n_where, float* out) {
  const int64_t OH = (H + 2 * pad - kh) / stride + 1, OW = (W + 2 * pad - kw) / stride + 1;
  double* Ad = unpack_to_double(vals, mask, Nb * Ci * H * W, dt);
  if (!Ad) return -1;
#pragma omp parallel for schedule(static)
  for (int64_t s = 0; s < n_where; ++s) {
    int64_t f = where[s];
    const int64_t v = f % kw;
    f /= kw;
    const int64_t u = f % kh;
    f /= kh;
    const int64_t ci = f % Ci, co = f / Ci;
    out[s] = (float)conv_dw_entry(Ad, dY, dt, Nb, Ci, H, W, Co, OH, OW, stride, pad, co, ci, u, v);
  }
  free(Ad);
  return 0;
}

/* Eq. 4 with N_i = number of weight elements: G = sqrt( sum dW_j^2 / n ) */
float oracle_grad_importance(const float* dW, int64_t n) {
  if (n <= 0) return 0.0f;
  double s = 0.0;
  for (int64_t j = 0; j < n; ++j) s += (double)dW[j] * (double)dW[j];
  return (float)sqrt(s / (double)n);
}

static double max_norm(double x, double xmax) {
  if (xmax == 0.0) return 1.0; /* 0/0 := 1: every layer equally important */
  return x / xmax;
}

/*
 * Eq. 5 (M_i), Eq. 6 (I_i, max-normalised factors) and Eq. 7 (p_i) in double.  Any of M, I, p may be NULL.
 * Returns 0, -1 on bad input (l < 1, m_i == 0, G_i negative or not finite).
 */
int oracle_layer_scores(const float* G, const uint64_t* m, int l, double* M, double* I, double* p) {
  if (l < 1) return -1;
  double m_sum = 0.0;
  for (int i = 0; i < l; ++i) {
    if (m[i] == 0 || !(G[i] >= 0.0f) || isinf(G[i])) return -1;
    m_sum += (double)m[i];
  }
  double* Mv = (double*)malloc(sizeof(double) * (size_t)l);
  double* Iv = (double*)malloc(sizeof(double) * (size_t)l);
  double M_max = 0.0, G_max = 0.0, I_max = 0.0;
  for (int i = 0; i < l; ++i) {
    Mv[i] = -log((double)m[i] / m_sum); /* Eq. 5 */
    if (Mv[i] > M_max) M_max = Mv[i];
    if ((double)G[i] > G_max) G_max = (double)G[i];
  }
  for (int i = 0; i < l; ++i) {
    Iv[i] = max_norm(Mv[i], M_max) * max_norm((double)G[i], G_max); /* Eq. 6 */
    if (Iv[i] > I_max) I_max = Iv[i];
  }
  for (int i = 0; i < l; ++i) {
    if (M) M[i] = Mv[i];
    if (I) I[i] = Iv[i];
    if (p) p[i] = (I_max == 0.0) ? 0.0 : 1.0 - Iv[i] / I_max; /* Eq. 7 */
  }
  free(Mv);
  free(Iv);
  return 0;
}

/* Eq. 7 followed by the benchmark's affine map r = r_lo + (r_hi - r_lo) * p, rounded once to float */
int oracle_layer_ratios(const float* G, const uint64_t* m, int l, float r_lo, float r_hi, float* r_out) {
  if (!(r_lo >= 0.0f && r_hi <= 1.0f && r_lo <= r_hi)) return -1;
  if (l < 1) return -1;
  double* p = (double*)malloc(sizeof(double) * (size_t)l);
  int rc = oracle_layer_scores(G, m, l, NULL, NULL, p);
  if (rc == 0)
    for (int i = 0; i < l; ++i) r_out[i] = (float)((double)r_lo + ((double)r_hi - (double)r_lo) * p[i]);
  free(p);
  return rc;
}


/* ---------------------------------------------------------------------------------------------------------
 * The rest of Alg. 1's backward step and the other layer types
 * --------------------------------------------------------------------------------------------------------- */

/* double -> bfloat16 bit pattern, round to nearest, ties to even, decided on the double itself (going through
 * float first would round twice) */
static uint16_t double_to_bf16(double x) {
  if (isnan(x)) return 0x7fc0u;
  float f = (float)x;
  uint32_t fb;
  memcpy(&fb, &f, 4);
  if (isinf(f)) return (uint16_t)(fb >> 16);
  /* candidates: the bfloat16 at or next to the truncated float pattern; pick the nearest to x, ties to even */
  uint32_t base = fb & 0xffff0000u;
  uint32_t best_bits = base;
  double best_err = -1.0;
  for (int d = -1; d <= 1; ++d) {
    uint32_t cb = base + (uint32_t)(d * 0x10000);
    if ((cb & 0x7f800000u) == 0x7f800000u && d != 0) {
      /* stepping into the infinity pattern is a legal rounding result only for values beyond the largest finite */
      if ((cb & 0x007f0000u) != 0) continue;
    }
    float cf;
    memcpy(&cf, &cb, 4);
    if ((cb ^ fb) & 0x80000000u) continue; /* crossed zero */
    double err = fabs(x - (double)cf);
    if (isinf(cf)) err = fabs(x) - 3.3961775292304601e38 >= 0 ? 0.0 : INFINITY; /* halfway point to infinity */
    if (best_err < 0.0 || err < best_err || (err == best_err && ((cb >> 16) & 1u) == 0u)) {
      best_err = err;
      best_bits = cb;
    }
  }
  return (uint16_t)(best_bits >> 16);
}

static void store_rounded(void* out, int dt, int64_t i, double x) {
  if (dt == ORACLE_F32) ((float*)out)[i] = (float)x;
  else ((uint16_t*)out)[i] = double_to_bf16(x);
}

/* Eq. 2, first line, linear layer: dA[m][k] = sum_n dY[m][n] * W[n][k]; dY is [M x N], W is [N x K] (the layout
 * of a framework's weight), dA is [M x K] in the dtype of dY and W */
int oracle_da_linear(const void* dY, const void* Wt, int64_t M, int64_t K, int64_t N, int dt, void* dA) {
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m) {
    for (int64_t k = 0; k < K; ++k) {
      double acc = 0.0;
      for (int64_t n = 0; n < N; ++n) acc += elem_as_double(dY, dt, m * N + n) * elem_as_double(Wt, dt, n * K + k);
      store_rounded(dA, dt, m * K + k, acc);
    }
  }
  return 0;
}

int oracle_da_linear_at(const void* dY, const void* Wt, int64_t M, int64_t K, int64_t N, int dt,
                        const int64_t* where, int64_t n_where, void* out) {
  (void)M;
#pragma omp parallel for schedule(static)
  for (int64_t s = 0; s < n_where; ++s) {
    const int64_t m = where[s] / K, k = where[s] % K;
    double acc = 0.0;
    for (int64_t n = 0; n < N; ++n) acc += elem_as_double(dY, dt, m * N + n) * elem_as_double(Wt, dt, n * K + k);
    store_rounded(out, dt, s, acc);
  }
  return 0;
}

/* one entry of the activation gradient of y = conv2d(A, W): every output position (oh, ow) and tap (u, v) with
 * oh*stride + u - pad == ih and ow*stride + v - pad == iw contributes dY[b][co][oh][ow] * W[co][ci][u][v] */
static double conv_da_entry(const void* dY, const void* Wt, int dt, int64_t Ci, int64_t Co, int64_t OH, int64_t OW,
                            int64_t kh, int64_t kw, int64_t stride, int64_t pad, int64_t b, int64_t ci, int64_t ih,
                            int64_t iw) {
  double acc = 0.0;
  for (int64_t co = 0; co < Co; ++co) {
    for (int64_t u = 0; u < kh; ++u) {
      const int64_t top = ih + pad - u;
      if (top < 0 || top % stride != 0 || top / stride >= OH) continue;
      for (int64_t v = 0; v < kw; ++v) {
        const int64_t left = iw + pad - v;
        if (left < 0 || left % stride != 0 || left / stride >= OW) continue;
        acc += elem_as_double(dY, dt, ((b * Co + co) * OH + top / stride) * OW + left / stride) *
               elem_as_double(Wt, dt, ((co * Ci + ci) * kh + u) * kw + v);
      }
    }
  }
  return acc;
}

/* Activation gradient of a 2-D convolution (cross-correlation, zero padding, no dilation, groups = 1):
 * dY [Nb, Co, OH, OW], W [Co, Ci, kh, kw]  ->  dA [Nb, Ci, H, W] in the dtype of the inputs */
int oracle_da_conv2d(const void* dY, const void* Wt, int64_t Nb, int64_t Ci, int64_t H, int64_t W, int64_t Co,
                     int64_t kh, int64_t kw, int64_t stride, int64_t pad, int dt, void* dA) {
  const int64_t OH = (H + 2 * pad - kh) / stride + 1, OW = (W + 2 * pad - kw) / stride + 1;
#pragma omp parallel for schedule(static) collapse(2)
  for (int64_t b = 0; b < Nb; ++b) {
    for (int64_t ci = 0; ci < Ci; ++ci) {
      for (int64_t ih = 0; ih < H; ++ih)
        for (int64_t iw = 0; iw < W; ++iw)
          store_rounded(dA, dt, ((b * Ci + ci) * H + ih) * W + iw,
                        conv_da_entry(dY, Wt, dt, Ci, Co, OH, OW, kh, kw, stride, pad, b, ci, ih, iw));
    }
  }
  return 0;
}

/* The same for a convolution with channel groups: W is [Co, Ci/groups, kh, kw]; input channel ci belongs to group
 * ci / (Ci/groups) and receives from that group's Co/groups output channels only. */
int oracle_da_conv2d_grouped(const void* dY, const void* Wt, int64_t Nb, int64_t Ci, int64_t H, int64_t W, int64_t Co,
                             int64_t kh, int64_t kw, int64_t stride, int64_t pad, int64_t groups, int dt, void* dA) {
  const int64_t OH = (H + 2 * pad - kh) / stride + 1, OW = (W + 2 * pad - kw) / stride + 1;
  const int64_t Cig = Ci / groups, Cog = Co / groups;
#pragma omp parallel for schedule(static) collapse(2)
  for (int64_t b = 0; b < Nb; ++b) {
    for (int64_t ci = 0; ci < Ci; ++ci) {
      const int64_t grp = ci / Cig, cig = ci % Cig;
      for (int64_t ih = 0; ih < H; ++ih)
        for (int64_t iw = 0; iw < W; ++iw) {
          double acc = 0.0;
          for (int64_t co = grp * Cog; co < (grp + 1) * Cog; ++co)
            for (int64_t u = 0; u < kh; ++u) {
              const int64_t top = ih + pad - u;
              if (top < 0 || top % stride != 0 || top / stride >= OH) continue;
              for (int64_t v = 0; v < kw; ++v) {
                const int64_t left = iw + pad - v;
                if (left < 0 || left % stride != 0 || left / stride >= OW) continue;
                acc += elem_as_double(dY, dt, ((b * Co + co) * OH + top / stride) * OW + left / stride) *
                       elem_as_double(Wt, dt, ((co * Cig + cig) * kh + u) * kw + v);
              }
            }
          store_rounded(dA, dt, ((b * Ci + ci) * H + ih) * W + iw, acc);
        }
    }
  }
  return 0;
}

int oracle_da_conv2d_at(const void* dY, const void* Wt, int64_t Nb, int64_t Ci, int64_t H, int64_t W, int64_t Co,
                        int64_t kh, int64_t kw, int64_t stride, int64_t pad, int dt, const int64_t* where,
                        int64_t n_where, void* out) {
  const int64_t OH = (H + 2 * pad - kh) / stride + 1, OW = (W + 2 * pad - kw) / stride + 1;
  (void)Nb;
#pragma omp parallel for schedule(static)
  for (int64_t s = 0; s < n_where; ++s) {
    int64_t f = where[s];
    const int64_t iw = f % W;
    f /= W;
    const int64_t ih = f % H;
    f /= H;
    const int64_t ci = f % Ci, b = f / Ci;
    store_rounded(out, dt, s, conv_da_entry(dY, Wt, dt, Ci, Co, OH, OW, kh, kw, stride, pad, b, ci, ih, iw));
  }
  return 0;
}

/* Alg. 1 line 14 as one plain gradient step: W_new[j] = W[j] - lr * dW[j]; W in the layer's dtype, dW float */
int oracle_weight_update(const void* Wt, const float* dW, int64_t n, float lr, int dt, void* W_new) {
  for (int64_t j = 0; j < n; ++j) store_rounded(W_new, dt, j, elem_as_double(Wt, dt, j) - (double)lr * (double)dW[j]);
  return 0;
}

/*
 * Scale and shift gradients of a normalisation layer y = gamma[c] * x_hat + beta[c] from the pruned normalised
 * activation: dgamma[c] = sum dY * x_hat_pruned, dbeta[c] = sum dY, both over every element of channel c.
 * Element (o, c, i) of the [outer, C, inner] tensor sits at (o*C + c)*inner + i: batch norm over NCHW is
 * (Nb, C, H*W), layer norm over [tokens, features] is (tokens, features, 1).
 */
int oracle_affine_grad(const void* vals, const uint64_t* mask, const void* dY, int64_t outer, int64_t C,
                       int64_t inner, int dt, float* dgamma, float* dbeta) {
  double* Xd = unpack_to_double(vals, mask, outer * C * inner, dt);
  if (!Xd) return -1;
#pragma omp parallel for schedule(static)
  for (int64_t c = 0; c < C; ++c) {
    double g = 0.0, b = 0.0;
    for (int64_t o = 0; o < outer; ++o) {
      for (int64_t i = 0; i < inner; ++i) {
        const int64_t e = (o * C + c) * inner + i;
        const double dy = elem_as_double(dY, dt, e);
        g += dy * Xd[e];
        b += dy;
      }
    }
    dgamma[c] = (float)g;
    dbeta[c] = (float)b;
  }
  free(Xd);
  return 0;
}

/* one entry of the weight gradient of a convolution with channel groups: output channel co belongs to group
 * co / (Co/groups) and sees the input channels of that group only; cig indexes them inside the group */
static double conv_dw_grouped_entry(const double* Ad, const void* dY, int dt, int64_t Nb, int64_t Ci, int64_t H,
                                    int64_t W, int64_t Co, int64_t OH, int64_t OW, int64_t stride, int64_t pad,
                                    int64_t groups, int64_t co, int64_t cig, int64_t u, int64_t v) {
  const int64_t ci = (co / (Co / groups)) * (Ci / groups) + cig;
  return conv_dw_entry(Ad, dY, dt, Nb, Ci, H, W, Co, OH, OW, stride, pad, co, ci, u, v);
}

/* dW [Co, Ci/groups, kh, kw]; groups == Ci == Co is a depthwise convolution */
int oracle_dw_conv2d_grouped(const void* vals, const uint64_t* mask, const void* dY, int64_t Nb, int64_t Ci,
                             int64_t H, int64_t W, int64_t Co, int64_t kh, int64_t kw, int64_t stride, int64_t pad,
                             int64_t groups, int dt, float* dW) {
  if (groups < 1 || Ci % groups || Co % groups) return -2;
  const int64_t OH = (H + 2 * pad - kh) / stride + 1, OW = (W + 2 * pad - kw) / stride + 1, Cig = Ci / groups;
  double* Ad = unpack_to_double(vals, mask, Nb * Ci * H * W, dt);
  if (!Ad) return -1;
#pragma omp parallel for schedule(static) collapse(2)
  for (int64_t co = 0; co < Co; ++co) {
    for (int64_t cig = 0; cig < Cig; ++cig) {
      for (int64_t u = 0; u < kh; ++u)
        for (int64_t v = 0; v < kw; ++v)
          dW[((co * Cig + cig) * kh + u) * kw + v] = (float)conv_dw_grouped_entry(
              Ad, dY, dt, Nb, Ci, H, W, Co, OH, OW, stride, pad, groups, co, cig, u, v);
    }
  }
  free(Ad);
  return 0;
}

int oracle_dw_conv2d_grouped_at(const void* vals, const uint64_t* mask, const void* dY, int64_t Nb, int64_t Ci,
                                int64_t H, int64_t W, int64_t Co, int64_t kh, int64_t kw, int64_t stride,
                                int64_t pad, int64_t groups, int dt, const int64_t* where, int64_t n_where,
                                float* out) {
  if (groups < 1 || Ci % groups || Co % groups) return -2;
  const int64_t OH = (H + 2 * pad - kh) / stride + 1, OW = (W + 2 * pad - kw) / stride + 1, Cig = Ci / groups;
  double* Ad = unpack_to_double(vals, mask, Nb * Ci * H * W, dt);
  if (!Ad) return -1;
#pragma omp parallel for schedule(static)
  for (int64_t s = 0; s < n_where; ++s) {
    int64_t f = where[s];
    const int64_t v = f % kw;
    f /= kw;
    const int64_t u = f % kh;
    f /= kh;
    const int64_t cig = f % Cig, co = f / Cig;
    out[s] = (float)conv_dw_grouped_entry(Ad, dY, dt, Nb, Ci, H, W, Co, OH, OW, stride, pad, groups, co, cig, u, v);
  }
  free(Ad);
  return 0;
}
