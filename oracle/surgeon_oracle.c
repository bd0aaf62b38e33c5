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
 *
 * Floating point: every accumulation is in double; results are rounded once to float.
 * Pins: tests/test_oracle_*.py check each function against brute-force rank counting, numpy float64
 * matmul, torch.nn.grad.conv2d_weight in float64, closed forms and hand-derived examples of Eq. 5-7.
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
