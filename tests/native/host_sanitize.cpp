// Host-side sanitizer run: the library's host-only entry points (size rules, Eq. 5-7) and the CPU oracle on small
// inputs, built with -fsanitize=address,undefined by tests/test_host_sanitizers.py.  No GPU call is made.
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "surgeon.h"

extern "C" {
int64_t oracle_keep_count(int64_t len, float r);
int oracle_prune_pack(const void* A, int64_t n, int64_t g, float r, int dt, void* vals, uint64_t* mask, uint32_t* idx,
                      int64_t* k_out);
void oracle_unpack(const void* vals, const uint64_t* mask, int64_t n, int dt, void* dense);
int oracle_dw_linear(const void* vals, const uint64_t* mask, const void* dY, int64_t M, int64_t K, int64_t N, int dt, float* dW);
int oracle_dw_conv2d(const void* vals, const uint64_t* mask, const void* dY, int64_t Nb, int64_t Ci, int64_t H, int64_t W,
                     int64_t Co, int64_t kh, int64_t kw, int64_t stride, int64_t pad, int dt, float* dW);
int oracle_dw_conv2d_grouped(const void* vals, const uint64_t* mask, const void* dY, int64_t Nb, int64_t Ci, int64_t H,
                             int64_t W, int64_t Co, int64_t kh, int64_t kw, int64_t stride, int64_t pad, int64_t groups,
                             int dt, float* dW);
float oracle_grad_importance(const float* dW, int64_t n);
int oracle_layer_ratios(const float* G, const uint64_t* m, int l, float r_lo, float r_hi, float* r_out);
int oracle_da_linear(const void* dY, const void* W, int64_t M, int64_t K, int64_t N, int dt, void* dA);
int oracle_da_conv2d(const void* dY, const void* W, int64_t Nb, int64_t Ci, int64_t H, int64_t Wd, int64_t Co, int64_t kh,
                     int64_t kw, int64_t stride, int64_t pad, int dt, void* dA);
int oracle_weight_update(const void* W, const float* dW, int64_t n, float lr, int dt, void* W_new);
int oracle_affine_grad(const void* vals, const uint64_t* mask, const void* dY, int64_t outer, int64_t C, int64_t inner, int dt,
                       float* dgamma, float* dbeta);
}

static uint32_t rng_state = 12345u;
static float frand() {
  rng_state = rng_state * 1664525u + 1013904223u;
  return (float)((rng_state >> 8) & 0xffff) / 32768.0f - 1.0f;
}

#define CHECK(cond)                                                    \
  do {                                                                 \
    if (!(cond)) {                                                     \
      fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #cond); \
      return 1;                                                        \
    }                                                                  \
  } while (0)

int main() {
  // ---- host entry points of the library
  for (int64_t len = 0; len < 300; len += 7)
    for (float r = 0.0f; r <= 1.0f; r += 0.125f) CHECK(surgeon_keep_count(len, r) == oracle_keep_count(len, r));
  CHECK(surgeon_keep_count(5, 2.0f) == -1);
  int64_t k = 0;
  size_t vb = 0, mb = 0, wb = 0;
  CHECK(surgeon_packed_sizes(1000, 300, 0.9f, SURGEON_BF16, &k, &vb, &mb, &wb) == SURGEON_OK && vb == (size_t)k * 2 && mb == 128);
  CHECK(surgeon_packed_sizes(1 << 20, 1 << 20, 0.5f, SURGEON_F32, &k, NULL, NULL, &wb) == SURGEON_OK && wb > 0);
  CHECK(surgeon_packed_sizes(-1, 4, 0.5f, SURGEON_F32, &k, &vb, &mb, &wb) == SURGEON_EINVAL);
  CHECK(strlen(surgeon_last_error()) > 0);
  const int l = 37;
  std::vector<float> G(l), r_lib(l), r_ora(l);
  std::vector<uint64_t> m(l);
  for (int i = 0; i < l; ++i) {
    G[i] = fabsf(frand()) + 0.01f;
    m[i] = 1000u + (uint64_t)(fabsf(frand()) * 1e6f);
  }
  CHECK(surgeon_layer_ratios(G.data(), m.data(), l, 0.3f, 0.9f, r_lib.data()) == SURGEON_OK);
  CHECK(oracle_layer_ratios(G.data(), m.data(), l, 0.3f, 0.9f, r_ora.data()) == 0);
  for (int i = 0; i < l; ++i) CHECK(fabsf(r_lib[i] - r_ora[i]) <= 1e-6f);
  CHECK(surgeon_layer_ratios(G.data(), m.data(), 0, 0.3f, 0.9f, r_lib.data()) == SURGEON_EINVAL);
  double ms[SURGEON_PROF_CLASSES];
  int64_t launches[SURGEON_PROF_CLASSES];
  CHECK(surgeon_profile_begin() == SURGEON_OK);
  CHECK(surgeon_profile_end(SURGEON_PROF_CLASSES, ms, launches) == SURGEON_OK && launches[0] == 0);
  CHECK(surgeon_profile_end(3, NULL, NULL) == SURGEON_EINVAL);

  // ---- the oracle on small, odd-sized inputs (fp32 and bf16)
  for (int dt = 0; dt < 2; ++dt) {
    const int64_t Nb = 2, Ci = 6, H = 7, W = 9, Co = 4, kh = 3, kw = 3, stride = 2, pad = 1;
    const int64_t OH = (H + 2 * pad - kh) / stride + 1, OW = (W + 2 * pad - kw) / stride + 1;
    const int64_t n = Nb * Ci * H * W, n_dy = Nb * Co * OH * OW, es = dt ? 2 : 4;
    std::vector<uint8_t> A((size_t)(n * es)), dY((size_t)(n_dy * es)), vals((size_t)(n * es)), dense((size_t)(n * es));
    std::vector<uint8_t> Wt((size_t)(Co * Ci * kh * kw * es)), dA((size_t)(n * es));
    auto fill = [&](std::vector<uint8_t>& buf, int64_t count) {
      for (int64_t i = 0; i < count; ++i) {
        const float f = frand();
        uint32_t b;
        memcpy(&b, &f, 4);
        if (dt) { const uint16_t h = (uint16_t)(b >> 16); memcpy(&buf[(size_t)i * 2], &h, 2); }
        else memcpy(&buf[(size_t)i * 4], &b, 4);
      }
    };
    fill(A, n); fill(dY, n_dy); fill(Wt, Co * Ci * kh * kw);
    std::vector<uint64_t> mask((size_t)((n + 63) / 64));
    std::vector<uint32_t> idx((size_t)n);
    for (int64_t g : {(int64_t)50, (int64_t)64, n}) {
      for (float r : {0.0f, 0.37f, 0.9f, 1.0f}) {
        std::fill(mask.begin(), mask.end(), 0);
        int64_t kk = -1;
        CHECK(oracle_prune_pack(A.data(), n, g, r, dt, vals.data(), mask.data(), idx.data(), &kk) == 0 && kk >= 0 && kk <= n);
        oracle_unpack(vals.data(), mask.data(), n, dt, dense.data());
        std::vector<float> dW((size_t)(Co * Ci * kh * kw)), dWg((size_t)(Co * (Ci / 2) * kh * kw));
        CHECK(oracle_dw_conv2d(vals.data(), mask.data(), dY.data(), Nb, Ci, H, W, Co, kh, kw, stride, pad, dt, dW.data()) == 0);
        CHECK(oracle_dw_conv2d_grouped(vals.data(), mask.data(), dY.data(), Nb, Ci, H, W, Co, kh, kw, stride, pad, 2, dt, dWg.data()) == 0);
        CHECK(isfinite(oracle_grad_importance(dW.data(), (int64_t)dW.size())));
        std::vector<float> dg((size_t)Ci), db((size_t)Ci);
        CHECK(oracle_affine_grad(vals.data(), mask.data(), A.data(), Nb, Ci, H * W, dt, dg.data(), db.data()) == 0);
      }
    }
    CHECK(oracle_da_conv2d(dY.data(), Wt.data(), Nb, Ci, H, W, Co, kh, kw, stride, pad, dt, dA.data()) == 0);
    // linear: A as [M x K] = [Nb*Ci x H*W], dY reused as [M x N] with N = 3
    const int64_t M = 5, K = 11, N = 3;
    std::vector<float> dWl((size_t)(N * K));
    std::fill(mask.begin(), mask.end(), 0);
    int64_t kk = -1;
    CHECK(oracle_prune_pack(A.data(), M * K, K, 0.5f, dt, vals.data(), mask.data(), idx.data(), &kk) == 0);
    CHECK(oracle_dw_linear(vals.data(), mask.data(), dY.data(), M, K, N, dt, dWl.data()) == 0);
    CHECK(oracle_da_linear(dY.data(), Wt.data(), M, K, N, dt, dA.data()) == 0);
    std::vector<uint8_t> Wn((size_t)(N * K * es));
    CHECK(oracle_weight_update(Wt.data(), dWl.data(), N * K, 0.01f, dt, Wn.data()) == 0);
  }
  printf("host sanitizer run ok\n");
  return 0;
}
