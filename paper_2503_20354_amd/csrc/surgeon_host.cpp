// Host-only part of libsurgeon: size rules, the ratio rule of Eq. 5-7, error text.
#include <math.h>
#include <stdarg.h>
#include <string.h>

#include <vector>

#include "common.hpp"

namespace surgeon {

static thread_local char g_err[512] = "no error";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

int fail(int status, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return status;
}

bool make_group_plan(int64_t n, int64_t group_len, float r, GroupPlan* p) {
  if (n < 0 || group_len < 1 || !(r >= 0.0f && r <= 1.0f)) return false;
  if (n > 0 && group_len > n) group_len = n;
  p->n = n;
  p->g = group_len;
  p->n_groups = n == 0 ? 0 : ceil_div(n, group_len);
  p->len_last = n == 0 ? 0 : n - (p->n_groups - 1) * group_len;
  p->k_full = surgeon_keep_count(group_len, r);
  p->k_last = surgeon_keep_count(p->len_last, r);
  p->k_total = n == 0 ? 0 : (p->n_groups - 1) * p->k_full + p->k_last;
  return true;
}

PrunePath choose_prune_path(const GroupPlan& p) {
  if (p.g >= kTwoReadMinGroup) return PATH_TWO_READ;
  if (p.g > kWaveRegMaxGroup) return PATH_GLOBAL;
  if (p.g % 64 == 0) return PATH_WAVE_REG;
  return PATH_WAVE_MEM;
}

int global_hist_replicas(const GroupPlan& p) {
  const int64_t blocks_per_group = ceil_div(p.g, kGlobalHistChunk);
  return (int)std::min<int64_t>(std::max<int64_t>(blocks_per_group / 32, 1), 16);
}

size_t prune_pack_ws_bytes(const GroupPlan& p) {
  const PrunePath path = choose_prune_path(p);
  if (p.n == 0 || (path != PATH_GLOBAL && path != PATH_TWO_READ)) return 0;
  const int64_t chunks_per_group = ceil_div(p.g, kGlobalWaveChunk);
  const int64_t n_chunks = p.n_groups * chunks_per_group;
  size_t bytes = 0;
  bytes += align_up((size_t)p.n_groups * 16, 256);       // per-group select state
  bytes += align_up((size_t)p.n_groups * global_hist_replicas(p) * kGlobalHistBins * 4, 256);  // per-group digit histograms
  bytes += align_up((size_t)n_chunks * 8, 256);          // per-chunk (greater, equal) counts
  bytes += align_up((size_t)n_chunks * 8, 256);          // per-chunk (equal-before, out-before) bases
  if (path == PATH_TWO_READ) {
    bytes += align_up((size_t)p.n_groups * 32, 256);     // per-group bracket and decision
    bytes += align_up((size_t)n_chunks * 16, 256);       // per-chunk counts relative to the bracket
    bytes += (size_t)n_chunks * kTwoReadSlotKeys * 4;    // per-chunk candidate keys
  }
  return bytes;
}

// ---- kernel timing aid -------------------------------------------------------------------------
struct ProfRecord {
  int kind;
  hipEvent_t start, stop;
};
static bool g_prof_on = false;
static thread_local int g_prof_kind = -1;  // class of the innermost live ProfScope on this thread
static std::vector<ProfRecord> g_prof;

static thread_local int g_prof_force = -1;  // class that every ProfScope of this thread books under while a ProfForce lives
ProfScope::ProfScope(int kind, hipStream_t) : prev_(g_prof_kind) { g_prof_kind = g_prof_force >= 0 ? g_prof_force : kind; }
ProfForce::ProfForce(int kind) : prev_(g_prof_force) { g_prof_force = kind; }
ProfForce::~ProfForce() { g_prof_force = prev_; }

ProfScope::~ProfScope() { g_prof_kind = prev_; }

// events are kept in a pool and reused by later profiling sessions: creating them costs host time per launch
static std::vector<hipEvent_t> g_event_pool;
static size_t g_events_used = 0;

static bool pool_event(hipEvent_t* e) {
  if (g_events_used == g_event_pool.size()) {
    hipEvent_t fresh;
    if (hipEventCreate(&fresh) != hipSuccess) return false;
    g_event_pool.push_back(fresh);
  }
  *e = g_event_pool[g_events_used++];
  return true;
}

bool prof_next_events(hipEvent_t* start, hipEvent_t* stop) {
  if (!g_prof_on || g_prof_kind < 0) return false;
  ProfRecord r;
  r.kind = g_prof_kind;
  if (!pool_event(&r.start)) return false;
  if (!pool_event(&r.stop)) {
    --g_events_used;
    return false;
  }
  g_prof.push_back(r);
  *start = r.start;
  *stop = r.stop;
  return true;
}

}  // namespace surgeon

using namespace surgeon;

extern "C" int surgeon_profile_begin(void) {
  g_prof.clear();
  g_events_used = 0;
  g_prof_on = true;
  return SURGEON_OK;
}

extern "C" int surgeon_profile_end(int n_classes, double* ms, int64_t* launches) {
  g_prof_on = false;
  if (n_classes < 0 || (n_classes > 0 && (!ms || !launches))) return fail(SURGEON_EINVAL, "profile_end: bad arguments");
  for (int i = 0; i < n_classes; ++i) {
    ms[i] = 0.0;
    launches[i] = 0;
  }
  int rc = SURGEON_OK;
  for (auto& r : g_prof) {
    float t = 0.0f;
    hipError_t e = hipEventSynchronize(r.stop);
    if (e == hipSuccess) e = hipEventElapsedTime(&t, r.start, r.stop);
    if (e != hipSuccess) rc = fail(SURGEON_EHIP, "profile_end: %s", hipGetErrorString(e));
    if (e == hipSuccess && r.kind >= 0 && r.kind < n_classes) {
      ms[r.kind] += (double)t;
      launches[r.kind] += 1;
    }
  }
  g_prof.clear();
  g_events_used = 0;
  return rc;
}

extern "C" {

const char* surgeon_last_error(void) { return g_err; }

const char* surgeon_version(void) { return "surgeon-gfx950 0.1"; }

int64_t surgeon_keep_count(int64_t len, float r) {
  if (len < 0 || !(r >= 0.0f && r <= 1.0f)) return -1;
  // two separately rounded double operations: the subtraction must not fuse into the product
  volatile double keep_fraction = 1.0 - (double)r;
  volatile double product = keep_fraction * (double)len;
  int64_t k = (int64_t)ceil(product);
  if (k < 0) k = 0;
  if (k > len) k = len;
  return k;
}

int surgeon_packed_sizes(int64_t n, int64_t group_len, float r, int dt, int64_t* k_total, size_t* vals_bytes,
                         size_t* mask_bytes, size_t* ws_bytes) {
  if (dt != SURGEON_F32 && dt != SURGEON_BF16) return fail(SURGEON_EINVAL, "packed_sizes: bad dtype %d", dt);
  GroupPlan p;
  if (!make_group_plan(n, group_len, r, &p))
    return fail(SURGEON_EINVAL, "packed_sizes: need n >= 0, group_len >= 1, 0 <= r <= 1 (n=%lld group_len=%lld r=%g)",
                (long long)n, (long long)group_len, (double)r);
  if (n > ((int64_t)1 << 31)) return fail(SURGEON_EUNSUPPORTED, "packed_sizes: n = %lld exceeds 2^31", (long long)n);
  if (k_total) *k_total = p.k_total;
  if (vals_bytes) *vals_bytes = (size_t)p.k_total * (dt == SURGEON_F32 ? 4 : 2);
  if (mask_bytes) *mask_bytes = (size_t)ceil_div(n, 64) * 8;
  if (ws_bytes) *ws_bytes = prune_pack_ws_bytes(p);
  return SURGEON_OK;
}

int surgeon_layer_ratios(const float* G, const uint64_t* m, int l, float r_lo, float r_hi, float* r_out) {
  if (!G || !m || !r_out) return fail(SURGEON_EINVAL, "layer_ratios: null pointer");
  if (l < 1) return fail(SURGEON_EINVAL, "layer_ratios: l = %d", l);
  if (!(r_lo >= 0.0f && r_hi <= 1.0f && r_lo <= r_hi))
    return fail(SURGEON_EINVAL, "layer_ratios: need 0 <= r_lo <= r_hi <= 1 (got %g, %g)", (double)r_lo, (double)r_hi);
  double total = 0.0;
  for (int i = 0; i < l; ++i) {
    if (m[i] == 0) return fail(SURGEON_EINVAL, "layer_ratios: m[%d] == 0", i);
    if (!(G[i] >= 0.0f) || isinf(G[i])) return fail(SURGEON_EINVAL, "layer_ratios: G[%d] = %g", i, (double)G[i]);
    total += (double)m[i];
  }
  // Eq. 5: memory score; Eq. 6: product of the two max-normalised scores; Eq. 7: ratio
  std::vector<double> score(l);
  double mem_max = 0.0, grad_max = 0.0;
  for (int i = 0; i < l; ++i) {
    score[i] = -log((double)m[i] / total);
    mem_max = fmax(mem_max, score[i]);
    grad_max = fmax(grad_max, (double)G[i]);
  }
  double ind_max = 0.0;
  for (int i = 0; i < l; ++i) {
    const double mem_n = mem_max > 0.0 ? score[i] / mem_max : 1.0;
    const double grad_n = grad_max > 0.0 ? (double)G[i] / grad_max : 1.0;
    score[i] = mem_n * grad_n;
    ind_max = fmax(ind_max, score[i]);
  }
  const double span = (double)r_hi - (double)r_lo;
  for (int i = 0; i < l; ++i) {
    const double p = ind_max > 0.0 ? 1.0 - score[i] / ind_max : 0.0;
    r_out[i] = (float)((double)r_lo + span * p);
  }
  return SURGEON_OK;
}

}  // extern "C"
