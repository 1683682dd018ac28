// Host-side parts of libcake: error strings, argument checks, workspace layout and the
// cascading budget allocation (Sec. 4.1 Eq. 7, Sec. 4.2 Eq. 9).  No GPU code here.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <vector>

#include "cake_internal.h"

namespace cake {

static thread_local char g_error[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_error, sizeof(g_error), fmt, ap);
  va_end(ap);
  return code;
}
void clear_error() { g_error[0] = '\0'; }

int check_shape_basic(const cake_shape* s) {
  CAKE_REQUIRE(s != nullptr, "shape is NULL");
  CAKE_REQUIRE(s->batch >= 1 && s->batch <= kMaxLaunchEntries, "batch %d outside [1, %d]", s->batch, kMaxLaunchEntries);
  CAKE_REQUIRE(s->n_layers >= 1 && s->n_layers <= 1024, "n_layers %d outside [1, 1024]", s->n_layers);
  CAKE_REQUIRE(s->n_kv_heads >= 1 && s->n_q_heads >= s->n_kv_heads && s->n_q_heads % s->n_kv_heads == 0,
               "n_q_heads %d must be a positive multiple of n_kv_heads %d", s->n_q_heads, s->n_kv_heads);
  CAKE_REQUIRE((int64_t)s->batch * s->n_kv_heads <= 65535, "batch*n_kv_heads = %lld exceeds 65535",
               (long long)s->batch * s->n_kv_heads);
  CAKE_REQUIRE(s->window >= 1, "window %d must be positive", s->window);
  CAKE_REQUIRE(s->head_dim >= 1, "head_dim %d must be positive", s->head_dim);
  if (s->dtype != CAKE_BF16 && s->dtype != CAKE_F32)
    return fail(CAKE_ERR_UNSUPPORTED, "dtype %d is neither CAKE_BF16 nor CAKE_F32", s->dtype);
  if ((size_t)s->head_dim * elem_bytes(s->dtype) % 16 != 0)
    return fail(CAKE_ERR_UNSUPPORTED, "rows of head_dim %d are not a multiple of 16 bytes", s->head_dim);
  return CAKE_OK;
}

int check_shape_scores(const cake_shape* s) {
  if (int rc = check_shape_basic(s)) return rc;
  CAKE_REQUIRE(s->seq_len > s->window, "seq_len %d must exceed window %d", s->seq_len, s->window);
  if (s->head_dim != 64 && s->head_dim != 128)
    return fail(CAKE_ERR_UNSUPPORTED, "head_dim %d: score kernels exist for 64 and 128", s->head_dim);
  if (s->window != 32 && s->window != 64)
    return fail(CAKE_ERR_UNSUPPORTED, "window %d: score kernels exist for 32 and 64", s->window);
  int g = s->n_q_heads / s->n_kv_heads;
  if (g > 8) return fail(CAKE_ERR_UNSUPPORTED, "group size %d: score kernels handle at most 8 query heads per KV head", g);
  return CAKE_OK;
}

ScoreLayout score_layout(const cake_shape& s) {
  ScoreLayout w{};
  const int g = s.n_q_heads / s.n_kv_heads;
  const int64_t n_p = (int64_t)s.seq_len - s.window;
  w.n_slices = (int64_t)s.n_layers * s.batch * s.n_kv_heads;
  w.rows = g * s.window;
  // The chunk depends on N alone, so that a layer's sums are grouped the same way (and come out
  // bit-identical) whether it is scored alone (cascading) or batched with other layers.
  const int chunk = s.seq_len >= 32768 ? 2048 : s.seq_len >= 8192 ? 1024 : s.seq_len >= 2048 ? 512 : 256;
  w.chunk = chunk;
  w.n_chunks = (s.seq_len + chunk - 1) / chunk;
  w.n_chunks_p = (int32_t)((n_p + chunk - 1) / chunk);
  size_t off = 0;
  w.off_lse = off;   off = align_up(off + sizeof(float) * w.n_slices * w.rows, 256);
  w.off_part = off;  off = align_up(off + sizeof(float) * w.n_slices * w.n_chunks * w.rows * 2, 256);
  w.off_hv = off;    off = align_up(off + sizeof(float) * w.n_slices * w.n_chunks_p * g * 2, 256);
  w.off_raw = off;   off = align_up(off + sizeof(float) * w.n_slices * n_p, 256);
  w.total = off;
  return w;
}

}  // namespace cake

using namespace cake;

extern "C" int cake_version(void) { return 100; }

extern "C" const char* cake_last_error(void) { return g_error; }

extern "C" int cake_workspace_bytes(const cake_shape* shape, size_t* bytes) {
  CAKE_REQUIRE(bytes != nullptr, "bytes is NULL");
  if (int rc = check_shape_scores(shape)) return rc;
  *bytes = score_layout(*shape).total;
  return CAKE_OK;
}

// Number of seat counts s in [window, n-1] whose priority p/(s + 1/2) is strictly above lam.
// The quotient never increases with s, so the boundary is found by bisection on s with the
// same fp64 division the award loop uses.
static int64_t seats_above(double p, double lam, int32_t window, int32_t n) {
  if (!(p / (window + 0.5) > lam)) return 0;
  int64_t lo = window, hi = n - 1;          // invariant: quotient(lo) > lam
  while (lo < hi) {
    int64_t mid = lo + (hi - lo + 1) / 2;
    if (p / ((double)mid + 0.5) > lam) lo = mid; else hi = mid - 1;
  }
  return lo - window + 1;
}

extern "C" int cake_keep_counts(const int32_t* budgets, const int32_t* cur_len, int32_t n, int32_t window, int32_t* keep) {
  CAKE_REQUIRE(budgets && cur_len && keep, "budgets, cur_len or keep is NULL");
  CAKE_REQUIRE(n >= 0 && window >= 1, "n %d must be >= 0 and window %d >= 1", n, window);
  for (int i = 0; i < n; ++i) {
    CAKE_REQUIRE(cur_len[i] >= 0, "cur_len[%d] = %d is negative", i, cur_len[i]);
    keep[i] = std::min(std::max(budgets[i] - window, 0), cur_len[i]);
  }
  return CAKE_OK;
}

extern "C" int cake_cascade_allocate(const double* pref, int32_t n_seen, int64_t total_budget,
                                     int32_t window, int32_t seq_len, int32_t* budgets) {
  CAKE_REQUIRE(pref != nullptr && budgets != nullptr, "pref or budgets is NULL");
  CAKE_REQUIRE(n_seen >= 1, "n_seen %d must be positive", n_seen);
  CAKE_REQUIRE(window >= 1 && seq_len > window, "need 1 <= window (%d) < seq_len (%d)", window, seq_len);
  CAKE_REQUIRE(total_budget >= (int64_t)n_seen * window,
               "total_budget %lld is below n_seen*window = %lld", (long long)total_budget,
               (long long)n_seen * window);
  bool all_zero = true;
  for (int l = 0; l < n_seen; ++l) {
    CAKE_REQUIRE(std::isfinite(pref[l]) && pref[l] >= 0.0, "pref[%d] = %g is not finite and >= 0", l, pref[l]);
    if (pref[l] != 0.0) all_zero = false;
  }
  if ((int64_t)n_seen * seq_len <= total_budget) {   // every layer fits whole: nothing to evict
    for (int l = 0; l < n_seen; ++l) budgets[l] = seq_len;
    return CAKE_OK;
  }
  std::vector<double> p(pref, pref + n_seen);
  if (all_zero) std::fill(p.begin(), p.end(), 1.0);

  // The award loop takes seats in descending priority.  Jump ahead: find a level `hi` such
  // that the seats with priority strictly above it number at most R; all of them are taken
  // before any seat at or below `hi`, so taking them at once reaches a state of the loop.
  const int64_t r_total = total_budget - (int64_t)n_seen * window;
  auto taken_above = [&](double lam) {
    int64_t t = 0;
    for (int l = 0; l < n_seen; ++l) t += seats_above(p[l], lam, window, seq_len);
    return t;
  };
  double hi = 0.0;
  for (int l = 0; l < n_seen; ++l) hi = std::max(hi, p[l] / (window + 0.5));   // nothing lies above this
  double lo = 0.0;
  if (taken_above(lo) <= r_total) {
    hi = lo;
  } else {
    for (int it = 0; it < 80; ++it) {
      double mid = 0.5 * (lo + hi);
      if (!(mid > lo && mid < hi)) break;
      if (taken_above(mid) <= r_total) hi = mid; else lo = mid;
    }
  }
  std::vector<int64_t> b(n_seen);
  int64_t remaining = r_total;
  for (int l = 0; l < n_seen; ++l) {
    int64_t t = seats_above(p[l], hi, window, seq_len);
    b[l] = window + t;
    remaining -= t;
  }
  // Award what is left one seat at a time: largest pref/(B + 1/2), ties to the lower layer.
  std::vector<double> prio(n_seen);
  for (int l = 0; l < n_seen; ++l) prio[l] = b[l] < seq_len ? p[l] / ((double)b[l] + 0.5) : -1.0;
  while (remaining > 0) {
    int best = 0;
    for (int l = 1; l < n_seen; ++l) if (prio[l] > prio[best]) best = l;
    if (prio[best] < 0.0) break;
    b[best] += 1;
    remaining -= 1;
    prio[best] = b[best] < seq_len ? p[best] / ((double)b[best] + 0.5) : -1.0;
  }
  for (int l = 0; l < n_seen; ++l) budgets[l] = (int32_t)b[l];
  return CAKE_OK;
}
