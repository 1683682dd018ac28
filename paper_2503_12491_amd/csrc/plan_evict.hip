// cake_plan_eviction / cake_evict_planned: the allocation step and EVICT of a one-shot pass with
// no host round trip in between.
//
// Preference-prioritised allocation (Sec. 4.1 Eq. 7; Sec. 4.2 Eq. 9, Prop. 1) on the device, with
// the same integers as the host routine cake_cascade_allocate: divisor (Webster) apportionment,
// every layer first holds its S_w window tokens, the rest go one at a time to the layer with the
// largest pref/(B + 1/2) among layers below N, ties to the lower layer.  The retained prefix
// counts k = clamp(B - S_w, 0, cur_len) (Sec. 4.3 Eq. 11-12: the window tokens are kept
// structurally and count towards B) and the places of every layer's outputs in four pools are
// derived in the same launches and left in a device-resident plan, from which the top-k and the
// compaction of all layers read their counts and output addresses.
//
// One wave per sequence.  The award loop is entered from a state it passes through: for a level
// lambda found by bisection every layer takes at once all seats whose priority is strictly above
// lambda (counted exactly, with the very division the loop compares), which is what the loop
// would have awarded before touching any seat at or below lambda.  Only fp64 divisions and
// comparisons decide, so host and device agree bit for bit.
#include <cmath>

#include "cake_internal.h"

namespace cake {
namespace {

constexpr int kMaxLayers = 1024;

// p/(s + 1/2) > lam, decided exactly as the fp64 division and comparison would.  The rounded
// quotient lies within one part in 2^52 of p/x, so away from a narrow band around p = lam*x a
// multiplication settles it; inside the band the division itself is done.
__device__ __forceinline__ bool seat_above(double p, double lam, int64_t s) {
  const double x = (double)s + 0.5;
  const double t = lam * x;
  if (!(lam > 0x1p-900 && t < 0x1p900)) return p / x > lam;     // products near the ends of the range: no shortcut
  if (p > t * (1.0 + 0x1p-50)) return true;
  if (p < t * (1.0 - 0x1p-50)) return false;
  return p / x > lam;
}

// Number of seat counts s in [window, n-1] with p/(s + 1/2) > lam.  The quotient never increases
// with s, so the count is fixed by the last s that passes; a closed-form guess is corrected with
// the exact predicate.
__device__ int64_t seats_above(double p, double lam, int window, int n) {
  if (!seat_above(p, lam, window)) return 0;
  int64_t s = n - 1;
  if (lam > 0.0) {
    const double guess = floor(p / lam - 0.5);
    s = guess >= (double)(n - 1) ? (int64_t)(n - 1) : guess <= (double)window ? (int64_t)window : (int64_t)guess;
  }
  while (s < n - 1 && seat_above(p, lam, s + 1)) ++s;
  while (s > window && !seat_above(p, lam, s)) --s;
  return s - window + 1;
}

__device__ __forceinline__ int64_t wave_sum(int64_t x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off);
  return x;
}
__device__ __forceinline__ double wave_max(double x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x = fmax(x, __shfl_xor(x, off));
  return x;
}

// budgets[l*B + b], keep[l*B + b], cur_out[l*B + b] for sequence b = blockIdx.x.
// status[b] = 1 if a preference of the sequence is NaN, negative or infinite (the budgets are then
// those of equal preferences, so that everything downstream stays in bounds), else 0.
__global__ __launch_bounds__(64) void allocate_kernel(const double* pref, int n_layers, int batch, int64_t total_budget,
                                                      int window, int seq_len, const int32_t* cur_len,
                                                      int32_t* budgets, int32_t* keep, int32_t* cur_out, int32_t* status) {
  __shared__ double p[kMaxLayers];
  __shared__ double prio[kMaxLayers];
  __shared__ int32_t bud[kMaxLayers];
  const int b = blockIdx.x, lane = threadIdx.x;
  const int n_p = seq_len - window;

  bool bad = false, any_pos = false;
  for (int l = lane; l < n_layers; l += 64) {
    const double x = pref[(int64_t)b * n_layers + l];
    p[l] = x;
    bad = bad || !(x >= 0.0) || isinf(x);
    any_pos = any_pos || x != 0.0;
  }
  bad = __any(bad);
  any_pos = __any(any_pos);
  if (lane == 0) status[b] = bad ? 1 : 0;
  if (!any_pos || bad)                            // all-zero preferences count as equal ones
    for (int l = lane; l < n_layers; l += 64) p[l] = 1.0;
  __syncthreads();

  if ((int64_t)n_layers * seq_len <= total_budget) {   // every layer fits whole: nothing to evict
    for (int l = lane; l < n_layers; l += 64) bud[l] = seq_len;
  } else {
    const int64_t r_total = total_budget - (int64_t)n_layers * window;
    auto taken_above = [&](double lam) {
      int64_t t = 0;
      for (int l = lane; l < n_layers; l += 64) t += seats_above(p[l], lam, window, seq_len);
      return wave_sum(t);
    };
    double hi = 0.0;
    for (int l = lane; l < n_layers; l += 64) hi = fmax(hi, p[l] / (window + 0.5));
    hi = wave_max(hi);                              // nothing lies above this
    double lo = 0.0;
    if (taken_above(lo) <= r_total) {
      hi = lo;
    } else {
      // Any level with at most r_total seats above it is a state of the award loop; the bisection
      // stops as soon as the seats left for the loop are few.
      int64_t at_hi = 0;
      // Without floors and caps the budgets are pref/lambda - 1/2 and sum to the total at
      // lambda = sum(pref)/(total + L/2): try a narrow bracket around that level first.
      double sum_p = 0.0;
      for (int l = lane; l < n_layers; l += 64) sum_p += p[l];
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) sum_p += __shfl_xor(sum_p, off);
      const double lam0 = sum_p / ((double)total_budget + 0.5 * n_layers);
      const double a = lam0 * (1.0 - 0x1p-9), c = lam0 * (1.0 + 0x1p-9);
      if (a > lo && c < hi) {
        const int64_t ta = taken_above(a), tc = taken_above(c);
        if (tc <= r_total) { hi = c; at_hi = tc; }
        if (ta > r_total) lo = a; else if (ta >= at_hi) { hi = a; at_hi = ta; }
      }
      for (int it = 0; it < 64 && r_total - at_hi > 8; ++it) {
        const double mid = 0.5 * (lo + hi);
        if (!(mid > lo && mid < hi)) break;
        const int64_t t = taken_above(mid);
        if (t <= r_total) { hi = mid; at_hi = t; } else lo = mid;
      }
    }
    int64_t taken = 0;
    for (int l = lane; l < n_layers; l += 64) {
      const int64_t t = seats_above(p[l], hi, window, seq_len);
      bud[l] = window + (int32_t)t;
      prio[l] = bud[l] < seq_len ? p[l] / ((double)bud[l] + 0.5) : -1.0;
      taken += t;
    }
    int64_t remaining = r_total - wave_sum(taken);
    __syncthreads();
    // Award what is left one seat at a time: largest pref/(B + 1/2), ties to the lower layer.
    while (remaining > 0) {
      double best = -2.0;
      int best_l = kMaxLayers;
      for (int l = lane; l < n_layers; l += 64)
        if (prio[l] > best) { best = prio[l]; best_l = l; }      // first maximum within the lane's layers
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) {
        const double ob = __shfl_xor(best, off);
        const int ol = __shfl_xor(best_l, off);
        if (ob > best || (ob == best && ol < best_l)) { best = ob; best_l = ol; }
      }
      if (best < 0.0) break;
      // A layer of zero preference keeps the priority 0 until it is full, and the lowest such
      // layer wins every tie: it takes all it can hold at once.
      const int64_t take = best == 0.0 ? min(remaining, (int64_t)(seq_len - bud[best_l])) : 1;
      __syncthreads();
      if (lane == 0) {
        bud[best_l] += (int32_t)take;
        prio[best_l] = bud[best_l] < seq_len ? p[best_l] / ((double)bud[best_l] + 0.5) : -1.0;
      }
      remaining -= take;
      __syncthreads();
    }
  }
  __syncthreads();
  for (int l = lane; l < n_layers; l += 64) {
    const int64_t e = (int64_t)l * batch + b;
    const int cur = cur_len ? cur_len[e] : n_p;
    budgets[e] = bud[l];
    keep[e] = min(max(bud[l] - window, 0), cur);
    cur_out[e] = cur;
  }
}

// Row capacities of every layer (the largest count over the batch), the places of the
// layers' outputs, one after the other, in the four pools, and the compaction's work list.
__global__ __launch_bounds__(64) void place_kernel(int n_layers, int batch, int h_kv, int window, int row_bytes,
                                                   const int32_t* keep, const int32_t* cur, int32_t* cap_keep,
                                                   int32_t* cap_cur, int32_t* copy_blocks, char* pool_idx, char* pool_k, char* pool_v,
                                                   char* pool_ind, void** idx_tbl, void** k_tbl, void** v_tbl,
                                                   void** ind_tbl) {
  const int lane = threadIdx.x;
  for (int l = lane; l < n_layers; l += 64) {
    int ck = 0, cc = 0;
    for (int b = 0; b < batch; ++b) {
      ck = max(ck, keep[(int64_t)l * batch + b]);
      cc = max(cc, cur[(int64_t)l * batch + b]);
    }
    cap_keep[l] = ck;
    cap_cur[l] = cc;
  }
  __threadfence_block();
  __syncthreads();
  // Running sums over the layers (output places) and over the (layer, sequence) entries (the
  // work list): every lane sums a run of consecutive items, a wave scan gives the runs' starts.
  auto scan = [&](int64_t own) {           // exclusive prefix sum over the lanes
    int64_t incl = own;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int64_t t = __shfl_up(incl, off);
      if (lane >= off) incl += t;
    }
    return incl - own;
  };
  const int64_t bh = (int64_t)batch * h_kv;
  {
    const int per = (n_layers + 63) / 64;
    const int l0 = min(lane * per, n_layers), l1 = min(l0 + per, n_layers);
    int64_t rows = 0;
    for (int l = l0; l < l1; ++l) rows += cap_keep[l];
    int64_t before = scan(rows);            // rows of capacity in the layers before l0
    for (int l = l0; l < l1; ++l) {
      const int64_t off_i = bh * before, off_kv = bh * (before + (int64_t)l * window) * row_bytes;
      idx_tbl[l] = pool_idx + off_i * 4;
      ind_tbl[l] = pool_ind + off_i * 4;
      k_tbl[l] = pool_k + off_kv;
      v_tbl[l] = pool_v + off_kv;
      before += cap_keep[l];
    }
  }
  {
    const int64_t n = (int64_t)n_layers * batch, pieces = row_bytes / 16;
    const int64_t per = (n + 63) / 64;
    const int64_t e0 = min(lane * per, n), e1 = min(e0 + per, n);
    auto blocks_of = [&](int64_t e) { return ((keep[e] + window) * pieces + kCopyBlockPieces - 1) / kCopyBlockPieces; };
    int64_t own = 0;
    for (int64_t e = e0; e < e1; ++e) own += blocks_of(e);
    int64_t before = scan(own);
    for (int64_t e = e0; e < e1; ++e) {
      copy_blocks[e] = (int32_t)before;
      before += blocks_of(e);
    }
    if (lane == 63) copy_blocks[n] = (int32_t)before;     // the last lane's run ends the list
  }
}

}  // namespace
}  // namespace cake

using namespace cake;

extern "C" int cake_plan_bytes(const cake_shape* shape, size_t* bytes) {
  CAKE_REQUIRE(bytes != nullptr, "bytes is NULL");
  if (int rc = check_shape_basic(shape)) return rc;
  *bytes = plan_layout(shape->n_layers, shape->batch).total;
  return CAKE_OK;
}

extern "C" int cake_plan_eviction(const cake_shape* shape, const double* pref, int64_t total_budget,
                                  const int32_t* cur_len,
                                  void* pool_idx, void* pool_k, void* pool_v, void* pool_ind,
                                  void* plan, size_t plan_bytes, int32_t* status, void* stream) {
  if (int rc = check_shape_basic(shape)) return rc;
  CAKE_REQUIRE(pref && pool_idx && pool_k && pool_v && pool_ind && plan && status, "a pointer argument is NULL");
  CAKE_REQUIRE(shape->seq_len > shape->window, "seq_len %d must exceed window %d", shape->seq_len, shape->window);
  CAKE_REQUIRE(total_budget >= (int64_t)shape->n_layers * shape->window,
               "total_budget %lld is below n_layers*window = %lld", (long long)total_budget,
               (long long)shape->n_layers * shape->window);
  CAKE_REQUIRE((reinterpret_cast<uintptr_t>(plan) & 7) == 0, "plan must be 8-byte aligned");
  const PlanLayout lay = plan_layout(shape->n_layers, shape->batch);
  CAKE_REQUIRE(plan_bytes >= lay.total, "plan has %zu bytes, %zu needed", plan_bytes, lay.total);
  for (void* q : {pool_idx, pool_k, pool_v, pool_ind})
    CAKE_REQUIRE((reinterpret_cast<uintptr_t>(q) & 15) == 0, "pools must be 16-byte aligned");
  char* b = static_cast<char*>(plan);
  int32_t* budgets = reinterpret_cast<int32_t*>(b + lay.off_budgets);
  int32_t* keep = reinterpret_cast<int32_t*>(b + lay.off_keep);
  int32_t* cur = reinterpret_cast<int32_t*>(b + lay.off_cur);
  int32_t* cap_keep = reinterpret_cast<int32_t*>(b + lay.off_cap_keep);
  int32_t* cap_cur = reinterpret_cast<int32_t*>(b + lay.off_cap_cur);
  int32_t* copy_blocks = reinterpret_cast<int32_t*>(b + lay.off_blocks);
  void** tables = reinterpret_cast<void**>(b + lay.off_tables);
  const int L = shape->n_layers;
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(allocate_kernel, dim3(shape->batch), dim3(64), 0, st, pref, L, shape->batch, total_budget,
                     shape->window, shape->seq_len, cur_len, budgets, keep, cur, status);
  hipLaunchKernelGGL(place_kernel, dim3(1), dim3(64), 0, st, L, shape->batch, shape->n_kv_heads, shape->window,
                     (int)(shape->head_dim * elem_bytes(shape->dtype)), keep, cur, cap_keep, cap_cur, copy_blocks,
                     static_cast<char*>(pool_idx), static_cast<char*>(pool_k), static_cast<char*>(pool_v),
                     static_cast<char*>(pool_ind), tables, tables + L, tables + 2 * L, tables + 3 * L);
  CAKE_HIP_TRY(hipGetLastError());
  return CAKE_OK;
}

extern "C" int cake_plan_layout(const cake_shape* shape, size_t* offsets) {
  CAKE_REQUIRE(offsets != nullptr, "offsets is NULL");
  if (int rc = check_shape_basic(shape)) return rc;
  const PlanLayout lay = plan_layout(shape->n_layers, shape->batch);
  const size_t tbl = (size_t)shape->n_layers * sizeof(void*);
  const size_t all[10] = {lay.off_budgets, lay.off_keep, lay.off_cur, lay.off_cap_keep, lay.off_cap_cur, lay.off_blocks,
                          lay.off_tables, lay.off_tables + tbl, lay.off_tables + 2 * tbl, lay.off_tables + 3 * tbl};
  for (int i = 0; i < 10; ++i) offsets[i] = all[i];
  return CAKE_OK;
}

extern "C" int cake_evict_planned(const cake_shape* shape, const float* const* indicator,
                                  const void* const* k_in, const void* const* v_in, const int64_t* kv_strides,
                                  const uint8_t* compacted,
                                  const void* plan, size_t plan_bytes, void* stream) {
  if (int rc = check_shape_basic(shape)) return rc;
  CAKE_REQUIRE(indicator && k_in && v_in && kv_strides && plan, "a pointer argument is NULL");
  CAKE_REQUIRE((int64_t)shape->n_layers * shape->batch * shape->n_kv_heads <= 65535 * 64,
               "too many (layer, sequence, head) rows for one call");
  const int eb = (int)elem_bytes(shape->dtype);
  for (int j = 0; j < 3; ++j) {
    CAKE_REQUIRE(kv_strides[j] >= 0, "negative stride");
    CAKE_REQUIRE((kv_strides[j] * eb) % 16 == 0, "strides must be multiples of 16 bytes");
  }
  const PlanLayout lay = plan_layout(shape->n_layers, shape->batch);
  CAKE_REQUIRE(plan_bytes >= lay.total, "plan has %zu bytes, %zu needed", plan_bytes, lay.total);
  const PlanView view = plan_view(plan, shape->n_layers, shape->batch);
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (int rc = launch_topk_planned(shape, indicator, view, st)) return rc;
  return launch_compact_planned(shape, k_in, v_in, kv_strides, compacted, indicator, view, st);
}
