// cake_select_topk: per-head top-k of the eviction indicator (Sec. 4.3 Eq. 12).
//
// One workgroup per (layer, sequence, KV head) row.  The k-th largest value is found by an
// MSB-first radix select on order-preserving 32-bit keys (digits of 11, 11 and 10 bits, LDS
// histograms), which also yields how many entries equal to the threshold belong to the top k.
// A final ordered pass writes, in ascending position, every entry above the threshold and the
// first `need` entries equal to it: the total order (value descending, position ascending).
// Each of the four sweeps reads the row with 16-byte loads (the row start is brought to a
// 16-byte boundary by a virtual offset); after the first sweep the row comes from the last-level cache.
#include <algorithm>

#include "cake_internal.h"

namespace cake {
namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / 64;
constexpr int kBatch = 8;                           // 16-byte loads in flight per thread in the histogram sweeps
constexpr int kSlotsPerThread = 4;                  // consecutive 4-entry slots per thread in the ordered sweep
constexpr int kTileSlots = kThreads * kSlotsPerThread;
constexpr int kMaxBins = 2048;
constexpr int kCopies = 4;                          // histogram copies, chosen by lane: fewer lanes meet on one LDS address

struct TopkArgs {
  const float* const* indicator;
  int32_t* const* idx;
  int32_t batch, h_kv;
  int32_t cap_cur[kMaxLaunchLayers];
  int32_t cap_keep[kMaxLaunchLayers];
};
// The same dimensions when they live in device memory (an eviction plan).
struct TopkPlan {
  const int32_t* cur_len;     // [L*B]
  const int32_t* keep;        // [L*B]
  const int32_t* cap_cur;     // [L]
  const int32_t* cap_keep;    // [L]
};

// Larger float <=> larger key.  -0 is folded onto +0 first so that they compare equal.
__device__ __forceinline__ uint32_t order_key(float x) {
  uint32_t u = __float_as_uint(x + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// A row seen as slots of four entries whose addresses are 16-byte aligned: slot s holds
// positions 4s - pad .. 4s - pad + 3, pad in 0..3 chosen from the row's address.  Positions
// outside [0, cur) are absent (flagged invalid).
struct Row {
  const float* base;
  int cur, pad, n_slots;
  __device__ __forceinline__ void init(const float* row, int cur_) {
    base = row;
    cur = cur_;
    pad = (int)((reinterpret_cast<uintptr_t>(row) >> 2) & 3);
    n_slots = (cur + pad + 3) >> 2;
  }
  // values of slot s (0 where the position does not exist) and a 4-bit mask of the positions that exist
  __device__ __forceinline__ uint32_t load(int s, float4& x) const {
    const int p0 = 4 * s - pad;
    if (p0 >= 0 && p0 + 3 < cur) {
      x = *reinterpret_cast<const float4*>(base + p0);
      return 0xFu;
    }
    float v[4];
    uint32_t valid = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bool in = p0 + j >= 0 && p0 + j < cur;
      v[j] = in ? base[p0 + j] : 0.f;
      valid |= in ? 1u << j : 0u;
    }
    x = float4{v[0], v[1], v[2], v[3]};
    return valid;
  }
  static __device__ __forceinline__ void keys(const float4& x, uint32_t (&key)[4]) {
    key[0] = order_key(x.x); key[1] = order_key(x.y); key[2] = order_key(x.z); key[3] = order_key(x.w);
  }
};

template <bool kPlanned>
__global__ __launch_bounds__(kThreads) void select_topk_kernel(TopkArgs a, RaggedDims dims, TopkPlan plan) {
  __shared__ __attribute__((aligned(16))) uint32_t hist[kMaxBins * kCopies];     // [digit][copy]
  __shared__ uint32_t sel_prefix, sel_need;
  __shared__ uint32_t wave_tot[2][kWaves];

  const int ll = blockIdx.y;                         // layer within this launch
  const int b = blockIdx.x / a.h_kv, h = blockIdx.x % a.h_kv;
  const int cur = kPlanned ? plan.cur_len[ll * a.batch + b] : dims.cur_len[ll * a.batch + b];
  const int keep = kPlanned ? plan.keep[ll * a.batch + b] : dims.keep[ll * a.batch + b];
  if (keep <= 0) return;
  const int cap_cur = kPlanned ? plan.cap_cur[ll] : a.cap_cur[ll];
  const int cap_keep = kPlanned ? plan.cap_keep[ll] : a.cap_keep[ll];
  Row row;
  row.init(a.indicator[ll] + ((int64_t)b * a.h_kv + h) * cap_cur, cur);
  int32_t* out = a.idx[ll] + ((int64_t)b * a.h_kv + h) * cap_keep;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int copy = lane & (kCopies - 1);

  // ---- radix select: threshold key and number of threshold-equal entries to take ----------
  uint32_t prefix = 0, mask = 0, need = (uint32_t)keep;
#pragma unroll
  for (int pass = 0; pass < 3; ++pass) {
    const int shift = pass == 0 ? 21 : pass == 1 ? 10 : 0;
    const int bits = pass == 2 ? 10 : 11;
    const int n_bins = 1 << bits;
    for (int i = tid; i < n_bins * kCopies; i += kThreads) hist[i] = 0;
    __syncthreads();
    // kBatch independent 16-byte loads are in flight before the first histogram update
    for (int s0 = tid; s0 < row.n_slots; s0 += kThreads * kBatch) {
      float4 x[kBatch];
      uint32_t valid[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        valid[u] = 0;
        if (s0 + u * kThreads < row.n_slots) valid[u] = row.load(s0 + u * kThreads, x[u]);
      }
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        uint32_t key[4];
        Row::keys(x[u], key);
        // Neighbouring entries of a pooled indicator mostly share their leading digits: a slot
        // whose four entries agree takes one update instead of four.
        uint32_t dig[4];
        bool take[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          take[j] = (valid[u] >> j & 1u) && (key[j] & mask) == prefix;
          dig[j] = (key[j] >> shift) & (n_bins - 1);
        }
        if (take[0] && take[1] && take[2] && take[3] && dig[0] == dig[1] && dig[1] == dig[2] && dig[2] == dig[3]) {
          atomicAdd(&hist[dig[0] * kCopies + copy], 4u);
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (take[j]) atomicAdd(&hist[dig[j] * kCopies + copy], 1u);
        }
      }
    }
    __syncthreads();
    if (wave == 0) {
      // lane i owns the per = n_bins/64 digits below n_bins - per*i; scan from the top digit downwards.
      // The sum over a lane's digits is taken in a rotated order so that the lanes hit different banks.
      const int per = n_bins / 64;
      const int top = n_bins - 1 - per * lane;          // this lane's highest digit
      auto bin_count = [&](int d) {
        const uint4 c = *reinterpret_cast<const uint4*>(&hist[d * kCopies]);
        return c.x + c.y + c.z + c.w;
      };
      static_assert(kCopies == 4, "bin_count reads the copies of a digit as one 16-byte word");
      uint32_t s = 0;
      for (int j = 0; j < per; ++j) s += bin_count(top - ((j + lane) & (per - 1)));
      uint32_t incl = s;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        uint32_t t = __shfl_up(incl, off);
        if (lane >= off) incl += t;
      }
      const uint32_t excl = incl - s;
      if (excl < need && need <= incl) {              // exactly one lane
        uint32_t above = excl;
        for (int j = 0; j < per; ++j) {
          const uint32_t c = bin_count(top - j);
          if (need <= above + c) {
            sel_prefix = prefix | ((uint32_t)(top - j) << shift);
            sel_need = need - above;
            break;
          }
          above += c;
        }
      }
    }
    __syncthreads();
    prefix = sel_prefix;
    need = sel_need;
    mask |= (uint32_t)(n_bins - 1) << shift;
  }
  const uint32_t thr = prefix;   // key of the k-th largest entry; `need` entries equal to it are taken

  // ---- ordered output ------------------------------------------------------------------------
  uint32_t base_gt = 0, base_eq = 0;                  // entries above / equal before this tile
  int parity = 0;
  // the next tile's slots are loaded while the current tile is scanned and written
  float4 nx[kSlotsPerThread];
  uint32_t nvalid[kSlotsPerThread];
#pragma unroll
  for (int u = 0; u < kSlotsPerThread; ++u) {
    nvalid[u] = 0;
    if (tid * kSlotsPerThread + u < row.n_slots) nvalid[u] = row.load(tid * kSlotsPerThread + u, nx[u]);
  }
  for (int t0 = 0; t0 < row.n_slots; t0 += kTileSlots, parity ^= 1) {
    const int s0 = t0 + tid * kSlotsPerThread;
    uint32_t key[kSlotsPerThread][4], valid[kSlotsPerThread];
    uint32_t cnt = 0;                                 // low 16 bits: above, high 16 bits: equal
#pragma unroll
    for (int u = 0; u < kSlotsPerThread; ++u) {
      valid[u] = nvalid[u];
      Row::keys(nx[u], key[u]);
      nvalid[u] = 0;
      if (s0 + kTileSlots + u < row.n_slots) nvalid[u] = row.load(s0 + kTileSlots + u, nx[u]);
    }
    // few entries reach the threshold: a slot whose largest key is below it costs four
    // instructions; only the others are counted and written entry by entry
    bool hot[kSlotsPerThread];
#pragma unroll
    for (int u = 0; u < kSlotsPerThread; ++u) {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (!(valid[u] >> j & 1u)) key[u][j] = 0u;       // absent positions: below every real key
      hot[u] = max(max(key[u][0], key[u][1]), max(key[u][2], key[u][3])) >= thr && valid[u] != 0;
      if (hot[u]) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const bool in = valid[u] >> j & 1u;
          cnt += (in && key[u][j] > thr ? 1u : 0u) + (in && key[u][j] == thr ? 0x10000u : 0u);
        }
      }
    }
    uint32_t incl = cnt;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      uint32_t t = __shfl_up(incl, off);
      if (lane >= off) incl += t;
    }
    if (lane == 63) wave_tot[parity][wave] = incl;
    __syncthreads();
    uint32_t before = 0, total = 0;
#pragma unroll
    for (int ww = 0; ww < kWaves; ++ww) {
      uint32_t t = wave_tot[parity][ww];
      if (ww < wave) before += t;
      total += t;
    }
    const uint32_t excl = before + incl - cnt;
    uint32_t gt_before = base_gt + (excl & 0xFFFFu);
    uint32_t eq_before = base_eq + (excl >> 16);
#pragma unroll
    for (int u = 0; u < kSlotsPerThread; ++u) {
      if (!hot[u]) continue;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const bool in = valid[u] >> j & 1u;
        const bool gt = in && key[u][j] > thr;
        const bool eq = in && key[u][j] == thr;
        if (gt || (eq && eq_before < need)) out[gt_before + min(eq_before, need)] = 4 * (s0 + u) - row.pad + j;
        gt_before += gt ? 1u : 0u;
        eq_before += eq ? 1u : 0u;
      }
    }
    base_gt += total & 0xFFFFu;
    base_eq += total >> 16;
  }
}

}  // namespace
}  // namespace cake

int cake::launch_topk_planned(const cake_shape* shape, const float* const* indicator, const PlanView& plan, hipStream_t stream) {
  TopkArgs a{};
  a.indicator = indicator;
  a.idx = reinterpret_cast<int32_t* const*>(plan.idx);
  a.batch = shape->batch;
  a.h_kv = shape->n_kv_heads;
  const TopkPlan tp{plan.cur_len, plan.keep, plan.cap_cur, plan.cap_keep};
  hipLaunchKernelGGL(select_topk_kernel<true>, dim3(shape->batch * shape->n_kv_heads, shape->n_layers), dim3(kThreads), 0,
                     stream, a, RaggedDims{}, tp);
  CAKE_HIP_TRY(hipGetLastError());
  return CAKE_OK;
}

using namespace cake;

extern "C" int cake_select_topk(const cake_shape* shape, const float* const* indicator,
                                const int32_t* cur_len, const int32_t* k, int32_t* const* idx,
                                void* workspace, size_t workspace_bytes, void* stream) {
  (void)workspace; (void)workspace_bytes;
  if (int rc = check_shape_basic(shape)) return rc;
  CAKE_REQUIRE(indicator && idx && cur_len && k, "indicator, idx, cur_len or k is NULL");
  const int B = shape->batch, L = shape->n_layers;
  for (int i = 0; i < L * B; ++i) {
    CAKE_REQUIRE(cur_len[i] >= 0, "cur_len[%d] = %d is negative", i, cur_len[i]);
    CAKE_REQUIRE(k[i] >= 0 && k[i] <= cur_len[i], "k[%d] = %d outside [0, cur_len = %d]", i, k[i], cur_len[i]);
  }
  CAKE_REQUIRE((int64_t)B * shape->n_kv_heads <= 0x7fffffff, "too many rows");
  hipStream_t st = static_cast<hipStream_t>(stream);
  for (int l0 = 0; l0 < L;) {
    const int nl = launch_layers(L - l0, B);
    TopkArgs a{};
    RaggedDims dims{};
    a.indicator = indicator + l0;
    a.idx = idx + l0;
    a.batch = B;
    a.h_kv = shape->n_kv_heads;
    bool any = false;
    for (int ll = 0; ll < nl; ++ll) {
      int cc = 0, ck = 0;
      for (int b = 0; b < B; ++b) {
        const int i = (l0 + ll) * B + b;
        dims.cur_len[ll * B + b] = cur_len[i];
        dims.keep[ll * B + b] = k[i];
        cc = std::max(cc, cur_len[i]);
        ck = std::max(ck, k[i]);
      }
      a.cap_cur[ll] = cc;
      a.cap_keep[ll] = ck;
      any = any || ck > 0;
    }
    if (any)
      hipLaunchKernelGGL(select_topk_kernel<false>, dim3(B * shape->n_kv_heads, nl), dim3(kThreads), 0, st, a, dims, TopkPlan{});
    l0 += nl;
  }
  CAKE_HIP_TRY(hipGetLastError());
  return CAKE_OK;
}
