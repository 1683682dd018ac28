// cake_select_topk: per-head top-k of the eviction indicator (Sec. 4.3 Eq. 12).
//
// One workgroup per (layer, sequence, KV head) row.  The k-th largest value is found by an
// MSB-first radix select on order-preserving 32-bit keys (four 8-bit digits, LDS histograms),
// which also yields how many entries equal to the threshold belong to the top k.  A final
// ordered pass writes, in ascending position, every entry above the threshold and the first
// `need` entries equal to it: the total order (value descending, position ascending).
// The row stays in the L2 of the compute unit's XCD between passes.
#include <algorithm>

#include "cake_internal.h"

namespace cake {
namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / 64;
constexpr int kPerThread = 4;                       // consecutive entries per thread in the ordered pass
constexpr int kTile = kThreads * kPerThread;
constexpr int kBatch = 8;                           // loads in flight per thread in the histogram passes

struct TopkArgs {
  const float* const* indicator;
  int32_t* const* idx;
  int32_t batch, h_kv;
  int32_t cap_cur[kMaxLaunchLayers];
  int32_t cap_keep[kMaxLaunchLayers];
};

// Larger float <=> larger key.  -0 is folded onto +0 first so that they compare equal.
__device__ __forceinline__ uint32_t order_key(float x) {
  uint32_t u = __float_as_uint(x + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__global__ __launch_bounds__(kThreads) void select_topk_kernel(TopkArgs a, RaggedDims dims) {
  __shared__ uint32_t hist[256];
  __shared__ uint32_t sel_prefix, sel_need;
  __shared__ uint32_t wave_tot[2][kWaves];

  const int ll = blockIdx.y;                         // layer within this launch
  const int b = blockIdx.x / a.h_kv, h = blockIdx.x % a.h_kv;
  const int cur = dims.cur_len[ll * a.batch + b];
  const int keep = dims.keep[ll * a.batch + b];
  if (keep <= 0) return;
  const float* row = a.indicator[ll] + ((int64_t)b * a.h_kv + h) * a.cap_cur[ll];
  int32_t* out = a.idx[ll] + ((int64_t)b * a.h_kv + h) * a.cap_keep[ll];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  // ---- radix select: threshold key and number of threshold-equal entries to take ----------
  uint32_t prefix = 0, mask = 0, need = (uint32_t)keep;
  for (int shift = 24; shift >= 0; shift -= 8) {
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    // kBatch independent loads are in flight before the first histogram update, so that the
    // pass runs at memory throughput rather than one load latency per element
    for (int i0 = tid; i0 < cur; i0 += kThreads * kBatch) {
      float x[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) x[u] = (i0 + u * kThreads < cur) ? row[i0 + u * kThreads] : 0.f;
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const uint32_t key = order_key(x[u]);
        if (i0 + u * kThreads < cur && (key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 0xFF], 1u);
      }
    }
    __syncthreads();
    if (wave == 0) {
      // lane i owns digits 255-4i .. 252-4i; scan from the top digit downwards
      uint32_t c[4], s = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) { c[j] = hist[255 - (4 * lane + j)]; s += c[j]; }
      uint32_t incl = s;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        uint32_t t = __shfl_up(incl, off);
        if (lane >= off) incl += t;
      }
      uint32_t excl = incl - s;
      if (excl < need && need <= incl) {              // exactly one lane
        uint32_t above = excl;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if (need <= above + c[j]) {
            sel_prefix = prefix | ((uint32_t)(255 - (4 * lane + j)) << shift);
            sel_need = need - above;
            break;
          }
          above += c[j];
        }
      }
    }
    __syncthreads();
    prefix = sel_prefix;
    need = sel_need;
    mask |= 0xFFu << shift;
  }
  const uint32_t thr = prefix;   // key of the k-th largest entry; `need` entries equal to it are taken

  // ---- ordered output ------------------------------------------------------------------------
  uint32_t base_gt = 0, base_eq = 0;                  // entries above / equal before this tile
  int parity = 0;
  for (int t0 = 0; t0 < cur; t0 += kTile, parity ^= 1) {
    const int i0 = t0 + tid * kPerThread;
    uint32_t key[kPerThread];
    uint32_t cnt = 0;                                 // low 16 bits: above, high 16 bits: equal
#pragma unroll
    for (int j = 0; j < kPerThread; ++j) {
      key[j] = (i0 + j < cur) ? order_key(row[i0 + j]) : 0u;   // key 0 is below every float's key
      cnt += (key[j] > thr ? 1u : 0u) + (key[j] == thr && i0 + j < cur ? 0x10000u : 0u);
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
    uint32_t excl = before + incl - cnt;
    uint32_t gt_before = base_gt + (excl & 0xFFFFu);
    uint32_t eq_before = base_eq + (excl >> 16);
#pragma unroll
    for (int j = 0; j < kPerThread; ++j) {
      const bool gt = key[j] > thr;
      const bool eq = key[j] == thr && i0 + j < cur;
      if (gt || (eq && eq_before < need)) out[gt_before + min(eq_before, need)] = i0 + j;
      gt_before += gt ? 1u : 0u;
      eq_before += eq ? 1u : 0u;
    }
    base_gt += total & 0xFFFFu;
    base_eq += total >> 16;
  }
}

}  // namespace
}  // namespace cake

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
      hipLaunchKernelGGL(select_topk_kernel, dim3(B * shape->n_kv_heads, nl), dim3(kThreads), 0, st, a, dims);
    l0 += nl;
  }
  CAKE_HIP_TRY(hipGetLastError());
  return CAKE_OK;
}
