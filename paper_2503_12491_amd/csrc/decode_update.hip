// cake_decode_update: indicator maintenance for one generated token (implementation appendix,
// decoding branch of the listing: the new query's attention over the cached keys outside the
// window is pooled and folded into the stored eviction indicator; the layer is then evicted
// back to its fixed budget with cake_select_topk / cake_compact_kv at k = cur_len - 1).
//
// One workgroup per (layer, sequence, KV head).  The cache of that head holds cur_len scored
// rows followed by the S_w window rows, the last of which is the new token's key.  The G query
// heads of the group attend to all cur_len + S_w rows (one query row each: a matrix-vector
// product, done on the vector ALU); the weights on the scored rows are averaged over the group,
// max-pooled along the row axis and added to the stored indicator.  Caches at their budget are a
// few thousand rows per head, so the kernel is latency-bound by design; the keys are read
// twice (normaliser, then weights) rather than keeping G logits per row.
#include <algorithm>
#include <cmath>

#include "cake_internal.h"

namespace cake {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kMaxGroup = 8;
constexpr float kMasked = -1.0e30f;

struct DecodeArgs {
  const void* const* q_new;
  const void* const* k_cache;
  float* const* indicator;
  int64_t qs[2];             // element strides of q_new: batch, head
  int32_t batch, h_kv, group, window, pool;
  int32_t obs_stride;        // floats per slice in `obs`
  float c;                   // scale * log2(e)
  float inv_g;
  float* obs;                // [slice][obs_stride]: group-mean weights on the scored rows
  int32_t cap_cur[kMaxLaunchLayers];
};

template <typename T> struct Row16;      // sixteen bytes of a key row as floats
template <> struct Row16<__bf16> {
  static constexpr int kElems = 8;
  static __device__ __forceinline__ void load(const __bf16* p, float (&x)[8]) {
    typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
    const bf16x8 v = *reinterpret_cast<const bf16x8*>(p);
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = (float)v[i];
  }
};
template <> struct Row16<float> {
  static constexpr int kElems = 4;
  static __device__ __forceinline__ void load(const float* p, float (&x)[4]) {
    const float4 v = *reinterpret_cast<const float4*>(p);
    x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
  }
};

// t[h] = c * <q_h, k_row> for the G heads of the group; q lies in LDS as floats [G][D].
template <typename T, int D>
__device__ __forceinline__ void row_logits(const T* k_row, const float* q_lds, int group, float c, float (&t)[kMaxGroup]) {
  using R = Row16<T>;
  float acc[kMaxGroup];
#pragma unroll
  for (int h = 0; h < kMaxGroup; ++h) acc[h] = 0.f;
#pragma unroll
  for (int e0 = 0; e0 < D; e0 += R::kElems) {
    float x[R::kElems];
    R::load(k_row + e0, x);
#pragma unroll
    for (int h = 0; h < kMaxGroup; ++h) {
      if (h < group) {
#pragma unroll
        for (int i = 0; i < R::kElems; ++i) acc[h] = fmaf(x[i], q_lds[h * D + e0 + i], acc[h]);
      }
    }
  }
#pragma unroll
  for (int h = 0; h < kMaxGroup; ++h) t[h] = acc[h] * c;
}

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void decode_update_kernel(DecodeArgs a, RaggedDims dims, LayerStrides ks) {
  __shared__ float q_lds[kMaxGroup * D];
  __shared__ float red_m[kWaves][kMaxGroup], red_l[kWaves][kMaxGroup];
  __shared__ float lse_lds[kMaxGroup];

  const int ll = blockIdx.y;
  const int b = blockIdx.x / a.h_kv, g = blockIdx.x % a.h_kv;
  const int cur = dims.cur_len[ll * a.batch + b];
  const int n = cur + a.window;                                  // rows the new query sees
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const T* q = reinterpret_cast<const T*>(a.q_new[ll]) + b * a.qs[0] + (int64_t)(g * a.group) * a.qs[1];
  const T* k = reinterpret_cast<const T*>(a.k_cache[ll]) + b * ks.s[ll][0] + g * ks.s[ll][1];
  const int64_t tok = ks.s[ll][2];
  for (int i = tid; i < a.group * D; i += kThreads) q_lds[i] = (float)q[(i / D) * a.qs[1] + (i % D)];
  __syncthreads();

  // ---- normaliser of every head: running (reference, sum) per thread, then over the workgroup
  float m[kMaxGroup], l[kMaxGroup];
#pragma unroll
  for (int h = 0; h < kMaxGroup; ++h) { m[h] = kMasked; l[h] = 0.f; }
  for (int j = tid; j < n; j += kThreads) {
    float t[kMaxGroup];
    row_logits<T, D>(k + j * tok, q_lds, a.group, a.c, t);
#pragma unroll
    for (int h = 0; h < kMaxGroup; ++h) {
      if (h < a.group) {
        const float mn = fmaxf(m[h], t[h]);
        l[h] = l[h] * exp2f(m[h] - mn) + exp2f(t[h] - mn);
        m[h] = mn;
      }
    }
  }
#pragma unroll
  for (int h = 0; h < kMaxGroup; ++h) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      const float om = __shfl_xor(m[h], off), ol = __shfl_xor(l[h], off);
      const float mn = fmaxf(m[h], om);
      l[h] = l[h] * exp2f(m[h] - mn) + ol * exp2f(om - mn);
      m[h] = mn;
    }
    if (lane == 0) { red_m[wave][h] = m[h]; red_l[wave][h] = l[h]; }
  }
  __syncthreads();
  if (tid < kMaxGroup) {
    float mm = kMasked, s = 0.f;
    for (int w = 0; w < kWaves; ++w) mm = fmaxf(mm, red_m[w][tid]);
    for (int w = 0; w < kWaves; ++w) s += red_l[w][tid] * exp2f(red_m[w][tid] - mm);
    lse_lds[tid] = mm + log2f(s);            // heads >= G: never read
  }
  __syncthreads();

  // ---- weights of the scored rows, averaged over the group
  float* obs = a.obs + (int64_t)((ll * a.batch + b) * a.h_kv + g) * a.obs_stride;
  for (int j = tid; j < cur; j += kThreads) {
    float t[kMaxGroup];
    row_logits<T, D>(k + j * tok, q_lds, a.group, a.c, t);
    float s = 0.f;
#pragma unroll
    for (int h = 0; h < kMaxGroup; ++h)
      if (h < a.group) s += exp2f(t[h] - lse_lds[h]);
    obs[j] = s * a.inv_g;
  }
  __threadfence_block();
  __syncthreads();

  // ---- pooled weights are added to the stored indicator
  float* ind = a.indicator[ll] + ((int64_t)b * a.h_kv + g) * a.cap_cur[ll];
  const int half = a.pool / 2;
  for (int j = tid; j < cur; j += kThreads) {
    float mx = obs[j];
    for (int d = 1; d <= half; ++d) {
      if (j - d >= 0) mx = fmaxf(mx, obs[j - d]);
      if (j + d < cur) mx = fmaxf(mx, obs[j + d]);
    }
    ind[j] += mx;
  }
}

}  // namespace
}  // namespace cake

using namespace cake;

extern "C" int cake_decode_update(const cake_shape* shape, const cake_params* params,
                                  const void* const* q_new, const int64_t* q_strides,
                                  const void* const* k_cache, const int64_t* k_strides,
                                  const int32_t* cur_len, float* const* indicator,
                                  void* workspace, size_t workspace_bytes, void* stream) {
  if (int rc = check_shape_scores(shape)) return rc;
  CAKE_REQUIRE(params != nullptr, "params is NULL");
  CAKE_REQUIRE(q_new && k_cache && indicator && q_strides && k_strides && cur_len, "a pointer argument is NULL");
  CAKE_REQUIRE(params->pool_kernel >= 1 && params->pool_kernel % 2 == 1 && params->pool_kernel <= 129,
               "pool_kernel %d must be odd and within [1, 129]", params->pool_kernel);
  CAKE_REQUIRE(std::isfinite(params->scale) && params->scale >= 0.f, "scale must be finite and >= 0");
  const int B = shape->batch, L = shape->n_layers;
  const int G = shape->n_q_heads / shape->n_kv_heads;
  const int n_p = shape->seq_len - shape->window;
  const size_t eb = elem_bytes(shape->dtype);
  CAKE_REQUIRE(q_strides[0] >= 0 && q_strides[1] >= shape->head_dim && (q_strides[0] * eb) % 16 == 0 &&
                   (q_strides[1] * eb) % 16 == 0, "q_new strides must be multiples of 16 bytes, head stride >= head_dim");
  for (int i = 0; i < L * 3; ++i)
    CAKE_REQUIRE(k_strides[i] >= 0 && (k_strides[i] * eb) % 16 == 0, "k_cache strides must be non-negative multiples of 16 bytes");
  for (int i = 0; i < L * B; ++i)
    CAKE_REQUIRE(cur_len[i] >= 0 && cur_len[i] <= n_p, "cur_len[%d] = %d outside [0, seq_len - window = %d]", i, cur_len[i], n_p);
  const ScoreLayout lay = score_layout(*shape);
  if (workspace == nullptr || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0)
    return fail(CAKE_ERR_WORKSPACE, "workspace is NULL or not 256-byte aligned");
  if (workspace_bytes < lay.total)
    return fail(CAKE_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, lay.total);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const double scale = params->scale > 0.f ? (double)params->scale : 1.0 / std::sqrt((double)shape->head_dim);
  for (int l0 = 0; l0 < L;) {
    const int nl = launch_layers(L - l0, B);
    DecodeArgs a{};
    RaggedDims dims{};
    LayerStrides ks{};
    a.q_new = q_new + l0; a.k_cache = k_cache + l0; a.indicator = indicator + l0;
    a.qs[0] = q_strides[0]; a.qs[1] = q_strides[1];
    a.batch = B; a.h_kv = shape->n_kv_heads; a.group = G; a.window = shape->window; a.pool = params->pool_kernel;
    a.obs_stride = n_p;
    a.c = (float)(scale * 1.4426950408889634);
    a.inv_g = 1.0f / (float)G;
    a.obs = reinterpret_cast<float*>(static_cast<char*>(workspace) + lay.off_raw) + (int64_t)l0 * B * shape->n_kv_heads * n_p;
    for (int ll = 0; ll < nl; ++ll) {
      int cc = 0;
      for (int b = 0; b < B; ++b) {
        dims.cur_len[ll * B + b] = cur_len[(l0 + ll) * B + b];
        cc = std::max(cc, cur_len[(l0 + ll) * B + b]);
      }
      a.cap_cur[ll] = cc;
      for (int i = 0; i < 3; ++i) ks.s[ll][i] = k_strides[(l0 + ll) * 3 + i];
    }
    dim3 grid(B * shape->n_kv_heads, nl), block(kThreads);
#define CAKE_DECODE(T, D) hipLaunchKernelGGL((decode_update_kernel<T, D>), grid, block, 0, st, a, dims, ks)
    const bool bf = shape->dtype == CAKE_BF16;
    if (bf && shape->head_dim == 128) CAKE_DECODE(__bf16, 128);
    else if (bf && shape->head_dim == 64) CAKE_DECODE(__bf16, 64);
    else if (!bf && shape->head_dim == 128) CAKE_DECODE(float, 128);
    else if (!bf && shape->head_dim == 64) CAKE_DECODE(float, 64);
    else return fail(CAKE_ERR_UNSUPPORTED, "no decode kernel for this shape");
#undef CAKE_DECODE
    l0 += nl;
  }
  CAKE_HIP_TRY(hipGetLastError());
  return CAKE_OK;
}
