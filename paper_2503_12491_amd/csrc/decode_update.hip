// cake_decode_update: indicator maintenance for one generated token (implementation appendix,
// decoding branch of the listing: the new query's attention over the cached keys outside the
// window is pooled and folded into the stored eviction indicator; the layer is then evicted
// back to its fixed budget with cake_select_topk / cake_compact_kv at k = cur_len - 1).
//
// The cache of a (layer, sequence, KV head) holds cur_len scored rows followed by the S_w window
// rows, the last of which is the new token's key.  The G query heads of the group attend to all
// cur_len + S_w rows (one query row each: a matrix-vector product, done on the vector ALU, one
// row per thread); the weights on the scored rows are averaged over the group, max-pooled along
// the row axis and added to the stored indicator.  Two launches over chunks of 256 rows, so
// that a few thousand rows per head still spread over the chip: per-chunk softmax partials, then
// normaliser + weights (with the pooling halo recomputed) + update.  The keys are read twice
// rather than keeping G logits per row.
#include <algorithm>
#include <cmath>
#include <mutex>

#include "cake_internal.h"

namespace cake {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kMaxGroup = 8;
constexpr float kMasked = -1.0e30f;
constexpr int kMaxHalf = 64;               // widest pooling window: 2*64+1

struct DecodeArgs {
  const void* const* q_new;
  const void* const* k_cache;
  float* const* indicator;
  int64_t qs[2];             // element strides of q_new: batch, head
  int32_t batch, h_kv, group, window, pool;
  int32_t n_chunks;          // chunks of kThreads rows per slice in `part`
  float c;                   // scale * log2(e)
  float inv_g;
  float* part;               // [slice][n_chunks][kMaxGroup][2]: (reference, sum) of each chunk and head
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

// Kernel 1: per chunk of kThreads rows and per head, (reference, sum of 2^(t - reference)).
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void decode_partials_kernel(DecodeArgs a, RaggedDims dims, LayerStrides ks) {
  __shared__ float q_lds[kMaxGroup * D];
  __shared__ float red_m[kWaves][kMaxGroup], red_l[kWaves][kMaxGroup];

  const int chunk = blockIdx.x, ll = blockIdx.z;
  const int b = blockIdx.y / a.h_kv, g = blockIdx.y % a.h_kv;
  const int n = dims.cur_len[ll * a.batch + b] + a.window;       // rows the new query sees
  if (chunk * kThreads >= n) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const T* q = reinterpret_cast<const T*>(a.q_new[ll]) + b * a.qs[0] + (int64_t)(g * a.group) * a.qs[1];
  const T* k = reinterpret_cast<const T*>(a.k_cache[ll]) + b * ks.s[ll][0] + g * ks.s[ll][1];
  for (int i = tid; i < a.group * D; i += kThreads) q_lds[i] = (float)q[(i / D) * a.qs[1] + (i % D)];
  __syncthreads();

  const int j = chunk * kThreads + tid;
  float m[kMaxGroup], l[kMaxGroup];
#pragma unroll
  for (int h = 0; h < kMaxGroup; ++h) { m[h] = kMasked; l[h] = 0.f; }
  if (j < n) {
    row_logits<T, D>(k + j * ks.s[ll][2], q_lds, a.group, a.c, m);
#pragma unroll
    for (int h = 0; h < kMaxGroup; ++h) l[h] = 1.f;
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
  if (tid < a.group) {
    float mm = kMasked, sum = 0.f;
    for (int w = 0; w < kWaves; ++w) mm = fmaxf(mm, red_m[w][tid]);
    for (int w = 0; w < kWaves; ++w) sum += red_l[w][tid] * exp2f(red_m[w][tid] - mm);
    float* o = a.part + ((((int64_t)(ll * a.batch + b) * a.h_kv + g) * a.n_chunks + chunk) * kMaxGroup + tid) * 2;
    o[0] = mm;
    o[1] = sum;
  }
}

// Kernel 2: normalisers from the chunks' pairs, then for this chunk's scored rows (and the pooling
// halo on either side) the group-mean weights, pooled and added to the stored indicator.
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void decode_apply_kernel(DecodeArgs a, RaggedDims dims, LayerStrides ks) {
  __shared__ float q_lds[kMaxGroup * D];
  __shared__ float lse_lds[kMaxGroup];
  __shared__ float obs[kThreads + 2 * kMaxHalf];

  const int chunk = blockIdx.x, ll = blockIdx.z;
  const int b = blockIdx.y / a.h_kv, g = blockIdx.y % a.h_kv;
  const int cur = dims.cur_len[ll * a.batch + b];
  const int n = cur + a.window;
  if (chunk * kThreads >= cur) return;
  const int tid = threadIdx.x;
  const T* q = reinterpret_cast<const T*>(a.q_new[ll]) + b * a.qs[0] + (int64_t)(g * a.group) * a.qs[1];
  const T* k = reinterpret_cast<const T*>(a.k_cache[ll]) + b * ks.s[ll][0] + g * ks.s[ll][1];
  for (int i = tid; i < a.group * D; i += kThreads) q_lds[i] = (float)q[(i / D) * a.qs[1] + (i % D)];
  if (tid < a.group) {
    const int used = (n + kThreads - 1) / kThreads;               // chunks that hold rows
    const float* p = a.part + (((int64_t)(ll * a.batch + b) * a.h_kv + g) * a.n_chunks * kMaxGroup + tid) * 2;
    float mm = kMasked;
    for (int c = 0; c < used; ++c) mm = fmaxf(mm, p[(int64_t)c * kMaxGroup * 2]);
    float sum = 0.f;
    for (int c = 0; c < used; ++c) sum += p[(int64_t)c * kMaxGroup * 2 + 1] * exp2f(p[(int64_t)c * kMaxGroup * 2] - mm);
    lse_lds[tid] = mm + log2f(sum);
  }
  __syncthreads();

  const int half = a.pool / 2;
  const int j0 = chunk * kThreads - half;                          // first row of the halo
  for (int i = tid; i < kThreads + 2 * half; i += kThreads) {
    const int j = j0 + i;
    float w = -INFINITY;                                           // clipped edges never win the max
    if (j >= 0 && j < cur) {
      float t[kMaxGroup];
      row_logits<T, D>(k + j * ks.s[ll][2], q_lds, a.group, a.c, t);
      float s = 0.f;
#pragma unroll
      for (int h = 0; h < kMaxGroup; ++h)
        if (h < a.group) s += exp2f(t[h] - lse_lds[h]);
      w = s * a.inv_g;
    }
    obs[i] = w;
  }
  __syncthreads();
  const int j = chunk * kThreads + tid;
  if (j < cur) {
    float mx = obs[tid + half];
    for (int d = 1; d <= half; ++d) mx = fmaxf(mx, fmaxf(obs[tid + half - d], obs[tid + half + d]));
    float* ind = a.indicator[ll] + ((int64_t)b * a.h_kv + g) * a.cap_cur[ll];
    ind[j] += mx;
  }
}


// ------------------------------------------------------------------------------------------
// In-place decode step (cake_decode_step).  The cache of a (layer, sequence, KV head) lives in
// fixed physical slots; `order` lists the slots in logical order: the cur scored rows by position,
// then the S_w window rows, oldest first.  One generated token: its key and value go to the free
// slot and are appended to the list, so the oldest window row becomes the last scored row (with
// indicator 0); the indicator is updated as in cake_decode_update; the scored row with the
// smallest indicator (the later one among equals: what top-k at k = cur under (value descending,
// position ascending) leaves out) is deleted from the list and its slot becomes the free one.
// K and V are touched at one row per head; only the 4-byte list entries and indicators move.
// ------------------------------------------------------------------------------------------
struct StepArgs {
  const void* q_new; const void* k_new; const void* v_new;
  void* const* k_slots; void* const* v_slots;
  float* const* indicator; int32_t* const* order; int32_t* const* state;
  int64_t qs[3], ns[3];             // element strides of q_new / k_new, v_new: layer, batch, head
  int64_t ss[kMaxLaunchLayers][3];  // element strides of every layer's slots: batch, head, slot
  int32_t batch, h_kv, group, window, pool, n_chunks, rows_max;
  float c, inv_g;
  float* logits;      // [slice][rows_max][kMaxGroup]
  float* part;        // [slice][n_chunks][kMaxGroup][2]
  float* amin;        // [slice][n_chunks][2]: (value, logical index as float bits)
  int32_t cap[kMaxLaunchLayers];
};

// Step kernel 1: the new row goes to its slot and onto the list; logits of the G heads for every
// listed row (kept for the second kernel) and the chunks' (reference, sum) pairs.
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void step_logits_kernel(StepArgs a) {
  __shared__ float q_lds[kMaxGroup * D];
  __shared__ float red_m[kWaves][kMaxGroup], red_l[kWaves][kMaxGroup];
  const int chunk = blockIdx.x, ll = blockIdx.z;
  const int b = blockIdx.y / a.h_kv, g = blockIdx.y % a.h_kv;
  const int64_t slice = ((int64_t)ll * a.batch + b) * a.h_kv + g;
  const int32_t* st = a.state[ll] + ((int64_t)b * a.h_kv + g) * 4;
  const int cur = st[0], free_slot = st[1];
  const int n = cur + 1 + a.window;                       // rows the new query sees
  if (chunk * kThreads >= n) return;
  const int cap = a.cap[ll];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const T* q = reinterpret_cast<const T*>(a.q_new) + ll * a.qs[0] + b * a.qs[1] + (int64_t)(g * a.group) * a.qs[2];
  T* ks = reinterpret_cast<T*>(a.k_slots[ll]) + b * a.ss[ll][0] + g * a.ss[ll][1];
  int32_t* order = a.order[ll] + ((int64_t)b * a.h_kv + g) * (cap + a.window + 1);
  for (int i = tid; i < a.group * D; i += kThreads) q_lds[i] = (float)q[(i / D) * a.qs[2] + (i % D)];
  __syncthreads();

  const int j = chunk * kThreads + tid;
  float m[kMaxGroup], l[kMaxGroup];
#pragma unroll
  for (int h = 0; h < kMaxGroup; ++h) { m[h] = kMasked; l[h] = 0.f; }
  if (j < n) {
    const T* row;
    if (j == n - 1) {
      // the generated token: copy its key and value into the free slot, list it, start its
      // predecessor in the scored part (the row that just left the window) at indicator 0
      const T* kn = reinterpret_cast<const T*>(a.k_new) + ll * a.ns[0] + b * a.ns[1] + g * a.ns[2];
      const T* vn = reinterpret_cast<const T*>(a.v_new) + ll * a.ns[0] + b * a.ns[1] + g * a.ns[2];
      T* kd = ks + free_slot * a.ss[ll][2];
      T* vd = reinterpret_cast<T*>(a.v_slots[ll]) + b * a.ss[ll][0] + g * a.ss[ll][1] + free_slot * a.ss[ll][2];
      for (int e = 0; e < D; e += 16 / (int)sizeof(T)) {
        *reinterpret_cast<uint4*>(kd + e) = *reinterpret_cast<const uint4*>(kn + e);
        *reinterpret_cast<uint4*>(vd + e) = *reinterpret_cast<const uint4*>(vn + e);
      }
      order[j] = free_slot;
      a.indicator[ll][((int64_t)b * a.h_kv + g) * (cap + 1) + cur] = 0.f;
      row = kn;
    } else {
      row = ks + order[j] * a.ss[ll][2];
    }
    row_logits<T, D>(row, q_lds, a.group, a.c, m);
    float* lg = a.logits + (slice * a.rows_max + j) * kMaxGroup;
#pragma unroll
    for (int h = 0; h < kMaxGroup; ++h) { lg[h] = m[h]; l[h] = 1.f; }
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
  if (tid < a.group) {
    float mm = kMasked, sum = 0.f;
    for (int w = 0; w < kWaves; ++w) mm = fmaxf(mm, red_m[w][tid]);
    for (int w = 0; w < kWaves; ++w) sum += red_l[w][tid] * exp2f(red_m[w][tid] - mm);
    float* o = a.part + ((slice * a.n_chunks + chunk) * kMaxGroup + tid) * 2;
    o[0] = mm;
    o[1] = sum;
  }
}

// Step kernel 2: normalisers, pooled group-mean weights added to the indicator of the cur + 1
// scored rows, and this chunk's candidate for eviction: the smallest updated indicator, the later
// row among equals.
__global__ __launch_bounds__(kThreads) void step_apply_kernel(StepArgs a) {
  __shared__ float lse_lds[kMaxGroup];
  __shared__ float obs[kThreads + 2 * kMaxHalf];
  __shared__ float cand_v[kWaves];
  __shared__ int cand_j[kWaves];
  const int chunk = blockIdx.x, ll = blockIdx.z;
  const int b = blockIdx.y / a.h_kv, g = blockIdx.y % a.h_kv;
  const int64_t slice = ((int64_t)ll * a.batch + b) * a.h_kv + g;
  const int32_t* st = a.state[ll] + ((int64_t)b * a.h_kv + g) * 4;
  const int cur1 = st[0] + 1;                              // scored rows, the newcomer included
  const int n = cur1 + a.window;
  if (chunk * kThreads >= cur1) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid < a.group) {
    const int used = (n + kThreads - 1) / kThreads;
    const float* p = a.part + (slice * a.n_chunks * kMaxGroup + tid) * 2;
    float mm = kMasked;
    for (int c = 0; c < used; ++c) mm = fmaxf(mm, p[(int64_t)c * kMaxGroup * 2]);
    float sum = 0.f;
    for (int c = 0; c < used; ++c) sum += p[(int64_t)c * kMaxGroup * 2 + 1] * exp2f(p[(int64_t)c * kMaxGroup * 2] - mm);
    lse_lds[tid] = mm + log2f(sum);
  }
  __syncthreads();
  const int half = a.pool / 2;
  const int j0 = chunk * kThreads - half;
  const float* lg = a.logits + slice * a.rows_max * kMaxGroup;
  for (int i = tid; i < kThreads + 2 * half; i += kThreads) {
    const int j = j0 + i;
    float w = -INFINITY;                                   // clipped edges never win the max
    if (j >= 0 && j < cur1) {
      float s = 0.f;
#pragma unroll
      for (int h = 0; h < kMaxGroup; ++h)
        if (h < a.group) s += exp2f(lg[(int64_t)j * kMaxGroup + h] - lse_lds[h]);
      w = s * a.inv_g;
    }
    obs[i] = w;
  }
  __syncthreads();
  const int j = chunk * kThreads + tid;
  float val = INFINITY;
  int best = -1;
  if (j < cur1) {
    float mx = obs[tid + half];
    for (int d = 1; d <= half; ++d) mx = fmaxf(mx, fmaxf(obs[tid + half - d], obs[tid + half + d]));
    float* ind = a.indicator[ll] + ((int64_t)b * a.h_kv + g) * (a.cap[ll] + 1);
    val = ind[j] + mx;
    ind[j] = val;
    best = j;
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const float ov = __shfl_xor(val, off);
    const int oj = __shfl_xor(best, off);
    if (ov < val || (ov == val && oj > best)) { val = ov; best = oj; }
  }
  if (lane == 0) { cand_v[wave] = val; cand_j[wave] = best; }
  __syncthreads();
  if (tid == 0) {
    for (int w = 1; w < kWaves; ++w)
      if (cand_v[w] < val || (cand_v[w] == val && cand_j[w] > best)) { val = cand_v[w]; best = cand_j[w]; }
    float* o = a.amin + (slice * a.n_chunks + chunk) * 2;
    o[0] = val;
    o[1] = __int_as_float(best);
  }
}

// Step kernel 3: the row to evict over all chunks; it is deleted from the list and from the
// indicator (the later entries move down by one), its slot becomes the free one.
__global__ __launch_bounds__(kThreads) void step_evict_kernel(StepArgs a) {
  __shared__ int evict_lds;
  const int ll = blockIdx.y;
  const int b = blockIdx.x / a.h_kv, g = blockIdx.x % a.h_kv;
  const int64_t slice = ((int64_t)ll * a.batch + b) * a.h_kv + g;
  int32_t* st = a.state[ll] + ((int64_t)b * a.h_kv + g) * 4;
  const int cur = st[0], cur1 = cur + 1, n = cur1 + a.window;
  const int cap = a.cap[ll];
  const int tid = threadIdx.x;
  int32_t* order = a.order[ll] + ((int64_t)b * a.h_kv + g) * (cap + a.window + 1);
  float* ind = a.indicator[ll] + ((int64_t)b * a.h_kv + g) * (cap + 1);
  if (tid == 0) {
    const int used = (cur1 + kThreads - 1) / kThreads;
    const float* p = a.amin + slice * a.n_chunks * 2;
    float val = p[0];
    int best = __float_as_int(p[1]);
    for (int c = 1; c < used; ++c) {
      const float v = p[2 * c];
      const int jj = __float_as_int(p[2 * c + 1]);
      if (v < val || (v == val && jj > best)) { val = v; best = jj; }
    }
    evict_lds = best;
  }
  __syncthreads();
  const int e = evict_lds;
  const int freed = order[e];
  __syncthreads();
  for (int base = e; base < n - 1; base += kThreads) {     // entries base+1.. move to base..: read all, then write
    const int jj = base + tid;
    const bool live = jj < n - 1;
    const int32_t o = live ? order[jj + 1] : 0;
    const float x = (live && jj + 1 < cur1) ? ind[jj + 1] : 0.f;
    __syncthreads();
    if (live) order[jj] = o;
    if (live && jj + 1 < cur1) ind[jj] = x;
    __syncthreads();
  }
  if (tid == 0) {
    st[1] = freed;
    st[2] = e;          // logical index of the evicted scored row (for inspection)
  }
}

}  // namespace
}  // namespace cake

using namespace cake;

namespace {

// Scratch of the entry point that may not take a workspace from its caller: the chunks'
// (reference, sum) pairs.  Every GPU the library runs on holds its own copy of this array until
// the process ends.  In host code the array's name is only a handle: its device address is
// looked up once per device and only that address is ever handed to a kernel.
constexpr size_t kStaticScratchBytes = size_t(1) << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device.
int static_scratch(void** out) {
  int dev = -1;
  CAKE_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(CAKE_ERR_UNSUPPORTED, "device ordinal %d outside [0, %d)", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    CAKE_HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (ptr == nullptr) return fail(CAKE_ERR_HIP, "hipGetSymbolAddress returned a null address");
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return CAKE_OK;
}

// Bytes of (reference, sum) pairs a call with this shape writes.
size_t decode_part_bytes(const cake_shape& shape) {
  const size_t n_chunks = ((size_t)shape.seq_len + kThreads - 1) / kThreads;
  return sizeof(float) * (size_t)shape.n_layers * shape.batch * shape.n_kv_heads * n_chunks * kMaxGroup * 2;
}

// Argument checks and the two launches; `part` is device memory of at least decode_part_bytes.
int decode_update_impl(const cake_shape* shape, const cake_params* params,
                       const void* const* q_new, const int64_t* q_strides,
                       const void* const* k_cache, const int64_t* k_strides,
                       const int32_t* cur_len, float* const* indicator,
                       float* part, void* stream) {
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
  const int n_chunks = (shape->seq_len + kThreads - 1) / kThreads;
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
    a.n_chunks = n_chunks;
    a.c = (float)(scale * 1.4426950408889634);
    a.inv_g = 1.0f / (float)G;
    a.part = part + (int64_t)l0 * B * shape->n_kv_heads * n_chunks * kMaxGroup * 2;
    int max_cur = 0;
    for (int ll = 0; ll < nl; ++ll) {
      int cc = 0;
      for (int b = 0; b < B; ++b) {
        dims.cur_len[ll * B + b] = cur_len[(l0 + ll) * B + b];
        cc = std::max(cc, cur_len[(l0 + ll) * B + b]);
      }
      a.cap_cur[ll] = cc;
      max_cur = std::max(max_cur, cc);
      for (int i = 0; i < 3; ++i) ks.s[ll][i] = k_strides[(l0 + ll) * 3 + i];
    }
    const int used = (max_cur + shape->window + kThreads - 1) / kThreads;
    dim3 grid(used, B * shape->n_kv_heads, nl), block(kThreads);
#define CAKE_DECODE(T, D)                                                                        \
  do {                                                                                           \
    hipLaunchKernelGGL((decode_partials_kernel<T, D>), grid, block, 0, st, a, dims, ks);         \
    hipLaunchKernelGGL((decode_apply_kernel<T, D>), grid, block, 0, st, a, dims, ks);            \
  } while (0)
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

}  // namespace

extern "C" int cake_decode_update(const cake_shape* shape, const cake_params* params,
                                  const void* const* q_new, const int64_t* q_strides,
                                  const void* const* k_cache, const int64_t* k_strides,
                                  const int32_t* cur_len, float* const* indicator,
                                  void* workspace, size_t workspace_bytes, void* stream) {
  if (int rc = check_shape_scores(shape)) return rc;
  CAKE_REQUIRE(params != nullptr, "params is NULL");
  CAKE_REQUIRE(q_new && k_cache && indicator && q_strides && k_strides && cur_len, "a pointer argument is NULL");
  const ScoreLayout lay = score_layout(*shape);
  if (workspace == nullptr || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0)
    return fail(CAKE_ERR_WORKSPACE, "workspace is NULL or not 256-byte aligned");
  if (workspace_bytes < lay.total)
    return fail(CAKE_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, lay.total);
  // the chunks' (reference, sum) pairs live where the score pass keeps its own partial pairs
  const size_t part_bytes = decode_part_bytes(*shape);
  if (lay.off_part + part_bytes > lay.total)
    return fail(CAKE_ERR_WORKSPACE, "workspace layout leaves %zu bytes for the decode partials, %zu needed",
                lay.total - lay.off_part, part_bytes);
  return decode_update_impl(shape, params, q_new, q_strides, k_cache, k_strides, cur_len, indicator,
                            reinterpret_cast<float*>(static_cast<char*>(workspace) + lay.off_part), stream);
}

extern "C" int cake_decode_update_static(const cake_shape* shape, const cake_params* params,
                                         const void* const* q_new, const int64_t* q_strides,
                                         const void* const* k_cache, const int64_t* k_strides,
                                         const int32_t* cur_len, float* const* indicator, void* stream) {
  if (int rc = check_shape_scores(shape)) return rc;
  CAKE_REQUIRE(params != nullptr, "params is NULL");
  CAKE_REQUIRE(q_new && k_cache && indicator && q_strides && k_strides && cur_len, "a pointer argument is NULL");
  const size_t part_bytes = decode_part_bytes(*shape);
  if (part_bytes > kStaticScratchBytes)
    return fail(CAKE_ERR_UNSUPPORTED,
                "cake_decode_update_static: n_layers*batch*n_kv_heads*ceil(seq_len/%d) = %zu chunk entries need %zu bytes, "
                "the built-in scratch holds %zu (use cake_decode_update with a workspace)",
                kThreads, part_bytes / (sizeof(float) * kMaxGroup * 2), part_bytes, kStaticScratchBytes);
  void* ptr = nullptr;
  if (int rc = static_scratch(&ptr)) return rc;
  return decode_update_impl(shape, params, q_new, q_strides, k_cache, k_strides, cur_len, indicator,
                            static_cast<float*>(ptr), stream);
}

extern "C" int cake_decode_step_workspace_bytes(const cake_shape* shape, size_t* bytes) {
  CAKE_REQUIRE(bytes != nullptr, "bytes is NULL");
  if (int rc = check_shape_scores(shape)) return rc;
  const size_t slices = (size_t)shape->n_layers * shape->batch * shape->n_kv_heads;
  const size_t n_chunks = ((size_t)shape->seq_len + kThreads - 1) / kThreads;
  *bytes = align_up(sizeof(float) * slices * shape->seq_len * kMaxGroup, 256) +
           align_up(sizeof(float) * slices * n_chunks * kMaxGroup * 2, 256) + align_up(sizeof(float) * slices * n_chunks * 2, 256);
  return CAKE_OK;
}

extern "C" int cake_decode_step(const cake_shape* shape, const cake_params* params,
                                const void* q_new, const int64_t* q_strides,
                                const void* k_new, const void* v_new, const int64_t* kv_new_strides,
                                void* const* k_slots, void* const* v_slots, const int64_t* slot_strides,
                                float* const* indicator, int32_t* const* order, int32_t* const* state,
                                const int32_t* cap, void* workspace, size_t workspace_bytes, void* stream) {
  if (int rc = check_shape_scores(shape)) return rc;
  CAKE_REQUIRE(params != nullptr, "params is NULL");
  CAKE_REQUIRE(q_new && k_new && v_new && k_slots && v_slots && indicator && order && state && q_strides && kv_new_strides &&
                   slot_strides && cap, "a pointer argument is NULL");
  CAKE_REQUIRE(params->pool_kernel >= 1 && params->pool_kernel % 2 == 1 && params->pool_kernel <= 129,
               "pool_kernel %d must be odd and within [1, 129]", params->pool_kernel);
  CAKE_REQUIRE(std::isfinite(params->scale) && params->scale >= 0.f, "scale must be finite and >= 0");
  const int B = shape->batch, L = shape->n_layers, G = shape->n_q_heads / shape->n_kv_heads;
  CAKE_REQUIRE(L <= kMaxLaunchLayers, "at most %d layers per cake_decode_step call", kMaxLaunchLayers);
  const size_t eb = elem_bytes(shape->dtype);
  for (int i = 0; i < 3; ++i) {
    CAKE_REQUIRE(q_strides[i] >= 0 && kv_new_strides[i] >= 0, "negative stride");
    CAKE_REQUIRE((q_strides[i] * eb) % 16 == 0 && (kv_new_strides[i] * eb) % 16 == 0, "strides must be multiples of 16 bytes");
  }
  for (int i = 0; i < 3 * L; ++i) {
    CAKE_REQUIRE(slot_strides[i] >= 0, "negative stride");
    CAKE_REQUIRE((slot_strides[i] * eb) % 16 == 0, "strides must be multiples of 16 bytes");
  }
  for (int l = 0; l < L; ++l)
    CAKE_REQUIRE(cap[l] >= 0 && cap[l] + shape->window + 1 <= shape->seq_len,
                 "cap[%d] = %d: cap + window + 1 must not exceed shape.seq_len = %d", l, cap[l], shape->seq_len);
  size_t need = 0;
  if (int rc = cake_decode_step_workspace_bytes(shape, &need)) return rc;
  if (workspace == nullptr || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0)
    return fail(CAKE_ERR_WORKSPACE, "workspace is NULL or not 256-byte aligned");
  if (workspace_bytes < need) return fail(CAKE_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, need);

  StepArgs a{};
  a.q_new = q_new; a.k_new = k_new; a.v_new = v_new;
  a.k_slots = k_slots; a.v_slots = v_slots; a.indicator = indicator; a.order = order; a.state = state;
  for (int i = 0; i < 3; ++i) { a.qs[i] = q_strides[i]; a.ns[i] = kv_new_strides[i]; }
  for (int l = 0; l < L; ++l)
    for (int i = 0; i < 3; ++i) a.ss[l][i] = slot_strides[l * 3 + i];
  a.batch = B; a.h_kv = shape->n_kv_heads; a.group = G; a.window = shape->window; a.pool = params->pool_kernel;
  a.rows_max = shape->seq_len;
  a.n_chunks = (shape->seq_len + kThreads - 1) / kThreads;
  const double scale = params->scale > 0.f ? (double)params->scale : 1.0 / std::sqrt((double)shape->head_dim);
  a.c = (float)(scale * 1.4426950408889634);
  a.inv_g = 1.0f / (float)G;
  const size_t slices = (size_t)L * B * shape->n_kv_heads;
  char* ws = static_cast<char*>(workspace);
  a.logits = reinterpret_cast<float*>(ws);
  ws += align_up(sizeof(float) * slices * shape->seq_len * kMaxGroup, 256);
  a.part = reinterpret_cast<float*>(ws);
  ws += align_up(sizeof(float) * slices * a.n_chunks * kMaxGroup * 2, 256);
  a.amin = reinterpret_cast<float*>(ws);
  int cap_max = 0;
  for (int l = 0; l < L; ++l) { a.cap[l] = cap[l]; cap_max = std::max(cap_max, cap[l]); }
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int used = (cap_max + shape->window + 1 + kThreads - 1) / kThreads;
  const dim3 grid(used, B * shape->n_kv_heads, L), block(kThreads);
  const bool bf = shape->dtype == CAKE_BF16;
  if (bf && shape->head_dim == 128) hipLaunchKernelGGL((step_logits_kernel<__bf16, 128>), grid, block, 0, st, a);
  else if (bf && shape->head_dim == 64) hipLaunchKernelGGL((step_logits_kernel<__bf16, 64>), grid, block, 0, st, a);
  else if (!bf && shape->head_dim == 128) hipLaunchKernelGGL((step_logits_kernel<float, 128>), grid, block, 0, st, a);
  else if (!bf && shape->head_dim == 64) hipLaunchKernelGGL((step_logits_kernel<float, 64>), grid, block, 0, st, a);
  else return fail(CAKE_ERR_UNSUPPORTED, "no decode kernel for this shape");
  hipLaunchKernelGGL(step_apply_kernel, grid, block, 0, st, a);
  hipLaunchKernelGGL(step_evict_kernel, dim3(B * shape->n_kv_heads, L), block, 0, st, a);
  CAKE_HIP_TRY(hipGetLastError());
  return CAKE_OK;
}
