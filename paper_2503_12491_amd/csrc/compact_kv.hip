// cake_compact_kv: EVICT's gather (Sec. 4.3 Eq. 12, K_hat = K[D,:], V_hat = V[D,:]; Alg. 1
// cache and indicator update).  Pure data movement: every output row is one contiguous run
// of head_dim elements, copied as 16-byte pieces with consecutive lanes on consecutive pieces,
// so a 256-byte bf16 row is one coalesced access of 16 lanes.
#include <algorithm>

#include "cake_internal.h"

namespace cake {
namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 4;   // pieces per thread

struct CompactArgs {
  const void* const* k_in;
  const void* const* v_in;
  const int32_t* const* idx;
  const float* const* ind_in;
  void* const* k_out;
  void* const* v_out;
  float* const* ind_out;
  int32_t batch, h_kv, window, pieces;   // pieces: 16-byte pieces per row
  int32_t elem_bytes;
  int32_t cap_cur[kMaxLaunchLayers];
  int32_t cap_keep[kMaxLaunchLayers];
};

// The same dimensions when they live in device memory (an eviction plan); the strides are then
// the same for every layer.
struct CompactPlan {
  const int32_t* cur_len;     // [L*B]
  const int32_t* keep;        // [L*B]
  const int32_t* cap_cur;     // [L]
  const int32_t* cap_keep;    // [L]
  const int32_t* copy_blocks; // [L*B + 1] running block counts (the work list)
  int32_t n_entries;          // L*B
  int64_t s[3];               // strides of the layers that come as the caller laid them out
  // Bit l set: layer l's K and V are themselves outputs of an earlier planned compaction,
  // contiguous [B, H_kv, cap_cur[l] + S_w, d]; their strides follow from the plan.
  uint32_t compacted[kPlanMaskWords];
};
static_assert(kThreads * kUnroll == kCopyBlockPieces, "a workgroup step is one block of the plan's work list");
constexpr int kListLds = 4096;       // work-list entries searched from LDS (longer lists are searched in memory)

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store_streaming(char* dst, const uint4& x) {
  const u32x4 v = {x.x, x.y, x.z, x.w};
  __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(dst));
}

// A workgroup moves kThreads*kUnroll pieces of one (layer, sequence, head) slice per step.
// Launches that know the row counts on the host give every slice the blocks it needs.  Planned
// launches (counts known only on the device) run a fixed number of workgroups that stride over
// the plan's work list, the blocks of all (layer, sequence) entries in one sequence, head by
// blockIdx.y: the entry of a block is found by bisection of the running counts.
template <bool kPlanned>
__global__ __launch_bounds__(kThreads) void compact_kernel(CompactArgs a, RaggedDims dims, LayerStrides st, CompactPlan plan) {
  __shared__ int32_t list[kPlanned ? kListLds + 1 : 1];
  const int32_t* blocks = plan.copy_blocks;
  int32_t n_blocks = 1;
  if (kPlanned) {
    if (plan.n_entries <= kListLds) {
      for (int i = threadIdx.x; i <= plan.n_entries; i += kThreads) list[i] = plan.copy_blocks[i];
      __syncthreads();
      blocks = list;
    }
    n_blocks = blocks[plan.n_entries];
  }
  const int32_t blk_end = kPlanned ? n_blocks : (int32_t)blockIdx.x + 1;      // host-sized launches: one step per workgroup
  for (int32_t blk = blockIdx.x; blk < blk_end; blk += gridDim.x) {
  int ll, b, h;
  int64_t first;
  if (kPlanned) {
    int lo = 0, hi = plan.n_entries;          // largest e with blocks[e] <= blk (entries without blocks share a count)
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (blocks[mid] <= blk) lo = mid; else hi = mid;
    }
    ll = lo / a.batch; b = lo % a.batch; h = blockIdx.y;
    first = (int64_t)(blk - blocks[lo]) * (kThreads * kUnroll);
  } else {
    ll = blockIdx.z; b = blockIdx.y / a.h_kv; h = blockIdx.y % a.h_kv;
    first = (int64_t)blockIdx.x * (kThreads * kUnroll);
  }
  const int cur = kPlanned ? plan.cur_len[ll * a.batch + b] : dims.cur_len[ll * a.batch + b];
  const int keep = kPlanned ? plan.keep[ll * a.batch + b] : dims.keep[ll * a.batch + b];
  const int cap_cur = kPlanned ? plan.cap_cur[ll] : a.cap_cur[ll];
  const int cap_keep = kPlanned ? plan.cap_keep[ll] : a.cap_keep[ll];
  int64_t s0 = kPlanned ? plan.s[0] : st.s[ll][0], s1 = kPlanned ? plan.s[1] : st.s[ll][1],
          s2 = kPlanned ? plan.s[2] : st.s[ll][2];
  if (kPlanned && (plan.compacted[ll >> 5] >> (ll & 31) & 1u)) {
    s2 = (int64_t)a.pieces * 16 / a.elem_bytes;
    s1 = (int64_t)(cap_cur + a.window) * s2;
    s0 = (int64_t)a.h_kv * s1;
  }
  const int rows_out = keep + a.window;
  const int64_t total = (int64_t)rows_out * a.pieces;

  const int64_t in_off = (b * s0 + h * s1) * a.elem_bytes;
  const int64_t in_row = s2 * a.elem_bytes;
  const int64_t out_row = (int64_t)a.pieces * 16;
  const int64_t out_off = ((int64_t)b * a.h_kv + h) * (cap_keep + a.window) * out_row;
  const char* kin = static_cast<const char*>(a.k_in[ll]) + in_off;
  const char* vin = static_cast<const char*>(a.v_in[ll]) + in_off;
  char* kout = static_cast<char*>(a.k_out[ll]) + out_off;
  char* vout = static_cast<char*>(a.v_out[ll]) + out_off;
  const int32_t* idx = a.idx[ll] + ((int64_t)b * a.h_kv + h) * cap_keep;

  if (first >= total) { if (kPlanned) continue; else return; }
  uint4 kv[kUnroll], vv[kUnroll];
  int64_t dst[kUnroll];
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const int64_t p = first + (int64_t)u * kThreads + threadIdx.x;
    dst[u] = -1;
    if (p < total) {
      const int r = (int)(p / a.pieces), piece = (int)(p % a.pieces);
      // selected prefix rows first, then the window rows that follow the cur prefix rows
      int src = r < keep ? min(max(idx[r], 0), cur - 1) : cur + (r - keep);
      const int64_t so = (int64_t)src * in_row + piece * 16;
      kv[u] = *reinterpret_cast<const uint4*>(kin + so);
      vv[u] = *reinterpret_cast<const uint4*>(vin + so);
      dst[u] = (int64_t)r * out_row + piece * 16;
    }
  }
  // Streaming stores: the compacted rows are not read again by this pass, and plain stores were
  // measured to cost twice their bytes in memory writes (the rows pass through the cache first).
#pragma unroll
  for (int u = 0; u < kUnroll; ++u)
    if (dst[u] >= 0) {
      store_streaming(kout + dst[u], kv[u]);
      store_streaming(vout + dst[u], vv[u]);
    }

  // indicator entries of the retained prefix positions
  if (a.ind_in != nullptr) {
    const float* iin = a.ind_in[ll] + ((int64_t)b * a.h_kv + h) * cap_cur;
    float* iout = a.ind_out[ll] + ((int64_t)b * a.h_kv + h) * cap_keep;
    const int64_t r0 = first / a.pieces;                               // rows this block touches
    const int64_t r1 = min((first + kThreads * kUnroll + a.pieces - 1) / a.pieces, (int64_t)keep);
    // a row split between two blocks is written by the block that holds its piece 0
    for (int64_t r = r0 + threadIdx.x; r < r1; r += kThreads)
      if (r * a.pieces >= first) iout[r] = iin[min(max(idx[r], 0), cur - 1)];
  }
  }
}

}  // namespace
}  // namespace cake

int cake::launch_compact_planned(const cake_shape* shape, const void* const* k_in, const void* const* v_in,
                                 const int64_t* kv_strides, const uint8_t* compacted, const float* const* ind_in,
                                 const PlanView& plan, hipStream_t stream) {
  const int eb = (int)elem_bytes(shape->dtype);
  CompactArgs a{};
  a.k_in = k_in; a.v_in = v_in;
  a.idx = reinterpret_cast<const int32_t* const*>(plan.idx);
  a.ind_in = ind_in;
  a.k_out = plan.k_out; a.v_out = plan.v_out;
  a.ind_out = ind_in ? reinterpret_cast<float* const*>(plan.ind_out) : nullptr;
  a.batch = shape->batch; a.h_kv = shape->n_kv_heads; a.window = shape->window;
  a.pieces = shape->head_dim * eb / 16;
  a.elem_bytes = eb;
  CompactPlan cp{plan.cur_len, plan.keep, plan.cap_cur, plan.cap_keep, plan.copy_blocks, shape->n_layers * shape->batch,
                 {kv_strides[0], kv_strides[1], kv_strides[2]}, {}};
  if (compacted != nullptr)
    for (int l = 0; l < shape->n_layers; ++l)
      if (compacted[l]) cp.compacted[l >> 5] |= 1u << (l & 31);
  // 8192 workgroups in all (a few rounds of what the chip holds at once), striding over the work list
  const unsigned gx = (unsigned)std::max(1, 8192 / shape->n_kv_heads);
  hipLaunchKernelGGL(compact_kernel<true>, dim3(gx, shape->n_kv_heads), dim3(kThreads), 0,
                     stream, a, RaggedDims{}, LayerStrides{}, cp);
  CAKE_HIP_TRY(hipGetLastError());
  return CAKE_OK;
}

using namespace cake;

extern "C" int cake_compact_kv(const cake_shape* shape,
                               const void* const* k_in, const void* const* v_in, const int64_t* kv_strides,
                               const int32_t* cur_len, const int32_t* k, const int32_t* const* idx,
                               const float* const* ind_in,
                               void* const* k_out, void* const* v_out, float* const* ind_out,
                               void* stream) {
  if (int rc = check_shape_basic(shape)) return rc;
  CAKE_REQUIRE(k_in && v_in && kv_strides && cur_len && k && idx && k_out && v_out, "a required pointer is NULL");
  CAKE_REQUIRE((ind_in == nullptr) == (ind_out == nullptr), "ind_in and ind_out must both be given or both be NULL");
  const int B = shape->batch, L = shape->n_layers;
  const int eb = (int)elem_bytes(shape->dtype);
  for (int i = 0; i < L * B; ++i) {
    CAKE_REQUIRE(cur_len[i] >= 0, "cur_len[%d] = %d is negative", i, cur_len[i]);
    CAKE_REQUIRE(k[i] >= 0 && k[i] <= cur_len[i], "k[%d] = %d outside [0, cur_len = %d]", i, k[i], cur_len[i]);
    CAKE_REQUIRE(k[i] == 0 || cur_len[i] > 0, "k > 0 with an empty prefix");
  }
  for (int l = 0; l < L; ++l)
    for (int j = 0; j < 3; ++j) {
      CAKE_REQUIRE(kv_strides[l * 3 + j] >= 0, "negative stride");
      CAKE_REQUIRE((kv_strides[l * 3 + j] * eb) % 16 == 0, "strides must be multiples of 16 bytes");
    }
  hipStream_t st = static_cast<hipStream_t>(stream);
  for (int l0 = 0; l0 < L;) {
    const int nl = launch_layers(L - l0, B);
    CompactArgs a{};
    RaggedDims dims{};
    LayerStrides ls{};
    a.k_in = k_in + l0; a.v_in = v_in + l0; a.idx = idx + l0;
    a.ind_in = ind_in ? ind_in + l0 : nullptr;
    a.k_out = k_out + l0; a.v_out = v_out + l0;
    a.ind_out = ind_out ? ind_out + l0 : nullptr;
    a.batch = B; a.h_kv = shape->n_kv_heads; a.window = shape->window;
    a.pieces = shape->head_dim * eb / 16;
    a.elem_bytes = eb;
    int max_rows = 0;
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
      max_rows = std::max(max_rows, ck + shape->window);
      for (int j = 0; j < 3; ++j) ls.s[ll][j] = kv_strides[(l0 + ll) * 3 + j];
    }
    const int64_t pieces_total = (int64_t)max_rows * a.pieces;
    const unsigned gx = (unsigned)((pieces_total + kThreads * kUnroll - 1) / (kThreads * kUnroll));
    hipLaunchKernelGGL(compact_kernel<false>, dim3(gx, B * shape->n_kv_heads, nl), dim3(kThreads), 0, st, a, dims, ls, CompactPlan{});
    l0 += nl;
  }
  CAKE_HIP_TRY(hipGetLastError());
  return CAKE_OK;
}
