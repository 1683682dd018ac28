// cake_quantize_kv: b-bit storage of the retained cache (appendix "Comparison and compatibility
// with quantization methods": eviction combined with a key-per-channel / value-per-token
// quantiser).  Asymmetric uniform quantisation over groups of 32: the keys of a head per channel
// over 32 consecutive retained tokens, the values per token over 32 consecutive channels;
// zero = group minimum, scale = (max - min) / (2^b - 1), code = round-half-even((x - zero) / scale).
// The window rows are not touched: they stay in the compacted arrays as they are.
//
// One workgroup per (layer, sequence, head, group of 32 tokens): the 32 x d tile of K and of V is
// read once with 16-byte loads into LDS as fp32, statistics and codes are formed there, and the
// packed codes leave as whole rows.  Pure streaming: bound by HBM.
#include <algorithm>

#include "cake_internal.h"

namespace cake {
namespace {

constexpr int kThreads = 256;
constexpr int kGroup = 32;       // tokens per key group, channels per value group

struct QuantArgs {
  const void* const* k_hat;
  const void* const* v_hat;
  uint8_t* const* k_codes; float* const* k_scale; float* const* k_zero;
  uint8_t* const* v_codes; float* const* v_scale; float* const* v_zero;
  int32_t batch, h_kv, bits;
  int32_t cap[kMaxLaunchLayers];
};

__device__ __forceinline__ float to_float(__bf16 x) { return (float)x; }
__device__ __forceinline__ float to_float(float x) { return x; }

// code of x in a group with minimum lo and step sc (sc = 0: a constant group, code 0)
__device__ __forceinline__ uint32_t encode(float x, float lo, float sc, float levels) {
  if (!(sc > 0.f)) return 0u;
  const float c = rintf((x - lo) / sc);
  return (uint32_t)fminf(fmaxf(c, 0.f), levels);
}

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void quantize_kernel(QuantArgs a, RaggedDims dims, LayerStrides st) {
  constexpr int kPad = D + 1;                        // column reads of the tile without bank conflicts
  constexpr int kVGroups = D / kGroup;
  constexpr int kPer16 = 16 / (int)sizeof(T);        // elements per 16-byte piece
  constexpr int kPieces = D / kPer16;                // pieces per row
  constexpr int kMine = kGroup * kPieces / kThreads; // pieces of a tile per thread
  constexpr int kParts = kThreads / D;               // threads that share a key channel's statistics
  static_assert(kGroup * kPieces % kThreads == 0 && kThreads % D == 0, "tile does not divide over the workgroup");
  __shared__ float tile[kGroup * kPad];
  __shared__ float lo_s[kThreads], hi_s[kThreads];   // partial (min, max), then (zero, scale), per channel or per (token, channel group)

  const int tg = blockIdx.x, ll = blockIdx.z;
  const int b = blockIdx.y / a.h_kv, h = blockIdx.y % a.h_kv;
  const int keep = dims.keep[ll * a.batch + b];
  const int r0 = tg * kGroup;
  if (r0 >= keep) return;
  const int rows = min(kGroup, keep - r0);
  const int cap = a.cap[ll];
  const int tid = threadIdx.x;
  const float levels = (float)((1 << a.bits) - 1);
  const int64_t head = (int64_t)b * a.h_kv + h;
  const int64_t in_off = b * st.s[ll][0] + h * st.s[ll][1] + (int64_t)r0 * st.s[ll][2];
  const int64_t tok = st.s[ll][2];

  // Both tiles' loads are issued before anything waits: 2 x 8 KiB in flight per workgroup.
  uint4 kraw[kMine], vraw[kMine];
  const T* ksrc = reinterpret_cast<const T*>(a.k_hat[ll]) + in_off;
  const T* vsrc = reinterpret_cast<const T*>(a.v_hat[ll]) + in_off;
#pragma unroll
  for (int m = 0; m < kMine; ++m) {
    const int p = m * kThreads + tid, r = min(p / kPieces, rows - 1), q = p % kPieces;     // rows past the end repeat the last one
    kraw[m] = *reinterpret_cast<const uint4*>(ksrc + (int64_t)r * tok + q * kPer16);
    vraw[m] = *reinterpret_cast<const uint4*>(vsrc + (int64_t)r * tok + q * kPer16);
  }
  auto to_tile = [&](const uint4 (&raw)[kMine]) {
#pragma unroll
    for (int m = 0; m < kMine; ++m) {
      const int p = m * kThreads + tid, r = p / kPieces, q = p % kPieces;
      const T* e = reinterpret_cast<const T*>(&raw[m]);
#pragma unroll
      for (int i = 0; i < kPer16; ++i) tile[r * kPad + q * kPer16 + i] = to_float(e[i]);
    }
  };
  // Codes of eight consecutive channels of a row, packed low channel first, leave as `bits` bytes.
  auto encode_and_store = [&](uint8_t* out_rows, auto zero_scale_of) {
    const int row_bytes = D * a.bits / 8;
    for (int e8 = tid; e8 < rows * (D / 8); e8 += kThreads) {
      const int r = e8 / (D / 8), c0 = (e8 % (D / 8)) * 8;
      uint64_t packed = 0;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        float lo, sc;
        zero_scale_of(r, c0 + i, lo, sc);
        packed |= (uint64_t)encode(tile[r * kPad + c0 + i], lo, sc, levels) << (i * a.bits);
      }
      uint8_t* dst = out_rows + (int64_t)r * row_bytes + (c0 / 8) * a.bits;
      if (a.bits == 8) *reinterpret_cast<uint64_t*>(dst) = packed;
      else if (a.bits == 4) *reinterpret_cast<uint32_t*>(dst) = (uint32_t)packed;
      else *reinterpret_cast<uint16_t*>(dst) = (uint16_t)packed;
    }
  };

  // ---- keys: per channel over the tile's tokens -------------------------------------------
  to_tile(kraw);
  __syncthreads();
  {
    const int c = tid % D, part = tid / D;
    float lo = tile[c], hi = lo;                     // row 0 exists
    for (int r = part; r < rows; r += kParts) {
      const float x = tile[r * kPad + c];
      lo = fminf(lo, x);
      hi = fmaxf(hi, x);
    }
    lo_s[tid] = lo;
    hi_s[tid] = hi;
  }
  __syncthreads();
  float k_lo = 0.f, k_sc = 0.f;
  if (tid < D) {
    float hi = hi_s[tid];
    k_lo = lo_s[tid];
#pragma unroll
    for (int part = 1; part < kParts; ++part) {
      k_lo = fminf(k_lo, lo_s[part * D + tid]);
      hi = fmaxf(hi, hi_s[part * D + tid]);
    }
    k_sc = (hi - k_lo) / levels;
    const int64_t n_groups = (cap + kGroup - 1) / kGroup;
    const int64_t o = (head * n_groups + tg) * D + tid;
    a.k_scale[ll][o] = k_sc;
    a.k_zero[ll][o] = k_lo;
  }
  __syncthreads();                                   // everyone has read the partial values
  if (tid < D) {
    lo_s[tid] = k_lo;
    hi_s[tid] = k_sc;
  }
  __syncthreads();
  encode_and_store(a.k_codes[ll] + (head * cap + r0) * (D * a.bits / 8),
                   [&](int, int c, float& lo, float& sc) { lo = lo_s[c]; sc = hi_s[c]; });
  __syncthreads();

  // ---- values: per token over groups of 32 channels -------------------------------------
  to_tile(vraw);
  __syncthreads();
  {
    // two threads per (token, channel group): 16 channels each, merged across the lane pair
    const int pair = tid >> 1, halfsel = tid & 1;
    const int r = min(pair / kVGroups, rows - 1), cg = pair % kVGroups;
    float lo = 0.f, hi = 0.f;
    if (pair < kGroup * kVGroups) {
      const float* x = &tile[r * kPad + cg * kGroup + halfsel * 16];
      lo = hi = x[0];
#pragma unroll
      for (int i = 1; i < 16; ++i) {
        lo = fminf(lo, x[i]);
        hi = fmaxf(hi, x[i]);
      }
    }
    lo = fminf(lo, __shfl_xor(lo, 1));
    hi = fmaxf(hi, __shfl_xor(hi, 1));
    if (pair < kGroup * kVGroups && halfsel == 0) {
      const float sc = (hi - lo) / levels;
      lo_s[pair] = lo;
      hi_s[pair] = sc;
      if (pair / kVGroups < rows) {
        const int64_t o = (head * cap + r0 + r) * kVGroups + cg;
        a.v_scale[ll][o] = sc;
        a.v_zero[ll][o] = lo;
      }
    }
  }
  __syncthreads();
  encode_and_store(a.v_codes[ll] + (head * cap + r0) * (D * a.bits / 8),
                   [&](int r, int c, float& lo, float& sc) { lo = lo_s[r * kVGroups + c / kGroup]; sc = hi_s[r * kVGroups + c / kGroup]; });
}

}  // namespace
}  // namespace cake

using namespace cake;

extern "C" int cake_quantize_kv(const cake_shape* shape, int32_t bits,
                                const void* const* k_hat, const void* const* v_hat, const int64_t* kv_strides,
                                const int32_t* keep,
                                uint8_t* const* k_codes, float* const* k_scale, float* const* k_zero,
                                uint8_t* const* v_codes, float* const* v_scale, float* const* v_zero,
                                void* stream) {
  if (int rc = check_shape_basic(shape)) return rc;
  CAKE_REQUIRE(bits == 2 || bits == 4 || bits == 8, "bits = %d must be 2, 4 or 8", bits);
  CAKE_REQUIRE(k_hat && v_hat && kv_strides && keep && k_codes && k_scale && k_zero && v_codes && v_scale && v_zero,
               "a pointer argument is NULL");
  const int B = shape->batch, L = shape->n_layers;
  const int eb = (int)elem_bytes(shape->dtype);
  for (int i = 0; i < L * B; ++i) CAKE_REQUIRE(keep[i] >= 0, "keep[%d] = %d is negative", i, keep[i]);
  for (int i = 0; i < 3 * L; ++i) {
    CAKE_REQUIRE(kv_strides[i] >= 0, "negative stride");
    CAKE_REQUIRE((kv_strides[i] * eb) % 16 == 0, "strides must be multiples of 16 bytes");
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  for (int l0 = 0; l0 < L;) {
    const int nl = launch_layers(L - l0, B);
    QuantArgs a{};
    RaggedDims dims{};
    LayerStrides ls{};
    a.k_hat = k_hat + l0; a.v_hat = v_hat + l0;
    a.k_codes = k_codes + l0; a.k_scale = k_scale + l0; a.k_zero = k_zero + l0;
    a.v_codes = v_codes + l0; a.v_scale = v_scale + l0; a.v_zero = v_zero + l0;
    a.batch = B; a.h_kv = shape->n_kv_heads; a.bits = bits;
    int cap_max = 0;
    for (int ll = 0; ll < nl; ++ll) {
      int ck = 0;
      for (int b = 0; b < B; ++b) {
        dims.keep[ll * B + b] = keep[(l0 + ll) * B + b];
        ck = std::max(ck, keep[(l0 + ll) * B + b]);
      }
      a.cap[ll] = ck;
      cap_max = std::max(cap_max, ck);
      for (int j = 0; j < 3; ++j) ls.s[ll][j] = kv_strides[(l0 + ll) * 3 + j];
    }
    if (cap_max > 0) {
      const dim3 grid((cap_max + kGroup - 1) / kGroup, B * shape->n_kv_heads, nl), block(kThreads);
      const bool bf = shape->dtype == CAKE_BF16;
      if (bf && shape->head_dim == 128) hipLaunchKernelGGL((quantize_kernel<__bf16, 128>), grid, block, 0, st, a, dims, ls);
      else if (bf && shape->head_dim == 64) hipLaunchKernelGGL((quantize_kernel<__bf16, 64>), grid, block, 0, st, a, dims, ls);
      else if (!bf && shape->head_dim == 128) hipLaunchKernelGGL((quantize_kernel<float, 128>), grid, block, 0, st, a, dims, ls);
      else if (!bf && shape->head_dim == 64) hipLaunchKernelGGL((quantize_kernel<float, 64>), grid, block, 0, st, a, dims, ls);
      else return fail(CAKE_ERR_UNSUPPORTED, "no quantiser for head_dim %d", shape->head_dim);
    }
    l0 += nl;
  }
  CAKE_HIP_TRY(hipGetLastError());
  return CAKE_OK;
}
