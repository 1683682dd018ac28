// cake_quantize_kv: b-bit storage of the retained cache (appendix "Comparison and compatibility
// with quantization methods": eviction combined with a key-per-channel / value-per-token
// quantiser).  Asymmetric uniform quantisation over groups of 32: the keys of a head per channel
// over 32 consecutive retained tokens, the values per token over 32 consecutive channels;
// zero = group minimum, scale = (max - min) / (2^b - 1), code = round-half-even((x - zero) / scale).
// The window rows are not touched: they stay in the compacted arrays as they are.
//
// Two wavefronts per (layer, sequence, head, group of 32 tokens), one for the keys and one for the
// values, no LDS and no barrier: a lane owns one 16-byte piece of a row (the same channels in every
// row it loads), so the keys' per-channel extremes are element-wise over the lane's rows plus a few
// cross-lane steps, the values' per-token extremes are over the lanes of one row that share a
// 32-channel group, and every lane packs and stores the codes of its own pieces.  Pure streaming:
// bound by HBM.
#include <algorithm>
#include <type_traits>

#include "cake_internal.h"

namespace cake {
namespace {

constexpr int kThreads = 256;
constexpr int kGroupsPerBlock = kThreads / 64 / 2;     // a wavefront for the keys and one for the values of each token group
constexpr int kGroup = 32;       // tokens per key group, channels per value group

struct QuantArgs {
  const void* const* k_hat;
  const void* const* v_hat;
  uint8_t* const* k_codes; float* const* k_scale; float* const* k_zero;
  uint8_t* const* v_codes; float* const* v_scale; float* const* v_zero;
  int32_t batch, h_kv, bits, n_entries;
  int32_t cap[kMaxLaunchLayers];
  int32_t keep[kMaxLaunchEntries];                 // [layer of the launch][sequence]
  // workgroups before those of entry e: a workgroup serves kGroupsPerBlock consecutive token groups of
  // one (layer, sequence), so the grid holds no workgroup without rows however uneven the layers' counts are
  int32_t first_block[kMaxLaunchEntries + 1];
};

__device__ __forceinline__ float to_float(__bf16 x) { return (float)x; }
__device__ __forceinline__ float to_float(float x) { return x; }

// Codes of the N values of one piece, packed low channel first.  The code of x in a group with
// minimum lo and step sc is round-half-even of the fp32 quotient (x - lo) / sc, clamped to
// [0, levels]; inv = 1 / sc to within one unit in the last place (0 for a constant group, whose
// codes are 0).  The product with inv lies within 2^-22 of the rounded quotient, relatively, and
// the quotients are at most 2^b, so unless it comes within 2^(b-21) of a rounding boundary (twice
// the bound) it rounds to the same integer; a
// lane that meets a value near a boundary (or a product that is not finite) redoes its piece with
// the division itself.
template <int kBits, int N, typename Lo, typename Sc, typename Inv>
__device__ __forceinline__ uint64_t encode_piece(const float (&x)[N], Lo lo, Sc sc, Inv inv) {
  constexpr float levels = (float)((1 << kBits) - 1);
  constexpr float kSafe = 0.5f - (float)(1 << kBits) * 0x1p-21f;
  float c[N];
  bool near = false;
#pragma unroll
  for (int i = 0; i < N; ++i) {
    const float t = (x[i] - lo(i)) * inv(i);
    c[i] = rintf(t);
    near = near || !(fabsf(t - c[i]) < kSafe);
  }
  if (near) {
#pragma unroll
    for (int i = 0; i < N; ++i) c[i] = sc(i) > 0.f ? rintf((x[i] - lo(i)) / sc(i)) : 0.f;
  }
  uint64_t packed = 0;
#pragma unroll
  for (int i = 0; i < N; ++i) packed |= (uint64_t)(uint32_t)__builtin_amdgcn_fmed3f(c[i], 0.f, levels) << (i * kBits);
  return packed;
}
__device__ __forceinline__ float step_inverse(float sc) { return sc > 0.f ? __builtin_amdgcn_rcpf(sc) : 0.f; }   // v_rcp_f32: 1 ulp

// The low `bytes` bytes of `packed` (1, 2, 4 or 8; dst is aligned to that size).
__device__ __forceinline__ void store_codes(uint8_t* dst, uint64_t packed, int bytes) {
  if (bytes == 8) *reinterpret_cast<uint64_t*>(dst) = packed;
  else if (bytes == 4) *reinterpret_cast<uint32_t*>(dst) = (uint32_t)packed;
  else if (bytes == 2) *reinterpret_cast<uint16_t*>(dst) = (uint16_t)packed;
  else *dst = (uint8_t)packed;
}

template <typename T, int D, int kBits>
__global__ __launch_bounds__(kThreads) void quantize_kernel(QuantArgs a, LayerStrides st) {
  constexpr int kPer16 = 16 / (int)sizeof(T);        // elements per 16-byte piece
  constexpr int kPieces = D / kPer16;                // pieces per row = lanes per row
  constexpr int kRowsPerLoad = 64 / kPieces;         // rows a wave-wide load covers
  constexpr int kLoads = kGroup / kRowsPerLoad;      // loads per lane and tile
  constexpr int kVLanes = kGroup / kPer16;           // lanes of a row that share a value group
  constexpr int kVGroups = D / kGroup;
  static_assert(64 % kPieces == 0 && kGroup % kRowsPerLoad == 0 && kPieces % kVLanes == 0, "tile does not divide over a wavefront");

  const int lane = threadIdx.x & 63;
  int e = 0;
  for (int hi = a.n_entries; hi - e > 1;) {          // first_block[e] <= blockIdx.x < first_block[e + 1]
    const int mid = (e + hi) >> 1;
    if (a.first_block[mid] <= (int)blockIdx.x) e = mid; else hi = mid;
  }
  const int ll = e / a.batch, b = e % a.batch, h = blockIdx.y;
  const int wave = threadIdx.x >> 6;
  const bool keys = (wave & 1) == 0;                  // even wavefronts take the keys, odd ones the values
  const int tg = ((int)blockIdx.x - a.first_block[e]) * kGroupsPerBlock + (wave >> 1);
  const int keep = a.keep[e];
  const int r0 = tg * kGroup;
  if (r0 >= keep) return;                            // the whole wavefront: there is no barrier below
  const int rows = min(kGroup, keep - r0);
  const int cap = a.cap[ll];
  const int q = lane % kPieces, rg = lane / kPieces;
  constexpr float levels = (float)((1 << kBits) - 1);
  constexpr int code_bytes = kPer16 * kBits / 8;     // of one piece
  constexpr int row_bytes = D * kBits / 8;
  const int64_t head = (int64_t)b * a.h_kv + h;
  const int64_t in_off = b * st.s[ll][0] + h * st.s[ll][1] + (int64_t)r0 * st.s[ll][2] + q * kPer16;
  const int64_t tok = st.s[ll][2];
  const T* src = reinterpret_cast<const T*>(keys ? a.k_hat[ll] : a.v_hat[ll]) + in_off;

  auto load_tile = [&](const T* src, uint4 (&raw)[kLoads]) {
#pragma unroll
    for (int m = 0; m < kLoads; ++m) {
      const int r = min(m * kRowsPerLoad + rg, rows - 1);        // rows past the end repeat the last one
      raw[m] = *reinterpret_cast<const uint4*>(src + (int64_t)r * tok);
    }
  };
  auto value = [](const uint4& piece, int i) { return to_float(reinterpret_cast<const T*>(&piece)[i]); };

  uint4 raw[kLoads];
  load_tile(src, raw);

  // ---- keys: per channel over the tile's tokens -------------------------------------------
  if (keys) {
    float lo[kPer16], sc[kPer16], inv[kPer16];
#pragma unroll
    for (int i = 0; i < kPer16; ++i) {
      float l = value(raw[0], i), hi = l;
#pragma unroll
      for (int m = 1; m < kLoads; ++m) {
        const float x = value(raw[m], i);
        l = fminf(l, x);
        hi = fmaxf(hi, x);
      }
#pragma unroll
      for (int off = kPieces; off < 64; off <<= 1) {            // the lanes that hold the same piece of other rows
        l = fminf(l, __shfl_xor(l, off));
        hi = fmaxf(hi, __shfl_xor(hi, off));
      }
      lo[i] = l;
      sc[i] = (hi - l) / levels;
      inv[i] = step_inverse(sc[i]);
    }
    if (rg == 0) {
      const int64_t n_groups = (cap + kGroup - 1) / kGroup;
      const int64_t o = (head * n_groups + tg) * D + q * kPer16;
#pragma unroll
      for (int i = 0; i < kPer16; ++i) {
        a.k_scale[ll][o + i] = sc[i];
        a.k_zero[ll][o + i] = lo[i];
      }
    }
    uint8_t* out = a.k_codes[ll] + (head * cap + r0) * row_bytes + q * code_bytes;
#pragma unroll
    for (int m = 0; m < kLoads; ++m) {
      const int r = m * kRowsPerLoad + rg;
      float x[kPer16];
#pragma unroll
      for (int i = 0; i < kPer16; ++i) x[i] = value(raw[m], i);
      const uint64_t packed = encode_piece<kBits>(x, [&](int i) { return lo[i]; }, [&](int i) { return sc[i]; },
                                                  [&](int i) { return inv[i]; });
      if (r < rows) store_codes(out + (int64_t)r * row_bytes, packed, code_bytes);
    }
  } else {
    // ---- values: per token over groups of 32 channels -----------------------------------
    uint8_t* out = a.v_codes[ll] + (head * cap + r0) * row_bytes + q * code_bytes;
#pragma unroll
    for (int m = 0; m < kLoads; ++m) {
      const int r = m * kRowsPerLoad + rg;
      float x[kPer16];
#pragma unroll
      for (int i = 0; i < kPer16; ++i) x[i] = value(raw[m], i);
      float lo = x[0], hi = x[0];
#pragma unroll
      for (int i = 1; i < kPer16; ++i) {
        lo = fminf(lo, x[i]);
        hi = fmaxf(hi, x[i]);
      }
#pragma unroll
      for (int off = 1; off < kVLanes; off <<= 1) {              // the lanes of this row's channel group
        lo = fminf(lo, __shfl_xor(lo, off));
        hi = fmaxf(hi, __shfl_xor(hi, off));
      }
      const float sc = (hi - lo) / levels, inv = step_inverse(sc);
      const uint64_t packed = encode_piece<kBits>(x, [&](int) { return lo; }, [&](int) { return sc; }, [&](int) { return inv; });
      if (r < rows) {
        if (q % kVLanes == 0) {
          const int64_t o = (head * cap + r0 + r) * kVGroups + q / kVLanes;
          a.v_scale[ll][o] = sc;
          a.v_zero[ll][o] = lo;
        }
        store_codes(out + (int64_t)r * row_bytes, packed, code_bytes);
      }
    }
  }
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
    LayerStrides ls{};
    a.k_hat = k_hat + l0; a.v_hat = v_hat + l0;
    a.k_codes = k_codes + l0; a.k_scale = k_scale + l0; a.k_zero = k_zero + l0;
    a.v_codes = v_codes + l0; a.v_scale = v_scale + l0; a.v_zero = v_zero + l0;
    a.batch = B; a.h_kv = shape->n_kv_heads; a.bits = bits; a.n_entries = nl * B;
    int64_t n_blocks = 0;
    for (int ll = 0; ll < nl; ++ll) {
      int ck = 0;
      for (int b = 0; b < B; ++b) {
        const int kp = keep[(l0 + ll) * B + b];
        a.keep[ll * B + b] = kp;
        a.first_block[ll * B + b] = (int32_t)n_blocks;
        n_blocks += ((kp + kGroup - 1) / kGroup + kGroupsPerBlock - 1) / kGroupsPerBlock;
        ck = std::max(ck, kp);
      }
      a.cap[ll] = ck;
      for (int j = 0; j < 3; ++j) ls.s[ll][j] = kv_strides[(l0 + ll) * 3 + j];
    }
    a.first_block[nl * B] = (int32_t)n_blocks;
    CAKE_REQUIRE(n_blocks <= 0x7fffffff, "too many rows for one launch");
    if (n_blocks > 0) {
      const dim3 grid((unsigned)n_blocks, shape->n_kv_heads), block(kThreads);
      const bool bf = shape->dtype == CAKE_BF16;
      auto launch = [&](auto bits_c) {
        constexpr int kBits = decltype(bits_c)::value;
        if (bf && shape->head_dim == 128) hipLaunchKernelGGL((quantize_kernel<__bf16, 128, kBits>), grid, block, 0, st, a, ls);
        else if (bf && shape->head_dim == 64) hipLaunchKernelGGL((quantize_kernel<__bf16, 64, kBits>), grid, block, 0, st, a, ls);
        else if (!bf && shape->head_dim == 128) hipLaunchKernelGGL((quantize_kernel<float, 128, kBits>), grid, block, 0, st, a, ls);
        else hipLaunchKernelGGL((quantize_kernel<float, 64, kBits>), grid, block, 0, st, a, ls);
      };
      if (shape->head_dim != 64 && shape->head_dim != 128) return fail(CAKE_ERR_UNSUPPORTED, "no quantiser for head_dim %d", shape->head_dim);
      if (bits == 2) launch(std::integral_constant<int, 2>{});
      else if (bits == 4) launch(std::integral_constant<int, 4>{});
      else launch(std::integral_constant<int, 8>{});
    }
    l0 += nl;
  }
  CAKE_HIP_TRY(hipGetLastError());
  return CAKE_OK;
}
