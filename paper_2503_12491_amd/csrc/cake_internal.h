// Internal declarations shared by the translation units of libcake.  Not installed.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstddef>
#include <cstdint>

#include "cake.h"

namespace cake {

// ---- error reporting -----------------------------------------------------------------
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

#define CAKE_HIP_TRY(expr)                                                              \
  do {                                                                                  \
    hipError_t e__ = (expr);                                                            \
    if (e__ != hipSuccess)                                                              \
      return ::cake::fail(CAKE_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e__)); \
  } while (0)

#define CAKE_REQUIRE(cond, ...)                                       \
  do {                                                                \
    if (!(cond)) return ::cake::fail(CAKE_ERR_INVALID_ARG, __VA_ARGS__); \
  } while (0)

// ---- shape checks common to the entry points -------------------------------------------
int check_shape_basic(const cake_shape* s);   // batch/heads/head_dim/window/dtype/layers
int check_shape_scores(const cake_shape* s);  // + N > S_w and the kernels' supported set

inline size_t elem_bytes(int32_t dtype) { return dtype == CAKE_BF16 ? 2 : 4; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- workspace layout of the score pass -------------------------------------------------
// One "slice" is (layer, sequence, KV head).  Keys of a slice are cut into chunks of
// `chunk` keys; one workgroup handles one chunk in each of the two passes.
struct ScoreLayout {
  int32_t chunk;        // keys per workgroup, multiple of 64
  int32_t n_chunks;     // chunks over all N keys (pass 1)
  int32_t n_chunks_p;   // chunks over the N_p prefix keys (pass 2)
  int64_t n_slices;     // L * B * H_kv
  int32_t rows;         // G * S_w window rows per slice
  size_t off_lse;       // f32 [n_slices][rows]            log2-domain row normaliser
  size_t off_part;      // f32 [n_slices][n_chunks][rows][2]      pass-1 (reference, sum) per window row
  size_t off_hv;        // f32 [n_slices][n_chunks_p][G][2]       pass-2 (entropy, variance) sums
  size_t off_raw;       // f32 [n_slices][N_p]             un-pooled indicator
  size_t total;
};
ScoreLayout score_layout(const cake_shape& s);

// ---- ragged per-launch dimensions, passed to kernels by value ----------------------------
constexpr int kMaxLaunchLayers = 32;
constexpr int kMaxLaunchEntries = 256;   // (layer, sequence) pairs per launch

struct RaggedDims {
  int32_t cur_len[kMaxLaunchEntries];
  int32_t keep[kMaxLaunchEntries];
};
struct LayerStrides {
  int64_t s[kMaxLaunchLayers][3];
};

// Layers [l0, l0+nl) that fit one launch under the two limits above.
inline int launch_layers(int n_layers_left, int batch) {
  int by_entries = kMaxLaunchEntries / batch;
  int nl = n_layers_left < kMaxLaunchLayers ? n_layers_left : kMaxLaunchLayers;
  return nl < by_entries ? nl : by_entries;
}

}  // namespace cake
