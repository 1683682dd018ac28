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

// ---- device-resident eviction plan (cake_plan_eviction writes it, cake_evict_planned reads it) ----
// int32 budgets[L*B], keep[L*B], cur_len[L*B], cap_keep[L], cap_cur[L], copy_blocks[L*B + 1];
// then, 8-byte aligned, four tables of L device pointers: idx, k_out, v_out, ind_out.
// copy_blocks[e] = number of kCopyBlockPieces-piece blocks that the output rows of the entries
// before e (entry l*B + b) fill, each entry rounded up: the planned compaction's work list.
constexpr int kCopyBlockPieces = 1024;       // 16-byte pieces a compaction workgroup moves per step
struct PlanLayout {
  size_t off_budgets, off_keep, off_cur, off_cap_keep, off_cap_cur, off_blocks, off_tables, total;
};
inline PlanLayout plan_layout(int n_layers, int batch) {
  PlanLayout p{};
  const size_t lb = (size_t)n_layers * batch * sizeof(int32_t), l4 = (size_t)n_layers * sizeof(int32_t);
  size_t off = 0;
  p.off_budgets = off;  off += lb;
  p.off_keep = off;     off += lb;
  p.off_cur = off;      off += lb;
  p.off_cap_keep = off; off += l4;
  p.off_cap_cur = off;  off += l4;
  p.off_blocks = off;   off += lb + sizeof(int32_t);
  off = align_up(off, 8);
  p.off_tables = off;   off += 4 * (size_t)n_layers * sizeof(void*);
  p.total = align_up(off, 256);
  return p;
}
struct PlanView {               // device addresses inside a plan buffer
  const int32_t* keep;
  const int32_t* cur_len;
  const int32_t* cap_keep;
  const int32_t* cap_cur;
  const int32_t* copy_blocks;
  void* const* idx;
  void* const* k_out;
  void* const* v_out;
  void* const* ind_out;
};
inline PlanView plan_view(const void* plan, int n_layers, int batch) {
  const PlanLayout lay = plan_layout(n_layers, batch);
  const char* b = static_cast<const char*>(plan);
  void* const* t = reinterpret_cast<void* const*>(b + lay.off_tables);
  return PlanView{reinterpret_cast<const int32_t*>(b + lay.off_keep), reinterpret_cast<const int32_t*>(b + lay.off_cur),
                  reinterpret_cast<const int32_t*>(b + lay.off_cap_keep), reinterpret_cast<const int32_t*>(b + lay.off_cap_cur),
                  reinterpret_cast<const int32_t*>(b + lay.off_blocks), t, t + n_layers, t + 2 * n_layers, t + 3 * n_layers};
}
// top-k and compaction of all layers with the counts and output places read from a plan
int launch_topk_planned(const cake_shape* shape, const float* const* indicator, const PlanView& plan, hipStream_t stream);
constexpr int kPlanMaskWords = 32;       // one bit per layer, n_layers <= 1024
int launch_compact_planned(const cake_shape* shape, const void* const* k_in, const void* const* v_in,
                           const int64_t* kv_strides, const uint8_t* compacted, const float* const* ind_in,
                           const PlanView& plan, hipStream_t stream);

// Layers [l0, l0+nl) that fit one launch under the two limits above.
inline int launch_layers(int n_layers_left, int batch) {
  int by_entries = kMaxLaunchEntries / batch;
  int nl = n_layers_left < kMaxLaunchLayers ? n_layers_left : kMaxLaunchLayers;
  return nl < by_entries ? nl : by_entries;
}

}  // namespace cake
