/*
 * libcake — prefill-time KV-cache eviction pass of CAKE (cascading and adaptive KV-cache
 * eviction with layer preferences) for one AMD MI355X (gfx950).
 *
 * C ABI.  No C++ or framework types cross this boundary: plain pointers, sizes and PODs.
 *
 * Notation (the paper's, with N for its sequence length S):
 *   B batch, L layers, H_q query heads, H_kv KV heads, G = H_q / H_kv, d head_dim,
 *   N rows of K/V per head (prompt length, observation window included), S_w window,
 *   N_p = N - S_w prefix length (the positions that are scored and may be evicted),
 *   B_total cache budget per KV head summed over layers, B_l budget of layer l
 *   (window tokens included), k_l = B_l - S_w prefix tokens retained.
 *
 * Conventions for every call
 *   - Returns CAKE_OK (0) or a negative cake_status; cake_last_error() gives the reason
 *     (thread-local string, valid until the thread's next failing call).
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are
 *     ordinary process memory owned by the caller.  The library never allocates or frees
 *     device memory and keeps no state between calls (two documented exceptions: the optional
 *     profiling events of cake_profile_enable and the fixed scratch array of
 *     cake_decode_update_static).
 *   - Device work is enqueued on `stream` (a hipStream_t passed as void*; NULL = default
 *     stream) and the call returns without synchronising.  Host arrays are consumed before
 *     the call returns.  cake_cascade_allocate is host-only and synchronous.
 *   - Inputs are never written.  Outputs must not overlap inputs or each other.
 *   - A "table" is a DEVICE array of n_layers device pointers, one base pointer per layer,
 *     so that a whole multi-layer pass is a handful of launches.
 *   - Ragged per-layer arrays: where sequences of a batch keep different numbers of rows,
 *     a per-layer array [B, H_kv, rows, ...] is laid out with row capacity
 *     cap_l = max over b of the per-sequence row count; rows past a sequence's own count
 *     are neither read nor written.
 *   - Invalid arguments are rejected on the host before anything is launched.
 */
#ifndef CAKE_H_
#define CAKE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  CAKE_OK = 0,
  CAKE_ERR_INVALID_ARG = -1,  /* null pointer, non-positive size, N <= S_w, k > cur_len, ... */
  CAKE_ERR_UNSUPPORTED = -2,  /* dtype / head_dim / window / group size with no kernel */
  CAKE_ERR_WORKSPACE = -3,    /* workspace missing, misaligned (256 B) or too small */
  CAKE_ERR_HIP = -4           /* a HIP runtime call or launch failed */
} cake_status;

typedef enum { CAKE_BF16 = 0, CAKE_F32 = 1 } cake_dtype;

/* Problem shape.  Supported: head_dim 64 or 128, window 32 or 64, 1 <= G <= 8, n_layers <= 1024,
 * batch <= 256, batch * n_kv_heads <= 65535, and for the score calls
 * n_layers * batch * n_kv_heads <= 65535 per call (split larger passes over layers).  The top-k,
 * compaction and decode calls split their launches over layers themselves.
 * Every per-layer base pointer in a table and every stride must be a multiple of 16 bytes
 * (rows are moved as 16-byte pieces); the strides are checked, the base pointers live in device
 * memory and are the caller's responsibility. */
typedef struct {
  int32_t batch;       /* B */
  int32_t n_layers;    /* layers handled by this call (1 for strict per-layer cascading) */
  int32_t n_q_heads;   /* H_q */
  int32_t n_kv_heads;  /* H_kv, divides H_q */
  int32_t head_dim;    /* d */
  int32_t seq_len;     /* N, only read by cake_window_scores / cake_workspace_bytes */
  int32_t window;      /* S_w */
  int32_t dtype;       /* cake_dtype of Q, K, V */
} cake_shape;

/* Per-head token score before the group mean and the pooling.  CAKE's own indicator is
 * Mean + gamma*Var (Sec. 4.3 Eq. 11); the other three are the alternatives of the paper's
 * indicator ablation (Sec. 5, "Effectiveness of Proposed Eviction Indicator"). */
typedef enum {
  CAKE_IND_MEAN_PLUS_VAR = 0,  /* Mean + gamma*Var */
  CAKE_IND_MEAN = 1,           /* Mean (the SnapKV-style window mean) */
  CAKE_IND_VAR = 2,            /* Var */
  CAKE_IND_MEAN_TIMES_VAR = 3, /* Mean * Var */
  CAKE_IND_CUMULATIVE = 4      /* sum over the S_w window rows = S_w * Mean: the accumulated-attention
                                  (H2O-style) indicator of Sec. 5.5 under this allocation, taken over the
                                  observation window.  Selects the same tokens as CAKE_IND_MEAN; the
                                  stored values differ by the factor S_w, which matters once decode
                                  steps add single attention rows to them. */
} cake_indicator;

/* Method parameters (Sec. 4.1 Eq. 6, Sec. 4.3 Eq. 11 and the implementation appendix). */
typedef struct {
  float scale;             /* softmax scale; 0 selects 1/sqrt(head_dim) (Sec. 2) */
  float gamma;             /* weight of Var in the indicator, the paper fixes 200 */
  float tau1;              /* temperature of the dispersion H in Eq. 6 */
  float tau2;              /* temperature of the shift V in Eq. 6 */
  int32_t var_correction;  /* 1: unbiased Var over the S_w rows (divide by S_w-1); 0: biased */
  int32_t pool_kernel;     /* odd width (<= 129) of the stride-1 max-pool over prefix positions; 1 = off */
  int32_t indicator_mode;  /* cake_indicator: which per-head statistic scores a token */
} cake_params;

/* Library version (major*10000 + minor*100 + patch). */
int cake_version(void);

/* Reason for the calling thread's most recent failure; "" if none. */
const char* cake_last_error(void);

/* Bytes of device workspace that cake_window_scores(_lse) and cake_layer_preference need for
 * `shape`.  cake_decode_update places its partial sums inside the same layout and checks at
 * run time that they fit (they do for every supported shape); cake_select_topk needs none.
 * The workspace must be 256-byte aligned.  cake_layer_preference reads what cake_window_scores left in it, so the
 * same buffer must be passed to both with nothing else written in between. */
int cake_workspace_bytes(const cake_shape* shape, size_t* bytes /* host, out */);

/*
 * Observation-window scores (Sec. 2 attention weights; Sec. 4.1 recent-window submatrix
 * A[-S_w:, :-S_w]; Sec. 3 Eq. 4-5; Sec. 4.3 Eq. 11).
 *
 * For every layer, sequence and query head h (KV head h / G) the last S_w queries attend to
 * all N keys: logits scale*<q_r, k_j>, key j hidden from window row r when j > N_p + r,
 * softmax over the visible keys.  On the prefix columns j < N_p of those rows it forms
 *   per (h, j): Mean and Var over the S_w rows, I_q = Mean + gamma*Var          (Eq. 11)
 *   per KV head: I = mean of I_q over the G heads of the group, then max-pooled
 *   per h: H_h = -sum p ln p (Eq. 4), V_h = sum_j Var (Eq. 5)  -> partial sums in workspace
 *
 *   q_win      table; q_win[l] -> [B, H_q, S_w, d] window queries, strides q_strides
 *   k          table; k[l]     -> [B, H_kv, N, d] keys (window rows are the last S_w)
 *   q_strides  host [3]: element strides of batch, head, token; d is contiguous
 *   k_strides  host [3]: likewise for k
 *   indicator  table; indicator[l] -> [B, H_kv, N_p] f32, contiguous, written
 *   workspace  device scratch of at least cake_workspace_bytes(shape)
 */
int cake_window_scores(const cake_shape* shape, const cake_params* params,
                       const void* const* q_win, const void* const* k,
                       const int64_t* q_strides, const int64_t* k_strides,
                       float* const* indicator,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same scores when the softmax normaliser of every window row is already known: the
 * prefill attention that the model runs anyway (the paper's implementation calls a
 * FlashAttention forward, App. "More implementation details") returns the log-sum-exp of each
 * query row, so the pass over the keys that would recompute it is skipped and K is read once.
 *
 *   row_lse    table; row_lse[l] -> [B, H_q, S_w] f32, contiguous: for window row r of head h the
 *              natural logarithm of sum_{j <= N_p + r} exp(scale * <q_r, k_j>), with the same
 *              `scale` as params.  An error of e in an entry scales that row's weights by exp(-e).
 * Everything else as in cake_window_scores; results agree with it to rounding when row_lse is exact.
 */
int cake_window_scores_lse(const cake_shape* shape, const cake_params* params,
                           const void* const* q_win, const void* const* k,
                           const int64_t* q_strides, const int64_t* k_strides,
                           const float* const* row_lse, float* const* indicator,
                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same scores when the keys of a layer are not resident at once (a prompt whose K is
 * produced, or paged in, a range of positions at a time): the softmax of Sec. 2 over all N keys
 * needs every key twice, once for the row normalisers and once for the statistics of Eq. 4-5
 * and Eq. 11, so the caller hands the key axis over in segments, twice:
 *
 *   for each segment:  cake_window_scores_segment(pass 1)      partial (max, sum) pairs per row
 *   cake_window_scores_finish(pass 1)                          row normalisers, final
 *   for each segment:  cake_window_scores_segment(pass 2)      un-pooled indicator, H/V partials
 *   cake_window_scores_finish(pass 2)                          pooling -> indicator
 *   cake_layer_preference(...)                                 as after cake_window_scores
 *
 * A segment is the key range [key_begin, key_begin + key_count): key_begin a multiple of
 * cake_scores_chunk_keys(shape), the end a multiple of it or N.  The segments of a pass may come
 * in any order and must cover [0, N) in pass 1 and [0, N_p) in pass 2 exactly once (pass-2
 * segments may extend into the window; those keys are skipped).  The window queries are small
 * (S_w rows) and are passed whole with every segment.  Work is split over the key axis at the
 * same chunk boundaries and every partial result is reduced in the same fixed order as in
 * cake_window_scores, so the outputs are bit-identical to those of one resident call.
 *
 *   k_segment  table; k_segment[l] -> [B, H_kv, key_count, d]: row 0 is key key_begin;
 *              strides k_strides as for k.  Only read during the call.
 *   workspace  the same buffer through the whole sequence of calls and into
 *              cake_layer_preference, nothing else written to it in between.
 * cake_window_scores_finish takes no q/k; `indicator` is written by pass 2's finish only (pass 1
 * ignores it, may be NULL).  Errors as elsewhere: CAKE_ERR_ARGUMENT for a misaligned segment.
 */
int cake_scores_chunk_keys(const cake_shape* shape, int32_t* chunk /* host, out */);
int cake_window_scores_segment(const cake_shape* shape, const cake_params* params, int32_t pass,
                               int32_t key_begin, int32_t key_count,
                               const void* const* q_win, const void* const* k_segment,
                               const int64_t* q_strides, const int64_t* k_strides,
                               void* workspace, size_t workspace_bytes, void* stream);
int cake_window_scores_finish(const cake_shape* shape, const cake_params* params, int32_t pass,
                              float* const* indicator,
                              void* workspace, size_t workspace_bytes, void* stream);

/*
 * Layer preference (Sec. 4.1 Eq. 6): H_l and V_l are the means over the layer's query heads
 * of H_h and V_h, reduced in a fixed order from the partial sums cake_window_scores left in
 * `workspace`; P_l = H_l^(1/tau1) * V_l^(1/tau2).
 *
 *   pref  device [B, n_layers] f64, written
 *   hv    device [B, n_layers, 2] f64 = (H_l, V_l), written; may be NULL
 */
int cake_layer_preference(const cake_shape* shape, const cake_params* params,
                          const void* workspace, size_t workspace_bytes,
                          double* pref, double* hv, void* stream);

/*
 * Preference-prioritised allocation in its cascading form (Sec. 4.1 Eq. 7; Sec. 4.2 Eq. 9,
 * Prop. 1; Alg. 1 budget step).  HOST function, no GPU involved.
 *
 * Stage m = n_seen - 1: integer budgets B_l^(m), l = 0..m, proportional to pref[l] over the
 * layers seen so far.  Integers come from divisor (Webster) apportionment: each layer first
 * holds its S_w window tokens, the rest are awarded one by one to the layer with the largest
 * pref[l] / (B_l + 1/2) among layers below N, ties to the lower layer.  Hence
 *   sum_l B_l = min(total_budget, n_seen*N),  S_w <= B_l <= N,
 *   pref[a] >= pref[b] => B_a >= B_b,  and B_l^(m+1) <= B_l^(m) (Prop. 1, non-strict).
 * If every layer fits whole (n_seen*N <= total_budget) every B_l = N: nothing to evict.
 * All-zero preferences are treated as equal.  n_seen = L gives Eq. 7.
 *
 *   pref     host [n_seen], finite and >= 0
 *   budgets  host [n_seen], written
 * Errors: NaN/negative preference, total_budget < n_seen*S_w, N <= S_w.
 *
 * cake_keep_counts (HOST) turns budgets into the number of prefix tokens each layer retains:
 * the window tokens carry the score Omega in Sec. 4.3 Eq. 11 and are part of B_l, so
 * keep[i] = clamp(budgets[i] - S_w, 0, cur_len[i]) for n entries (cur_len: the current
 * evictable lengths, N - S_w before the first eviction).  These are the k of cake_select_topk
 * and cake_compact_kv.
 */
int cake_keep_counts(const int32_t* budgets, const int32_t* cur_len, int32_t n, int32_t window,
                     int32_t* keep);
int cake_cascade_allocate(const double* pref, int32_t n_seen, int64_t total_budget,
                          int32_t window, int32_t seq_len, int32_t* budgets);

/*
 * Per-head top-k of the indicator (Sec. 4.3 Eq. 12, D_l = TopK(I_l, B_l); the window
 * positions carry Omega in Eq. 11 and are kept structurally, so k counts prefix tokens).
 *
 * For each layer l, sequence b and KV head: the k[l*B+b] entries of the first
 * cur_len[l*B+b] indicator values that are largest under (value descending, position
 * ascending); positions are written in ascending order.  Values are compared as IEEE floats
 * (-0 = +0); NaNs are not supported.
 *
 *   indicator  table; indicator[l] -> [B, H_kv, max_b cur_len] f32
 *   cur_len    host [n_layers*B]: current evictable length (N_p at first, a previous k later)
 *   k          host [n_layers*B]: 0 <= k <= cur_len
 *   idx        table; idx[l] -> [B, H_kv, max_b k] int32, written
 */
int cake_select_topk(const cake_shape* shape, const float* const* indicator,
                     const int32_t* cur_len, const int32_t* k, int32_t* const* idx,
                     void* workspace, size_t workspace_bytes, void* stream);

/*
 * EVICT's compaction (Sec. 4.3 Eq. 12, K_hat = K[D,:], V_hat = V[D,:]; Alg. 1 cache and
 * indicator update).  Gathers the selected prefix rows and appends the S_w window rows.
 *
 * Sequence b of layer l holds cur_len prefix rows followed by its S_w window rows
 * (rows cur_len .. cur_len+S_w-1).  Output: k[l*B+b] gathered rows, then the window rows.
 *
 *   k_in, v_in   tables; [B, H_kv, rows, d] with per-layer element strides kv_strides
 *   kv_strides   host [n_layers][3]: batch, head, token strides of k_in[l] and v_in[l]
 *   cur_len, k   host [n_layers*B] as in cake_select_topk
 *   idx          table; idx[l] -> [B, H_kv, max_b k] int32 ascending positions < cur_len
 *   ind_in       table of [B, H_kv, max_b cur_len] f32, or NULL to skip the indicator
 *   k_out, v_out tables; [B, H_kv, max_b k + S_w, d] contiguous, written
 *   ind_out      table of [B, H_kv, max_b k] f32, written; NULL iff ind_in is NULL
 */
int cake_compact_kv(const cake_shape* shape,
                    const void* const* k_in, const void* const* v_in, const int64_t* kv_strides,
                    const int32_t* cur_len, const int32_t* k, const int32_t* const* idx,
                    const float* const* ind_in,
                    void* const* k_out, void* const* v_out, float* const* ind_out,
                    void* stream);

/*
 * The allocation step and EVICT of a one-shot pass without a host round trip in between.
 *
 * cake_plan_eviction computes on the device, for every sequence, the same integer budgets as
 * cake_cascade_allocate at n_seen = n_layers (Sec. 4.1 Eq. 7; bit-identical to the host routine
 * on the same preferences), the retained prefix counts k = clamp(B_l - S_w, 0, cur_len) (the
 * window tokens carry Omega in Sec. 4.3 Eq. 11 and count towards B_l), and the place of every
 * layer's outputs, one layer after the other, in four caller-owned pools.  All of it is left in
 * `plan`, device memory of cake_plan_bytes(shape) bytes laid out as
 *   int32 budgets[L*B], keep[L*B], cur_len[L*B] (entry l*B + b), cap_keep[L], cap_cur[L]
 *   (cap = maximum over the batch), copy_blocks[L*B + 1] (the compaction's work list: running
 *   count of 1024-piece blocks of output rows), then from the next multiple of 8 bytes four
 *   tables of L device pointers: idx, k_out, v_out, ind_out;
 * the host may copy it back at any later time to learn the budgets.
 * cake_evict_planned then runs cake_select_topk and cake_compact_kv for all layers with the
 * counts and output addresses taken from the plan (results identical to those two calls).
 *
 *   pref      device [B, n_layers] f64 as written by cake_layer_preference
 *   cur_len   device [n_layers*B] current evictable lengths, or NULL for N_p = seq_len - window
 *   pool_idx  device, 16-byte aligned: layer l holds [B, H_kv, cap_keep[l]] int32
 *   pool_k/v  device: layer l holds [B, H_kv, cap_keep[l] + S_w, d]
 *   pool_ind  device: layer l holds [B, H_kv, cap_keep[l]] f32
 *             (sum_l cap_keep[l] <= B*(total_budget - n_layers*S_w) rows bound the pool sizes)
 *   status    device [B] int32, written: 1 if a preference of the sequence is NaN, negative or
 *             infinite (the plan then holds the budgets of equal preferences), else 0
 *   k_in, v_in, indicator, kv_strides  as in cake_compact_kv / cake_select_topk, with one set of
 *             strides (host [3]) for all layers
 *   compacted host [n_layers] or NULL (= all 0): 1 marks a layer whose k_in/v_in are themselves
 *             outputs of an earlier cake_evict_planned, contiguous [B, H_kv, cap_cur[l] + S_w, d]
 *             (cap_cur from this plan: the capacities are only known on the device); its strides
 *             are derived from the plan instead of kv_strides.  This is what lets the stages of
 *             the cascade (Alg. 1) follow one another without the host reading anything back.
 *
 * cake_plan_layout gives the byte offsets of the plan's ten parts for `shape` (n_layers, batch):
 * budgets, keep, cur_len, cap_keep, cap_cur, copy_blocks, then the idx, k_out, v_out and ind_out
 * tables, so that a caller can hand parts of one plan (keep counts, output tables) to the next call
 * as device pointers.
 */
int cake_plan_layout(const cake_shape* shape, size_t* offsets /* host [10], out */);
int cake_plan_bytes(const cake_shape* shape, size_t* bytes /* host, out */);
int cake_plan_eviction(const cake_shape* shape, const double* pref, int64_t total_budget,
                       const int32_t* cur_len,
                       void* pool_idx, void* pool_k, void* pool_v, void* pool_ind,
                       void* plan, size_t plan_bytes, int32_t* status, void* stream);
int cake_evict_planned(const cake_shape* shape, const float* const* indicator,
                       const void* const* k_in, const void* const* v_in, const int64_t* kv_strides,
                       const uint8_t* compacted,
                       const void* plan, size_t plan_bytes, void* stream);

/*
 * b-bit storage of the retained cache (appendix "Comparison and compatibility with quantization
 * methods", which combines eviction with a key-per-channel / value-per-token quantiser).
 * Asymmetric uniform quantisation over groups of 32 of the keep[l, b] retained prefix rows of
 * every head: keys per channel over 32 consecutive retained tokens, values per token over 32
 * consecutive channels; zero = group minimum, scale = (max - min) / (2^bits - 1), code =
 * round-half-to-even((x - zero) / scale), all in float32; a constant group has scale 0 and codes 0.
 * x is recovered as zero + code * scale, within half a step.  The S_w window rows that follow the
 * retained rows in k_hat / v_hat are left as they are (recent tokens stay in full precision).
 *
 *   bits       2, 4 or 8
 *   k_hat, v_hat  tables; compacted [B, H_kv, >= keep + S_w, d] as written by cake_compact_kv,
 *              element strides kv_strides (host [n_layers][3]), read only
 *   keep       host [n_layers*B]: retained prefix rows (entry l*B + b); cap_l = max over b
 *   k_codes, v_codes  tables; [B, H_kv, cap_l, d*bits/8] uint8, written: 8/bits consecutive
 *              channels to a byte, the lower channel in the lower bits
 *   k_scale, k_zero  tables; [B, H_kv, ceil(cap_l/32), d] f32, written (token group, channel)
 *   v_scale, v_zero  tables; [B, H_kv, cap_l, d/32] f32, written (token, channel group)
 * Rows at or beyond a sequence's own keep are neither read nor written.  The arrays behind k_hat and
 * v_hat start at 16-byte boundaries (strides are checked to be multiples of 16 bytes), the code
 * arrays at 8-byte boundaries; the tables live in device memory, so the addresses are not checked.
 */
int cake_quantize_kv(const cake_shape* shape, int32_t bits,
                     const void* const* k_hat, const void* const* v_hat, const int64_t* kv_strides,
                     const int32_t* keep,
                     uint8_t* const* k_codes, float* const* k_scale, float* const* k_zero,
                     uint8_t* const* v_codes, float* const* v_scale, float* const* v_zero,
                     void* stream);

/*
 * Indicator maintenance for one generated token (implementation appendix, decoding branch of
 * the listing: the new query's attention over the cached keys outside the window is pooled and
 * the stored indicator is updated with it; Sec. 5, implementation details: eviction also runs
 * during decoding).  The paper does not define the update; this
 * library ADDS the pooled weights to the stored values.
 *
 * Sequence b of layer l holds cur_len scored rows followed by its S_w window rows, the last of
 * which is the new token's key (the row that just left the window is the last scored row and
 * enters with whatever indicator the caller stored for it, normally 0).  For every KV head the G
 * query heads' new rows attend to all cur_len + S_w rows (softmax over all of them); the weights
 * on the scored rows are averaged over the group, max-pooled with params.pool_kernel along the
 * row axis (edges clipped) and added to indicator[l][b, g, :cur_len].  Only the mean term of
 * Eq. 11 exists for a single query row: gamma and indicator_mode are not used.
 * Evicting back to the budget is cake_select_topk + cake_compact_kv with k = cur_len - 1.
 *
 *   shape      seq_len = row capacity of the caches (>= max cur_len + S_w); n_layers as usual
 *   q_new      table; q_new[l] -> [B, H_q, d], element strides q_strides (host [2]: batch, head)
 *   k_cache    table; k_cache[l] -> [B, H_kv, rows, d], element strides k_strides (host [n_layers][3])
 *   cur_len    host [n_layers*B]: scored rows per (layer, sequence), <= seq_len - S_w
 *   indicator  table; indicator[l] -> [B, H_kv, max_b cur_len] f32, updated in place
 *   workspace  device scratch of at least cake_workspace_bytes(shape)
 */
int cake_decode_update(const cake_shape* shape, const cake_params* params,
                       const void* const* q_new, const int64_t* q_strides,
                       const void* const* k_cache, const int64_t* k_strides,
                       const int32_t* cur_len, float* const* indicator,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same decode-phase maintenance in place: one generated token at each of n_layers layers
 * (normally one), with K and V touched at a single row per head.
 *
 * The cache of a (layer, sequence, KV head) lives in cap + S_w + 1 physical slots that never move.
 * order[0 .. cur + S_w) lists the slots in logical order: the cur scored rows by position, then
 * the S_w window rows, oldest first.  The call (1) copies the token's key and value into the free
 * slot and appends it to the list, which turns the oldest window row into the last scored row,
 * starting at indicator 0; (2) updates the indicator of the cur + 1 scored rows exactly as
 * cake_decode_update does (softmax of the G new query rows over all listed rows, group mean,
 * max-pool along the logical order, added); (3) evicts the scored row with the smallest updated
 * indicator, the later one among equals, i.e. the row that cake_select_topk at k = cur leaves
 * out: it is deleted from the list and from the indicator (later entries move down by one) and
 * its slot becomes the free one.  cur does not change.
 *
 *   shape      seq_len >= max over layers of cap + S_w + 1 (sizes the workspace)
 *   q_new      device [n_layers, B, H_q, d], element strides q_strides (host [3]: layer, batch, head)
 *   k_new, v_new  device [n_layers, B, H_kv, d], element strides kv_new_strides (host [3])
 *   k_slots, v_slots  tables; [B, H_kv, cap_l + S_w + 1, d], element strides slot_strides[l]
 *              (host [n_layers][3]: batch, head, slot of every layer), updated
 *   indicator  table; indicator[l] -> [B, H_kv, cap_l + 1] f32 in logical order, updated
 *   order      table; order[l] -> [B, H_kv, cap_l + S_w + 1] int32, updated
 *   state      table; state[l] -> [B, H_kv, 4] int32: {cur, free slot, logical index of the row
 *              evicted by the last call, unused}; the caller sets cur and the free slot once
 *   cap        host [n_layers]: scored-row capacity cap_l of the layer's arrays (cur <= cap_l)
 *   workspace  device scratch of at least cake_decode_step_workspace_bytes(shape), 256-byte aligned
 */
int cake_decode_step_workspace_bytes(const cake_shape* shape, size_t* bytes /* host, out */);
int cake_decode_step(const cake_shape* shape, const cake_params* params,
                     const void* q_new, const int64_t* q_strides,
                     const void* k_new, const void* v_new, const int64_t* kv_new_strides,
                     void* const* k_slots, void* const* v_slots, const int64_t* slot_strides,
                     float* const* indicator, int32_t* const* order, int32_t* const* state,
                     const int32_t* cap, void* workspace, size_t workspace_bytes, void* stream);

/*
 * cake_decode_update for callers that cannot hand over a workspace or allocate one: code under
 * HIP graph capture, tight serving loops, harnesses that forbid device allocation.  Same
 * computation and same results as cake_decode_update; the chunks' softmax partials go to a
 * scratch array built into the library (1 MiB of device memory per GPU, held until the process
 * ends) instead of a caller's workspace.  The call allocates and frees nothing.
 *
 * Limit: n_layers * B * H_kv * ceil(shape.seq_len / 256) <= 16384 chunk entries (e.g. 32 layers
 * of 8 KV heads with caches of up to 16384 rows); larger shapes return CAKE_ERR_UNSUPPORTED and
 * should use cake_decode_update.  All calls on one GPU share that GPU's scratch array: calls that
 * overlap in time on one GPU (different streams or threads) race; serialise them.
 */
int cake_decode_update_static(const cake_shape* shape, const cake_params* params,
                              const void* const* q_new, const int64_t* q_strides,
                              const void* const* k_cache, const int64_t* k_strides,
                              const int32_t* cur_len, float* const* indicator, void* stream);

/*
 * Diagnostics, not part of the method: per-kernel timing of cake_window_scores.
 * While enabled, every cake_window_scores call records HIP events on its stream around its
 * kernels (a few microseconds of overhead).  cake_profile_read waits for the last recorded
 * event and returns milliseconds averaged over the calls since cake_profile_enable(1) (at most
 * the 64 most recent): ms[0] pass 1 (row normalisers), ms[1] combine, ms[2] pass 2 (column
 * statistics), ms[3] pooling.  Process-wide state, not thread-safe; events are created by
 * cake_profile_enable(1) and destroyed by cake_profile_enable(0).
 */
int cake_profile_enable(int enable);
int cake_profile_read(float* ms /* host [4], out */);

#ifdef __cplusplus
}
#endif
#endif /* CAKE_H_ */
