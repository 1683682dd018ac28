// cake_window_scores / cake_layer_preference: observation-window attention statistics.
//
// Sec. 2 (attention weights), Sec. 4.1 (recent-window submatrix A[-S_w:, :-S_w]),
// Sec. 3 Eq. 4-5 (dispersion, shift), Sec. 4.3 Eq. 11 (Mean + gamma*Var indicator).
//
// A "slice" is one (layer, sequence, KV head).  Its G*S_w window rows (G query heads of the
// group, S_w rows each) attend to the slice's N keys.  The softmax normaliser of a row needs
// every key, the column statistics need the normalised weights, so the keys are visited twice:
//
//   pass 1  logits via MFMA (keys on the M side, window rows on the N side, so that each lane
//           owns ONE window row per 32-row block and keeps a running (reference, sum) pair for
//           it with no cross-lane traffic); partial pairs per chunk of keys        -> workspace
//   combine partial pairs -> log2-domain normaliser per window row                  -> workspace
//   pass 2  logits again (window rows on the M side, keys on the N side, so that each lane owns
//           ONE key column and the Mean/Var over the S_w rows are in-register sums); weights
//           p = exp2(t), t = logit*scale*log2(e) - lse2; per column sum p, sum p^2; entropy
//           sum p*t; group mean of I_q through LDS                      -> un-pooled indicator
//           (software-pipelined for bf16 at S_w = 64: the MFMAs of one 32-key sub-tile are
//           interleaved with the statistics of the previous one)
//   pool    stride-1 max-pool over prefix positions                              -> indicator
//   pref    fixed-order fp64 reduction of the per-chunk entropy/variance sums    -> P_l, H_l, V_l
//
// One workgroup = G wavefronts = one chunk of keys of one slice; wave w serves query head
// g*G + w.  K tiles of 64 keys go from global memory straight into LDS (global_load_lds, 16
// bytes per lane), double-buffered so that tile t+1 is in flight while tile t is consumed, and
// are shared by the G waves.  Rows are stored unpadded with their 16-byte pieces XOR-swizzled by
// the row index so that the MFMA operand reads spread over the banks.
// With the row normalisers supplied by the caller (cake_window_scores_lse) pass 1 and the
// combine give way to a kernel that converts them to the log2 domain.
// Everything is deterministic: no float atomics, fixed reduction orders.
#include <cmath>
#include <type_traits>

#include "cake_internal.h"

namespace cake {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(1))) const void* global_cptr;
typedef __attribute__((address_space(3))) void* lds_ptr;

constexpr int kTileKeys = 64;        // keys staged per LDS tile (two 32-key MFMA sub-tiles)
constexpr float kMasked = -1.0e30f;  // stands for -inf without producing NaN in differences

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }  // v_exp_f32

template <typename T, int D>
struct Tile {
  static constexpr int kRowBytes = D * (int)sizeof(T);
  static constexpr int kPieces = kRowBytes / 16;         // 16-byte pieces per key row (power of two)
  static constexpr int kBytes = kTileKeys * kRowBytes;
  static constexpr int kGroups = kBytes / 1024;          // one wave-wide 1 KiB transfer each
  // LDS byte offset of piece q of row r: pieces are permuted within the row by r.
  static __device__ __forceinline__ int offset(int r, int q) { return r * kRowBytes + ((q ^ (r & (kPieces - 1))) << 4); }
};

// MFMA operand fragments.  For both the A and the B operand of the 32x32 instructions lane
// (c32, hh) supplies, for its row/column c32, a group of consecutive reduction elements chosen
// by hh; A and B use the same element order, so the dot products come out complete.
template <typename T> struct Frag;
template <> struct Frag<__bf16> {
  using type = bf16x8;
  static constexpr int kElems = 16;  // reduction elements per MFMA
  static __device__ __forceinline__ type load_global(const __bf16* row, int step, int hh) {
    return *reinterpret_cast<const bf16x8*>(row + step * 16 + hh * 8);
  }
  template <typename TL>
  static __device__ __forceinline__ type load_lds(const char* tile, int r, int step, int hh) {
    return *reinterpret_cast<const bf16x8*>(tile + TL::offset(r, 2 * step + hh));
  }
  static __device__ __forceinline__ f32x16 mfma(type a, type b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  }
};
template <> struct Frag<float> {
  using type = float;
  static constexpr int kElems = 2;
  static __device__ __forceinline__ type load_global(const float* row, int step, int hh) { return row[step * 2 + hh]; }
  template <typename TL>
  static __device__ __forceinline__ type load_lds(const char* tile, int r, int step, int hh) {
    const int e = step * 2 + hh;
    return *reinterpret_cast<const float*>(tile + TL::offset(r, e >> 2) + (e & 3) * 4);
  }
  static __device__ __forceinline__ f32x16 mfma(type a, type b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
  }
};

struct ScoreArgs {
  const void* const* q_win;
  const void* const* k;
  float* const* indicator;
  int64_t qs[3], ks[3];      // element strides: batch, head, token
  int32_t batch, h_kv, group, n, n_p, chunk, n_chunks, n_chunks_p, pool;
  int32_t key_lo, key_hi;    // keys [key_lo, key_hi) are behind the k pointers (row 0 = key key_lo); the whole layer: 0, n
  int32_t chunk0;            // chunk of the first workgroup of a launch
  int32_t n_slices, pack;    // slices in all; slices that share a workgroup (packed kernels), else 1
  float c;                   // scale * log2(e): logits are handled in the log2 domain
  float inv_sw, inv_swc, inv_g;
  float w_mean, w_var, w_prod;   // I_q = w_mean*Mean + w_var*Var + w_prod*Mean*Var (Eq. 11 and the ablation's variants)
  float* lse;                // [slice][G*S_w]
  float* part;               // [slice][n_chunks][G*S_w][2]
  float* hv;                 // [slice][n_chunks_p][G][2]
  float* raw;                // [slice][n_p]
};

// Transfer of keys [t0, t0+64) of one slice into an LDS tile.  The tile is moved as 1 KiB
// groups, one wave-wide instruction each, group i by wave i mod G.  Lane j of a group fills LDS
// bytes [16 j, 16 j + 16) of that group and fetches the piece of the key row that the swizzle
// assigns to that place: group i holds rows i*kRows + lr (lr = j / kPieces), and since kRows is a
// power of two the swizzle splits into a per-lane part (slot ^ lr) and a per-group part
// (i*kRows mod kPieces) that is XORed in with one instruction.  The per-lane offsets are computed
// once per kernel; per transfer there remain a scalar base, one XOR and one add, and no branch.
// Rows past the last key are clamped to it (their logits are masked later), so every access
// stays inside the slice.
// Cache-policy bits of the tile transfers: non-temporal.  Every key byte is used once per pass
// and the whole K of a pass is far larger than the caches, so the tiles should not displace the
// small arrays that are reused (partial sums, normalisers, the un-pooled indicator); measured
// 5-12 % faster on the 32K-context shapes, neutral at 128K.
constexpr int kStreamPolicy = 2;

template <typename T, int D>
struct TileMover {
  using TL = Tile<T, D>;
  static constexpr int kRows = 1024 / TL::kRowBytes;                           // key rows per group
  uint32_t row_off, piece_off;              // per-lane: lr * token stride; (slot ^ lr) * 16
  const char* kbase;
  int64_t tok_bytes;
  int last_key, wave, n_waves, lane;

  __device__ __forceinline__ void init(const char* kbase_, int64_t tok_bytes_, int last_key_, int wave_, int n_waves_,
                                       int lane_) {
    kbase = kbase_; tok_bytes = tok_bytes_; last_key = last_key_; wave = wave_; n_waves = n_waves_; lane = lane_;
    const int lr = lane / TL::kPieces, slot = lane % TL::kPieces;
    row_off = (uint32_t)(lr * tok_bytes);
    piece_off = (uint32_t)((slot ^ lr) << 4);
  }
  __device__ __forceinline__ void issue(char* tile, int t0) const {
    if (t0 + kTileKeys - 1 <= last_key) {       // whole tile inside the slice
      const char* base = kbase + (int64_t)t0 * tok_bytes;
      for (int i = wave; i < TL::kGroups; i += n_waves) {
        const uint32_t group_bits = (uint32_t)(((i * kRows) & (TL::kPieces - 1)) << 4);
        const char* src = base + (int64_t)i * kRows * tok_bytes + (row_off + (piece_off ^ group_bits));
        __builtin_amdgcn_global_load_lds((global_cptr)src, (lds_ptr)(tile + i * 1024), 16, 0, kStreamPolicy);
      }
    } else {
      for (int i = wave; i < TL::kGroups; i += n_waves) {
        const int off = i * 1024 + lane * 16;
        const int r = off / TL::kRowBytes, slot = (off % TL::kRowBytes) >> 4;
        const int q = slot ^ (r & (TL::kPieces - 1));
        const char* src = kbase + (int64_t)min(t0 + r, last_key) * tok_bytes + q * 16;
        __builtin_amdgcn_global_load_lds((global_cptr)src, (lds_ptr)(tile + i * 1024), 16, 0, kStreamPolicy);
      }
    }
  }
};

// All of this wave's outstanding vector-memory operations (the tile transfers) have landed.
__device__ __forceinline__ void wait_vmem() { __builtin_amdgcn_s_waitcnt(0x0F70); }   // vmcnt(0)

__device__ __forceinline__ void slice_coords(const ScoreArgs& a, int slice, int& l, int& b, int& g) {
  g = slice % a.h_kv;
  b = (slice / a.h_kv) % a.batch;
  l = slice / (a.h_kv * a.batch);
}

template <typename T, int D, int MB>
__device__ __forceinline__ void load_q(typename Frag<T>::type (&qf)[MB][D / Frag<T>::kElems], const T* q,
                                       int64_t tok_stride, int c32, int hh) {
  using F = Frag<T>;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int s = 0; s < D / F::kElems; ++s) qf[mb][s] = F::load_global(q + (int64_t)(mb * 32 + c32) * tok_stride, s, hh);
}

// ------------------------------------------------------------------------------------------
// Pass 1: per window row, (reference, sum of 2^(t - reference)) over one chunk of keys.
// ------------------------------------------------------------------------------------------
// Logits of sub-tile `sub` of `tile` (32 keys) against the wave's window rows.
// acc[nb][v]: key = kb + 8*(v/4) + 4*hh + (v%4), window row = nb*32 + c32.
template <typename T, int D, int MB>
__device__ __forceinline__ void pass1_logits(const char* tile, int sub,
                                             const typename Frag<T>::type (&qf)[MB][D / Frag<T>::kElems],
                                             f32x16 (&acc)[MB], int c32, int hh) {
  using F = Frag<T>;
  using TL = Tile<T, D>;
  constexpr int kSteps = D / F::kElems;
#pragma unroll
  for (int s = 0; s < kSteps; ++s) {
    const typename F::type kf = F::template load_lds<TL>(tile, sub * 32 + c32, s, hh);
#pragma unroll
    for (int nb = 0; nb < MB; ++nb) {
      if (s == 0) {
        f32x16 zero;
#pragma unroll
        for (int v = 0; v < 16; ++v) zero[v] = 0.f;
        acc[nb] = F::mfma(kf, qf[nb][s], zero);
      } else {
        acc[nb] = F::mfma(kf, qf[nb][s], acc[nb]);
      }
    }
  }
}

// The finished logits of a sub-tile (first key kb) folded into the rows' running
// (reference, sum) pairs.  Key j is visible to window row r iff j <= n_p + r (and j < n);
// kTail: some key of the sub-tile may be hidden or lie past the end.
template <int MB, bool kTail>
__device__ __forceinline__ void pass1_sums(const f32x16 (&acc)[MB], int kb, float (&mref)[MB], float (&lsum)[MB],
                                           float cv, int n, int n_p, int c32, int hh) {
#pragma unroll
  for (int nb = 0; nb < MB; ++nb) {
    const int last_visible = min(n_p + nb * 32 + c32, n - 1);
    auto hidden = [&](int v) { return kTail && kb + 8 * (v / 4) + 4 * hh + (v % 4) > last_visible; };
    float bsum[2];                        // two chains: consecutive additions do not wait on each other
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const float e = hidden(v) ? 0.f : fast_exp2(fmaf(acc[nb][v], cv, -mref[nb]));
      if (v < 2) bsum[v] = e;
      else bsum[v & 1] += e;
    }
    float block = bsum[0] + bsum[1];
    // Sixteen terms of at most 2^40 each add at most 2^44.  Anything above that (or inf/NaN)
    // means a logit outran the row's reference: redo the block with a reference of its own.
    if (!(block <= 16.f * 1.0995116e12f)) {
      float rmax = kMasked;
#pragma unroll
      for (int v = 0; v < 16; ++v) rmax = fmaxf(rmax, hidden(v) ? kMasked : acc[nb][v] * cv);
      lsum[nb] *= fast_exp2(mref[nb] - rmax);
      mref[nb] = rmax;
      block = 0.f;
#pragma unroll
      for (int v = 0; v < 16; ++v) block += hidden(v) ? 0.f : fast_exp2(acc[nb][v] * cv - rmax);
    }
    lsum[nb] += block;
  }
}

// Packed kernels (kPack): a.pack slices share a workgroup, G waves each, every slice with its own
// tile buffers.  A workgroup's waves are dealt over the compute unit's four SIMDs in turn, so a
// group of 5 or 6 heads alone leaves two waves on one SIMD and one on the others, and the
// barriers make every wave wait for the doubled SIMD; three slices of 5 waves (or two of 6) fill
// the SIMDs almost evenly.  Slices past the last one (the final workgroup) repeat the last
// slice's work and store nothing.
extern __shared__ __attribute__((aligned(1024))) char packed_lds[];

struct WaveRole {
  int slice, w;      // the wave's slice and its head within the group
  int first_wave;    // index of the slice's first wave in the workgroup
  bool live;         // false: a repeat of the last slice, stores nothing
};
template <bool kPack>
__device__ __forceinline__ WaveRole wave_role(const ScoreArgs& a) {
  const int w_all = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave index, known uniform
  WaveRole r;
  if (kPack) {
    const int hg = w_all / a.group;
    const int slice = blockIdx.y * a.pack + hg;
    r.live = slice < a.n_slices;
    r.slice = min(slice, a.n_slices - 1);
    r.first_wave = hg * a.group;
    r.w = w_all - r.first_wave;
  } else {
    r.slice = blockIdx.y; r.w = w_all; r.first_wave = 0; r.live = true;
  }
  return r;
}

template <typename T, int D, int MB, bool kPack>
__global__ __launch_bounds__(kPack ? 1024 : 512) void scores_pass1(ScoreArgs a) {
  using F = Frag<T>;
  using TL = Tile<T, D>;
  constexpr int kSteps = D / F::kElems;
  // double buffer: tile t+1 is in flight while tile t is consumed (rings of three and four tiles
  // measured no faster, and 4 % slower in the packed kernels)
  __shared__ __attribute__((aligned(1024))) char own_tiles[kPack ? 1024 : 2 * TL::kBytes];

  const WaveRole role = wave_role<kPack>(a);
  const int chunk_id = blockIdx.x + a.chunk0, slice = role.slice;
  int l, b, g;
  slice_coords(a, slice, l, b, g);
  const int w = role.w;
  char* tiles = kPack ? packed_lds + (role.first_wave / a.group) * (2 * TL::kBytes) : own_tiles;
  const int lane = threadIdx.x & 63, c32 = lane & 31, hh = lane >> 5;
  const int n_waves = a.group;
  constexpr int s_w = MB * 32;
  const T* q = reinterpret_cast<const T*>(a.q_win[l]) + b * a.qs[0] + (int64_t)(g * a.group + w) * a.qs[1];
  const int64_t tok_bytes = a.ks[2] * (int64_t)sizeof(T);
  // address of key 0 of the slice (keys below key_lo are not behind the pointer and never touched)
  const char* kbase = reinterpret_cast<const char*>(reinterpret_cast<const T*>(a.k[l]) + b * a.ks[0] + (int64_t)g * a.ks[1]) -
                      (int64_t)a.key_lo * tok_bytes;

  const int key0 = chunk_id * a.chunk;
  const int key_end = min(key0 + a.chunk, min(a.n, a.key_hi));
  const int n_tiles = (key_end - key0 + kTileKeys - 1) / kTileKeys;
  TileMover<T, D> mover;
  mover.init(kbase, tok_bytes, min(a.n, a.key_hi) - 1, w, n_waves, lane);
  mover.issue(tiles, key0);

  typename F::type qf[MB][kSteps];
  load_q<T, D, MB>(qf, q, a.qs[2], c32, hh);
  float mref[MB], lsum[MB];
#pragma unroll
  for (int nb = 0; nb < MB; ++nb) { mref[nb] = kMasked; lsum[nb] = 0.f; }
  float cv = a.c;
  asm volatile("" : "+v"(cv));     // a vector register: a scalar operand halves the issue rate of the multiply

  // The MFMAs of a 32-key sub-tile, then the exponentials and sums of its logits.  An explicit
  // software pipeline over two accumulator sets (each k-step's MFMAs followed by a share of the
  // previous sub-tile's vector work, as in pass 2) measured 10 % slower here: it costs a wave
  // per SIMD in registers, and under the chip's power limit overlapping the two pipes buys no time.
  f32x16 acc[MB];
  auto tail_of = [&](int kb) { return kb + 31 > a.n_p; };      // some key of the sub-tile may be hidden or past the end

  // Stage t consumes buffer t mod 2 (known at compile time: the operand reads then address LDS
  // with immediate offsets) and refills the other one, which stage t-1 consumed.
  auto stage = [&](auto slot_c, int t) {
    constexpr int kSlot = decltype(slot_c)::value;
    const char* cur = tiles + kSlot * TL::kBytes;
    char* nxt = tiles + (kSlot ^ 1) * TL::kBytes;
    wait_vmem();
    __syncthreads();                 // tile t complete in `cur`; everyone is done reading `nxt`
    const int t0 = key0 + t * kTileKeys;
    if (t + 1 < n_tiles) mover.issue(nxt, t0 + kTileKeys);
#pragma unroll
    for (int sub = 0; sub < kTileKeys / 32; ++sub) {
      const int kb = t0 + sub * 32;
      if (kb >= key_end) break;
      pass1_logits<T, D, MB>(cur, sub, qf, acc, c32, hh);
      if (tail_of(kb))
        pass1_sums<MB, true>(acc, kb, mref, lsum, cv, a.n, a.n_p, c32, hh);
      else
        pass1_sums<MB, false>(acc, kb, mref, lsum, cv, a.n, a.n_p, c32, hh);
    }
  };
  for (int t = 0; t < n_tiles; t += 2) {
    stage(std::integral_constant<int, 0>{}, t);
    if (t + 1 < n_tiles) stage(std::integral_constant<int, 1>{}, t + 1);
  }

  // Merge the two lane halves of each window row and store the chunk's pair.
  float* out = a.part + (((int64_t)slice * a.n_chunks + chunk_id) * (a.group * s_w) + w * s_w) * 2;
#pragma unroll
  for (int nb = 0; nb < MB; ++nb) {
    float om = __shfl_xor(mref[nb], 32), ol = __shfl_xor(lsum[nb], 32);
    float m = fmaxf(mref[nb], om);
    float s = lsum[nb] * fast_exp2(mref[nb] - m) + ol * fast_exp2(om - m);
    if (hh == 0 && role.live) {
      out[(nb * 32 + c32) * 2 + 0] = m;
      out[(nb * 32 + c32) * 2 + 1] = s;
    }
  }
}

// Combine the chunks' pairs of every window row into lse2 = log2 sum_j 2^(t_j).  Four lanes share
// a row: each folds every fourth chunk into a running (reference, sum) pair in one sweep, the four
// pairs are merged in a fixed order.
__global__ __launch_bounds__(256) void scores_combine(ScoreArgs a, int rows_per_slice, int64_t total_rows) {
  const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 2;
  const int part = threadIdx.x & 3;
  const bool live = i < total_rows;
  const int64_t slice = live ? i / rows_per_slice : 0;
  const int row = live ? (int)(i % rows_per_slice) : 0;
  const float* p = a.part + (slice * a.n_chunks * rows_per_slice + row) * 2;
  float m = kMasked;
  double s = 0.0;
  for (int c = part; live && c < a.n_chunks; c += 4) {
    const float2 pc = *reinterpret_cast<const float2*>(p + (int64_t)c * rows_per_slice * 2);
    if (pc.x > m) { s *= (double)exp2f(m - pc.x); m = pc.x; }
    s += (double)pc.y * (double)exp2f(pc.x - m);
  }
#pragma unroll
  for (int off = 1; off <= 2; off <<= 1) {
    const float om = __shfl_xor(m, off);
    const double os = __shfl_xor(s, off);
    const float mm = fmaxf(m, om);
    // the lower lane's pair first: the same order in both partners
    const double lo_s = (part & off) ? os : s, hi_s = (part & off) ? s : os;
    const float lo_m = (part & off) ? om : m, hi_m = (part & off) ? m : om;
    s = lo_s * (double)exp2f(lo_m - mm) + hi_s * (double)exp2f(hi_m - mm);
    m = mm;
  }
  if (live && part == 0) a.lse[i] = m + (float)log2(s);
}

// Row normalisers handed over by the caller (natural log, [B, H_q, S_w] per layer) -> log2 domain
// in the workspace layout, which is the same order: slice (l, b, g), then head within the group, row.
__global__ void scores_import_lse(ScoreArgs a, const float* const* row_lse, int64_t per_layer, int64_t total) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  a.lse[i] = row_lse[i / per_layer][i % per_layer] * 1.4426950408889634f;
}

// ------------------------------------------------------------------------------------------
// Pass 2: normalised weights on the prefix columns; column Mean/Var, entropy, group mean.
// ------------------------------------------------------------------------------------------
// Column sums of one finished sub-tile, still split over the two lane halves.
struct ColSums {
  float sp, sp2;     // sum of (p - pivot), sum of (p - pivot)^2 over this half's window rows
  float pivot;       // 0 unless the pivoted form is used
};

// One period of pass 2.  kMfma: the MFMAs of sub-tile `sub` of `tile` accumulate into `dst`,
// starting from `init`, which holds -lse2/c of the lane's window rows, so that the accumulator
// times c is already the log2 of the weight.  kValu: the finished accumulators in `src` are
// turned into weights and column sums; with both, the vector work is dealt out over the MFMA
// steps and a scheduling barrier per step pins the interleaving.
// src[mb][v]: window row mb*32 + 8*(v/4) + 4*hh + (v%4) of the key column this lane owns.
// kTail: the column may lie at or beyond the end of the chunk (col_valid false): its weights are
// forced to zero.  kPivot: the sums are taken about the weight of window row 0 (Var and Mean*Var
// indicators: sum p^2 - (sum p)^2/S_w would cancel in fp32 where the weights barely move).
template <typename T, int D, int MB, bool kMfma, bool kValu, bool kTail, bool kPivot>
__device__ __forceinline__ void pass2_period(const char* tile, int sub,
                                             const typename Frag<T>::type (&qf)[MB][D / Frag<T>::kElems],
                                             const f32x16 (&init)[MB], f32x16 (&dst)[MB], const f32x16 (&src)[MB],
                                             float cv, bool col_valid, float (&entv)[2], ColSums& out,
                                             int c32, int hh) {
  using F = Frag<T>;
  using TL = Tile<T, D>;
  constexpr int kSteps = D / F::kElems;
  constexpr int kGroups = 4 * MB;      // groups of four logits per lane in a sub-tile
  constexpr int kAhead = 2;            // operand reads in flight ahead of their MFMA step
  float spv[2] = {0.f, 0.f}, sp2v[2] = {0.f, 0.f};
  float pivot = 0.f;
  auto logit = [&](int mb, int v) { return (kTail && !col_valid) ? -1.0e30f : src[mb][v]; };
  if (kValu && kPivot) {
    // the weight of window row 0 lives in the lower lane half (mb 0, v 0); both halves take it
    const float p0 = fast_exp2(logit(0, 0) * cv);
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(p0), __float_as_uint(p0), false, false);
    pivot = __uint_as_float(r[0]);
  }
  typename F::type kf[kSteps];
  if (kMfma) {
#pragma unroll
    for (int s = 0; s < kAhead && s < kSteps; ++s) kf[s] = F::template load_lds<TL>(tile, sub * 32 + c32, s, hh);
  }
#pragma unroll
  for (int s = 0; s < kSteps; ++s) {
    if (kMfma) {
      if (s + kAhead < kSteps) kf[s + kAhead] = F::template load_lds<TL>(tile, sub * 32 + c32, s + kAhead, hh);
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) dst[mb] = F::mfma(qf[mb][s], kf[s], s == 0 ? init[mb] : dst[mb]);
    }
    if (kValu) {
#pragma unroll
      for (int gi = 0; gi < kGroups; ++gi) {
        if (gi * kSteps / kGroups != s) continue;
        const int mb = gi / 4, v4 = (gi % 4) * 4;
        float x[4], p[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) x[i] = logit(mb, v4 + i);
#pragma unroll
        for (int i = 0; i < 4; ++i) p[i] = fast_exp2(x[i] * cv);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float pd = kPivot ? p[i] - pivot : p[i];
          spv[i & 1] += pd;
          sp2v[i & 1] = fmaf(pd, pd, sp2v[i & 1]);
          entv[i & 1] = fmaf(p[i], x[i], entv[i & 1]);      // sum p * log2(p) / c
        }
        // keep the accumulation in this step (it would otherwise be sunk to the end of the period)
        asm volatile("" : "+v"(spv[0]), "+v"(spv[1]), "+v"(sp2v[0]), "+v"(sp2v[1]), "+v"(entv[0]), "+v"(entv[1]));
      }
    }
    if (kMfma && kValu) __builtin_amdgcn_sched_barrier(0);
  }
  if (kValu) {
    out.sp = spv[0] + spv[1];
    out.sp2 = sp2v[0] + sp2v[1];
    out.pivot = pivot;
  }
}

// Statistics of the 64 key columns of one tile from the half sums of its two sub-tiles.  One
// swap of lane halves per quantity leaves lanes 0-31 with the complete sums of sub-tile 0's
// columns and lanes 32-63 with those of sub-tile 1's: lane L ends up owning key L of the tile.
template <bool kPivot>
__device__ __forceinline__ void pass2_tile_stats(const ColSums& s0, const ColSums& s1, const ScoreArgs& a, int hh,
                                                 float& var_acc, float* iq_row /* [64], this wave's */, int lane) {
  auto r1 = __builtin_amdgcn_permlane32_swap(__float_as_uint(s0.sp), __float_as_uint(s1.sp), false, false);
  auto r2 = __builtin_amdgcn_permlane32_swap(__float_as_uint(s0.sp2), __float_as_uint(s1.sp2), false, false);
  const float sp = __uint_as_float(r1[0]) + __uint_as_float(r1[1]);
  const float sp2 = __uint_as_float(r2[0]) + __uint_as_float(r2[1]);
  const float dmean = sp * a.inv_sw;                               // mean of (p - pivot)
  const float var = fmaxf((sp2 - sp * dmean) * a.inv_swc, 0.f);    // the variance does not see the pivot
  const float mean = kPivot ? dmean + (hh ? s1.pivot : s0.pivot) : dmean;
  var_acc += var;
  iq_row[lane] = fmaf(a.w_prod * mean, var, fmaf(a.w_var, var, a.w_mean * mean));
}

constexpr int kPackMaxWaves = 16;      // waves of a packed workgroup

template <typename T, int D, int MB, bool kPivot, bool kPack>
__global__ __launch_bounds__(kPack ? 1024 : 512) void scores_pass2(ScoreArgs a) {
  using F = Frag<T>;
  using TL = Tile<T, D>;
  constexpr int kSteps = D / F::kElems;
  // double buffer: tile t+1 is in flight while tile t is consumed (deeper rings measured no faster)
  __shared__ __attribute__((aligned(1024))) char own_tiles[kPack ? 1024 : 2 * TL::kBytes];
  // I_q of the G heads for two tiles in turn: the flush of one tile reads one buffer in the
  // stage in which the other is written, and a barrier separates the stages
  __shared__ float own_iq[kPack ? 1 : 2 * 8 * kTileKeys];

  const WaveRole role = wave_role<kPack>(a);
  const int chunk_id = blockIdx.x + a.chunk0, slice = role.slice;
  int l, b, g;
  slice_coords(a, slice, l, b, g);
  const int w = role.w;
  char* tiles = kPack ? packed_lds + (role.first_wave / a.group) * (2 * TL::kBytes) : own_tiles;
  constexpr int kIqWaves = kPack ? kPackMaxWaves : 8;
  // [2][kIqWaves][64]; the packed kernels keep it behind the slices' tile buffers
  float* iq_lds = kPack ? reinterpret_cast<float*>(packed_lds + a.pack * (2 * TL::kBytes)) : own_iq;
  auto iq_row = [&](int buf, int wave) { return iq_lds + (buf * kIqWaves + role.first_wave + wave) * kTileKeys; };
  const int lane = threadIdx.x & 63, c32 = lane & 31, hh = lane >> 5;
  const int n_waves = a.group;
  constexpr int s_w = MB * 32;
  const T* q = reinterpret_cast<const T*>(a.q_win[l]) + b * a.qs[0] + (int64_t)(g * a.group + w) * a.qs[1];
  const int64_t tok_bytes = a.ks[2] * (int64_t)sizeof(T);
  // address of key 0 of the slice (keys below key_lo are not behind the pointer and never touched)
  const char* kbase = reinterpret_cast<const char*>(reinterpret_cast<const T*>(a.k[l]) + b * a.ks[0] + (int64_t)g * a.ks[1]) -
                      (int64_t)a.key_lo * tok_bytes;

  const int key0 = chunk_id * a.chunk;
  const int key_end = min(key0 + a.chunk, min(a.n_p, a.key_hi));
  const int n_tiles = (key_end - key0 + kTileKeys - 1) / kTileKeys;
  TileMover<T, D> mover;
  mover.init(kbase, tok_bytes, min(a.n, a.key_hi) - 1, w, n_waves, lane);
  mover.issue(tiles, key0);

  typename F::type qf[MB][kSteps];
  load_q<T, D, MB>(qf, q, a.qs[2], c32, hh);
  // -lse2/c of the lane's window rows, in the accumulator layout: the MFMA chain of a sub-tile
  // starts from it, so its result times c is the log2 of the normalised weight.
  f32x16 init[MB];
  const float* lse = a.lse + (int64_t)slice * (a.group * s_w) + w * s_w;
  const float neg_inv_c = -1.0f / a.c;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int v = 0; v < 16; ++v) init[mb][v] = lse[mb * 32 + 8 * (v / 4) + 4 * hh + (v % 4)] * neg_inv_c;
  float cv = a.c;
  asm volatile("" : "+v"(cv));     // a vector register: a scalar operand halves the issue rate of the multiply

  float entv[2] = {0.f, 0.f};      // sum p * log2(p) / c over this lane's logits, two chains
  float var_acc = 0.f;
  float* raw = a.raw + (int64_t)slice * a.n_p;
  // Two accumulator sets (logits of even / odd sub-tiles) let one sub-tile's MFMAs overlap the
  // previous one's statistics.  Measured, this pays for bf16 with two row blocks per wave
  // (S_w = 64); with one row block the periods are too short and the plain order is faster, and
  // the fp32 kernels hold four times the query fragments and would spill.  Those run the two
  // phases of a sub-tile one after the other on a single set.
  constexpr bool kPipelined = sizeof(T) == 2 && MB == 2;
  f32x16 acc_a[MB], acc_b[MB];
  ColSums cs0{}, cs1{};

  // Group mean of the G heads' I_q for the 64 keys of tile t, one key per lane; the waves take
  // the tiles in turn.
  auto flush = [&](int t) {
    if (t % n_waves != w) return;
    const int key = key0 + t * kTileKeys + lane;
    float s = 0.f;
    for (int ww = 0; ww < a.group; ++ww) s += iq_row(t & 1, ww)[lane];
    if (key < key_end && role.live) raw[key] = s * a.inv_g;
  };
  // Tile t: its first sub-tile's MFMAs run beside the statistics of tile t-1's second sub-tile,
  // its second sub-tile's MFMAs beside the statistics of its first.  Only the last tile of a
  // chunk can hold columns at or beyond key_end.
  // Stage t consumes buffer t mod 2 (known at compile time: the operand reads then address LDS
  // with immediate offsets) and refills the other one, which stage t-1 consumed.
  constexpr int kFlushLag = kPipelined ? 2 : 1;     // stages between a tile's MFMAs and the flush of its I_q
  auto stage = [&](auto slot_c, int t, auto tail_c) {
    constexpr int kSlot = decltype(slot_c)::value;
    constexpr bool kTail = decltype(tail_c)::value;
    const char* cur = tiles + kSlot * TL::kBytes;
    char* nxt = tiles + (kSlot ^ 1) * TL::kBytes;
    wait_vmem();
    __syncthreads();       // tile t complete in `cur`; every wave is done with `nxt` and with the I_q buffer written next
    const int t0 = key0 + t * kTileKeys;
    if (t + 1 < n_tiles) mover.issue(nxt, t0 + kTileKeys);
    if (t >= kFlushLag) flush(t - kFlushLag);
    const bool v0 = t0 + c32 < key_end, v1 = t0 + 32 + c32 < key_end;
    if (kPipelined) {
      if (t == 0) {
        pass2_period<T, D, MB, true, false, false, kPivot>(cur, 0, qf, init, acc_a, acc_b, cv, true, entv, cs1, c32, hh);
      } else {
        // statistics of tile t-1's second sub-tile: never a tail, tile t-1 is not the last
        pass2_period<T, D, MB, true, true, false, kPivot>(cur, 0, qf, init, acc_a, acc_b, cv, true, entv, cs1, c32, hh);
        pass2_tile_stats<kPivot>(cs0, cs1, a, hh, var_acc, iq_row((t - 1) & 1, w), lane);
      }
      pass2_period<T, D, MB, true, true, kTail, kPivot>(cur, 1, qf, init, acc_b, acc_a, cv, v0, entv, cs0, c32, hh);
    } else {
      pass2_period<T, D, MB, true, false, false, kPivot>(cur, 0, qf, init, acc_a, acc_a, cv, true, entv, cs0, c32, hh);
      pass2_period<T, D, MB, false, true, kTail, kPivot>(cur, 0, qf, init, acc_a, acc_a, cv, v0, entv, cs0, c32, hh);
      pass2_period<T, D, MB, true, false, false, kPivot>(cur, 1, qf, init, acc_a, acc_a, cv, true, entv, cs1, c32, hh);
      pass2_period<T, D, MB, false, true, kTail, kPivot>(cur, 1, qf, init, acc_a, acc_a, cv, v1, entv, cs1, c32, hh);
      pass2_tile_stats<kPivot>(cs0, cs1, a, hh, var_acc, iq_row(t & 1, w), lane);
    }
  };
  const bool last_partial = (key_end - key0) % kTileKeys != 0;
  auto stage_at = [&](auto slot_c, int t) {
    if (t + 1 == n_tiles && last_partial) stage(slot_c, t, std::true_type{});
    else stage(slot_c, t, std::false_type{});
  };
  for (int t = 0; t < n_tiles; t += 2) {
    stage_at(std::integral_constant<int, 0>{}, t);
    if (t + 1 < n_tiles) stage_at(std::integral_constant<int, 1>{}, t + 1);
  }
  if (kPipelined) {    // drain: statistics of the last sub-tile, then of the last tile
    const bool v1 = key0 + (n_tiles - 1) * kTileKeys + 32 + c32 < key_end;
    if (last_partial)
      pass2_period<T, D, MB, false, true, true, kPivot>(tiles, 0, qf, init, acc_a, acc_b, cv, v1, entv, cs1, c32, hh);
    else
      pass2_period<T, D, MB, false, true, false, kPivot>(tiles, 0, qf, init, acc_a, acc_b, cv, true, entv, cs1, c32, hh);
    pass2_tile_stats<kPivot>(cs0, cs1, a, hh, var_acc, iq_row((n_tiles - 1) & 1, w), lane);
  }
  __syncthreads();
  if (kFlushLag == 2 && n_tiles >= 2) flush(n_tiles - 2);
  flush(n_tiles - 1);

  // Per-wave sums in a fixed order.
  float ent_acc = (entv[0] + entv[1]) * cv;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    ent_acc += __shfl_xor(ent_acc, off);
    var_acc += __shfl_xor(var_acc, off);
  }
  if (lane == 0 && role.live) {
    float* o = a.hv + (((int64_t)slice * a.n_chunks_p + chunk_id) * a.group + w) * 2;
    o[0] = ent_acc;
    o[1] = var_acc;
  }
}

// Stride-1 max-pool over the prefix positions, edges clipped (Sec. 4.3 pooling layer).
// A workgroup stages kPoolSpan consecutive positions plus the halo in LDS with coalesced loads,
// so that every un-pooled value is read from memory once.
constexpr int kPoolSpan = 2048;
constexpr int kPoolMaxHalf = 64;        // widest supported pooling window: 2*64+1
constexpr int kPoolQuadHalf = 4;        // widest half window of the four-outputs-per-lane path

// Four consecutive outputs from the twelve staged values around them (w[4..7] are the outputs' own
// positions).
template <int kHalf>
__device__ __forceinline__ float4 pool_quad(const float (&w)[12]) {
  float o[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    float m = w[4 + k];
#pragma unroll
    for (int d = 1; d <= kHalf; ++d) m = fmaxf(m, fmaxf(w[4 + k - d], w[4 + k + d]));
    o[k] = m;
  }
  return make_float4(o[0], o[1], o[2], o[3]);
}

__global__ __launch_bounds__(256) void pool_indicator(ScoreArgs a) {
  // position j0 + i of the span sits at win[kPoolMaxHalf + i]
  __shared__ __attribute__((aligned(16))) float win[kPoolSpan + 2 * kPoolMaxHalf];
  const int slice = blockIdx.y;
  int l, b, g;
  slice_coords(a, slice, l, b, g);
  const int half = a.pool / 2;
  const int j0 = blockIdx.x * kPoolSpan;
  const int span = min(kPoolSpan, a.n_p - j0);
  const float* raw = a.raw + (int64_t)slice * a.n_p;
  float* out = a.indicator[l] + ((int64_t)b * a.h_kv + g) * a.n_p;
  // Rows of a multiple of four positions at 16-byte aligned addresses, windows of at most nine:
  // 16-byte loads and stores, four outputs per lane from three 16-byte LDS reads.
  const bool quads = a.n_p % 4 == 0 && half <= kPoolQuadHalf &&
                     ((reinterpret_cast<uintptr_t>(raw) | reinterpret_cast<uintptr_t>(out)) & 15) == 0;
  if (quads) {
    const float4* raw4 = reinterpret_cast<const float4*>(raw + j0);
    for (int q = threadIdx.x; q < span / 4; q += 256)
      *reinterpret_cast<float4*>(&win[kPoolMaxHalf + 4 * q]) = raw4[q];
    if (threadIdx.x < 8) {            // four positions on either side; clipped edges never win the max
      const int i = threadIdx.x < 4 ? (int)threadIdx.x - 4 : span + (int)threadIdx.x - 4;
      const int j = j0 + i;
      win[kPoolMaxHalf + i] = (j >= 0 && j < a.n_p) ? raw[j] : -INFINITY;
    }
    __syncthreads();
    float4* out4 = reinterpret_cast<float4*>(out + j0);
    for (int q = threadIdx.x; q < span / 4; q += 256) {
      float w[12];
#pragma unroll
      for (int v = 0; v < 3; ++v) {
        const float4 x = *reinterpret_cast<const float4*>(&win[kPoolMaxHalf + 4 * q - 4 + 4 * v]);
        w[4 * v] = x.x; w[4 * v + 1] = x.y; w[4 * v + 2] = x.z; w[4 * v + 3] = x.w;
      }
      float4 r;
      switch (half) {
        case 0: r = pool_quad<0>(w); break;
        case 1: r = pool_quad<1>(w); break;
        case 2: r = pool_quad<2>(w); break;
        case 3: r = pool_quad<3>(w); break;
        default: r = pool_quad<4>(w); break;
      }
      out4[q] = r;
    }
    return;
  }
  for (int i = (int)threadIdx.x - half; i < span + half; i += 256) {
    const int j = j0 + i;
    win[kPoolMaxHalf + i] = (j >= 0 && j < a.n_p) ? raw[j] : -INFINITY;     // clipped edges never win the max
  }
  __syncthreads();
  for (int i = threadIdx.x; i < span; i += 256) {
    float m = win[kPoolMaxHalf + i];
    for (int k = 1; k <= half; ++k) m = fmaxf(m, fmaxf(win[kPoolMaxHalf + i - k], win[kPoolMaxHalf + i + k]));
    out[j0 + i] = m;
  }
}

// Eq. 6 per (layer, sequence): fixed-order fp64 reduction of the chunk sums, then the powers.
__global__ void layer_preference_kernel(const float* hv, int n_layers, int batch, int h_kv, int group,
                                        int n_chunks_p, double inv_tau1, double inv_tau2,
                                        double* pref, double* hv_out) {
  const int l = blockIdx.x / batch, b = blockIdx.x % batch;
  const int lane = threadIdx.x;
  const int per_head = n_chunks_p * group;                 // entries of one KV head
  const float* base = hv + ((int64_t)(l * batch + b) * h_kv) * per_head * 2;
  const int count = h_kv * per_head;
  double e = 0.0, v = 0.0;
  for (int i = lane; i < count; i += 64) {
    e += (double)base[2 * i];
    v += (double)base[2 * i + 1];
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    e += __shfl_xor(e, off);
    v += __shfl_xor(v, off);
  }
  if (lane == 0) {
    const double heads = (double)(h_kv * group);
    // Both are non-negative by definition; with nearly one-hot attention the fp32 sums can come
    // out a rounding error below zero, which the fractional powers below would turn into NaN.
    const double h_l = fmax(-0.6931471805599453 * e / heads, 0.0);   // sum p*log2 p -> -sum p ln p
    const double v_l = fmax(v / heads, 0.0);
    pref[(int64_t)b * n_layers + l] = pow(h_l, inv_tau1) * pow(v_l, inv_tau2);
    if (hv_out) {
      hv_out[((int64_t)b * n_layers + l) * 2 + 0] = h_l;
      hv_out[((int64_t)b * n_layers + l) * 2 + 1] = v_l;
    }
  }
}

// Optional event timing of the four kernels (diagnostics).  Process-wide and not thread-safe:
// one set of five events per profiled call, the last kProfileSets calls are kept.
constexpr int kProfileSets = 64;
struct Profile {
  bool enabled = false, created = false;
  int64_t calls = 0;                       // profiled calls since cake_profile_enable(1)
  hipEvent_t ev[kProfileSets][5] = {};
};
Profile g_profile;

inline void mark(int i, hipStream_t stream) {
  if (g_profile.enabled && g_profile.created) (void)hipEventRecord(g_profile.ev[g_profile.calls % kProfileSets][i], stream);
}

// Which parts of the score stage a call runs: everything on a resident layer, or one of the
// four steps of the segment-wise form (keys handed over a range at a time).
enum ScoreParts { kPartsAll, kPartsPass1Segment, kPartsCombine, kPartsPass2Segment, kPartsPool };

// Slices per workgroup: group sizes whose waves would load the four SIMDs unevenly share a
// workgroup (3 x 5 or 2 x 6 waves).  Only the kernels that fit 16 waves on a compute unit
// (bf16, one row block) have a packed form.
template <typename T, int MB>
constexpr bool can_pack() { return sizeof(T) == 2 && MB == 1; }
inline int slices_per_workgroup(int group) { return group == 5 ? 3 : group == 6 ? 2 : 1; }

template <typename T, int D, int MB, bool kPivot>
int launch_scores(const ScoreArgs& a_in, int64_t n_slices, const float* const* row_lse, ScoreParts parts, hipStream_t stream) {
  ScoreArgs a = a_in;
  const bool packing = a_in.pack > 1;
  auto set_pack = [&](int pass, dim3& block, unsigned& gy, size_t& packed_bytes) {
    (void)pass;
    a.pack = packing ? slices_per_workgroup(a.group) : 1;
    block = dim3(64 * a.group * a.pack);
    gy = (unsigned)((n_slices + a.pack - 1) / a.pack);
    packed_bytes = (size_t)a.pack * 2 * Tile<T, D>::kBytes + sizeof(float) * 2 * kPackMaxWaves * kTileKeys;
  };
  dim3 block;
  unsigned gy;
  size_t packed_bytes;
  auto run_pass1 = [&](int chunks) -> hipError_t {
    set_pack(1, block, gy, packed_bytes);
    if constexpr (can_pack<T, MB>()) {
      if (a.pack > 1) {
        auto kern = scores_pass1<T, D, MB, true>;
        if (hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                               (int)packed_bytes); e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, dim3(chunks, gy), block, packed_bytes, stream, a);
        return hipSuccess;
      }
    }
    hipLaunchKernelGGL((scores_pass1<T, D, MB, false>), dim3(chunks, gy), block, 0, stream, a);
    return hipSuccess;
  };
  auto run_pass2 = [&](int chunks) -> hipError_t {
    set_pack(2, block, gy, packed_bytes);
    if constexpr (can_pack<T, MB>()) {
      if (a.pack > 1) {
        auto kern = scores_pass2<T, D, MB, kPivot, true>;
        if (hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                               (int)packed_bytes); e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, dim3(chunks, gy), block, packed_bytes, stream, a);
        return hipSuccess;
      }
    }
    hipLaunchKernelGGL((scores_pass2<T, D, MB, kPivot, false>), dim3(chunks, gy), block, 0, stream, a);
    return hipSuccess;
  };
  const int rows = a.group * MB * 32;
  const int64_t total_rows = n_slices * rows;
  if (parts != kPartsAll) {
    // chunks of this launch: those that hold keys of [key_lo, key_hi) (pass 2: below n_p as well)
    const int hi1 = min(a.n, a.key_hi), hi2 = min(a.n_p, a.key_hi);
    const int c1 = (hi1 - a.key_lo + a.chunk - 1) / a.chunk, c2 = hi2 > a.key_lo ? (hi2 - a.key_lo + a.chunk - 1) / a.chunk : 0;
    if (parts == kPartsPass1Segment)
      CAKE_HIP_TRY(run_pass1(c1));
    else if (parts == kPartsCombine)
      hipLaunchKernelGGL(scores_combine, dim3((unsigned)((total_rows * 4 + 255) / 256)), dim3(256), 0, stream, a, rows, total_rows);
    else if (parts == kPartsPass2Segment && c2 > 0)
      CAKE_HIP_TRY(run_pass2(c2));
    else if (parts == kPartsPool)
      hipLaunchKernelGGL(pool_indicator, dim3((a.n_p + kPoolSpan - 1) / kPoolSpan, (unsigned)n_slices), dim3(256), 0, stream, a);
    CAKE_HIP_TRY(hipGetLastError());
    return CAKE_OK;
  }
  mark(0, stream);
  if (row_lse == nullptr) {
    CAKE_HIP_TRY(run_pass1(a.n_chunks));
    mark(1, stream);
    hipLaunchKernelGGL(scores_combine, dim3((unsigned)((total_rows * 4 + 255) / 256)), dim3(256), 0, stream, a, rows, total_rows);
  } else {
    const int64_t per_layer = (int64_t)a.batch * a.h_kv * rows;
    hipLaunchKernelGGL(scores_import_lse, dim3((unsigned)((total_rows + 255) / 256)), dim3(256), 0, stream, a, row_lse,
                       per_layer, total_rows);
    mark(1, stream);
  }
  mark(2, stream);
  CAKE_HIP_TRY(run_pass2(a.n_chunks_p));
  mark(3, stream);
  hipLaunchKernelGGL(pool_indicator, dim3((a.n_p + kPoolSpan - 1) / kPoolSpan, (unsigned)n_slices), dim3(256), 0, stream, a);
  mark(4, stream);
  if (g_profile.enabled && g_profile.created) g_profile.calls += 1;
  CAKE_HIP_TRY(hipGetLastError());
  return CAKE_OK;
}

}  // namespace
}  // namespace cake

using namespace cake;

extern "C" int cake_profile_enable(int enable) {
  if (enable && !g_profile.created) {
    for (auto& set : g_profile.ev)
      for (auto& e : set) CAKE_HIP_TRY(hipEventCreate(&e));
    g_profile.created = true;
  }
  if (!enable && g_profile.created) {
    for (auto& set : g_profile.ev)
      for (auto& e : set) (void)hipEventDestroy(e);
    g_profile.created = false;
  }
  g_profile.calls = 0;
  g_profile.enabled = enable != 0;
  return CAKE_OK;
}

extern "C" int cake_profile_read(float* ms) {
  CAKE_REQUIRE(ms != nullptr, "ms is NULL");
  CAKE_REQUIRE(g_profile.enabled && g_profile.calls > 0, "no profiled cake_window_scores call to read");
  const int64_t n = g_profile.calls < kProfileSets ? g_profile.calls : kProfileSets;
  double sum[4] = {0, 0, 0, 0};
  for (int64_t c = g_profile.calls - n; c < g_profile.calls; ++c) {
    hipEvent_t* ev = g_profile.ev[c % kProfileSets];
    CAKE_HIP_TRY(hipEventSynchronize(ev[4]));
    for (int i = 0; i < 4; ++i) {
      float x = 0.f;
      CAKE_HIP_TRY(hipEventElapsedTime(&x, ev[i], ev[i + 1]));
      sum[i] += x;
    }
  }
  for (int i = 0; i < 4; ++i) ms[i] = (float)(sum[i] / (double)n);
  return CAKE_OK;
}

namespace {
int window_scores_impl(const cake_shape* shape, const cake_params* params,
                       const void* const* q_win, const void* const* k,
                       const int64_t* q_strides, const int64_t* k_strides,
                       const float* const* row_lse, float* const* indicator,
                       void* workspace, size_t workspace_bytes, void* stream,
                       ScoreParts parts = kPartsAll, int key_begin = 0, int key_count = 0) {
  if (int rc = check_shape_scores(shape)) return rc;
  CAKE_REQUIRE(params != nullptr, "params is NULL");
  // what the parts of this call touch: the two finishing steps read neither queries nor keys,
  // and only the resident form and the pooling step write the indicator
  const bool reads_keys = parts == kPartsAll || parts == kPartsPass1Segment || parts == kPartsPass2Segment;
  const bool writes_indicator = parts == kPartsAll || parts == kPartsPool;
  if (reads_keys) {
    CAKE_REQUIRE(q_win && k, "q_win or k table is NULL");
    CAKE_REQUIRE(q_strides && k_strides, "q_strides or k_strides is NULL");
  }
  CAKE_REQUIRE(!writes_indicator || indicator, "indicator table is NULL");
  CAKE_REQUIRE(params->pool_kernel >= 1 && params->pool_kernel % 2 == 1 && params->pool_kernel <= 2 * kPoolMaxHalf + 1,
               "pool_kernel %d must be odd and within [1, %d]", params->pool_kernel, 2 * kPoolMaxHalf + 1);
  CAKE_REQUIRE(params->indicator_mode >= CAKE_IND_MEAN_PLUS_VAR && params->indicator_mode <= CAKE_IND_CUMULATIVE,
               "indicator_mode %d is not a cake_indicator", params->indicator_mode);
  CAKE_REQUIRE(params->var_correction == 0 || params->var_correction == 1, "var_correction %d must be 0 or 1", params->var_correction);
  CAKE_REQUIRE(std::isfinite(params->gamma) && std::isfinite(params->scale) && params->scale >= 0.f, "gamma/scale must be finite, scale >= 0");
  const size_t eb = elem_bytes(shape->dtype);
  if (reads_keys) {
    for (int i = 0; i < 3; ++i) {
      CAKE_REQUIRE(q_strides[i] >= 0 && k_strides[i] >= 0, "negative stride");
      CAKE_REQUIRE((q_strides[i] * eb) % 16 == 0 && (k_strides[i] * eb) % 16 == 0, "strides must be multiples of 16 bytes");
    }
    CAKE_REQUIRE(q_strides[2] >= shape->head_dim && k_strides[2] >= shape->head_dim, "token stride below head_dim");
    CAKE_REQUIRE(k_strides[2] * (int64_t)eb <= (int64_t)1 << 27, "key token stride above 128 MiB");
  }
  const ScoreLayout lay = score_layout(*shape);
  if (workspace == nullptr || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0)
    return fail(CAKE_ERR_WORKSPACE, "workspace is NULL or not 256-byte aligned");
  if (workspace_bytes < lay.total)
    return fail(CAKE_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, lay.total);
  if (lay.n_slices > 65535) return fail(CAKE_ERR_UNSUPPORTED, "layers*batch*kv_heads = %lld exceeds 65535 per call", (long long)lay.n_slices);

  ScoreArgs a{};
  a.q_win = q_win; a.k = k; a.indicator = indicator;
  if (reads_keys)
    for (int i = 0; i < 3; ++i) { a.qs[i] = q_strides[i]; a.ks[i] = k_strides[i]; }
  a.batch = shape->batch; a.h_kv = shape->n_kv_heads; a.group = shape->n_q_heads / shape->n_kv_heads;
  a.n = shape->seq_len; a.n_p = shape->seq_len - shape->window;
  a.chunk = lay.chunk; a.n_chunks = lay.n_chunks; a.n_chunks_p = lay.n_chunks_p; a.pool = params->pool_kernel;
  a.key_lo = 0; a.key_hi = a.n; a.chunk0 = 0;
  a.n_slices = (int32_t)lay.n_slices;
  a.pack = (shape->dtype == CAKE_BF16 && shape->window == 32) ? slices_per_workgroup(a.group) : 1;
  if (parts == kPartsPass1Segment || parts == kPartsPass2Segment) {
    CAKE_REQUIRE(key_begin >= 0 && key_count > 0 && (int64_t)key_begin + key_count <= a.n,
                 "segment [%d, %d + %d) outside [0, seq_len = %d)", key_begin, key_begin, key_count, a.n);
    CAKE_REQUIRE(key_begin % a.chunk == 0, "key_begin %d is not a multiple of the chunk of %d keys", key_begin, a.chunk);
    CAKE_REQUIRE((key_begin + key_count) % a.chunk == 0 || key_begin + key_count == a.n,
                 "a segment must end on a multiple of the chunk of %d keys or at seq_len", a.chunk);
    a.key_lo = key_begin; a.key_hi = key_begin + key_count; a.chunk0 = key_begin / a.chunk;
  }
  const int mode = params->indicator_mode;     // Eq. 11; Mean, Var, Mean*Var of the indicator ablation; the window's column sum
  a.w_mean = (mode == CAKE_IND_MEAN_PLUS_VAR || mode == CAKE_IND_MEAN) ? 1.f
             : mode == CAKE_IND_CUMULATIVE ? (float)shape->window : 0.f;     // Sec. 5.5: column sum = S_w * Mean
  a.w_var = mode == CAKE_IND_MEAN_PLUS_VAR ? params->gamma : mode == CAKE_IND_VAR ? 1.f : 0.f;
  a.w_prod = mode == CAKE_IND_MEAN_TIMES_VAR ? 1.f : 0.f;
  const double scale = params->scale > 0.f ? (double)params->scale : 1.0 / std::sqrt((double)shape->head_dim);
  a.c = (float)(scale * 1.4426950408889634);
  a.inv_sw = 1.0f / (float)shape->window;
  a.inv_swc = 1.0f / (float)(shape->window - params->var_correction);
  a.inv_g = 1.0f / (float)a.group;
  char* ws = static_cast<char*>(workspace);
  a.lse = reinterpret_cast<float*>(ws + lay.off_lse);
  a.part = reinterpret_cast<float*>(ws + lay.off_part);
  a.hv = reinterpret_cast<float*>(ws + lay.off_hv);
  a.raw = reinterpret_cast<float*>(ws + lay.off_raw);
  hipStream_t st = static_cast<hipStream_t>(stream);

  // Var and Mean*Var score a token by the variance alone or by a product with it: those take the
  // pivoted column sums.  Eq. 11's sum and the plain mean do not need them.
  const bool pivot = mode == CAKE_IND_VAR || mode == CAKE_IND_MEAN_TIMES_VAR;
#define CAKE_DISPATCH(T, D, MB)                                                         \
  return pivot ? launch_scores<T, D, MB, true>(a, lay.n_slices, row_lse, parts, st)     \
               : launch_scores<T, D, MB, false>(a, lay.n_slices, row_lse, parts, st)
  const bool bf = shape->dtype == CAKE_BF16;
  const int d = shape->head_dim, mb = shape->window / 32;
  if (bf && d == 128 && mb == 1) CAKE_DISPATCH(__bf16, 128, 1);
  if (bf && d == 128 && mb == 2) CAKE_DISPATCH(__bf16, 128, 2);
  if (bf && d == 64 && mb == 1) CAKE_DISPATCH(__bf16, 64, 1);
  if (bf && d == 64 && mb == 2) CAKE_DISPATCH(__bf16, 64, 2);
  if (!bf && d == 128 && mb == 1) CAKE_DISPATCH(float, 128, 1);
  if (!bf && d == 128 && mb == 2) CAKE_DISPATCH(float, 128, 2);
  if (!bf && d == 64 && mb == 1) CAKE_DISPATCH(float, 64, 1);
  if (!bf && d == 64 && mb == 2) CAKE_DISPATCH(float, 64, 2);
#undef CAKE_DISPATCH
  return fail(CAKE_ERR_UNSUPPORTED, "no score kernel for this shape");
}
}  // namespace

extern "C" int cake_window_scores(const cake_shape* shape, const cake_params* params,
                                  const void* const* q_win, const void* const* k,
                                  const int64_t* q_strides, const int64_t* k_strides,
                                  float* const* indicator,
                                  void* workspace, size_t workspace_bytes, void* stream) {
  return window_scores_impl(shape, params, q_win, k, q_strides, k_strides, nullptr, indicator, workspace,
                            workspace_bytes, stream);
}

extern "C" int cake_window_scores_lse(const cake_shape* shape, const cake_params* params,
                                      const void* const* q_win, const void* const* k,
                                      const int64_t* q_strides, const int64_t* k_strides,
                                      const float* const* row_lse, float* const* indicator,
                                      void* workspace, size_t workspace_bytes, void* stream) {
  CAKE_REQUIRE(row_lse != nullptr, "row_lse table is NULL");
  return window_scores_impl(shape, params, q_win, k, q_strides, k_strides, row_lse, indicator, workspace,
                            workspace_bytes, stream);
}

extern "C" int cake_scores_chunk_keys(const cake_shape* shape, int32_t* chunk) {
  CAKE_REQUIRE(chunk != nullptr, "chunk is NULL");
  if (int rc = check_shape_scores(shape)) return rc;
  *chunk = score_layout(*shape).chunk;
  return CAKE_OK;
}

extern "C" int cake_window_scores_segment(const cake_shape* shape, const cake_params* params, int32_t pass,
                                          int32_t key_begin, int32_t key_count,
                                          const void* const* q_win, const void* const* k_segment,
                                          const int64_t* q_strides, const int64_t* k_strides,
                                          void* workspace, size_t workspace_bytes, void* stream) {
  CAKE_REQUIRE(pass == 1 || pass == 2, "pass %d must be 1 or 2", pass);
  return window_scores_impl(shape, params, q_win, k_segment, q_strides, k_strides, nullptr, nullptr, workspace,
                            workspace_bytes, stream, pass == 1 ? kPartsPass1Segment : kPartsPass2Segment, key_begin, key_count);
}

extern "C" int cake_window_scores_finish(const cake_shape* shape, const cake_params* params, int32_t pass,
                                         float* const* indicator, void* workspace, size_t workspace_bytes, void* stream) {
  CAKE_REQUIRE(pass == 1 || pass == 2, "pass %d must be 1 or 2", pass);
  return window_scores_impl(shape, params, nullptr, nullptr, nullptr, nullptr, nullptr, indicator, workspace,
                            workspace_bytes, stream, pass == 1 ? kPartsCombine : kPartsPool);
}

extern "C" int cake_layer_preference(const cake_shape* shape, const cake_params* params,
                                     const void* workspace, size_t workspace_bytes,
                                     double* pref, double* hv, void* stream) {
  if (int rc = check_shape_scores(shape)) return rc;
  CAKE_REQUIRE(params != nullptr && pref != nullptr, "params or pref is NULL");
  CAKE_REQUIRE(params->tau1 > 0.f && params->tau2 > 0.f && std::isfinite(params->tau1) && std::isfinite(params->tau2),
               "tau1 and tau2 must be positive and finite");
  const ScoreLayout lay = score_layout(*shape);
  if (workspace == nullptr || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0)
    return fail(CAKE_ERR_WORKSPACE, "workspace is NULL or not 256-byte aligned");
  if (workspace_bytes < lay.total)
    return fail(CAKE_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, lay.total);
  const float* hv_part = reinterpret_cast<const float*>(static_cast<const char*>(workspace) + lay.off_hv);
  hipLaunchKernelGGL(layer_preference_kernel, dim3(shape->n_layers * shape->batch), dim3(64), 0,
                     static_cast<hipStream_t>(stream), hv_part, shape->n_layers, shape->batch, shape->n_kv_heads,
                     shape->n_q_heads / shape->n_kv_heads, lay.n_chunks_p, 1.0 / (double)params->tau1,
                     1.0 / (double)params->tau2, pref, hv);
  CAKE_HIP_TRY(hipGetLastError());
  return CAKE_OK;
}
