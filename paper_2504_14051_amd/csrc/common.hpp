// Shared declarations of the CAOTE HIP kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "caote.h"

namespace caote {

constexpr int kWave = 64;
constexpr int kVChunk = 256;      // tokens per workgroup in the value sweeps
constexpr int kMaxD = 128;        // largest head_dim
constexpr int kHistBins = 4096;   // selection histogram: top 12 bits of the score key
constexpr int kHistShift = 20;
constexpr int kSelSpan = 2048;    // tokens per workgroup in the selection kernels
constexpr int kMaxSpans = 1024;   // spans per head the selection supports (2M tokens)
constexpr int kOneWgCap = 16384;  // largest cache whose selection one workgroup per head does alone
constexpr int kVSideSlots = 34;   // short caches: value rows a lane keeps in registers (k_vside)
constexpr int kJointMaxCap = CAOTE_JOINT_MAX_CAPACITY;   // greedy joint eviction: weights of a head fit LDS

struct SegTab { long long first; int tiles; int pad; };   // (see Params::seg_tab)

// Everything a kernel needs to know about one call.  Passed by value.
struct Params {
  const void* q;
  void* K;
  void* V;
  float* base;        // H2O accumulator (in/out) or nullptr
  float* scores;      // out
  const int32_t* seq_lens;
  const float* lse_in;// [B][Hq][W] natural-log row normalisers from the caller, or nullptr
  int32_t* kept;      // [BH][budget]
  int B, Hq, Hkv, G, D, W, R, cap;
  int64_t ksb, ksh, ksn, vsb, vsh, vsn, qsb, qsh, qsw;
  int base_mode, pool, wic, ph, pt, variant, dtype;
  int budget, mode;
  float c2;           // softmax_scale * log2(e): logits are handled in the log2 domain
  float rcpW;         // 1 / W, for row -> (query head, window position) without integer division
  // ---- workspace ----
  float* stats;       // [BH][n_split][Rp][2]  partial (max, sum) per query row
  float* lse2;        // [BH][Rp]              log2-sum-exp2 per query row
  float* S;           // [BH][s_rows][s_pitch] stored logits (few-row path only)
  int small_r, s_rows;// few-row path: R <= 8, logits kept instead of a second key sweep
  int s_pitch;        // cap rounded up to a multiple of 4 (16-byte aligned rows of S)
  float* a;           // [BH][cap]             column sums of attention
  float* h;           // [BH][cap]             base score (aliases `base` for H2O)
  float* opart;       // [BH][n_vpart][D]      partial sum of h_j v_j
  float* zpart;       // [BH][n_vpart]         partial sum of h_j
  float* osum;        // [BH][kMaxD+1]         sum h_j v_j (un-normalised) and, last, Z
  uint32_t* hist;     // [BH][kHistBins]       histogram of the score keys
  uint32_t* sel_cand; // [BH][cap]             keys of the threshold bin, one list per span
  int32_t* sel_rec;   // [BH][n_span][2]       per span: keys in higher bins, list length
  int32_t* sel_head;  // [BH][4]               threshold bin, rank inside it, its population
  int n_span;
  int hist_zeroed;    // an earlier kernel of this call has cleared `hist` (fused call)
  int hist_in_vscore; // fused call, long cache: k_vscore builds the selection's histogram
  int select_swaps;   // fused call on a short cache: the selection also does the evict-one row swap
  void* stage;        // compaction staging
  // greedy joint eviction (capacity <= kJointMaxCap); its per-token weights reuse sel_cand
  float* j_part;      // [2][BH][j_c][4 + kMaxD] per slice and step parity: best candidate and its w (o - v)
  float* j_u;         // [2][BH][kMaxD]          running sum u, by step parity
  double* j_rest;     // [2][BH]                 1 - evicted weight, by step parity
  int j_c, j_slice;   // slices per head, tokens per slice
  int n_split, split_len, Rp, n_vchunk, vchunk_len;
  // the first key sweep and the merge of its row statistics: the same split unless the
  // matrix-core sweep has several row groups, which then go into the grid with longer splits
  int n_split0, split_len0, n_rg0;
  // Ragged batches on the matrix-core path: the key tiles of all heads, laid end to end, are cut
  // into equal shares, one per workgroup, wherever the cuts fall (a workgroup may finish one
  // head and start the next); a head's pieces are its splits.  k_plan_splits fills the tables.
  int dyn_split;      // the key sweeps take their splits from the tables below
  int dyn_wgs;        // workgroups per sweep launch (shares)
  int dyn_min_tiles;  // a share is at least this long, so that no head has more than n_split pieces
  SegTab* seg_tab;    // [BH]       per head: index of its first tile in the end-to-end order, tiles
  int32_t* wg_tab;    // [dyn_wgs]  per workgroup: the head its share starts in, -1: no work
  int32_t* seg_glob;  // [0]        tiles per share
  int vrep, n_vsum;   // value sum: 256-token chunks per workgroup, partial sums per head
  int use_mfma;       // key sweeps on the matrix cores (bf16, head_dim 128, R > 16)
  int halo;           // SnapKV: pooling half-width (0 otherwise)
  int vside_cs;       // short cache: column workgroups per head of the one-read value kernel (0: not used)
  float* d2part;      // [vside_cs][BH][cap]   per column slice: its part of ||v_j - o||^2
  int merge_in_vside; // few query rows: k_vside merges the row statistics itself (no merge kernel)
  int combine_in_select;  // fused call: the one-workgroup selection adds the column slices up (no k_vcombine)
  int fuse_v;         // the second key sweep also forms the value partial sums (one per split)
  int n_vpart;        // partial sums per head in opart / zpart: n_split if fuse_v, else n_vsum
};

__device__ __forceinline__ int seq_len(const Params& p, int b) {
  if (p.seq_lens == nullptr) return p.cap;
  int n = p.seq_lens[b];
  return n < 0 ? 0 : (n > p.cap ? p.cap : n);
}

// Key splits of head bh on the matrix-core path: how many there are, and the keys [c0, c1) of
// split s.  Equal lengths: cap cut into pieces of `split_len` keys.  Ragged batches: the pieces
// that the workgroups' equal shares of the end-to-end tile sequence cut the head into.
__device__ __forceinline__ int split_count(const Params& p, int bh, int N, int split_len) {
  if (!p.dyn_split) return (N + split_len - 1) / split_len;
  const SegTab t = p.seg_tab[bh];
  if (t.tiles == 0) return 0;
  const long long tpw = p.seg_glob[0];
  return (int)((t.first + t.tiles - 1) / tpw - t.first / tpw) + 1;
}
__device__ __forceinline__ void split_range(const Params& p, int bh, int s, int N, int split_len, int& c0, int& c1) {
  if (!p.dyn_split) {
    c0 = s * split_len;
    c1 = min(N, c0 + split_len);
    return;
  }
  const SegTab t = p.seg_tab[bh];
  const long long tpw = p.seg_glob[0], w = t.first / tpw + s;
  const long long t0 = max(0ll, w * tpw - t.first), t1 = min((long long)t.tiles, (w + 1) * tpw - t.first);
  c0 = (int)t0 * 64;
  c1 = min(N, (int)t1 * 64);
}

// ---- 8-element row fragments ---------------------------------------------------
struct bf16_t { uint16_t bits; };

__device__ __forceinline__ void load8(const float* ptr, float (&x)[8]) {
  const float4 lo = *reinterpret_cast<const float4*>(ptr);
  const float4 hi = *reinterpret_cast<const float4*>(ptr + 4);
  x[0] = lo.x; x[1] = lo.y; x[2] = lo.z; x[3] = lo.w;
  x[4] = hi.x; x[5] = hi.y; x[6] = hi.z; x[7] = hi.w;
}

__device__ __forceinline__ void load8(const bf16_t* ptr, float (&x)[8]) {
  const uint4 u = *reinterpret_cast<const uint4*>(ptr);
  x[0] = __uint_as_float(u.x << 16); x[1] = __uint_as_float(u.x & 0xffff0000u);
  x[2] = __uint_as_float(u.y << 16); x[3] = __uint_as_float(u.y & 0xffff0000u);
  x[4] = __uint_as_float(u.z << 16); x[5] = __uint_as_float(u.z & 0xffff0000u);
  x[6] = __uint_as_float(u.w << 16); x[7] = __uint_as_float(u.w & 0xffff0000u);
}

// Sum over a team of TL consecutive lanes (TL a power of two <= 64); every lane
// of the team receives the total.
template <int TL>
__device__ __forceinline__ float team_sum(float v) {
#pragma unroll
  for (int m = TL / 2; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
  return v;
}

// x + (x of another lane of the same 16-lane row), the lane chosen by a DPP control word.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
  const int y = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, false);
  return x + __builtin_bit_cast(float, y);
}
// Sum over a team of TL (2, 4, 8 or 16) consecutive lanes, total in every lane: fold the row
// (lane i <-> 15-i), fold each half (i <-> 7-i), then the two quad exchanges.
template <int TL>
__device__ __forceinline__ float team_sum_dpp(float x) {
  static_assert(TL == 2 || TL == 4 || TL == 8 || TL == 16, "team size");
  if (TL >= 16) x = dpp_add<0x140>(x);   // row_mirror
  if (TL >= 8) x = dpp_add<0x141>(x);    // row_half_mirror
  x = dpp_add<0xB1>(x);                  // quad_perm [1,0,3,2]
  if (TL >= 4) x = dpp_add<0x4E>(x);     // quad_perm [2,3,0,1]
  return x;
}

// r = q * W + m with 0 <= m < W, for 0 <= r < 2^22: float estimate, one correction step.
__device__ __forceinline__ void divmod_w(const Params& p, int r, int& q, int& m) {
  q = (int)((float)r * p.rcpW);
  m = r - q * p.W;
  if (m < 0) { m += p.W; --q; }
  else if (m >= p.W) { m -= p.W; ++q; }
}

// log2-domain normaliser of query row r of head bh = (b, hk): the caller's, or the one the
// first key sweep left in the workspace.
__device__ __forceinline__ float row_lse2(const Params& p, int b, int hk, int bh, int r) {
  if (p.lse_in) {
    int g, iw;
    divmod_w(p, r, g, iw);
    return p.lse_in[((int64_t)b * p.Hq + hk * p.G + g) * p.W + iw] * 1.4426950408889634f;
  }
  return p.lse2[(int64_t)bh * p.Rp + r];
}

// log2-domain normaliser of query row r from the partial (max, sum) pairs that the first key
// sweep left per split: lse2_r = log2 sum_j exp2(t_rj).
__device__ __forceinline__ float merged_lse2(const Params& p, int bh, int r, int N) {
  const int ns = (N + p.split_len0 - 1) / p.split_len0;
  const float* st = p.stats + ((int64_t)bh * p.n_split0 * p.Rp + r) * 2;
  float M = -INFINITY;
  for (int s = 0; s < ns; ++s) M = fmaxf(M, st[(int64_t)s * p.Rp * 2]);
  float L = 0.f;
  for (int s = 0; s < ns; ++s) {
    const float ms = st[(int64_t)s * p.Rp * 2];
    if (ms > -INFINITY) L += st[(int64_t)s * p.Rp * 2 + 1] * exp2f(ms - M);
  }
  return L > 0.f ? M + log2f(L) : INFINITY;
}

// Score of token j from what k_vside left: c_j = h_j / (Z - h_j) * sqrt(sum over the column
// slices of their part of ||v_j - o||^2) (Sec. 3.2), +INF for protected rows and for a lone
// scored token.  Also writes the score and, for H2O, the updated accumulator.
__device__ __forceinline__ float combine_score(const Params& p, int bh, int j, int N) {
  const int lo = min(p.ph, N), hi = max(lo, N - p.pt);
  const float Z = p.osum[(int64_t)bh * (kMaxD + 1) + kMaxD];
  const float hj = p.h[(int64_t)bh * p.cap + j];
  float out = INFINITY;
  if (j >= lo && j < hi && hi - lo > 1) {
    float q = 0.f;
    for (int c = 0; c < p.vside_cs; ++c) q += p.d2part[((int64_t)c * p.B * p.Hkv + bh) * p.cap + j];
    out = Z > 0.f ? hj / fmaxf(Z - hj, 1.17549435e-38f) * sqrtf(q) : 0.f;
  }
  p.scores[(int64_t)bh * p.cap + j] = out;
  if (p.base_mode == CAOTE_BASE_H2O) p.base[(int64_t)bh * p.cap + j] = hj;   // the accumulator, all rows
  return out;
}

// Clears the per-head counters that later kernels of the same call accumulate into.
// Called by one workgroup per head of a kernel that runs before them.
__device__ __forceinline__ void reset_counters(const Params& p, int bh) {
  for (int i = threadIdx.x; i < kHistBins; i += blockDim.x) p.hist[(int64_t)bh * kHistBins + i] = 0u;
}

// Order-preserving map float -> uint32 (larger float <=> larger key; -0 and +0 share a key,
// as they compare equal).
__device__ __forceinline__ uint32_t float_key(float f) {
  uint32_t u = __float_as_uint(f);
  u = u == 0x80000000u ? 0u : u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// ---- launchers (one per source file) --------------------------------------------
// A launcher calls mark(hook, name) after each kernel it enqueues (measurement aid); a true
// return means: enqueue nothing more, return.
struct PhaseHook {
  virtual bool mark(const char* name) = 0;
  virtual bool full() const = 0;      // a launcher that another one called has been told to stop
 protected:
  ~PhaseHook() = default;
};
inline bool mark(PhaseHook* h, const char* name) { return h && h->mark(name); }
inline bool full(const PhaseHook* h) { return h && h->full(); }

hipError_t launch_score_generic(const Params& p, hipStream_t s, PhaseHook* hook);
hipError_t launch_score_mfma(const Params& p, hipStream_t s, PhaseHook* hook);
hipError_t launch_score_small(const Params& p, hipStream_t s, PhaseHook* hook);
hipError_t launch_score_few_mfma(const Params& p, hipStream_t s, PhaseHook* hook);
hipError_t launch_merge_stats(const Params& p, hipStream_t s, PhaseHook* hook);
constexpr int kDynMaxBatch = 1024;   // sequences the split planner handles in one workgroup
hipError_t launch_value_passes(const Params& p, hipStream_t s, PhaseHook* hook);
int vside_column_split(int cap);
hipError_t launch_value_side(const Params& p, hipStream_t s, PhaseHook* hook);
hipError_t launch_select(const Params& p, hipStream_t s, PhaseHook* hook);
int joint_slice_len();
hipError_t launch_select_joint(const Params& p, int32_t* order, float* err, int max_evict, hipStream_t s,
                               PhaseHook* hook);
hipError_t launch_compact(const Params& p, hipStream_t s, PhaseHook* hook);
hipError_t launch_read_stream(const void* buf, size_t bytes, void* sink, hipStream_t s);
hipError_t launch_issue_probe(int variant, int iters, float* out, hipStream_t s);
hipError_t launch_append(const Params& p, const void* k_new, const void* v_new, int n_at, int n_new,
                         hipStream_t s);

}  // namespace caote
