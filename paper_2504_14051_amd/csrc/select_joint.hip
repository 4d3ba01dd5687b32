// Greedy multi-token eviction under the joint error (App. "Extending CAOTE to Multi-token
// Eviction").  The joint error of an evicted set S is
//     c_S = || sum_{i in S} w_i (o - v_i) ||_2 / (1 - sum_{i in S} w_i),
// with o the output before any eviction.  Choosing the best set is combinatorial, so tokens
// leave one at a time: each step evicts the scored token j whose c_{S+j} is smallest, then
// folds it into the running sums  u = sum_{i in S} w_i (o - v_i)  and  1 - sum_{i in S} w_i.
//
// A step needs every value row of the head once and then one decision for the whole head.
// One compute unit is far too slow for a head (16 us per step at 2176 rows, measured: its
// vector units are busy all that time), so a head is cut into slices of 128 tokens, one
// workgroup each, and the decision
// crosses workgroups at a kernel boundary: ONE LAUNCH PER STEP, stream order is the only
// synchronisation.  Kernel t
//   1. (t > 0) reduces the slices' best candidates of step t-1 to the head's winner, adds
//      the winner's w_j (o - v_j), which its slice posted beside the candidate, to u, and
//      marks the winner evicted (the slice that owns it);
//   2. evaluates c_{S+j} for the tokens of its slice and posts the slice's best.
// Every workgroup of a head repeats step 1 (a few hundred bytes); buffers that one kernel
// writes and the next reads are double-buffered by step parity.  A last kernel applies the
// final winner and writes the kept rows in ascending order.
#include <math.h>

#include "common.hpp"

namespace caote {
namespace {

constexpr int kJT = 256;                  // threads per workgroup of a step
constexpr int kJW = kJT / kWave;
constexpr int kJPass = 8;                 // value rows per lane: slices hold at most kJPass * teams tokens
constexpr int kJSlice = 128;              // tokens per slice: few slices, so that a step reads few records
constexpr int kJMaxC = kJointMaxCap / kJSlice;   // slices per head at most
constexpr int kJPre = kJMaxC * (kMaxD / 4) / kJT;   // 16-byte pieces of the posted vectors per thread
static_assert(kJSlice <= kJPass * (kJT / (kMaxD / 8)), "a slice fits the lanes' row registers");
static_assert(kJMaxC <= kWave, "a wave reads all records of a head, one per lane");
constexpr int kET = 1024;                 // threads of the closing kernel
constexpr int kEW = kET / kWave;

struct Best { float q; int j; float w; };   // joint error^2, token (< 0: none), the token's weight
__device__ __forceinline__ bool better(const Best& a, const Best& b) {   // a ahead of b?
  if (a.j < 0) return false;
  return b.j < 0 || a.q < b.q || (a.q == b.q && a.j > b.j);   // equal errors: the higher index leaves
}

// The candidate of another lane of the same 16-lane row, chosen by a DPP control word.
template <int CTRL>
__device__ __forceinline__ void dpp_best(Best& v) {
  Best o;
  o.q = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v.q), CTRL, 0xf, 0xf, false));
  o.j = __builtin_amdgcn_update_dpp(0, v.j, CTRL, 0xf, 0xf, false);
  o.w = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v.w), CTRL, 0xf, 0xf, false));
  if (better(o, v)) v = o;
}
__device__ __forceinline__ Best lane_best(const Best& v, int lane) {
  Best o;
  o.q = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v.q), lane));
  o.j = __builtin_amdgcn_readlane(v.j, lane);
  o.w = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v.w), lane));
  return o;
}
// Best of the wave's 64 candidates (every token at most once), the same in every lane: the
// rows fold as in team_sum_dpp, then the four rows' results are read out lane by lane.
// No LDS traffic, no waiting.
__device__ __forceinline__ Best wave_best(Best v) {
  dpp_best<0x140>(v);                     // row_mirror
  dpp_best<0x141>(v);                     // row_half_mirror
  dpp_best<0xB1>(v);                      // quad_perm [1,0,3,2]
  dpp_best<0x4E>(v);                      // quad_perm [2,3,0,1]
  Best r = lane_best(v, 0);
#pragma unroll
  for (int row = 1; row < 4; ++row) {
    const Best o = lane_best(v, row * 16);
    if (better(o, r)) r = o;
  }
  return r;
}

struct Geometry { int N, lo, hi, m; };
__device__ __forceinline__ Geometry geometry(const Params& p, int b) {
  Geometry g;
  g.N = seq_len(p, b);
  g.lo = min(p.ph, g.N);
  g.hi = max(g.lo, g.N - p.pt);           // scored rows [lo,hi)
  g.m = min(g.N - min(g.N, p.budget), g.hi - g.lo);
  return g;
}

// Record a slice posts per step: (error^2, token, w_token, -) then w_token (o - v_token).
__device__ __forceinline__ float* record(const Params& p, int parity, int bh, int wg) {
  return p.j_part + (((int64_t)parity * p.B * p.Hkv + bh) * p.j_c + wg) * (4 + kMaxD);
}

// The head's winner of a step from the slices' records (at most 64 of them: one per lane, so
// every wave finds the winner by itself).  j < 0: no candidate was left.
__device__ __forceinline__ Best head_winner(const Params& p, int parity, int bh) {
  const int lane = threadIdx.x & 63;
  Best v = {INFINITY, -1, 0.f};
  const float4 r = *reinterpret_cast<const float4*>(record(p, parity, bh, min(lane, p.j_c - 1)));
  if (lane < p.j_c) { v.q = r.x; v.j = __float_as_int(r.y); v.w = r.z; }
  return wave_best(v);
}

template <typename T, int D>
__global__ __launch_bounds__(kJT) void k_joint_step(const Params p, int32_t* order_out, float* err_out,
                                                    int max_evict, int t) {
  constexpr int TL = D / 8;               // lanes per value row, 8 columns each
  constexpr int NT = kJT / TL;            // row teams per workgroup
  constexpr int F4 = kMaxD / 4;           // 16-byte pieces of a posted vector
  const int bh = blockIdx.y, wg = blockIdx.x, b = bh / p.Hkv, hk = bh % p.Hkv;
  const Geometry g = geometry(p, b);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, tl = tid % TL, team = tid / TL;
  int32_t* ord = order_out + (int64_t)bh * max_evict;
  float* er = err_out + (int64_t)bh * max_evict;
  if (t == 0 && wg == 0)
    for (int i = g.m + tid; i < max_evict; i += kJT) { ord[i] = -1; er[i] = NAN; }
  if (t >= g.m) return;                   // this head has evicted all it has to
  const int s0 = g.lo + wg * p.j_slice, s1 = min(g.hi, s0 + p.j_slice);

  __shared__ float4 sh[kJW];
  __shared__ float4 dl[kJMaxC * F4];      // the vectors every slice posted at step t-1

  // ---- everything the step reads is requested up front, in one round trip: the winner of
  // step t-1 is only known once the records are here, and its posted vector must not cost a
  // second trip, so all posted vectors come along (a few KB) ----
  const int par = t & 1;
  const int64_t head2 = (int64_t)par * p.B * p.Hkv + bh, head2p = (int64_t)(par ^ 1) * p.B * p.Hkv + bh;
  float4 pre[kJPre];
  float u[8];
  double rest_all = 1.0;                  // 1 - sum of the evicted weights
  Best win = {INFINITY, -1, 0.f};
  if (t > 0) {
#pragma unroll
    for (int i = 0; i < kJPre; ++i) {
      // a workgroup-uniform bound, and inside it a clamped index instead of a lane-dependent
      // condition: loads under one are waited for one by one
      if (i * kJT < p.j_c * F4) {
        const int idx = min(tid + i * kJT, p.j_c * F4 - 1);
        pre[i] = *reinterpret_cast<const float4*>(record(p, par ^ 1, bh, idx / F4) + 4 + (idx % F4) * 4);
      }
    }
    load8(p.j_u + head2p * kMaxD + tl * 8, u);
    rest_all = p.j_rest[head2p];
    win = head_winner(p, par ^ 1, bh);    // (its loads are requested here, used below)
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) u[e] = 0.f;
  }
  const T* Vb = reinterpret_cast<const T*>(p.V) + (int64_t)b * p.vsb + (int64_t)hk * p.vsh + tl * 8;
  float* alpha = reinterpret_cast<float*>(p.sel_cand) + (int64_t)bh * p.cap;
  const float* os = p.osum + (int64_t)bh * (kMaxD + 1);
  const float* wsrc = t == 0 ? p.h + (int64_t)bh * p.cap : alpha;
  // (every pass loads: a pass beyond the slice re-reads a scored row and is marked gone; loads
  // under a lane-dependent condition would be waited for one by one)
  float x[kJPass][8], al[kJPass], o[8];
#pragma unroll
  for (int k = 0; k < kJPass; ++k) {
    const int j = s0 + team + k * NT;
    const int jj = j < s1 ? j : g.lo;
    load8(Vb + (int64_t)jj * p.vsn, x[k]);
    al[k] = wsrc[jj];
  }
#pragma unroll
  for (int k = 0; k < kJPass; ++k)
    if (s0 + team + k * NT >= s1) al[k] = -1.f;
  load8(os + tl * 8, o);
  const float Z = os[kMaxD];
  const float invZ = Z > 0.f ? 1.f / Z : 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] *= invZ;

  // ---- the previous step's winner ----
  if (t > 0) {
#pragma unroll
    for (int i = 0; i < kJPre; ++i) {
      const int idx = tid + i * kJT;
      if (idx < p.j_c * F4) dl[idx] = pre[i];
    }
    __syncthreads();
    // (win.j >= 0: step t-1 ran with t-1 < m <= number of scored tokens, so a candidate existed)
    const int slice_of = win.j >= 0 ? (win.j - g.lo) / p.j_slice : 0;
    const float4 d0 = dl[slice_of * F4 + tl * 2], d1 = dl[slice_of * F4 + tl * 2 + 1];
    u[0] += d0.x; u[1] += d0.y; u[2] += d0.z; u[3] += d0.w;
    u[4] += d1.x; u[5] += d1.y; u[6] += d1.z; u[7] += d1.w;
    rest_all -= (double)win.w;
    if (wg == 0 && tid == 0) { ord[t - 1] = win.j; er[t - 1] = sqrtf(win.q); }
#pragma unroll
    for (int k = 0; k < kJPass; ++k)
      if (s0 + team + k * NT == win.j) {
        al[k] = -1.f;
        if (tl == 0) alpha[win.j] = -1.f;
      }
  } else {
#pragma unroll
    for (int k = 0; k < kJPass; ++k) {
      const int j = s0 + team + k * NT;
      if (j < s1) {
        al[k] *= invZ;
        if (tl == 0) alpha[j] = al[k];
      }
    }
  }
  if (wg == 0) {
    if (tid < TL) {
      float* un = p.j_u + head2 * kMaxD + tl * 8;
      *reinterpret_cast<float4*>(un) = make_float4(u[0], u[1], u[2], u[3]);
      *reinterpret_cast<float4*>(un + 4) = make_float4(u[4], u[5], u[6], u[7]);
    }
    if (tid == 0) p.j_rest[head2] = rest_all;
  }

  // ---- c_{S+j} for the slice ----
  const float rest_f = (float)rest_all;
  Best best = {INFINITY, -1, 0.f};
  float bx[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) bx[e] = 0.f;
#pragma unroll
  for (int k = 0; k < kJPass; ++k) {
    float n2 = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float y = fmaf(al[k], o[e] - x[k][e], u[e]);
      n2 = fmaf(y, y, n2);
    }
    n2 = team_sum_dpp<TL>(n2);
    const float rest = rest_f - al[k];
    const float r = __builtin_amdgcn_rcpf(rest);
    const float q = rest > 0.f ? n2 * r * r : INFINITY;
    // a lane meets its tokens in ascending order, so `<=` lets the higher index win a tie
    if (al[k] >= 0.f && q <= best.q) {
      best.q = q; best.j = s0 + team + k * NT; best.w = al[k];
#pragma unroll
      for (int e = 0; e < 8; ++e) bx[e] = x[k][e];
    }
  }
  // the lanes of a team hold the same candidate: one lane per team enters the wave's contest
  const Best mine = best;
  Best cand = best;
  if (tl != 0) cand.j = -1;
  const Best wb = wave_best(cand);
  if (lane == 0) sh[wave] = make_float4(wb.q, __int_as_float(wb.j), wb.w, 0.f);
  __syncthreads();
  Best sl = {INFINITY, -1, 0.f};
#pragma unroll
  for (int w = 0; w < kJW; ++w) {
    const float4 r = sh[w];
    const Best c = {r.x, __float_as_int(r.y), r.z};
    if (better(c, sl)) sl = c;
  }
  float* rec = record(p, par, bh, wg);
  if (sl.j < 0) {
    if (tid == 0) *reinterpret_cast<float4*>(rec) = make_float4(INFINITY, __int_as_float(-1), 0.f, 0.f);
    return;
  }
  if (mine.j == sl.j) {                   // the team that evaluated the slice's best
    const float ba = mine.w;
    if (tl == 0) *reinterpret_cast<float4*>(rec) = make_float4(sl.q, __int_as_float(sl.j), ba, 0.f);
    float4 d0, d1;
    d0.x = ba * (o[0] - bx[0]); d0.y = ba * (o[1] - bx[1]); d0.z = ba * (o[2] - bx[2]); d0.w = ba * (o[3] - bx[3]);
    d1.x = ba * (o[4] - bx[4]); d1.y = ba * (o[5] - bx[5]); d1.z = ba * (o[6] - bx[6]); d1.w = ba * (o[7] - bx[7]);
    *reinterpret_cast<float4*>(rec + 4 + tl * 8) = d0;
    *reinterpret_cast<float4*>(rec + 4 + tl * 8 + 4) = d1;
  }
}

// Applies the winner of the last step and writes the kept rows of the head, ascending.
__global__ __launch_bounds__(kET) void k_joint_emit(const Params p, int32_t* order_out, float* err_out,
                                                    int max_evict) {
  const int bh = blockIdx.x, b = bh / p.Hkv;
  const Geometry g = geometry(p, b);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  __shared__ int wave_tot[kEW];
  const float* alpha = reinterpret_cast<const float*>(p.sel_cand) + (int64_t)bh * p.cap;
  int last = -1;
  if (g.m > 0) {
    const Best win = head_winner(p, (g.m - 1) & 1, bh);
    last = win.j;
    if (tid == 0) {
      order_out[(int64_t)bh * max_evict + g.m - 1] = win.j;
      err_out[(int64_t)bh * max_evict + g.m - 1] = sqrtf(win.q);
    }
  } else if (max_evict > 0) {             // no step kernel ran for this head: nothing evicted
    for (int i = tid; i < max_evict; i += kET) {
      order_out[(int64_t)bh * max_evict + i] = -1;
      err_out[(int64_t)bh * max_evict + i] = NAN;
    }
  }
  auto is_kept = [&](int j) {
    if (j >= g.N) return false;
    if (j < g.lo || j >= g.hi || g.m == 0) return true;   // (m == 0: alpha was never written)
    return j != last && alpha[j] >= 0.f;
  };
  const int per = (p.cap + kET - 1) / kET;
  const int j_first = tid * per;
  int cnt = 0;
  for (int i = 0; i < per; ++i) cnt += is_kept(j_first + i) ? 1 : 0;
  int inc = cnt;
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const int up = __shfl_up(inc, off, kWave);
    if (lane >= off) inc += up;
  }
  if (lane == kWave - 1) wave_tot[wave] = inc;
  __syncthreads();
  int pos = inc - cnt, total = 0;
#pragma unroll
  for (int w = 0; w < kEW; ++w) {
    const int wt = wave_tot[w];
    pos += w < wave ? wt : 0;
    total += wt;
  }
  int32_t* kept = p.kept + (int64_t)bh * p.budget;
  for (int i = 0; i < per; ++i) {
    const int j = j_first + i;
    if (is_kept(j)) {
      if (pos < p.budget) kept[pos] = j;
      ++pos;
    }
  }
  for (int i = min(total, p.budget) + tid; i < p.budget; i += kET) kept[i] = -1;
}

template <typename T, int D>
hipError_t launch_t(const Params& p, int32_t* order, float* err, int max_evict, hipStream_t s, PhaseHook* hook) {
  const dim3 grid(p.j_c, p.B * p.Hkv);
  for (int t = 0; t < max_evict; ++t)
    hipLaunchKernelGGL((k_joint_step<T, D>), grid, dim3(kJT), 0, s, p, order, err, max_evict, t);
  if (max_evict > 0 && mark(hook, "select_joint_steps")) return hipGetLastError();
  hipLaunchKernelGGL(k_joint_emit, dim3(p.B * p.Hkv), dim3(kET), 0, s, p, order, err, max_evict);
  if (mark(hook, "select_joint_emit")) return hipGetLastError();
  return hipGetLastError();
}

}  // namespace

int joint_slice_len() { return kJSlice; }

hipError_t launch_select_joint(const Params& p, int32_t* order, float* err, int max_evict, hipStream_t s,
                               PhaseHook* hook) {
  if (p.dtype == CAOTE_F32)
    return p.D == 64 ? launch_t<float, 64>(p, order, err, max_evict, s, hook)
                     : launch_t<float, 128>(p, order, err, max_evict, s, hook);
  return p.D == 64 ? launch_t<bf16_t, 64>(p, order, err, max_evict, s, hook)
                   : launch_t<bf16_t, 128>(p, order, err, max_evict, s, hook);
}

}  // namespace caote
