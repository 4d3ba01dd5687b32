// Window attention over the key cache for few query rows (R = G*W <= 8): decode-time
// eviction (one query position, Sec. 2 "Generation" / Sec. 3.1) and other small windows.
//
// With so few rows the logits are cheaper to keep than to recompute: R floats per key
// against a 256-byte key row.  So K is swept ONCE: the kernel stores the scaled logits
// t_rj = c2 * q_r.k_j (masked ones as -inf) in the workspace and keeps the running
// (max, sum) of each row; after the merge the value sweep forms the attention mass of a
// key, a_j = sum_r exp2(t_rj - lse2_r), straight from the stored logits.  HBM-bound:
// 2 flop per byte, the vector ALUs are enough (a 32-row matrix-core tile would be padding).
//
// 16 (8) lanes share one 256-byte key row; each thread keeps 4 independent 16-byte loads in
// flight; the dot products are reduced inside the 16-lane DPP row (no LDS traffic).
#include "common.hpp"

namespace caote {
namespace {

constexpr int kThreads = 256;
constexpr int kKeysInFlight = 4;

template <typename T> struct KFrag;
template <> struct KFrag<bf16_t> { uint4 u; };
template <> struct KFrag<float> { float4 lo, hi; };
__device__ __forceinline__ void kfetch(const bf16_t* ptr, KFrag<bf16_t>& f) { f.u = *reinterpret_cast<const uint4*>(ptr); }
__device__ __forceinline__ void kfetch(const float* ptr, KFrag<float>& f) {
  f.lo = *reinterpret_cast<const float4*>(ptr);
  f.hi = *reinterpret_cast<const float4*>(ptr + 4);
}
__device__ __forceinline__ void kwiden(const KFrag<bf16_t>& f, float (&x)[8]) {
  x[0] = __uint_as_float(f.u.x << 16); x[1] = __uint_as_float(f.u.x & 0xffff0000u);
  x[2] = __uint_as_float(f.u.y << 16); x[3] = __uint_as_float(f.u.y & 0xffff0000u);
  x[4] = __uint_as_float(f.u.z << 16); x[5] = __uint_as_float(f.u.z & 0xffff0000u);
  x[6] = __uint_as_float(f.u.w << 16); x[7] = __uint_as_float(f.u.w & 0xffff0000u);
}
__device__ __forceinline__ void kwiden(const KFrag<float>& f, float (&x)[8]) {
  x[0] = f.lo.x; x[1] = f.lo.y; x[2] = f.lo.z; x[3] = f.lo.w;
  x[4] = f.hi.x; x[5] = f.hi.y; x[6] = f.hi.z; x[7] = f.hi.w;
}

template <typename T, int D, int RT>
__global__ __launch_bounds__(kThreads) void k_rowstats_small(const Params p) {
  constexpr int TL = D / 8;               // lanes that share one key row
  constexpr int KPI = kThreads / TL;      // teams = keys per step
  static_assert(RT <= TL, "one lane per query row inside a team");
  const int bh = blockIdx.y, b = bh / p.Hkv, hk = bh % p.Hkv;
  const int N = seq_len(p, b);
  const int c0 = blockIdx.x * p.split_len;
  if (c0 >= N) return;
  const int c1 = min(N, c0 + p.split_len);
  const int tid = threadIdx.x, team = tid / TL, tl = tid % TL;
  const int P = p.wic ? N - p.W : N;      // keys [0,P) are visible to every row
  const int myr = tl % RT;                // the row whose softmax this lane tracks

  __shared__ float red[KPI][RT][2];

  float qf[RT][8];
  int nvis_my = 0;                        // visible-key count of row myr
#pragma unroll
  for (int rr = 0; rr < RT; ++rr) {
#pragma unroll
    for (int e = 0; e < 8; ++e) qf[rr][e] = 0.f;
    if (rr < p.R) {
      int g, iw;
      divmod_w(p, rr, g, iw);
      load8(reinterpret_cast<const T*>(p.q) + (int64_t)b * p.qsb + (int64_t)(hk * p.G + g) * p.qsh +
                (int64_t)iw * p.qsw + tl * 8, qf[rr]);
      if (rr == myr) nvis_my = p.wic ? P + iw + 1 : N;
    }
  }
  const T* Kb = reinterpret_cast<const T*>(p.K) + (int64_t)b * p.ksb + (int64_t)hk * p.ksh + tl * 8;
  float* Sb = p.S + (int64_t)bh * RT * p.s_pitch;       // row r of the stored logits at Sb + r * s_pitch
  float m = -INFINITY, l = 0.f;

  for (int j0 = c0 + team; j0 < c1; j0 += KPI * kKeysInFlight) {
    KFrag<T> f[kKeysInFlight];
#pragma unroll
    for (int u = 0; u < kKeysInFlight; ++u) {
      const int j = min(j0 + u * KPI, c1 - 1);            // clamped: stays inside the chunk
      kfetch(Kb + (int64_t)j * p.ksn, f[u]);
    }
    float t[kKeysInFlight];               // this lane's row against the keys of the step
#pragma unroll
    for (int u = 0; u < kKeysInFlight; ++u) {
      const int j = j0 + u * KPI;
      float kf[8];
      kwiden(f[u], kf);
      float mine = 0.f;
#pragma unroll
      for (int rr = 0; rr < RT; ++rr) {
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) s = fmaf(qf[rr][e], kf[e], s);
        s = team_sum_dpp<TL>(s);
        mine = rr == myr ? s : mine;
      }
      const bool vis = j < c1 && j < nvis_my && myr < p.R;
      t[u] = vis ? mine * p.c2 : -INFINITY;
      if (j < c1 && tl < RT) Sb[(int64_t)tl * p.s_pitch + j] = t[u];   // lane tl holds row tl
    }
    // one rescale of the running sum per step, not per key
    float mx = t[0];
#pragma unroll
    for (int u = 1; u < kKeysInFlight; ++u) mx = fmaxf(mx, t[u]);
    const float mn = fmaxf(m, mx);
    if (mn > -INFINITY) {
      float s = 0.f;
#pragma unroll
      for (int u = 0; u < kKeysInFlight; ++u) s += __builtin_amdgcn_exp2f(t[u] - mn);   // exp2(-inf) = 0
      l = l * __builtin_amdgcn_exp2f(m - mn) + s;
      m = mn;
    }
  }
  if (tl < RT) { red[team][tl][0] = m; red[team][tl][1] = l; }
  __syncthreads();
  if (tid < p.R) {
    float M = -INFINITY;
    for (int t = 0; t < KPI; ++t) M = fmaxf(M, red[t][tid][0]);
    float L = 0.f;
    for (int t = 0; t < KPI; ++t)
      if (red[t][tid][0] > -INFINITY) L += red[t][tid][1] * exp2f(red[t][tid][0] - M);
    float* st = p.stats + (((int64_t)bh * p.n_split + blockIdx.x) * p.Rp + tid) * 2;
    st[0] = M; st[1] = L;
  }
}

template <typename T, int D>
hipError_t launch_t(const Params& p, hipStream_t s, PhaseHook* hook) {
  const dim3 grid(p.n_split, p.B * p.Hkv);
  if (p.s_rows == 4) hipLaunchKernelGGL((k_rowstats_small<T, D, 4>), grid, dim3(kThreads), 0, s, p);
  else               hipLaunchKernelGGL((k_rowstats_small<T, D, 8>), grid, dim3(kThreads), 0, s, p);
  if (mark(hook, "key_rowstats")) return hipGetLastError();
  if (p.lse_in) return hipGetLastError();   // the caller's normalisers: nothing to merge
  return launch_merge_stats(p, s, hook);
}

}  // namespace

// Requires R <= 8; p.s_rows (4 or 8) floats of logits are stored per key.
hipError_t launch_score_small(const Params& p, hipStream_t s, PhaseHook* hook) {
  if (p.dtype == CAOTE_F32) {
    return p.D == 64 ? launch_t<float, 64>(p, s, hook) : launch_t<float, 128>(p, s, hook);
  }
  return p.D == 64 ? launch_t<bf16_t, 64>(p, s, hook) : launch_t<bf16_t, 128>(p, s, hook);
}

}  // namespace caote
