// Value-side sweeps of the CAOTE score (Sec. 3.2 general form, Sec. 3.3 FastCAOTE).
//
//   k_vsum   : base score h from the column sums a (H2O accumulate / SnapKV max-pool),
//              then partial sums  sum_j h_j v_j  and  sum_j h_j  per chunk of tokens.
//   k_vscore : o = (sum h_j v_j) / Z,  score_j = h_j / (Z - h_j) * ||v_j - o||_2.
//
// ||v_j - o|| is taken directly on the differences (not via ||v||^2 - 2 v.o + ||o||^2,
// which cancels when v_j is close to o).  1 - w_j is formed as (Z - h_j) / Z.
#include <float.h>

#include "common.hpp"

namespace caote {
namespace {

constexpr int kThreads = 256;

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void k_vsum(const Params p) {
  constexpr int TL = D / 8;
  constexpr int RPI = kThreads / TL;      // rows in flight per iteration
  const int bh = blockIdx.y, b = bh / p.Hkv, hk = bh % p.Hkv;
  const int N = seq_len(p, b);
  const int c0 = blockIdx.x * p.vchunk_len;
  if (c0 >= N) return;
  const int c1 = min(N, c0 + p.vchunk_len);
  const int team = threadIdx.x / TL, tl = threadIdx.x % TL;
  const int lo = min(p.ph, N), hi = max(lo, N - p.pt);   // scored rows [lo,hi)
  const int half = p.pool / 2;

  const float* a = p.a + (int64_t)bh * p.cap;
  float* h = p.h + (int64_t)bh * p.cap;
  const T* Vb = reinterpret_cast<const T*>(p.V) + (int64_t)b * p.vsb + (int64_t)hk * p.vsh + tl * 8;

  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  float zacc = 0.f;
  for (int j = c0 + team; j < c1; j += RPI) {
    const bool scored = j >= lo && j < hi;
    float hj = a[j];
    if (p.base_mode == CAOTE_BASE_H2O) {
      hj += h[j];                           // h aliases the accumulator
    } else if (p.base_mode == CAOTE_BASE_SNAPKV && scored) {
      const int t0 = max(lo, j - half), t1 = min(hi - 1, j + half);
      for (int t = t0; t <= t1; ++t) hj = fmaxf(hj, a[t]);
    }
    if (tl == 0) h[j] = hj;
    if (scored) {
      float vf[8];
      load8(Vb + (int64_t)j * p.vsn, vf);
      const float wgt = p.variant == CAOTE_FAST ? 1.f : hj;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = fmaf(wgt, vf[e], acc[e]);
      zacc += hj;
    }
  }
  __shared__ float red[RPI][D + 1];
#pragma unroll
  for (int e = 0; e < 8; ++e) red[team][tl * 8 + e] = acc[e];
  if (tl == 0) red[team][D] = zacc;
  __syncthreads();
  if (threadIdx.x <= D) {
    float s = 0.f;
    for (int t = 0; t < RPI; ++t) s += red[t][threadIdx.x];
    if (threadIdx.x < D) p.opart[((int64_t)bh * p.n_vchunk + blockIdx.x) * D + threadIdx.x] = s;
    else p.zpart[(int64_t)bh * p.n_vchunk + blockIdx.x] = s;
  }
}

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void k_vscore(const Params p) {
  constexpr int TL = D / 8;
  constexpr int RPI = kThreads / TL;
  const int bh = blockIdx.y, b = bh / p.Hkv, hk = bh % p.Hkv;
  const int N = seq_len(p, b);
  const int c0 = blockIdx.x * p.vchunk_len;
  if (c0 >= N) return;
  const int c1 = min(N, c0 + p.vchunk_len);
  const int team = threadIdx.x / TL, tl = threadIdx.x % TL;
  const int lo = min(p.ph, N), hi = max(lo, N - p.pt);
  const int n_scored = hi - lo;
  const int nch = (N + p.vchunk_len - 1) / p.vchunk_len;

  __shared__ float o_lds[D];
  __shared__ float z_lds;
  if (threadIdx.x <= D) {
    float s = 0.f;
    if (threadIdx.x < D) {
      const float* op = p.opart + (int64_t)bh * p.n_vchunk * D + threadIdx.x;
      for (int cidx = 0; cidx < nch; ++cidx) s += op[(int64_t)cidx * D];
      o_lds[threadIdx.x] = s;
    } else {
      const float* zp = p.zpart + (int64_t)bh * p.n_vchunk;
      for (int cidx = 0; cidx < nch; ++cidx) s += zp[cidx];
      z_lds = s;
    }
  }
  __syncthreads();
  const float Z = z_lds;
  const float onorm = p.variant == CAOTE_FAST ? 1.f / (float)max(n_scored, 1)
                                              : (Z > 0.f ? 1.f / Z : 0.f);
  float of[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) of[e] = o_lds[tl * 8 + e] * onorm;

  const float* h = p.h + (int64_t)bh * p.cap;
  float* sc = p.scores + (int64_t)bh * p.cap;
  const T* Vb = reinterpret_cast<const T*>(p.V) + (int64_t)b * p.vsb + (int64_t)hk * p.vsh + tl * 8;
  for (int j = c0 + team; j < c1; j += RPI) {
    const bool scored = j >= lo && j < hi && n_scored > 1;
    float out = INFINITY;
    if (scored) {                           // uniform within the team
      float vf[8];
      load8(Vb + (int64_t)j * p.vsn, vf);
      float d2 = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) { const float t = vf[e] - of[e]; d2 = fmaf(t, t, d2); }
      d2 = team_sum<TL>(d2);
      const float hj = h[j];
      out = Z > 0.f ? hj / fmaxf(Z - hj, FLT_MIN) * sqrtf(d2) : 0.f;
    }
    if (tl == 0) sc[j] = out;
  }
}

template <typename T, int D>
hipError_t launch_t(const Params& p, hipStream_t s, PhaseHook* hook) {
  const dim3 grid(p.n_vchunk, p.B * p.Hkv);
  hipLaunchKernelGGL((k_vsum<T, D>), grid, dim3(kThreads), 0, s, p);
  mark(hook, "value_sum");
  hipLaunchKernelGGL((k_vscore<T, D>), grid, dim3(kThreads), 0, s, p);
  mark(hook, "value_score");
  return hipGetLastError();
}

}  // namespace

hipError_t launch_value_passes(const Params& p, hipStream_t s, PhaseHook* hook) {
  if (p.dtype == CAOTE_F32) {
    return p.D == 64 ? launch_t<float, 64>(p, s, hook) : launch_t<float, 128>(p, s, hook);
  }
  return p.D == 64 ? launch_t<bf16_t, 64>(p, s, hook) : launch_t<bf16_t, 128>(p, s, hook);
}

}  // namespace caote
