// Window attention over the key cache on the vector ALUs: any dtype, any number of
// query rows.  This is the path for fp32 caches and for small R = G*W (decode: one
// query position), where a 32-row matrix-core tile would be mostly padding.
//
// Two sweeps over K (Sec. 2, attention of the window queries over the cache):
//   1. per query row r: running (max, sum) of exp2(c2 * q_r.k_j)       -> stats
//      merged over the key splits into lse2_r = log2 sum_j exp2(.)      -> lse2
//   2. per key j: a_j = sum_r exp2(c2 * q_r.k_j - lse2_r)              -> a
// The second sweep needs every row's final normaliser, hence two sweeps; the
// attention matrix itself is never stored.
#include "common.hpp"

namespace caote {
namespace {

constexpr int kThreads = 256;
constexpr int kRT = 8;          // query rows handled together

// mode 0: row statistics, mode 1: column sums.
template <typename T, int D, int MODE>
__global__ __launch_bounds__(kThreads) void k_logits_generic(const Params p) {
  constexpr int TL = D / 8;               // lanes that share one key row
  constexpr int KPI = kThreads / TL;      // keys in flight per iteration
  const int bh = blockIdx.y, b = bh / p.Hkv, hk = bh % p.Hkv;
  const int N = seq_len(p, b);
  const int c0 = blockIdx.x * p.split_len;
  if (c0 >= N) return;
  const int c1 = min(N, c0 + p.split_len);
  const int team = threadIdx.x / TL, tl = threadIdx.x % TL;
  const int P = p.wic ? N - p.W : N;      // keys [0,P) are visible to every row

  __shared__ float red[KPI][kRT][2];
  extern __shared__ float a_lds[];        // MODE 1: [split_len]

  if (MODE == 1) {
    for (int i = threadIdx.x; i < p.split_len; i += kThreads) a_lds[i] = 0.f;
    __syncthreads();
  }
  const T* Kb = reinterpret_cast<const T*>(p.K) + (int64_t)b * p.ksb + (int64_t)hk * p.ksh + tl * 8;
  const T* Qb = reinterpret_cast<const T*>(p.q) + (int64_t)b * p.qsb + tl * 8;

  for (int r0 = 0; r0 < p.R; r0 += kRT) {
    float qf[kRT][8];
    int nvis[kRT];
    float lse[kRT], m[kRT], l[kRT];
#pragma unroll
    for (int rr = 0; rr < kRT; ++rr) {
      const int r = r0 + rr;
      m[rr] = -INFINITY; l[rr] = 0.f; lse[rr] = INFINITY; nvis[rr] = 0;
#pragma unroll
      for (int e = 0; e < 8; ++e) qf[rr][e] = 0.f;
      if (r < p.R) {
        const int g = r / p.W, i = r % p.W;
        load8(Qb + (int64_t)(hk * p.G + g) * p.qsh + (int64_t)i * p.qsw, qf[rr]);
        nvis[rr] = p.wic ? P + i + 1 : N;
        if (MODE == 1) lse[rr] = row_lse2(p, b, hk, bh, r);
      }
    }
    for (int j = c0 + team; j < c1; j += KPI) {
      float kf[8];
      load8(Kb + (int64_t)j * p.ksn, kf);
      float acc = 0.f;
#pragma unroll
      for (int rr = 0; rr < kRT; ++rr) {
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) s = fmaf(qf[rr][e], kf[e], s);
        s = team_sum<TL>(s);
        const float t = s * p.c2;
        const bool vis = j < nvis[rr];
        if (MODE == 0) {
          if (vis) {
            const float mn = fmaxf(m[rr], t);
            l[rr] = l[rr] * exp2f(m[rr] - mn) + exp2f(t - mn);
            m[rr] = mn;
          }
        } else {
          acc += vis ? exp2f(t - lse[rr]) : 0.f;
        }
      }
      if (MODE == 1 && tl == 0) a_lds[j - c0] += acc;   // one team owns key j
    }
    if (MODE == 0) {
      if (tl == 0) {
#pragma unroll
        for (int rr = 0; rr < kRT; ++rr) { red[team][rr][0] = m[rr]; red[team][rr][1] = l[rr]; }
      }
      __syncthreads();
      if (threadIdx.x < kRT && r0 + threadIdx.x < p.R) {
        const int rr = threadIdx.x;
        float M = -INFINITY;
        for (int t = 0; t < KPI; ++t) M = fmaxf(M, red[t][rr][0]);
        float L = 0.f;
        for (int t = 0; t < KPI; ++t)
          if (red[t][rr][0] > -INFINITY) L += red[t][rr][1] * exp2f(red[t][rr][0] - M);
        float* st = p.stats + (((int64_t)bh * p.n_split + blockIdx.x) * p.Rp + r0 + rr) * 2;
        st[0] = M; st[1] = L;
      }
      __syncthreads();
    }
  }
  if (MODE == 1) {
    __syncthreads();
    float* a = p.a + (int64_t)bh * p.cap;
    for (int i = threadIdx.x; i < c1 - c0; i += kThreads) a[c0 + i] = a_lds[i];
  }
}

// lse2_r = log2 sum_j exp2(t_rj), merged over the key splits that hold tokens.
__global__ void k_merge_stats(const Params p) {
  const int bh = blockIdx.y, b = bh / p.Hkv;
  if (blockIdx.x == 0) reset_counters(p, bh);
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= p.R) return;
  const int N = seq_len(p, b);
  const int ns = (N + p.split_len - 1) / p.split_len;
  const float* st = p.stats + ((int64_t)bh * p.n_split * p.Rp + r) * 2;
  float M = -INFINITY;
  for (int s = 0; s < ns; ++s) M = fmaxf(M, st[(int64_t)s * p.Rp * 2]);
  float L = 0.f;
  for (int s = 0; s < ns; ++s) {
    const float ms = st[(int64_t)s * p.Rp * 2];
    if (ms > -INFINITY) L += st[(int64_t)s * p.Rp * 2 + 1] * exp2f(ms - M);
  }
  // a row that sees no key contributes nothing: exp2(t - inf) = 0
  p.lse2[(int64_t)bh * p.Rp + r] = L > 0.f ? M + log2f(L) : INFINITY;
}

template <typename T, int D>
hipError_t launch_t(const Params& p, hipStream_t s, PhaseHook* hook) {
  const dim3 grid(p.n_split, p.B * p.Hkv);
  if (!p.lse_in) {                       // else the caller's attention pass has done sweep 1
    hipLaunchKernelGGL((k_logits_generic<T, D, 0>), grid, dim3(kThreads), 0, s, p);
    if (mark(hook, "key_rowstats")) return hipGetLastError();
    hipLaunchKernelGGL(k_merge_stats, dim3((p.R + 63) / 64, p.B * p.Hkv), dim3(64), 0, s, p);
    if (mark(hook, "merge_stats")) return hipGetLastError();
  }
  hipLaunchKernelGGL((k_logits_generic<T, D, 1>), grid, dim3(kThreads),
                     (size_t)p.split_len * sizeof(float), s, p);
  if (mark(hook, "key_colsum")) return hipGetLastError();
  return hipGetLastError();
}

}  // namespace

hipError_t launch_score_generic(const Params& p, hipStream_t s, PhaseHook* hook) {
  if (p.dtype == CAOTE_F32) {
    return p.D == 64 ? launch_t<float, 64>(p, s, hook) : launch_t<float, 128>(p, s, hook);
  }
  return p.D == 64 ? launch_t<bf16_t, 64>(p, s, hook) : launch_t<bf16_t, 128>(p, s, hook);
}

}  // namespace caote
