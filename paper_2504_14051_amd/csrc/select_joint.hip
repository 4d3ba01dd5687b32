// Greedy multi-token eviction under the joint error (App. "Extending CAOTE to Multi-token
// Eviction").  The joint error of an evicted set S is
//     c_S = || sum_{i in S} w_i (o - v_i) ||_2 / (1 - sum_{i in S} w_i),
// with o the output before any eviction.  Choosing the best set is combinatorial, so tokens
// leave one at a time: each step evicts the scored token j whose c_{S+j} is smallest, then
// folds it into the running sums  u = sum_{i in S} w_i (o - v_i)  and  1 - sum_{i in S} w_i.
//
// The steps depend on each other, so one workgroup walks all steps of a (sequence, KV head)
// and never leaves the compute unit: weights live in LDS (a negative entry marks an evicted
// token), u and o in registers (each lane of a row team holds its 8 columns), value rows
// are re-read every step (they stay in L2).  One barrier per step: every wave posts its best
// candidate together with that candidate's w_j (o - v_j), so that after the barrier all
// lanes update u from LDS without another trip to memory.
#include <math.h>

#include "common.hpp"

namespace caote {
namespace {

constexpr int kJT = 1024;                 // threads per workgroup
constexpr int kJW = kJT / kWave;          // waves
constexpr int kJU = 4;                    // value rows requested per lane before any is used

struct Best { float q; int j; };
__device__ __forceinline__ bool better(float q, int j, const Best& b) {
  return q < b.q || (q == b.q && j > b.j);   // equal errors: the higher index leaves
}

template <typename T, int D>
__global__ __launch_bounds__(kJT) void k_select_joint(const Params p, int32_t* order_out, float* err_out,
                                                      int max_evict) {
  constexpr int TL = D / 8;               // lanes per value row, 8 columns each
  constexpr int NT = kJT / TL;            // row teams per workgroup
  const int bh = blockIdx.x, b = bh / p.Hkv, hk = bh % p.Hkv;
  const int N = seq_len(p, b);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, tl = tid % TL, team = tid / TL;
  const int lo = min(p.ph, N), hi = max(lo, N - p.pt);   // scored rows [lo,hi)
  const int n_keep = min(N, p.budget);
  const int m = min(N - n_keep, hi - lo);

  __shared__ float alpha[kJointMaxCap];             // w_j, or < 0 once evicted
  __shared__ float4 res[2][kJW];                    // per wave: (error^2, token, w_token, -)
  __shared__ __attribute__((aligned(16))) float resv[2][kJW][D];   // per wave: w_j (o - v_j) of its best
  __shared__ int wave_tot[kJW];

  const float* os = p.osum + (int64_t)bh * (kMaxD + 1);
  const float Z = os[kMaxD];
  const float invZ = Z > 0.f ? 1.f / Z : 0.f;
  float o[8], u[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { o[e] = os[tl * 8 + e] * invZ; u[e] = 0.f; }
  const float* hb = p.h + (int64_t)bh * p.cap;
  for (int j = lo + tid; j < hi; j += kJT) alpha[j] = hb[j] * invZ;
  __syncthreads();

  const T* Vb = reinterpret_cast<const T*>(p.V) + (int64_t)b * p.vsb + (int64_t)hk * p.vsh + tl * 8;
  int32_t* ord = order_out + (int64_t)bh * max_evict;
  float* er = err_out + (int64_t)bh * max_evict;
  double rest_all = 1.0;                  // 1 - sum of the evicted weights
  int done = 0;
  for (int t = 0; t < m; ++t) {
    const float rest_f = (float)rest_all;
    Best best = {INFINITY, -1};
    for (int j0 = lo + team; j0 < hi; j0 += kJU * NT) {
      float al[kJU], x[kJU][8];
#pragma unroll
      for (int k = 0; k < kJU; ++k) {
        const int j = j0 + k * NT;
        al[k] = j < hi ? alpha[j] : -1.f;
        if (al[k] >= 0.f) load8(Vb + (int64_t)j * p.vsn, x[k]);
        else {
#pragma unroll
          for (int e = 0; e < 8; ++e) x[k][e] = 0.f;
        }
      }
#pragma unroll
      for (int k = 0; k < kJU; ++k) {
        float n2 = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float y = fmaf(al[k], o[e] - x[k][e], u[e]);
          n2 = fmaf(y, y, n2);
        }
        n2 = team_sum<TL>(n2);
        const float rest = rest_f - al[k];
        const float r = __builtin_amdgcn_rcpf(rest);
        const float q = rest > 0.f ? n2 * r * r : INFINITY;
        // a lane meets its tokens in ascending order, so `<=` lets the higher index win a tie
        if (al[k] >= 0.f && q <= best.q) { best.q = q; best.j = j0 + k * NT; }
      }
    }
    // ---- the wave's best, then its w_j (o - v_j) into LDS ----
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      const float oq = __shfl_xor(best.q, off, kWave);
      const int oj = __shfl_xor(best.j, off, kWave);
      if (better(oq, oj, best)) { best.q = oq; best.j = oj; }
    }
    const int buf = t & 1;
    if (best.j >= 0) {
      const float a = alpha[best.j];
      if (lane == 0) res[buf][wave] = make_float4(best.q, __int_as_float(best.j), a, 0.f);
      if (lane < TL) {
        float x[8];
        load8(Vb + (int64_t)best.j * p.vsn, x);
        float4 d0, d1;
        d0.x = a * (o[0] - x[0]); d0.y = a * (o[1] - x[1]); d0.z = a * (o[2] - x[2]); d0.w = a * (o[3] - x[3]);
        d1.x = a * (o[4] - x[4]); d1.y = a * (o[5] - x[5]); d1.z = a * (o[6] - x[6]); d1.w = a * (o[7] - x[7]);
        *reinterpret_cast<float4*>(&resv[buf][wave][tl * 8]) = d0;
        *reinterpret_cast<float4*>(&resv[buf][wave][tl * 8 + 4]) = d1;
      }
    } else if (lane == 0) {
      res[buf][wave] = make_float4(INFINITY, __int_as_float(-1), 0.f, 0.f);
    }
    __syncthreads();
    // ---- every thread: the workgroup's best ----
    Best g = {INFINITY, -1};
    float ga = 0.f;
    int gw = 0;
#pragma unroll
    for (int w = 0; w < kJW; ++w) {
      const float4 r = res[buf][w];
      const int rj = __float_as_int(r.y);
      if (rj >= 0 && (g.j < 0 || better(r.x, rj, g))) { g.q = r.x; g.j = rj; ga = r.z; gw = w; }
    }
    if (g.j < 0) break;                   // nothing left to evict (same decision in every thread)
    const float4 d0 = *reinterpret_cast<const float4*>(&resv[buf][gw][tl * 8]);
    const float4 d1 = *reinterpret_cast<const float4*>(&resv[buf][gw][tl * 8 + 4]);
    u[0] += d0.x; u[1] += d0.y; u[2] += d0.z; u[3] += d0.w;
    u[4] += d1.x; u[5] += d1.y; u[6] += d1.z; u[7] += d1.w;
    rest_all -= (double)ga;
    // only the team that owns the token reads its weight again, and it is the one that clears it
    if ((g.j - lo) % NT == team && tl == 0) alpha[g.j] = -1.f;
    if (tid == 0) { ord[t] = g.j; er[t] = sqrtf(g.q); }
    done = t + 1;
  }
  for (int t = done + tid; t < max_evict; t += kJT) { ord[t] = -1; er[t] = NAN; }
  __syncthreads();

  // ---- the kept rows, ascending ----
  const int per = (p.cap + kJT - 1) / kJT;
  const int j_first = tid * per;
  int cnt = 0;
  for (int i = 0; i < per; ++i) {
    const int j = j_first + i;
    cnt += (j < N && (j < lo || j >= hi || alpha[j] >= 0.f)) ? 1 : 0;
  }
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
  for (int w = 0; w < kJW; ++w) {
    const int wt = wave_tot[w];
    pos += w < wave ? wt : 0;
    total += wt;
  }
  int32_t* kept = p.kept + (int64_t)bh * p.budget;
  for (int i = 0; i < per; ++i) {
    const int j = j_first + i;
    if (j < N && (j < lo || j >= hi || alpha[j] >= 0.f)) {
      if (pos < p.budget) kept[pos] = j;
      ++pos;
    }
  }
  for (int i = min(total, p.budget) + tid; i < p.budget; i += kJT) kept[i] = -1;
}

}  // namespace

hipError_t launch_select_joint(const Params& p, int32_t* order, float* err, int max_evict, hipStream_t s,
                               PhaseHook* hook) {
  const dim3 grid(p.B * p.Hkv), block(kJT);
  if (p.dtype == CAOTE_F32) {
    if (p.D == 64) hipLaunchKernelGGL((k_select_joint<float, 64>), grid, block, 0, s, p, order, err, max_evict);
    else hipLaunchKernelGGL((k_select_joint<float, 128>), grid, block, 0, s, p, order, err, max_evict);
  } else {
    if (p.D == 64) hipLaunchKernelGGL((k_select_joint<bf16_t, 64>), grid, block, 0, s, p, order, err, max_evict);
    else hipLaunchKernelGGL((k_select_joint<bf16_t, 128>), grid, block, 0, s, p, order, err, max_evict);
  }
  mark(hook, "select_joint");
  return hipGetLastError();
}

}  // namespace caote
