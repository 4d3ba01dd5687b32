// Value-side sweeps of the CAOTE score (Sec. 3.2 general form, Sec. 3.3 FastCAOTE).
//
//   k_vsum   : base score h from the attention mass a (H2O accumulate / SnapKV max-pool),
//              then partial sums  sum_j h_j v_j  and  sum_j h_j  per workgroup (one or more
//              chunks of 256 tokens).  On the few-row path a_j comes straight from the
//              stored logits: a_j = sum_r exp2(t_rj - lse2_r).
//   k_vfinal : adds the partials of a head up in chunk order (fixed order: the result
//              does not depend on scheduling).
//   k_vscore : o = (sum h_j v_j) / Z,  score_j = h_j / (Z - h_j) * ||v_j - o||_2.
//
// ||v_j - o|| is taken directly on the differences (not via ||v||^2 - 2 v.o + ||o||^2,
// which cancels when v_j is close to o).  1 - w_j is formed as (Z - h_j) / Z.
// Both sweeps are HBM-bound streams over V: every thread keeps 8 independent 16-byte
// loads in flight, 16 lanes per 256-byte row.
#include <float.h>

#include "common.hpp"

namespace caote {
namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 8;
constexpr int kFinalThreads = 1024;

template <typename T> struct Frag;
template <> struct Frag<bf16_t> { uint4 u; };
template <> struct Frag<float> { float4 lo, hi; };

__device__ __forceinline__ void fetch(const bf16_t* ptr, Frag<bf16_t>& f) { f.u = *reinterpret_cast<const uint4*>(ptr); }
__device__ __forceinline__ void fetch(const float* ptr, Frag<float>& f) {
  f.lo = *reinterpret_cast<const float4*>(ptr);
  f.hi = *reinterpret_cast<const float4*>(ptr + 4);
}
__device__ __forceinline__ void zero(Frag<bf16_t>& f) { f.u = make_uint4(0, 0, 0, 0); }
__device__ __forceinline__ void zero(Frag<float>& f) { f.lo = make_float4(0, 0, 0, 0); f.hi = f.lo; }
__device__ __forceinline__ void widen(const Frag<bf16_t>& f, float (&x)[8]) {
  x[0] = __uint_as_float(f.u.x << 16); x[1] = __uint_as_float(f.u.x & 0xffff0000u);
  x[2] = __uint_as_float(f.u.y << 16); x[3] = __uint_as_float(f.u.y & 0xffff0000u);
  x[4] = __uint_as_float(f.u.z << 16); x[5] = __uint_as_float(f.u.z & 0xffff0000u);
  x[6] = __uint_as_float(f.u.w << 16); x[7] = __uint_as_float(f.u.w & 0xffff0000u);
}
__device__ __forceinline__ void widen(const Frag<float>& f, float (&x)[8]) {
  x[0] = f.lo.x; x[1] = f.lo.y; x[2] = f.lo.z; x[3] = f.lo.w;
  x[4] = f.hi.x; x[5] = f.hi.y; x[6] = f.hi.z; x[7] = f.hi.w;
}

// Attention mass of token j (Sec. 2, f_score,j = sum_i A_ij): from the column sums of
// the second key sweep, or, on the few-row path, from the stored logits.
__device__ __forceinline__ float mass_of(const Params& p, int bh, int j, const float (&lse)[8]) {
  if (!p.small_r) return p.a[(int64_t)bh * p.cap + j];
  const float* t = p.S + (int64_t)bh * p.s_rows * p.s_pitch + j;      // row r of S at t + r * s_pitch
  const int64_t sp = p.s_pitch;
  float a = (__builtin_amdgcn_exp2f(t[0] - lse[0]) + __builtin_amdgcn_exp2f(t[sp] - lse[1])) +
            (__builtin_amdgcn_exp2f(t[2 * sp] - lse[2]) + __builtin_amdgcn_exp2f(t[3 * sp] - lse[3]));
  if (p.s_rows == 8)
    a += (__builtin_amdgcn_exp2f(t[4 * sp] - lse[4]) + __builtin_amdgcn_exp2f(t[5 * sp] - lse[5])) +
         (__builtin_amdgcn_exp2f(t[6 * sp] - lse[6]) + __builtin_amdgcn_exp2f(t[7 * sp] - lse[7]));
  return a;
}

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void k_vsum(const Params p) {
  // Every wave owns 64 consecutive tokens of the chunk and works alone until the final
  // reduction: lane l weighs token l of the wave's share, the weight then travels to the
  // 16 (8) lanes that hold that token's value row by a lane shuffle.  No LDS and no barrier
  // between the weights and the value rows, whose loads are requested first.
  constexpr int TL = D / 8;               // lanes per value row
  constexpr int RPW = kWave / TL;         // rows per wave per load instruction
  constexpr int ITER = kWave / RPW;       // load instructions per wave per chunk (one per RPW rows)
  constexpr int NW = kThreads / kWave;
  static_assert(ITER % kUnroll == 0 && NW * kWave == kVChunk, "chunk geometry");
  const int bh = blockIdx.y, b = bh / p.Hkv, hk = bh % p.Hkv;
  const int N = seq_len(p, b);
  const int w0 = blockIdx.x * p.vrep * kVChunk;          // first token of this workgroup
  if (w0 >= N) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, tl = lane % TL, sub = lane / TL;
  const int lo = min(p.ph, N), hi = max(lo, N - p.pt);   // scored rows [lo,hi)
  const int half = p.pool / 2;

  __shared__ float red[NW][D + 1];

  // few-row path: normalisers of the (at most 8) query rows; rows that do not exist or see
  // no key have lse2 = +inf and stored logits -inf, both give exp2(-inf) = 0
  float lse[8];
#pragma unroll
  for (int r = 0; r < 8; ++r)
    lse[r] = p.small_r && r < p.R ? row_lse2(p, b, hk, bh, r) : INFINITY;

  const T* Vb = reinterpret_cast<const T*>(p.V) + (int64_t)b * p.vsb + (int64_t)hk * p.vsh + tl * 8;
  float* h = p.h + (int64_t)bh * p.cap;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  float zsum = 0.f;

  for (int rep = 0; rep < p.vrep; ++rep) {
    const int c0 = w0 + rep * kVChunk + wave * kWave;      // first token of this wave's share
    if (c0 >= N) break;                                    // (wave-uniform; no barrier in the loop)
    Frag<T> f[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int j = c0 + u * RPW + sub;
      if (j < N) fetch(Vb + (int64_t)j * p.vsn, f[u]); else zero(f[u]);
    }
    // ---- the weight of token c0 + lane ------------------------------------------------------
    float wj = 0.f;
    {
      const int j = c0 + lane;
      if (j < N) {
        const bool scored = j >= lo && j < hi;
        float hj = mass_of(p, bh, j, lse);
        if (p.base_mode == CAOTE_BASE_H2O) {
          hj += h[j];                           // h aliases the accumulator
        } else if (p.base_mode == CAOTE_BASE_SNAPKV && scored) {
          const int t0 = max(lo, j - half), t1 = min(hi - 1, j + half);
          for (int t = t0; t <= t1; ++t) hj = fmaxf(hj, t == j ? hj : mass_of(p, bh, t, lse));
        }
        h[j] = hj;
        wj = scored ? (p.variant == CAOTE_FAST ? 1.f : hj) : 0.f;
        zsum += scored ? hj : 0.f;
      }
    }
    // ---- the weighted sum over the wave's 64 value rows, kUnroll loads in flight -------------
#pragma unroll
    for (int it0 = 0; it0 < ITER; it0 += kUnroll) {
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const float w = __shfl(wj, (it0 + u) * RPW + sub, kWave);
        float x[8];
        widen(f[u], x);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = fmaf(w, x[e], acc[e]);
        if (it0 + kUnroll < ITER) {                          // the same slot, next group of rows
          const int j = c0 + (it0 + kUnroll + u) * RPW + sub;
          if (j < N) fetch(Vb + (int64_t)j * p.vsn, f[u]); else zero(f[u]);
        }
      }
    }
  }
  // ---- the rows of a wave, then the waves ----------------------------------------------------
#pragma unroll
  for (int o = TL; o < kWave; o <<= 1) {
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += __shfl_xor(acc[e], o, kWave);
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) zsum += __shfl_xor(zsum, o, kWave);
  if (lane < TL) {
#pragma unroll
    for (int e = 0; e < 8; ++e) red[wave][lane * 8 + e] = acc[e];
  }
  if (lane == 0) red[wave][D] = zsum;
  __syncthreads();
  if (tid <= D) {
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) s += red[w][tid];
    if (tid < D) p.opart[((int64_t)bh * p.n_vpart + blockIdx.x) * D + tid] = s;
    else         p.zpart[(int64_t)bh * p.n_vpart + blockIdx.x] = s;
  }
}

// Adds the per-workgroup partial sums of one head up, in order.  When the second key sweep
// formed the partial sums (one per split), the tokens within the pooling half-width of a
// split boundary are still open: their pooled base score needs column sums of two splits.
// They are few (2 * halo per split) and are finished here, from the column sums in memory.
__global__ __launch_bounds__(kFinalThreads) void k_vfinal(const Params p) {
  const int bh = blockIdx.x, b = bh / p.Hkv, hk = bh % p.Hkv;
  const int N = seq_len(p, b);
  const int nch = p.fuse_v ? split_count(p, bh, N, p.split_len) : (N + p.vrep * kVChunk - 1) / (p.vrep * kVChunk);
  const int tid = threadIdx.x, D = p.D;
  // kFinalThreads / 128 groups x 128 columns; group g takes partials g, g+G, ...
  constexpr int G = kFinalThreads / kMaxD;
  constexpr int NW = kFinalThreads / kWave;
  const int g = tid / kMaxD, col = tid % kMaxD;
  __shared__ float red[G][kMaxD + 1];
  __shared__ float edge[NW][kMaxD + 1];
  // The first partial sums are requested here and added up after the boundary tokens below,
  // whose loads are then in flight at the same time.
  float s = 0.f, z = 0.f;
  const float* op = p.opart + (int64_t)bh * p.n_vpart * D + (col < D ? col : 0);
  const float* zp = p.zpart + (int64_t)bh * p.n_vpart;
  float x0 = 0.f, x1 = 0.f, x2 = 0.f, x3 = 0.f, z0 = 0.f;
  if (col < D) {
    if (g < nch) x0 = op[(int64_t)g * D];
    if (g + G < nch) x1 = op[(int64_t)(g + G) * D];
    if (g + 2 * G < nch) x2 = op[(int64_t)(g + 2 * G) * D];
    if (g + 3 * G < nch) x3 = op[(int64_t)(g + 3 * G) * D];
  }
  if (col == 0 && g < nch) z0 = zp[g];
  const bool edges = p.fuse_v && p.halo > 0;    // bf16, head_dim 128: 16 lanes per value row
  if (edges) {
    const int team = tid >> 4, tl = tid & 15, halo = p.halo;
    const int lo = min(p.ph, N), hi = max(lo, N - p.pt);
    const float* a = p.a + (int64_t)bh * p.cap;
    const bf16_t* Vb = reinterpret_cast<const bf16_t*>(p.V) + (int64_t)b * p.vsb + (int64_t)hk * p.vsh + tl * 8;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    float zz = 0.f;
    // kEdgeBatch tokens per team at a time, all their loads requested before the first use:
    // the 16 lanes share the pooling window between them, and the value row does not wait
    // for the weight, so a batch costs one round trip to memory
    constexpr int kEdgeBatch = 4, kTeams = kFinalThreads / 16;
    const int n_edge = nch * 2 * halo;
    for (int idx0 = team; idx0 < n_edge; idx0 += kTeams * kEdgeBatch) {
      int jj[kEdgeBatch];
      bool sc[kEdgeBatch];
      float hj[kEdgeBatch], x[kEdgeBatch][8];
#pragma unroll
      for (int u = 0; u < kEdgeBatch; ++u) {
        const int idx = idx0 + u * kTeams;
        const int sp = idx / (2 * halo), o = idx - sp * 2 * halo;
        int c0, c1;
        split_range(p, bh, sp, N, p.split_len, c0, c1);
        const int j = o < halo ? c0 + o : c1 - 2 * halo + o;
        // front edge: the first `halo` tokens of the split; back edge: the last `halo`, unless
        // the split is so short that the front edge already covers them
        const bool valid = idx < n_edge && (o < halo ? j < c1 : j - c0 >= halo);
        jj[u] = valid ? j : -1;
        sc[u] = valid && j >= lo && j < hi;
        hj[u] = -INFINITY;
#pragma unroll
        for (int e = 0; e < 8; ++e) x[u][e] = 0.f;
        if (valid) {
          hj[u] = a[j];
          if (sc[u]) {
            load8(Vb + (int64_t)j * p.vsn, x[u]);
            const int t0 = max(lo, j - halo), t1 = min(hi - 1, j + halo);
            for (int t = t0 + tl; t <= t1; t += 16) hj[u] = fmaxf(hj[u], a[t]);
          }
        }
      }
#pragma unroll
      for (int u = 0; u < kEdgeBatch; ++u) {
#pragma unroll
        for (int m = 8; m >= 1; m >>= 1) hj[u] = fmaxf(hj[u], __shfl_xor(hj[u], m, kWave));
        if (jj[u] >= 0 && tl == 0) p.h[(int64_t)bh * p.cap + jj[u]] = hj[u];
        const float w = sc[u] ? (p.variant == CAOTE_FAST ? 1.f : hj[u]) : 0.f;
        if (tl == 0) zz += sc[u] ? hj[u] : 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = fmaf(w, x[u][e], acc[e]);
      }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      acc[e] += __shfl_xor(acc[e], 16, kWave);
      acc[e] += __shfl_xor(acc[e], 32, kWave);
    }
    zz += __shfl_xor(zz, 16, kWave);
    zz += __shfl_xor(zz, 32, kWave);
    const int lane = tid & 63, wave = tid >> 6;
    if (lane < 16) {
#pragma unroll
      for (int e = 0; e < 8; ++e) edge[wave][lane * 8 + e] = acc[e];
      if (lane == 0) edge[wave][kMaxD] = zz;
    }
  }
  if (col < D) {
    s += x0; s += x1; s += x2; s += x3;
    for (int c = g + 4 * G; c < nch; c += G) s += op[(int64_t)c * D];
  }
  if (col == 0) {
    z = z0;
    for (int c = g + G; c < nch; c += G) z += zp[c];
    red[g][kMaxD] = z;
  }
  red[g][col] = s;
  __syncthreads();
  if (tid <= kMaxD) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < G; ++i) t += red[i][tid];
    if (edges) {
#pragma unroll
      for (int i = 0; i < NW; ++i) t += edge[i][tid];
    }
    p.osum[(int64_t)bh * (kMaxD + 1) + tid] = t;
  }
}

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void k_vscore(const Params p) {
  constexpr int TL = D / 8;
  constexpr int RPI = kThreads / TL;
  constexpr int ITER = kVChunk / RPI;
  const int bh = blockIdx.y, b = bh / p.Hkv, hk = bh % p.Hkv;
  const int N = seq_len(p, b);
  const int c0 = blockIdx.x * kVChunk;
  if (c0 >= N) return;
  const int tid = threadIdx.x, team = tid / TL, tl = tid % TL;
  const int lo = min(p.ph, N), hi = max(lo, N - p.pt);
  const int n_scored = hi - lo;

  __shared__ float d_lds[kVChunk];        // ||v_j - o|| of each row of the chunk
  __shared__ uint32_t lh[kHistBins];      // hist_in_vscore: this chunk's histogram of score keys
  if (p.hist_in_vscore) {
#pragma unroll
    for (int u = 0; u < kHistBins / kThreads; ++u) lh[threadIdx.x + u * kThreads] = 0u;
  }

  const float* os = p.osum + (int64_t)bh * (kMaxD + 1);
  const float Z = os[kMaxD];
  const float onorm = p.variant == CAOTE_FAST ? 1.f / (float)max(n_scored, 1)
                                              : (Z > 0.f ? 1.f / Z : 0.f);
  float of[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) of[e] = os[tl * 8 + e] * onorm;

  const T* Vb = reinterpret_cast<const T*>(p.V) + (int64_t)b * p.vsb + (int64_t)hk * p.vsh + tl * 8;
#pragma unroll
  for (int it0 = 0; it0 < ITER; it0 += kUnroll) {
    Frag<T> f[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int j = c0 + (it0 + u) * RPI + team;
      if (j >= lo && j < hi) fetch(Vb + (int64_t)j * p.vsn, f[u]); else zero(f[u]);
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      float x[8];
      widen(f[u], x);
      float d2 = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) { const float t = x[e] - of[e]; d2 = fmaf(t, t, d2); }
      d2 = team_sum_dpp<TL>(d2);
      if (tl == 0) d_lds[(it0 + u) * RPI + team] = sqrtf(d2);
    }
  }
  __syncthreads();
  // ---- one thread per token: the score ------------------------------------------------------
  const int j = c0 + tid;
  float out = INFINITY;
  if (j < N) {
    if (j >= lo && j < hi && n_scored > 1) {
      const float hj = p.h[(int64_t)bh * p.cap + j];
      out = Z > 0.f ? hj / fmaxf(Z - hj, FLT_MIN) * d_lds[tid] : 0.f;
    }
    p.scores[(int64_t)bh * p.cap + j] = out;
  }
  // ---- fused call, long cache: the selection's 4096-bin histogram of the score keys, added up
  // per workgroup in LDS first (the scores of a head crowd into a few dozen bins, and
  // same-address device atomics serialise), then one global atomic per touched bin ----------
  if (p.hist_in_vscore) {
    if (j < N) atomicAdd(&lh[float_key(out) >> kHistShift], 1u);
    __syncthreads();
    uint32_t* gh = p.hist + (int64_t)bh * kHistBins;
#pragma unroll
    for (int u = 0; u < kHistBins / kThreads; ++u) {
      const uint32_t c = lh[tid + u * kThreads];
      if (c) atomicAdd(&gh[tid + u * kThreads], c);
    }
  }
}

template <typename T, int D>
hipError_t launch_t(const Params& p, hipStream_t s, PhaseHook* hook) {
  const int bh = p.B * p.Hkv;
  if (!p.fuse_v) {
    hipLaunchKernelGGL((k_vsum<T, D>), dim3(p.n_vsum, bh), dim3(kThreads), 0, s, p);
    if (mark(hook, "value_sum")) return hipGetLastError();
  }
  hipLaunchKernelGGL(k_vfinal, dim3(bh), dim3(kFinalThreads), 0, s, p);
  if (mark(hook, "value_final")) return hipGetLastError();
  hipLaunchKernelGGL((k_vscore<T, D>), dim3(p.n_vchunk, bh), dim3(kThreads), 0, s, p);
  if (mark(hook, "value_score")) return hipGetLastError();
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
