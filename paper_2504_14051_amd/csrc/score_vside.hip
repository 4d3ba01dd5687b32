// Value side of the CAOTE score on short caches (generation: a cache at its budget plus the
// new token), with V read from memory ONCE (Sec. 3.2: o = V (H^norm)^T, then
// c_j = w_j / (1 - w_j) ||v_j - o||).  The score needs every value row twice, first for o and
// then for the distance to o; k_vsum / k_vscore stream V twice and cross a kernel boundary in
// between.  Here a head's rows stay in registers between the two uses: a head is cut by
// COLUMNS into CS = 2 workgroups of 512 threads, each holding 128 / CS columns of all rows of the
// head (a lane keeps 8 columns of up to kSlots rows, 16 bytes each).  A column slice of o needs
// only that slice of V, so no workgroup waits for another:
//   1. request the slice's rows;  2. attention mass a_j of every token into LDS (from the
//   stored logits or the column sums);  3. base score h_j (H2O accumulate / SnapKV max-pool
//   over LDS) and Z = sum h;  4. o slice = sum_j w_j v_j / norm, reduced over the workgroup;
//   5. the slice's part of ||v_j - o||^2 for every row -> memory.
// k_vcombine adds the CS parts of a token up and writes the score (and the H2O accumulator,
// which the column workgroups of a head only read, so that none of them sees the others'
// update).
#include <float.h>

#include "common.hpp"

namespace caote {
namespace {

constexpr int kVT = 512;                  // threads per workgroup: 8 waves, up to 256 registers per lane
constexpr int kVW = kVT / kWave;
constexpr int kSlots = kVSideSlots;       // rows per lane

__device__ __forceinline__ float mass_at(const Params& p, int bh, int j, const float (&lse)[8]) {
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

__device__ __forceinline__ void widen8(const uint4& u, float (&x)[8]) {
  x[0] = __uint_as_float(u.x << 16); x[1] = __uint_as_float(u.x & 0xffff0000u);
  x[2] = __uint_as_float(u.y << 16); x[3] = __uint_as_float(u.y & 0xffff0000u);
  x[4] = __uint_as_float(u.z << 16); x[5] = __uint_as_float(u.z & 0xffff0000u);
  x[6] = __uint_as_float(u.w << 16); x[7] = __uint_as_float(u.w & 0xffff0000u);
}

// SR: rows of stored logits the token passes read per token (4 or 8; 1 when the mass comes
// from the column sums): a compile-time count keeps their registers to what is needed.
template <int CS, int SR>
__global__ __launch_bounds__(kVT) void k_vside(const Params p) {
  constexpr int TL = 16 / CS;             // lanes per row slice
  constexpr int NT = kVT / TL;            // rows per slot
  constexpr int COLS = kMaxD / CS;        // columns of this workgroup
  constexpr int NMAX = kSlots * NT;
  const int cs = blockIdx.x, bh = blockIdx.y, b = bh / p.Hkv, hk = bh % p.Hkv;
  const int N = seq_len(p, b);
  if (N <= 0) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, tl = tid % TL, team = tid / TL;
  const int lo = min(p.ph, N), hi = max(lo, N - p.pt);   // scored rows [lo,hi)
  const int n_scored = hi - lo;
  const int half = p.pool / 2;

  __shared__ float a_s[NMAX];             // attention mass per token
  __shared__ float h_s[NMAX];             // base score per token
  __shared__ float wsum[kVW][COLS];
  __shared__ float zred[kVW];
  __shared__ float o_s[COLS];

  // Order of the requests: loads return in the order they were issued, so what the base score
  // needs (stored logits or column sums, the accumulator) is requested BEFORE the value rows;
  // a_j, h_j and Z are then ready while the rows are still arriving, and step 4 takes each
  // row as it lands.  With two column workgroups a lane has at most 5 tokens in the token
  // passes and keeps their inputs in registers; with more, the token passes simply run first.
  constexpr int IMAX = (NMAX + kVT - 1) / kVT;     // tokens per thread in the token passes
  constexpr bool PRE = IMAX <= 5;
  // Row normalisers: the caller's, the merge kernel's, or (few query rows) merged here from the
  // first sweep's partial (max, sum) pairs, wave r taking row r as k_merge_stats_wave does.  The
  // partials are requested before everything else and reduced while the rows are in flight.
  const bool merge_here = SR > 1 && p.merge_in_vside && !p.lse_in;
  __shared__ float lse_s[8];
  const int ns = (N + p.split_len - 1) / p.split_len;
  float st_m[2] = {-INFINITY, -INFINITY}, st_l[2] = {0.f, 0.f};   // (n_split <= 128 on these caches)
  if (merge_here && wave < p.R) {
    const float* st = p.stats + ((int64_t)bh * p.n_split * p.Rp + wave) * 2;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int sp = min(lane + i * kWave, ns - 1);
      const float2 ml = *reinterpret_cast<const float2*>(st + (int64_t)sp * p.Rp * 2);
      if (lane + i * kWave < ns) { st_m[i] = ml.x; st_l[i] = ml.y; }
    }
  }
  float lse[8];
#pragma unroll
  for (int r = 0; r < 8; ++r)
    lse[r] = r < SR && p.small_r && r < p.R && !merge_here ? row_lse2(p, b, hk, bh, r) : INFINITY;
  const float* base_in = p.base + (p.base ? (int64_t)bh * p.cap : 0);
  const bool h2o = p.base_mode == CAOTE_BASE_H2O;
  float sv[PRE ? IMAX : 1][SR], bv[PRE ? IMAX : 1];
  if (PRE) {
#pragma unroll
    for (int i = 0; i < IMAX; ++i) {
      const int j = min(tid + i * kVT, N - 1);       // (clamped, not skipped: see request_rows)
      if (SR > 1) {
        const float* t = p.S + (int64_t)bh * SR * p.s_pitch + j;
#pragma unroll
        for (int r = 0; r < SR; ++r) sv[i][r] = t[(int64_t)r * p.s_pitch];
      } else {
        sv[i][0] = p.a[(int64_t)bh * p.cap + j];
      }
      bv[i] = h2o ? base_in[j] : 0.f;
    }
  }

  // ---- 1. the rows of this column slice (only scored rows enter o and get a distance) ----
  // (byte offsets inside the head's slab fit 32 bits: the host checks it; one register per
  // address instead of two keeps the rows' registers from spilling)
  const char* Vb = reinterpret_cast<const char*>(p.V) +
                   ((int64_t)b * p.vsb + (int64_t)hk * p.vsh + cs * COLS) * 2;   // workgroup-uniform
  const uint32_t row_bytes = (uint32_t)p.vsn * 2u;
  uint4 f[kSlots];
  // Every slot loads: a slot without a scored row re-reads a row that exists (its weight is 0
  // and its distance is not stored).  A load under a lane-dependent condition would make the
  // compiler wait for each one before the next.
  const int j_any = hi > lo ? lo : 0;
  auto request_rows = [&]() {
#pragma unroll
    for (int s = 0; s < kSlots; ++s) {
      const int j = team + s * NT;
      const int jj = (j >= lo && j < hi) ? j : j_any;
      f[s] = *reinterpret_cast<const uint4*>(Vb + ((uint32_t)jj * row_bytes + (uint32_t)tl * 16u));
      __builtin_amdgcn_sched_barrier(0);      // address, load, next address: no pile of live addresses
    }
  };
  if (PRE) request_rows();

  if (merge_here) {
    if (wave < p.R) {
      float M = fmaxf(st_m[0], st_m[1]);
#pragma unroll
      for (int o = 32; o >= 1; o >>= 1) M = fmaxf(M, __shfl_xor(M, o, kWave));
      float L = 0.f;
#pragma unroll
      for (int i = 0; i < 2; ++i)
        if (st_m[i] > -INFINITY) L += st_l[i] * exp2f(st_m[i] - M);
#pragma unroll
      for (int o = 32; o >= 1; o >>= 1) L += __shfl_xor(L, o, kWave);
      if (lane == 0) lse_s[wave] = L > 0.f ? M + log2f(L) : INFINITY;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < SR; ++r)
      if (r < p.R) lse[r] = lse_s[r];
  }

  // ---- 2. attention mass of every token (Sec. 2, f_score,j = sum_i A_ij) ----
  if (PRE) {
#pragma unroll
    for (int i = 0; i < IMAX; ++i) {
      const int j = tid + i * kVT;
      if (j < N) {
        float a = sv[i][0];
        if (SR > 1) {
          a = (__builtin_amdgcn_exp2f(sv[i][0] - lse[0]) + __builtin_amdgcn_exp2f(sv[i][1 % SR] - lse[1])) +
              (__builtin_amdgcn_exp2f(sv[i][2 % SR] - lse[2]) + __builtin_amdgcn_exp2f(sv[i][3 % SR] - lse[3]));
          if (SR == 8)
            a += (__builtin_amdgcn_exp2f(sv[i][4 % SR] - lse[4]) + __builtin_amdgcn_exp2f(sv[i][5 % SR] - lse[5])) +
                 (__builtin_amdgcn_exp2f(sv[i][6 % SR] - lse[6]) + __builtin_amdgcn_exp2f(sv[i][7 % SR] - lse[7]));
        }
        a_s[j] = a;
      }
    }
  } else {
    for (int j = tid; j < N; j += kVT) a_s[j] = mass_at(p, bh, j, lse);
  }
  __syncthreads();

  // ---- 3. base score and its sum over the scored rows ----
  float* h_out = p.h + (int64_t)bh * p.cap;
  float z = 0.f;
  auto base_score = [&](int j, float add) {
    const bool scored = j >= lo && j < hi;
    float hj = a_s[j] + add;
    if (p.base_mode == CAOTE_BASE_SNAPKV && scored) {
      const int t0 = max(lo, j - half), t1 = min(hi - 1, j + half);
      for (int t = t0; t <= t1; ++t) hj = fmaxf(hj, a_s[t]);
    }
    h_s[j] = hj;
    if (cs == 0) h_out[j] = hj;
    z += scored ? hj : 0.f;
  };
  if (PRE) {
#pragma unroll
    for (int i = 0; i < IMAX; ++i) {
      const int j = tid + i * kVT;
      if (j < N) base_score(j, bv[i]);
    }
  } else {
    for (int j = tid; j < N; j += kVT) base_score(j, h2o ? base_in[j] : 0.f);
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) z += __shfl_xor(z, o, kWave);
  if (lane == 0) zred[wave] = z;
  __syncthreads();
  float Z = 0.f;
#pragma unroll
  for (int w = 0; w < kVW; ++w) Z += zred[w];
  if (!PRE) request_rows();

  // ---- 4. this slice of o ----
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int s = 0; s < kSlots; ++s) {
    const int j = team + s * NT;
    const float w = (j >= lo && j < hi) ? (p.variant == CAOTE_FAST ? 1.f : h_s[j]) : 0.f;
    float x[8];
    widen8(f[s], x);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = fmaf(w, x[e], acc[e]);
  }
#pragma unroll
  for (int o = TL; o < kWave; o <<= 1) {
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += __shfl_xor(acc[e], o, kWave);
  }
  if (lane < TL) {
#pragma unroll
    for (int e = 0; e < 8; ++e) wsum[wave][lane * 8 + e] = acc[e];
  }
  __syncthreads();
  if (tid < COLS) {
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < kVW; ++w) t += wsum[w][tid];
    const float onorm = p.variant == CAOTE_FAST ? 1.f / (float)max(n_scored, 1) : (Z > 0.f ? 1.f / Z : 0.f);
    o_s[tid] = t * onorm;
    p.osum[(int64_t)bh * (kMaxD + 1) + cs * COLS + tid] = t;
  }
  if (cs == 0 && tid == 0) p.osum[(int64_t)bh * (kMaxD + 1) + kMaxD] = Z;
  __syncthreads();

  // ---- 5. this slice's part of || v_j - o ||^2 ----
  // (the rows stay packed between their two uses: unpacked copies would not fit the registers)
#pragma unroll
  for (int s = 0; s < kSlots; ++s) asm volatile("" : "+v"(f[s].x), "+v"(f[s].y), "+v"(f[s].z), "+v"(f[s].w));
  float of[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) of[e] = o_s[tl * 8 + e];
  float* d2 = p.d2part + ((int64_t)cs * p.B * p.Hkv + bh) * p.cap;
#pragma unroll
  for (int s = 0; s < kSlots; ++s) {
    const int j = team + s * NT;
    float x[8];
    widen8(f[s], x);
    float q = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) { const float t = x[e] - of[e]; q = fmaf(t, t, q); }
    q = team_sum_dpp<TL>(q);
    if (tl == 0 && j >= lo && j < hi) d2[j] = q;
  }
}

__global__ __launch_bounds__(256) void k_vcombine(const Params p) {
  const int bh = blockIdx.y, b = bh / p.Hkv;
  const int N = seq_len(p, b);
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j < N) combine_score(p, bh, j, N);
}

template <int CS>
hipError_t launch_cs(const Params& p, hipStream_t s, PhaseHook* hook) {
  const int bh = p.B * p.Hkv;
  const dim3 grid(CS, bh);
  if (!p.small_r)         hipLaunchKernelGGL((k_vside<CS, 1>), grid, dim3(kVT), 0, s, p);
  else if (p.s_rows == 4) hipLaunchKernelGGL((k_vside<CS, 4>), grid, dim3(kVT), 0, s, p);
  else                    hipLaunchKernelGGL((k_vside<CS, 8>), grid, dim3(kVT), 0, s, p);
  if (mark(hook, "value_side")) return hipGetLastError();
  if (!p.combine_in_select) {
    hipLaunchKernelGGL(k_vcombine, dim3((p.cap + 255) / 256, bh), dim3(256), 0, s, p);
    if (mark(hook, "value_combine")) return hipGetLastError();
  }
  return hipGetLastError();
}

}  // namespace

// Column workgroups per head, 0 if the streaming kernels should take the cache.  Only the
// two-way split is used: with four or eight workgroups per head the token passes repeat four
// or eight times, a row is fetched in 64- or 32-byte pieces, and a batch needs several rounds
// of workgroups; measured on 128 heads, 2177 rows cost 48 us with four against 25 us for 2049
// rows with two, and 8193 rows 216 us with eight against 110 us for the two streaming kernels.
int vside_column_split(int cap) {
  return cap <= kSlots * (kVT / 8) ? 2 : 0;
}

hipError_t launch_value_side(const Params& p, hipStream_t s, PhaseHook* hook) {
  if (p.vside_cs != 2) return hipErrorInvalidValue;
  return launch_cs<2>(p, s, hook);
}

}  // namespace caote
