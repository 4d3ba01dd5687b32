// Window attention over the key cache on the matrix cores: bf16, head_dim 128.
//
// Two sweeps over K (Sec. 2, attention of the window queries over the cache), as in the
// vector-ALU path, but the R x N logits come from v_mfma_f32_32x32x16_bf16 tiles:
//   sweep 1 (MODE 0)  S^T tile = K_tile (32 keys, M) x Q^T (32 query rows, N): a lane
//                     then holds 16 keys of ONE query row, so the running (max, sum)
//                     of the softmax is lane-local -- no cross-lane work per tile.
//   sweep 2 (MODE 1)  S tile = Q (32 rows, M) x K_tile^T (32 keys, N): a lane holds 16
//                     rows of ONE key, so the column sum a_j is lane-local.
// The A and B operands of this instruction have the same register layout (lane l holds
// row/column l%32, k = 8*(l/32)..+7), so the same Q registers and the same K reads from
// LDS serve both sweeps.
//
// A workgroup is 4 waves arranged WR (row waves) x WK (key waves); every wave keeps RBW
// 32-row blocks of Q in registers for the whole sweep.  K tiles of 64 keys go through a
// double-buffered, XOR-swizzled LDS stage: global -> registers one tile ahead -> LDS.
#include <type_traits>

#include "common.hpp"

namespace caote {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kTN = 64;                 // keys per LDS tile
constexpr int kD = 128;
constexpr int kRowBytes = kD * 2;       // 256
constexpr int kChunks = kRowBytes / 16; // 16-byte chunks per key row
constexpr int kNBuf = 3;                // LDS ring of key tiles: loads run kNBuf-1 tiles ahead

// global_load_lds_dwordx4: lane L of the wave copies 16 bytes from its own global address
// to LDS byte address lds_base + 16 L (lds_base is wave-uniform and travels in M0).  Issued
// through inline assembly so that the compiler does not serialise it against the LDS reads
// of other ring slots; the matching waits are wait_vmcnt<N>() below.
__device__ __forceinline__ void load_to_lds16(const void* gaddr, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               : : "v"(gaddr), "s"(lds_base) : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory"); }
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}

__device__ __forceinline__ int swz(int row, int chunk) { return row * kRowBytes + ((chunk ^ (row & 15)) << 4); }

// Key index inside a 32x32 output tile for accumulator register i when keys are the M
// dimension (sweep 1); also the row index when rows are the M dimension (sweep 2).
__device__ __forceinline__ int m_of(int i, int lane) { return 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3); }

template <int NWV, int WR, int RBW, int MODE>
__global__ __launch_bounds__(NWV * kWave) void k_logits_mfma(const Params p) {
  constexpr int kThreads = NWV * kWave; // NWV waves = WR row waves x WK key waves
  constexpr int LPT = 16 / NWV;         // 1 KiB loads per wave per K tile
  constexpr int WK = NWV / WR;          // key waves
  constexpr int KBW = (kTN / 32) / WK;  // 32-key blocks per wave per tile
  constexpr int ROWS = WR * RBW * 32;   // query rows per row group
  const int bh = blockIdx.y, b = bh / p.Hkv, hk = bh % p.Hkv;
  const int N = seq_len(p, b);
  const int c0 = blockIdx.x * p.split_len;
  if (c0 >= N) return;
  const int c1 = min(N, c0 + p.split_len);
  const int ntiles = (c1 - c0 + kTN - 1) / kTN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave / WK, kw = wave % WK;
  const int P = p.wic ? N - p.W : N;    // keys below P are visible to every row

  __shared__ __attribute__((aligned(16))) unsigned char Ks[kNBuf][kTN * kRowBytes];
  __shared__ float a_lds[2][WR][kTN];
  __shared__ int iw_lds[ROWS];          // window position of each row of the group
  __shared__ float lse_lds[ROWS];       // sweep 2: normaliser of each row of the group
  __shared__ float st_lds[WK][ROWS][2];

  const unsigned char* Kb = reinterpret_cast<const unsigned char*>(p.K) +
                            ((int64_t)b * p.ksb + (int64_t)hk * p.ksh) * 2;
  const int64_t krow = p.ksn * 2;
  float* a_out = p.a + (int64_t)bh * p.cap;

  for (int rg0 = 0; rg0 < p.R; rg0 += ROWS) {
    // ---- sweep over the key tiles of this split --------------------------------------
    // K tiles go from global memory straight into LDS (global_load_lds_dwordx4: lane L of
    // a wave fills the 16-byte slot base + 16 L), kNBuf-1 tiles ahead of the math.  The
    // XOR swizzle that keeps the fragment reads conflict-free is applied on the global
    // side: the lane that owns slot (row, pc) fetches chunk pc ^ (row & 15) of that row.
    auto issue = [&](int t, int buf) {
#pragma unroll
      for (int u = 0; u < LPT; ++u) {
        const int slot = (wave * LPT + u) * kWave + lane;    // 16-byte slot inside the tile
        const int row = slot / kChunks, pc = slot % kChunks;
        const int j = min(c0 + t * kTN + row, N - 1);        // rows past the end repeat the last one
        load_to_lds16(Kb + j * krow + ((pc ^ (row & 15)) << 4),
                      __builtin_amdgcn_readfirstlane(lds_addr(&Ks[buf][(wave * LPT + u) * kWave * 16])));
      }
    };
    // The first two K tiles are requested before anything else, so that their latency
    // overlaps the set-up below.
    __syncthreads();                     // previous row group is done with LDS
    for (int t = 0; t < kNBuf - 1 && t < ntiles; ++t) issue(t, t);
    // ---- per-row-group set-up: Q fragments, window positions, normalisers ----------
    for (int i = tid; i < ROWS; i += kThreads) {
      int g_unused, iw_i;
      divmod_w(p, rg0 + i, g_unused, iw_i);
      iw_lds[i] = (rg0 + i) < p.R ? iw_i : -1;
      if (MODE == 1) lse_lds[i] = (rg0 + i) < p.R ? p.lse2[(int64_t)bh * p.Rp + rg0 + i] : INFINITY;
    }
    bf16x8 qf[RBW][8];
    float lse[RBW][16];
    float m_run[RBW], l_run[RBW];
    int nvis_row[RBW];                  // MODE 0: visible-key count of this lane's row
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb) {
      const int rbase = rg0 + (wr * RBW + rb) * 32;
      const int r = rbase + (lane & 31);
      m_run[rb] = -INFINITY; l_run[rb] = 0.f; nvis_row[rb] = 0;
      if (r < p.R) {
        int g, iw;
        divmod_w(p, r, g, iw);
        const unsigned char* qp = reinterpret_cast<const unsigned char*>(p.q) +
            ((int64_t)b * p.qsb + (int64_t)(hk * p.G + g) * p.qsh + (int64_t)iw * p.qsw) * 2 + (lane >> 5) * 16;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
          qf[rb][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(qp + ks * 32));
        nvis_row[rb] = p.wic ? P + iw + 1 : N;
      } else {
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qf[rb][ks] = __builtin_bit_cast(bf16x8, make_uint4(0, 0, 0, 0));
      }
    }
    if (MODE == 1) {
      __syncthreads();
#pragma unroll
      for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
        for (int i = 0; i < 16; ++i) lse[rb][i] = lse_lds[(wr * RBW + rb) * 32 + m_of(i, lane)];
    }
    // One 64-key tile out of LDS buffer `buf`.  TAIL: some logits of the tile are masked
    // (keys past the end of the cache, or window keys a row must not see).
    auto tile = [&](auto tail_tag, int buf, int abuf, int tile0) {
      constexpr bool TAIL = decltype(tail_tag)::value;
#pragma unroll
      for (int kbi = 0; kbi < KBW; ++kbi) {
        const int kb = kw * KBW + kbi;                        // 32-key block inside the tile
        const int row = kb * 32 + (lane & 31);
        f32x16 acc[RBW];
        bf16x8 kf[8];                                         // all eight K fragments first, so
#pragma unroll                                                // that their LDS latencies overlap
        for (int ks = 0; ks < 8; ++ks)
          kf[ks] = __builtin_bit_cast(
              bf16x8, *reinterpret_cast<const uint4*>(&Ks[buf][swz(row, 2 * ks + (lane >> 5))]));
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
          for (int rb = 0; rb < RBW; ++rb) {
            const f32x16 cin = ks == 0 ? f32x16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f,
                                                0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f} : acc[rb];
            if (MODE == 0) acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[rb][ks], cin, 0, 0, 0);
            else           acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[rb][ks], kf[ks], cin, 0, 0, 0);
          }
        }
        const int jb = tile0 + kb * 32;                       // first key of the block
        if (MODE == 0) {
#pragma unroll
          for (int rb = 0; rb < RBW; ++rb) {
            if (TAIL) {                                         // masked logits become -inf
#pragma unroll
              for (int i = 0; i < 16; ++i)
                if (jb + m_of(i, lane) >= nvis_row[rb]) acc[rb][i] = -INFINITY;
            }
            float mx = acc[rb][0];
#pragma unroll
            for (int i = 1; i < 16; ++i) mx = __builtin_fmaxf(mx, acc[rb][i]);
            const float mn = __builtin_fmaxf(m_run[rb], mx * p.c2);     // c2 > 0
            if (!TAIL || mn > -INFINITY) {
              float e[16];                                      // independent terms, then a tree:
#pragma unroll                                                // no serial exp -> add chain
              for (int i = 0; i < 16; ++i) e[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(acc[rb][i], p.c2, -mn));
              const float s = (((e[0] + e[1]) + (e[2] + e[3])) + ((e[4] + e[5]) + (e[6] + e[7]))) +
                              (((e[8] + e[9]) + (e[10] + e[11])) + ((e[12] + e[13]) + (e[14] + e[15])));
              l_run[rb] = l_run[rb] * __builtin_amdgcn_exp2f(m_run[rb] - mn) + s;
              m_run[rb] = mn;
            }
          }
        } else {
          float cs = 0.f;
          const int j = jb + (lane & 31);
#pragma unroll
          for (int rb = 0; rb < RBW; ++rb) {
            const int rl = (wr * RBW + rb) * 32;                // row offset inside the group
            float e[16];                                        // independent terms, then a tree
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(acc[rb][i], p.c2, -lse[rb][i]));
              if (TAIL) {
                const int iw = iw_lds[rl + m_of(i, lane)];
                const bool vis = j < N && iw >= 0 && (!p.wic || j < P + iw + 1);
                pv = vis ? pv : 0.f;
              }
              e[i] = pv;
            }
            cs += (((e[0] + e[1]) + (e[2] + e[3])) + ((e[4] + e[5]) + (e[6] + e[7]))) +
                  (((e[8] + e[9]) + (e[10] + e[11])) + ((e[12] + e[13]) + (e[14] + e[15])));
          }
          cs += __shfl_xor(cs, 32, kWave);
          if (lane < 32) a_lds[abuf][wr][kb * 32 + lane] = cs;
        }
      }
    };
    auto math = [&](int t, int buf, int abuf) {
      const int tile0 = c0 + t * kTN;
      if (tile0 + kTN > min(P, N)) tile(std::true_type{}, buf, abuf, tile0);
      else                         tile(std::false_type{}, buf, abuf, tile0);
    };
    auto flush_a = [&](int t, int buf) {                     // after the barrier of step t
      const int tile0 = c0 + t * kTN;
      if (MODE == 1 && tid < kTN && tile0 + tid < c1) {
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < WR; ++w) s += a_lds[buf][w][tid];
        if (rg0 == 0) a_out[tile0 + tid] = s;
        else a_out[tile0 + tid] += s;                          // later row groups add on
      }
    };
    // Make the compiler finish its own global loads (Q fragments, normalisers) here: a wait
    // it placed inside the tile loop would also drain the LDS loads that must stay in flight.
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb) {
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) asm volatile("" : : "v"(qf[rb][ks]));
      if (MODE == 1) {
#pragma unroll
        for (int i = 0; i < 16; ++i) asm volatile("" : : "v"(lse[rb][i]));
      }
    }
    int buf = 0;
    for (int t = 0; t < ntiles; ++t) {
      // this wave's share of tile t has landed once at most the 4 loads of tile t+1 are
      // still in flight (loads complete in order; a store in between cannot hide a load)
      if (t + 1 < ntiles) wait_vmcnt<LPT>(); else wait_vmcnt<0>();
      __syncthreads();                   // ... and so has everyone else's; tile t-1 is done with
      if (t > 0) flush_a(t - 1, (t - 1) & 1);
      if (t + kNBuf - 1 < ntiles) issue(t + kNBuf - 1, buf == 0 ? kNBuf - 1 : buf - 1);
      math(t, buf, t & 1);
      buf = buf + 1 == kNBuf ? 0 : buf + 1;
    }
    __syncthreads();
    flush_a(ntiles - 1, (ntiles - 1) & 1);
    // ---- end of sweep 1: merge the two half-waves, then the key waves ------------------
    if (MODE == 0) {
#pragma unroll
      for (int rb = 0; rb < RBW; ++rb) {
        const float m2 = __shfl_xor(m_run[rb], 32, kWave), l2 = __shfl_xor(l_run[rb], 32, kWave);
        const float M = fmaxf(m_run[rb], m2);
        float L = 0.f;
        if (m_run[rb] > -INFINITY) L += l_run[rb] * exp2f(m_run[rb] - M);
        if (m2 > -INFINITY) L += l2 * exp2f(m2 - M);
        if (lane < 32) {
          const int rl = (wr * RBW + rb) * 32 + lane;
          st_lds[kw][rl][0] = M; st_lds[kw][rl][1] = L;
        }
      }
      __syncthreads();
      for (int rl = tid; rl < ROWS; rl += kThreads) {
        if (rg0 + rl >= p.R) continue;
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < WK; ++w) M = fmaxf(M, st_lds[w][rl][0]);
        float L = 0.f;
#pragma unroll
        for (int w = 0; w < WK; ++w)
          if (st_lds[w][rl][0] > -INFINITY) L += st_lds[w][rl][1] * exp2f(st_lds[w][rl][0] - M);
        float* st = p.stats + (((int64_t)bh * p.n_split + blockIdx.x) * p.Rp + rg0 + rl) * 2;
        st[0] = M; st[1] = L;
      }
    }
  }
}

// lse2_r = log2 sum_j exp2(t_rj): one wave per query row, lanes stride over the splits.
constexpr int kMergeThreads = 256;
__global__ __launch_bounds__(kMergeThreads) void k_merge_stats_wave(const Params p) {
  const int bh = blockIdx.y, b = bh / p.Hkv;
  if (blockIdx.x == 0) reset_counters(p, bh);
  const int r = blockIdx.x * (kMergeThreads / kWave) + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (r >= p.R) return;
  const int N = seq_len(p, b);
  const int ns = (N + p.split_len - 1) / p.split_len;
  const float* st = p.stats + ((int64_t)bh * p.n_split * p.Rp + r) * 2;
  float M = -INFINITY;
  for (int s = lane; s < ns; s += kWave) M = fmaxf(M, st[(int64_t)s * p.Rp * 2]);
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) M = fmaxf(M, __shfl_xor(M, o, kWave));
  float L = 0.f;
  for (int s = lane; s < ns; s += kWave) {
    const float ms = st[(int64_t)s * p.Rp * 2];
    if (ms > -INFINITY) L += st[(int64_t)s * p.Rp * 2 + 1] * exp2f(ms - M);
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) L += __shfl_xor(L, o, kWave);
  if (lane == 0) p.lse2[(int64_t)bh * p.Rp + r] = L > 0.f ? M + log2f(L) : INFINITY;
}

}  // namespace

hipError_t launch_merge_stats(const Params& p, hipStream_t s, PhaseHook* hook) {
  hipLaunchKernelGGL(k_merge_stats_wave, dim3((p.R + 3) / 4, p.B * p.Hkv), dim3(kMergeThreads), 0, s, p);
  mark(hook, "merge_stats");
  return hipGetLastError();
}

namespace {

template <int NWV, int WR, int RBW>
hipError_t launch_cfg(const Params& p, hipStream_t s, PhaseHook* hook) {
  const dim3 grid(p.n_split, p.B * p.Hkv);
  hipLaunchKernelGGL((k_logits_mfma<NWV, WR, RBW, 0>), grid, dim3(NWV * kWave), 0, s, p);
  mark(hook, "key_rowstats");
  if (launch_merge_stats(p, s, hook) != hipSuccess) return hipGetLastError();
  hipLaunchKernelGGL((k_logits_mfma<NWV, WR, RBW, 1>), grid, dim3(NWV * kWave), 0, s, p);
  mark(hook, "key_colsum");
  return hipGetLastError();
}

}  // namespace

// Requires: bf16, head_dim 128, split_len a multiple of 64.
hipError_t launch_score_mfma(const Params& p, hipStream_t s, PhaseHook* hook) {
  const int nrb = (p.R + 31) / 32;
  if (nrb <= 2) return launch_cfg<4, 2, 1>(p, s, hook);
  if (nrb <= 4) return launch_cfg<4, 2, 2>(p, s, hook);
  return launch_cfg<8, 4, 2>(p, s, hook);
}

}  // namespace caote
