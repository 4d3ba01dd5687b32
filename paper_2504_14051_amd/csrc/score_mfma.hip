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
// A workgroup is 4 or 8 waves arranged WR (row waves) x WK (key waves); every wave keeps RBW
// 32-row blocks of Q in registers for the whole sweep.  K tiles of 64 keys arrive in a
// three-slot, XOR-swizzled LDS ring by DMA (global_load_lds_dwordx4, two tiles ahead of the
// math, waits counted by hand); in the fused second sweep the V rows of each tile follow
// into a two-slot ring of their own, requested two iterations before they are added up.
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
// The 4-byte form: lane L fills lds_base + 4 L.
__device__ __forceinline__ void load_to_lds4(const void* gaddr, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off"
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
__global__ __launch_bounds__(NWV * kWave, 2) void k_logits_mfma(const Params p) {
  constexpr int kThreads = NWV * kWave; // NWV waves = WR row waves x WK key waves
  constexpr int LPT = 16 / NWV;         // 1 KiB loads per wave per K tile
  constexpr int WK = NWV / WR;          // key waves
  constexpr int KBW = (kTN / 32) / WK;  // 32-key blocks per wave per tile
  constexpr int ROWS = WR * RBW * 32;   // query rows per row group
  constexpr bool COLSUM = MODE >= 1;    // sweep 2
  constexpr bool FUSE = MODE == 2;      // sweep 2 that also accumulates sum_j h_j v_j
  // Q reaches its registers through LDS (where one workgroup per compute unit leaves room)
  constexpr bool QLDS = NWV == 8;
  const int tid = threadIdx.x, lane = tid & 63;
  // the wave index as a scalar: everything derived from it (ring addresses, row blocks) then
  // stays on the scalar unit
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wr = wave / WK, kw = wave % WK;
  // the first sweep may have its own split, with the row groups spread over the grid
  const int split_len = MODE == 0 ? p.split_len0 : p.split_len;

  __shared__ __attribute__((aligned(16))) unsigned char Ks[kNBuf][kTN * kRowBytes];
  __shared__ float a_lds[2][WR][kTN];
  __shared__ int iw_lds[ROWS];          // window position of each row of the group
  __shared__ __attribute__((aligned(16))) float lse_lds[ROWS];   // sweep 2: normaliser of each row of the group
  __shared__ float st_lds[WK][ROWS][2];
  __shared__ __attribute__((aligned(16))) unsigned char Qs[QLDS ? ROWS * kRowBytes : 16];
  // FUSE: attention mass of the last four tiles, weight of each row of the last four value
  // steps, the H2O accumulator rows of two steps, and one tile of V rows
  __shared__ float af[FUSE ? 4 * kTN : 1];
  __shared__ float hw[FUSE ? 4 * kTN : 1];
  __shared__ float bs[2][FUSE ? kTN : 1];
  __shared__ __attribute__((aligned(16))) unsigned char Vs[2][FUSE ? kTN * kRowBytes : 16];
  __shared__ float red[NWV][kD + 4];    // FUSE: the waves' partial value sums

  // ---- the pieces of work of this workgroup: (head, split, keys [c0, c1)) ------------------
  // Equal lengths: one piece, from the block index.  Ragged batches: this workgroup's share of
  // all heads' tiles laid end to end, which may end one head and start the next.
  int dyn_bh = -1;
  long long g = 0, g_end = 0, tpw = 1;
  if (p.dyn_split) {
    tpw = p.seg_glob[0];
    dyn_bh = p.wg_tab[blockIdx.x];
    g = (long long)blockIdx.x * tpw;
    g_end = g + tpw;
  }
  for (bool first_piece = true;; first_piece = false) {
  int bh, split, c0, c1_max;
  if (!p.dyn_split) {
    if (!first_piece) break;
    bh = blockIdx.y;
    // Which split of the head this workgroup takes rotates with the head: workgroups go to the
    // eight compute dies round-robin by their linear index, and a fixed blockIdx.x -> split
    // mapping would hand the dies unequal work when the splits near a sequence's end are short.
    split = (int)((blockIdx.x + (unsigned)bh) % gridDim.x);
    c0 = split * split_len;
    c1_max = c0 + split_len;
  } else {
    if (dyn_bh < 0 || dyn_bh >= p.B * p.Hkv || g >= g_end) break;
    const SegTab t = p.seg_tab[dyn_bh];
    if (t.first >= g_end) break;
    if (g >= t.first + t.tiles) { ++dyn_bh; continue; }     // past this head (or it is empty)
    const long long t0 = max(g, t.first), t1 = min(g_end, t.first + t.tiles);
    bh = dyn_bh;
    split = (int)((long long)blockIdx.x - t.first / tpw);
    c0 = (int)(t0 - t.first) * kTN;
    c1_max = (int)(t1 - t.first) * kTN;
    g = t1;
  }
  const int b = bh / p.Hkv, hk = bh % p.Hkv;
  const int N = seq_len(p, b);
  // with the caller's normalisers this is the first kernel of the call: it clears the
  // selection's counters (otherwise the merge of the row statistics does)
  if (COLSUM && p.lse_in && split == 0) reset_counters(p, bh);
  if (c0 >= N) continue;
  const int c1 = min(N, c1_max);
  const int ntiles = (c1 - c0 + kTN - 1) / kTN;
  const int P = p.wic ? N - p.W : N;    // keys below P are visible to every row

  const unsigned char* Kb = reinterpret_cast<const unsigned char*>(p.K) +
                            ((int64_t)b * p.ksb + (int64_t)hk * p.ksh) * 2;
  const int64_t krow = p.ksn * 2;
  float* a_out = p.a + (int64_t)bh * p.cap;

  const int rg_first = MODE == 0 ? blockIdx.z * ROWS : 0, rg_step = MODE == 0 ? gridDim.z * ROWS : ROWS;
  for (int rg0 = rg_first; rg0 < p.R; rg0 += rg_step) {
    // ---- sweep over the key tiles of this split --------------------------------------
    // K tiles go from global memory straight into LDS (global_load_lds_dwordx4: lane L of
    // a wave fills the 16-byte slot base + 16 L), kNBuf-1 tiles ahead of the math.  The
    // XOR swizzle that keeps the fragment reads conflict-free is applied on the global
    // side: the lane that owns slot (row, pc) fetches chunk pc ^ (row & 15) of that row.
    // this lane's piece of tile 0, per load: tiles that lie inside the cache are then one
    // 64-bit add away (the tile stride is a scalar); only the last tile clamps its rows
    const unsigned char* kp0[LPT];
#pragma unroll
    for (int u = 0; u < LPT; ++u) {
      const int slot = (wave * LPT + u) * kWave + lane;      // 16-byte slot inside the tile
      const int row = slot / kChunks, pc = slot % kChunks;
      kp0[u] = Kb + (int64_t)(c0 + row) * krow + ((pc ^ (row & 15)) << 4);
    }
    const int64_t ktile = (int64_t)kTN * krow;
    auto issue = [&](int t, int buf) {
      const uint32_t dst = lds_addr(&Ks[0][0]) + (uint32_t)(buf * kTN * kRowBytes + wave * LPT * kWave * 16);
      if (c0 + (t + 1) * kTN <= N) {
        const int64_t off = (int64_t)t * ktile;
#pragma unroll
        for (int u = 0; u < LPT; ++u) load_to_lds16(kp0[u] + off, dst + u * kWave * 16);
      } else {
#pragma unroll
        for (int u = 0; u < LPT; ++u) {
          const int slot = (wave * LPT + u) * kWave + lane;
          const int row = slot / kChunks, pc = slot % kChunks;
          const int j = min(c0 + t * kTN + row, N - 1);      // rows past the end repeat the last one
          load_to_lds16(Kb + j * krow + ((pc ^ (row & 15)) << 4), dst + u * kWave * 16);
        }
      }
    };
    // The first two K tiles are requested before anything else, so that their latency
    // overlaps the set-up below.
    __syncthreads();                     // previous row group is done with LDS
    if (QLDS) {
      // The Q rows of the group take the same road as the K tiles: whole 256-byte rows by
      // DMA into LDS (16 lanes per row, swizzled), fragments by ds_read_b128.  Loading the
      // fragments straight from global memory (32 rows x 32 bytes per instruction) keeps
      // the address unit busy for several microseconds per workgroup.
      // A load instruction of a wave covers four consecutive rows, its next one the four after
      // them: the lane's address is worked out once and then stepped (window position + 4, with
      // the carry into the next query head), the multiplications stay out of the loop.
      constexpr int kQLoads = ROWS * kChunks / kThreads;
      const int row0 = wave * kQLoads * (kWave / kChunks) + lane / kChunks, pc = lane % kChunks;
      int qg, qiw;
      divmod_w(p, rg0 + row0, qg, qiw);
      const unsigned char* qp = reinterpret_cast<const unsigned char*>(p.q) +
          ((int64_t)b * p.qsb + (int64_t)(hk * p.G + qg) * p.qsh + (int64_t)qiw * p.qsw) * 2;
      const int64_t q_step = (int64_t)(kWave / kChunks) * p.qsw * 2, q_carry = (p.qsh - (int64_t)p.W * p.qsw) * 2;
      const uint32_t q_dst = lds_addr(&Qs[0]) + (uint32_t)(wave * kQLoads * kWave * 16);
#pragma unroll 1
      for (int u = 0; u < kQLoads; ++u) {
        const int row = row0 + u * (kWave / kChunks);
        if (rg0 + row < p.R)              // rows past R are not fetched; their fragments are zeroed
          load_to_lds16(qp + ((pc ^ (row & 15)) << 4), q_dst + u * kWave * 16);
        qp += q_step;
        qiw += kWave / kChunks;
        while (qiw >= p.W) { qiw -= p.W; qp += q_carry; }
      }
    }
    for (int t = 0; t < kNBuf - 1 && t < ntiles; ++t) issue(t, t);
    // ---- per-row-group set-up: Q fragments, window positions, normalisers ----------
    for (int i = tid; i < ROWS; i += kThreads) {
      int g_unused, iw_i;
      divmod_w(p, rg0 + i, g_unused, iw_i);
      iw_lds[i] = (rg0 + i) < p.R ? iw_i : -1;
      if (COLSUM) lse_lds[i] = (rg0 + i) < p.R ? row_lse2(p, b, hk, bh, rg0 + i) : INFINITY;
    }
    bf16x8 qf[RBW][8];
    // normalisers of the rows a lane meets in sweep 2: in registers, or (fused sweep, which
    // is short of registers) read from LDS block by block, four consecutive rows per read
    constexpr bool LSE_REGS = COLSUM && !FUSE;
    float lse[LSE_REGS ? RBW : 1][16];
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
        if (!QLDS) {
          const unsigned char* qp = reinterpret_cast<const unsigned char*>(p.q) +
              ((int64_t)b * p.qsb + (int64_t)(hk * p.G + g) * p.qsh + (int64_t)iw * p.qsw) * 2 + (lane >> 5) * 16;
#pragma unroll
          for (int ks = 0; ks < 8; ++ks)
            qf[rb][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(qp + ks * 32));
        }
        nvis_row[rb] = p.wic ? P + iw + 1 : N;
      } else {
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qf[rb][ks] = __builtin_bit_cast(bf16x8, make_uint4(0, 0, 0, 0));
      }
    }
    if (QLDS) {
      // the Q rows are older than the K tiles requested after them
      if (ntiles >= kNBuf - 1) wait_vmcnt<(kNBuf - 1) * LPT>(); else wait_vmcnt<0>();
    }
    if (COLSUM || QLDS) __syncthreads();
    if (LSE_REGS) {
#pragma unroll
      for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
        for (int i = 0; i < 16; ++i) lse[rb][i] = lse_lds[(wr * RBW + rb) * 32 + m_of(i, lane)];
    }
    if (QLDS) {
#pragma unroll
      for (int rb = 0; rb < RBW; ++rb) {
        const int rl = (wr * RBW + rb) * 32 + (lane & 31);
        if (rg0 + rl < p.R) {
#pragma unroll
          for (int ks = 0; ks < 8; ++ks)
            qf[rb][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(&Qs[swz(rl, 2 * ks + (lane >> 5))]));
        }
      }
    }
    // One 64-key tile out of LDS buffer `buf`.  TAIL: some logits of the tile are masked
    // (keys past the end of the cache, or window keys a row must not see).
    // `mid` runs once, right after the matrix instructions of the first key block have been
    // issued: work that waits on LDS round trips of its own goes there, under their shadow.
    auto tile = [&](auto tail_tag, int buf, int abuf, int tile0, auto&& mid) {
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
        if (kbi == 0) mid();
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
            float nrm[16];
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
              if (LSE_REGS) {
#pragma unroll
                for (int i = 0; i < 4; ++i) nrm[4 * g4 + i] = lse[LSE_REGS ? rb : 0][4 * g4 + i];
              } else {
                const float4 v = *reinterpret_cast<const float4*>(&lse_lds[rl + 8 * g4 + 4 * (lane >> 5)]);
                nrm[4 * g4] = v.x; nrm[4 * g4 + 1] = v.y; nrm[4 * g4 + 2] = v.z; nrm[4 * g4 + 3] = v.w;
              }
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(acc[rb][i], p.c2, -nrm[i]));
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
    auto math = [&](int t, int buf, int abuf, auto&& mid) {
      const int tile0 = c0 + t * kTN;
      if (tile0 + kTN > min(P, N)) tile(std::true_type{}, buf, abuf, tile0, mid);
      else                         tile(std::false_type{}, buf, abuf, tile0, mid);
    };
    // ---- FUSE: the value sum rides along (Sec. 3.2: o = sum_j w_j v_j) ---------------------
    // Value step s covers the 64 keys c0 + 64 s - halo ... (shifted down by the pooling
    // half-width, so that every neighbour it needs belongs to tiles <= s).  The first wave
    // weighs its keys right after it has reduced the column sums of tile s (iteration s+1);
    // the V rows come straight into LDS like the K tiles, requested in iteration s+1 as well,
    // and every wave adds up the rows it fetched itself in iteration s+2.  Keys within `halo`
    // of a chunk boundary need a neighbouring workgroup's column sums and are left to the
    // kernel that adds the partial sums up.
    const bool vlast = FUSE && rg0 + ROWS >= p.R;           // column sums are final in this group
    constexpr int RW = LPT * 4;                             // value rows per wave per step
    const int halo = p.halo;
    const int lo = min(p.ph, N), hi = max(lo, N - p.pt);   // scored rows [lo,hi)
    float vacc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    float vz = 0.f;
    auto flush_a = [&](int t, int buf) {                     // after the barrier of step t+1
      const int tile0 = c0 + t * kTN;
      if (COLSUM && tid < kTN) {
        float s = 0.f;
        if (tile0 + tid < c1) {
#pragma unroll
          for (int w = 0; w < WR; ++w) s += a_lds[buf][w][tid];
          if (rg0 > 0) s += a_out[tile0 + tid];                // later row groups add on
          a_out[tile0 + tid] = s;
        }
        if (vlast) {
          af[(t & 3) * kTN + tid] = s;
          // base score and weight of key tid of value step t (same wave: the LDS writes above
          // are visible to the reads below without a barrier)
          const int j = tile0 - halo + tid;
          const bool mine = j >= c0 + halo && j < c1 - halo;
          const bool scored = mine && j >= lo && j < hi;
          float hj = 0.f;
          if (mine) {
            hj = af[(j - c0) & (4 * kTN - 1)];
            if (p.base_mode == CAOTE_BASE_H2O) {
              hj += bs[t & 1][tid];
            } else if (p.base_mode == CAOTE_BASE_SNAPKV && scored) {
              // eight neighbours per round of LDS reads (indices past the window's end repeat
              // its last key, which changes no maximum): pool width 7 is one round trip
              const int t0 = max(lo, j - halo), t1 = min(hi - 1, j + halo);
              for (int tb = t0; tb <= t1; tb += 8) {
                float x[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) x[u] = af[(min(tb + u, t1) - c0) & (4 * kTN - 1)];
                hj = fmaxf(fmaxf(fmaxf(hj, x[0]), fmaxf(x[1], x[2])),
                           fmaxf(fmaxf(x[3], x[4]), fmaxf(fmaxf(x[5], x[6]), x[7])));
              }
            }
            p.h[(int64_t)bh * p.cap + j] = hj;
          }
          hw[(t & 3) * kTN + tid] = scored ? (p.variant == CAOTE_FAST ? 1.f : hj) : 0.f;
          vz += scored ? hj : 0.f;
        }
      }
    };
    const unsigned char* Vb = reinterpret_cast<const unsigned char*>(p.V) +
                              ((int64_t)b * p.vsb + (int64_t)hk * p.vsh) * 2;
    const int64_t vrow = p.vsn * 2;
    const int jrow = c0 - halo + wave * RW + (lane >> 4);    // this lane's row of step 0, u = 0
    const unsigned char* vlane = Vb + (int64_t)jrow * vrow + ((lane & 15) << 4);
    const unsigned char* vp0[LPT];
#pragma unroll
    for (int u = 0; u < LPT; ++u) vp0[u] = vlane + (int64_t)(u * 4) * vrow;
    const int64_t vtile = (int64_t)kTN * vrow;
    auto v_issue = [&](int s, unsigned char* vs) {
      const int jw0 = c0 - halo + wave * RW + s * kTN;        // the wave's first row of step s
      const uint32_t dst = lds_addr(vs) + (uint32_t)(wave * LPT * kWave * 16);
      if (jw0 >= 0 && jw0 + RW <= N) {                        // wave-uniform: no clamping
        const int64_t off = (int64_t)s * vtile;
#pragma unroll
        for (int u = 0; u < LPT; ++u) load_to_lds16(vp0[u] + off, dst + u * kWave * 16);
      } else {
        const int j0 = jrow + s * kTN;
#pragma unroll
        for (int u = 0; u < LPT; ++u) {
          const int j = min(max(j0 + u * 4, 0), N - 1);
          load_to_lds16(Vb + j * vrow + ((lane & 15) << 4), dst + u * kWave * 16);
        }
      }
    };
    auto base_issue = [&](int s) {                           // first wave: H2O accumulator rows of step s
      const int j = min(max(c0 + s * kTN - halo + lane, 0), N - 1);
      load_to_lds4(p.base + (int64_t)bh * p.cap + j, __builtin_amdgcn_readfirstlane(lds_addr(&bs[s & 1][0])));
    };
    // The V rows of a step and their weights come out of LDS in v_load; v_fma adds them up
    // later, once the reads have surely returned.
    uint4 vraw[LPT];
    float vw[LPT];
    auto v_load = [&](int s, const unsigned char* vs) {
#pragma unroll
      for (int u = 0; u < LPT; ++u) {
        vw[u] = hw[(s & 3) * kTN + wave * RW + u * 4 + (lane >> 4)];
        vraw[u] = *reinterpret_cast<const uint4*>(vs + ((wave * LPT + u) * kWave + lane) * 16);
      }
    };
    auto v_fma = [&]() {
#pragma unroll
      for (int u = 0; u < LPT; ++u) {
        const float w = vw[u];
        const uint4 raw = vraw[u];
        vacc[0] = fmaf(w, __uint_as_float(raw.x << 16), vacc[0]);
        vacc[1] = fmaf(w, __uint_as_float(raw.x & 0xffff0000u), vacc[1]);
        vacc[2] = fmaf(w, __uint_as_float(raw.y << 16), vacc[2]);
        vacc[3] = fmaf(w, __uint_as_float(raw.y & 0xffff0000u), vacc[3]);
        vacc[4] = fmaf(w, __uint_as_float(raw.z << 16), vacc[4]);
        vacc[5] = fmaf(w, __uint_as_float(raw.z & 0xffff0000u), vacc[5]);
        vacc[6] = fmaf(w, __uint_as_float(raw.w << 16), vacc[6]);
        vacc[7] = fmaf(w, __uint_as_float(raw.w & 0xffff0000u), vacc[7]);
      }
    };
    auto v_consume = [&](int s, const unsigned char* vs) { v_load(s, vs); v_fma(); };
    // Make the compiler finish its own global loads (Q fragments, normalisers) here: a wait
    // it placed inside the tile loop would also drain the LDS loads that must stay in flight.
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb) {
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) asm volatile("" : : "v"(qf[rb][ks]));
      if (LSE_REGS) {
#pragma unroll
        for (int i = 0; i < 16; ++i) asm volatile("" : : "v"(lse[rb][i]));
      }
    }
    if (vlast && p.base_mode == CAOTE_BASE_H2O && wave == 0) base_issue(0);
    int buf = 0;
    for (int t = 0; t < ntiles; ++t) {
      // this wave's share of tile t has landed once only the loads requested after it are still
      // in flight (loads complete in order; a store in between cannot hide a load): the K tile
      // t+1 and, in the fused sweep, the V rows of step t-1, both requested in iteration t-1
      if (vlast && t >= 1) {
        if (t + 1 < ntiles) wait_vmcnt<2 * LPT>(); else wait_vmcnt<LPT>();
      } else {
        if (t + 1 < ntiles) wait_vmcnt<LPT>(); else wait_vmcnt<0>();
      }
      __syncthreads();                   // ... and so has everyone else's; tile t-1 is done with
      const int spare = buf == 0 ? kNBuf - 1 : buf - 1;     // ring slot of tile t-1
      if (t + kNBuf - 1 < ntiles) issue(t + kNBuf - 1, spare);
      // The first wave turns the column sums of tile t-1 into weights (for value step t-1,
      // next iteration).  Step t-2 of the value sum: its rows and weights are read out of LDS
      // now and added up after this tile's matrix instructions have been issued.  The V rows of
      // step t then go into the slot that step t-2 has been read from: two iterations pass
      // between the request and the use.
      if (t > 0) flush_a(t - 1, (t - 1) & 1);
      if (vlast && t >= 2) v_load(t - 2, Vs[t & 1]);
      math(t, buf, t & 1, [&]() {
        if (vlast) {
          if (t >= 2) v_fma();
          v_issue(t, Vs[t & 1]);
          if (p.base_mode == CAOTE_BASE_H2O && wave == 0 && t + 1 < ntiles) base_issue(t + 1);
        }
      });
      buf = buf + 1 == kNBuf ? 0 : buf + 1;
    }
    if (vlast) wait_vmcnt<0>();
    __syncthreads();
    flush_a(ntiles - 1, (ntiles - 1) & 1);
    if (vlast) {
      if (ntiles >= 2) v_consume(ntiles - 2, Vs[ntiles & 1]);
      __syncthreads();                   // the weights of the last step are in LDS
      v_consume(ntiles - 1, Vs[(ntiles - 1) & 1]);
      // partial sums of this chunk: over the four teams of a wave, then over the waves
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        vacc[e] += __shfl_xor(vacc[e], 16, kWave);
        vacc[e] += __shfl_xor(vacc[e], 32, kWave);
      }
#pragma unroll
      for (int o = 32; o >= 1; o >>= 1) vz += __shfl_xor(vz, o, kWave);
      if (lane < 16) {
#pragma unroll
        for (int e = 0; e < 8; ++e) red[wave][lane * 8 + e] = vacc[e];
        if (tid == 0) red[0][kD] = vz;
      }
      __syncthreads();
      if (tid < kD) {
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < NWV; ++w) sum += red[w][tid];
        p.opart[((int64_t)bh * p.n_vpart + split) * kD + tid] = sum;
      } else if (tid == kD) {
        p.zpart[(int64_t)bh * p.n_vpart + split] = red[0][kD];
      }
    }
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
        float* st = p.stats + (((int64_t)bh * p.n_split0 + split) * p.Rp + rg0 + rl) * 2;
        st[0] = M; st[1] = L;
      }
    }
  }
  }   // pieces of work
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
  const int ns = split_count(p, bh, N, p.split_len0);
  const float* st = p.stats + ((int64_t)bh * p.n_split0 * p.Rp + r) * 2;
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

// The same merge with one thread per query row: consecutive threads read consecutive rows of a
// split's statistics, so a batch of many heads moves whole cache lines.
__global__ __launch_bounds__(kMergeThreads) void k_merge_stats_rows(const Params p) {
  const int bh = blockIdx.y, b = bh / p.Hkv;
  if (blockIdx.x == 0) reset_counters(p, bh);
  const int r = blockIdx.x * kMergeThreads + threadIdx.x;
  if (r >= p.R) return;
  const int N = seq_len(p, b);
  const int ns = split_count(p, bh, N, p.split_len0);
  const float2* st = reinterpret_cast<const float2*>(p.stats) + (int64_t)bh * p.n_split0 * p.Rp + r;
  float M = -INFINITY;
#pragma unroll 8
  for (int s = 0; s < ns; ++s) M = fmaxf(M, st[(int64_t)s * p.Rp].x);
  float L = 0.f;
#pragma unroll 8
  for (int s = 0; s < ns; ++s) {
    const float2 ml = st[(int64_t)s * p.Rp];
    if (ml.x > -INFINITY) L += ml.y * exp2f(ml.x - M);
  }
  p.lse2[(int64_t)bh * p.Rp + r] = L > 0.f ? M + log2f(L) : INFINITY;
}

// ---------------------------------------------------------------------------------------
// Few query rows (R <= 8: decode-time eviction, Sec. 2 generation) on the matrix cores.
// One sweep over K that stores the scaled logits (see score_small.hip for why) and keeps the
// running (max, sum) of each row.  The R rows are padded to one 32-row block: the MFMA does
// the 128-long dot products and their reduction, which on the vector ALUs cost 25
// instructions per key; the padding is free, the matrix pipe is idle otherwise.
// Every wave works alone: it fetches its own 32-key blocks into a private ring of LDS slots
// (DMA, swizzled), so there is no barrier in the loop.  Keys on M, rows on N: lane l holds
// 16 keys of row l % 32, and only lanes with l % 32 < R carry anything.
// ---------------------------------------------------------------------------------------
constexpr int kFewWaves = 2;              // waves per workgroup
constexpr int kFewSlots = 3;              // LDS slots (8 KiB) per wave: two blocks in flight
constexpr int kFewBlock = 32;             // keys per block

__global__ __launch_bounds__(kFewWaves * kWave) void k_rowstats_few_mfma(const Params p) {
  const int bh = blockIdx.y, b = bh / p.Hkv, hk = bh % p.Hkv;
  const int N = seq_len(p, b);
  const int c0 = blockIdx.x * p.split_len;
  if (blockIdx.x == 0 && p.lse_in) reset_counters(p, bh);   // no merge kernel follows then
  if (c0 >= N) return;
  const int c1 = min(N, c0 + p.split_len);
  const int nblk = (c1 - c0 + kFewBlock - 1) / kFewBlock;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int P = p.wic ? N - p.W : N;
  const int n = lane & 31;                // query row of this lane

  __shared__ __attribute__((aligned(16))) unsigned char ring[kFewWaves][kFewSlots][kFewBlock * kRowBytes];
  __shared__ float st_lds[kFewWaves][8][2];

  const unsigned char* Kb = reinterpret_cast<const unsigned char*>(p.K) +
                            ((int64_t)b * p.ksb + (int64_t)hk * p.ksh) * 2;
  const int64_t krow = p.ksn * 2;
  // block i of this wave is block wave + kFewWaves * i of the chunk
  const int my_blocks = nblk > wave ? (nblk - wave + kFewWaves - 1) / kFewWaves : 0;
  auto issue = [&](int i, int slot) {
    const int j0 = c0 + (wave + kFewWaves * i) * kFewBlock;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int s16 = u * kWave + lane;                       // 16-byte slot inside the block
      const int row = s16 / kChunks, pc = s16 % kChunks;
      const int j = min(j0 + row, N - 1);                     // rows past the end repeat the last one
      load_to_lds16(Kb + j * krow + ((pc ^ (row & 15)) << 4),
                    __builtin_amdgcn_readfirstlane(lds_addr(&ring[wave][slot][u * kWave * 16])));
    }
  };
  for (int i = 0; i < kFewSlots - 1 && i < my_blocks; ++i) issue(i, i);

  bf16x8 qf[8];
  int nvis = 0;                           // keys visible to this lane's row (0: no such row)
  if (n < p.R) {
    int g, iw;
    divmod_w(p, n, g, iw);
    const unsigned char* qp = reinterpret_cast<const unsigned char*>(p.q) +
        ((int64_t)b * p.qsb + (int64_t)(hk * p.G + g) * p.qsh + (int64_t)iw * p.qsw) * 2 + (lane >> 5) * 16;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(qp + ks * 32));
    nvis = p.wic ? P + iw + 1 : N;
  } else {
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = __builtin_bit_cast(bf16x8, make_uint4(0, 0, 0, 0));
  }
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) asm volatile("" : : "v"(qf[ks]));   // the compiler's waits end here

  float* Srow = p.S + ((int64_t)bh * p.s_rows + n) * p.s_pitch;      // row n of the stored logits
  float m_run = -INFINITY, l_run = 0.f;
  int slot = 0;
  for (int i = 0; i < my_blocks; ++i) {
    const int ahead = min(kFewSlots - 2, my_blocks - 1 - i);         // blocks requested after block i
    if (i + kFewSlots - 1 < my_blocks) issue(i + kFewSlots - 1, slot == 0 ? kFewSlots - 1 : slot - 1);
    // (the slot of block i-1: this wave has read it)
    if (i + kFewSlots - 1 < my_blocks) wait_vmcnt<(kFewSlots - 1) * 8>();
    else if (ahead >= 1) wait_vmcnt<8>();
    else wait_vmcnt<0>();
    const unsigned char* tile = &ring[wave][slot][0];
    bf16x8 kf[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
      kf[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(&tile[swz(n, 2 * ks + (lane >> 5))]));
    f32x16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[ks], acc, 0, 0, 0);
    const int jb = c0 + (wave + kFewWaves * i) * kFewBlock;
    float t[16];
    float mx = -INFINITY;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int j = jb + m_of(e, lane);
      t[e] = (j < c1 && j < nvis) ? acc[e] * p.c2 : -INFINITY;
      mx = fmaxf(mx, t[e]);
    }
    if (n < p.s_rows) {                    // rows R..s_rows-1 are stored as -inf: exp2 gives 0
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {     // four consecutive keys per store
        const int j = jb + 8 * g4 + 4 * (lane >> 5);
        if (j + 3 < c1) {
          *reinterpret_cast<float4*>(Srow + j) = make_float4(t[4 * g4], t[4 * g4 + 1], t[4 * g4 + 2], t[4 * g4 + 3]);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (j + e < c1) Srow[j + e] = t[4 * g4 + e];
        }
      }
    }
    const float mn = fmaxf(m_run, mx);
    if (mn > -INFINITY) {
      float ssum = 0.f;
#pragma unroll
      for (int e = 0; e < 16; ++e) ssum += __builtin_amdgcn_exp2f(t[e] - mn);
      l_run = l_run * __builtin_amdgcn_exp2f(m_run - mn) + ssum;
      m_run = mn;
    }
    slot = slot + 1 == kFewSlots ? 0 : slot + 1;
  }
  // ---- the two half-waves, then the waves ------------------------------------------------------
  {
    const float m2 = __shfl_xor(m_run, 32, kWave), l2 = __shfl_xor(l_run, 32, kWave);
    const float M = fmaxf(m_run, m2);
    float L = 0.f;
    if (m_run > -INFINITY) L += l_run * exp2f(m_run - M);
    if (m2 > -INFINITY) L += l2 * exp2f(m2 - M);
    if (lane < 8) { st_lds[wave][lane][0] = M; st_lds[wave][lane][1] = L; }
  }
  __syncthreads();
  if (tid < p.R) {
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < kFewWaves; ++w) M = fmaxf(M, st_lds[w][tid][0]);
    float L = 0.f;
#pragma unroll
    for (int w = 0; w < kFewWaves; ++w)
      if (st_lds[w][tid][0] > -INFINITY) L += st_lds[w][tid][1] * exp2f(st_lds[w][tid][0] - M);
    float* st = p.stats + (((int64_t)bh * p.n_split + blockIdx.x) * p.Rp + tid) * 2;
    st[0] = M; st[1] = L;
  }
}

}  // namespace

// Few-row key sweep on the matrix cores.  Requires: bf16, head_dim 128, R <= 8, split_len a
// multiple of 32.
hipError_t launch_score_few_mfma(const Params& p, hipStream_t s, PhaseHook* hook) {
  hipLaunchKernelGGL(k_rowstats_few_mfma, dim3(p.n_split, p.B * p.Hkv), dim3(kFewWaves * kWave), 0, s, p);
  if (mark(hook, "key_rowstats")) return hipGetLastError();
  // the caller's normalisers: nothing to merge; short caches: the value kernel merges
  if (p.lse_in || p.merge_in_vside) return hipGetLastError();
  return launch_merge_stats(p, s, hook);
}


hipError_t launch_merge_stats(const Params& p, hipStream_t s, PhaseHook* hook) {
  // few rows in all: a wave per row keeps the launch short; many (batches): a thread per row,
  // whose loads coalesce over the rows
  if ((long long)p.B * p.Hkv * p.R >= 16384)
    hipLaunchKernelGGL(k_merge_stats_rows, dim3((p.R + kMergeThreads - 1) / kMergeThreads, p.B * p.Hkv),
                       dim3(kMergeThreads), 0, s, p);
  else
    hipLaunchKernelGGL(k_merge_stats_wave, dim3((p.R + 3) / 4, p.B * p.Hkv), dim3(kMergeThreads), 0, s, p);
  if (mark(hook, "merge_stats")) return hipGetLastError();
  return hipGetLastError();
}

namespace {

// Ragged batches: cuts the key tiles of all heads, laid end to end in (sequence, head) order,
// into p.dyn_wgs equal shares and writes the tables the sweeps read (Params::seg_tab, wg_tab,
// seg_glob).  One workgroup; the batch has at most kDynMaxBatch sequences.
__global__ __launch_bounds__(kDynMaxBatch) void k_plan_splits(const Params p) {
  __shared__ long long pre[kDynMaxBatch + 1];     // tiles of the sequences before b (one head each)
  __shared__ int wave_tot[kDynMaxBatch / kWave];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int nt = tid < p.B ? (seq_len(p, tid) + kTN - 1) / kTN : 0;
  int inc = nt;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const int up = __shfl_up(inc, o, kWave);
    if (lane >= o) inc += up;
  }
  if (lane == kWave - 1) wave_tot[wv] = inc;
  __syncthreads();
  long long before = 0;
  for (int w = 0; w < wv; ++w) before += wave_tot[w];
  pre[tid] = before + inc - nt;
  if (tid == kDynMaxBatch - 1) pre[kDynMaxBatch] = before + inc;
  __syncthreads();
  const long long T = pre[kDynMaxBatch] * p.Hkv;          // (threads past the batch added nothing)
  long long tpw = (T + p.dyn_wgs - 1) / p.dyn_wgs;
  tpw = max(tpw, (long long)p.dyn_min_tiles);
  if (tid == 0) p.seg_glob[0] = (int)tpw;
  for (int bh = tid; bh < p.B * p.Hkv; bh += kDynMaxBatch) {
    const int b = bh / p.Hkv, hk = bh % p.Hkv;
    const int n = (int)(pre[b + 1] - pre[b]);
    SegTab t;
    t.first = pre[b] * p.Hkv + (long long)hk * n;
    t.tiles = n;
    t.pad = 0;
    p.seg_tab[bh] = t;
  }
  for (int w = tid; w < p.dyn_wgs; w += kDynMaxBatch) {
    const long long g0 = (long long)w * tpw;
    int first = -1;
    if (g0 < T) {
      int lo = 0, hi = p.B;                 // the sequence b with pre[b] * Hkv <= g0 < pre[b+1] * Hkv
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (pre[mid] * p.Hkv <= g0) lo = mid; else hi = mid;
      }
      const long long n = pre[lo + 1] - pre[lo];
      first = lo * p.Hkv + (int)((g0 - pre[lo] * p.Hkv) / n);
    }
    p.wg_tab[w] = first;
  }
}

template <int NWV, int WR, int RBW>
hipError_t launch_cfg(const Params& p, hipStream_t s, PhaseHook* hook) {
  if (p.dyn_split) {
    hipLaunchKernelGGL(k_plan_splits, dim3(1), dim3(kDynMaxBatch), 0, s, p);
    if (mark(hook, "plan_splits")) return hipGetLastError();
  }
  const dim3 grid = p.dyn_split ? dim3(p.dyn_wgs) : dim3(p.n_split, p.B * p.Hkv);
  if (!p.lse_in) {                       // else the caller's attention pass has done sweep 1
    const dim3 grid0 = p.dyn_split ? dim3(p.dyn_wgs, 1, p.n_rg0) : dim3(p.n_split0, p.B * p.Hkv, p.n_rg0);
    hipLaunchKernelGGL((k_logits_mfma<NWV, WR, RBW, 0>), grid0, dim3(NWV * kWave), 0, s, p);
    if (mark(hook, "key_rowstats")) return hipGetLastError();
    const hipError_t e = launch_merge_stats(p, s, hook);
    if (e != hipSuccess || full(hook)) return e;
  }
  if (p.fuse_v) hipLaunchKernelGGL((k_logits_mfma<NWV, WR, RBW, 2>), grid, dim3(NWV * kWave), 0, s, p);
  else          hipLaunchKernelGGL((k_logits_mfma<NWV, WR, RBW, 1>), grid, dim3(NWV * kWave), 0, s, p);
  if (mark(hook, "key_colsum")) return hipGetLastError();
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
