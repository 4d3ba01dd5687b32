// In-place cache update after selection (Sec. 2: attention afterwards uses only the
// kept rows i_1..i_b): rows of K, V and the H2O accumulator move to the front of
// their slab.
//
// kept_idx is ascending, so rank i reads row kept_idx[i] >= i and writes row i; a
// row inside the destination range [0, n_keep) may be overwritten by one rank while
// another rank still has to read it.  Those source rows are first gathered into staging
// memory (first kernel); the second kernel writes every destination row, from staging or,
// for source rows at or beyond n_keep, which nobody writes, straight from the cache (stream
// order is the barrier).  On a long cache cut to a small budget nearly all kept rows come
// from beyond n_keep and move once.  Rows that already sit at their rank are not touched.
//
// Evict-one sequences in SWAP_LAST mode move a single row (k_swap_last): the last row drops
// into the hole.  A sequence that evicts any other number of tokens is compacted stably.
// FILL mode generalises the swap to any number of evictions (k_fill_holes).
#include "common.hpp"

namespace caote {
namespace {

constexpr int kThreads = 256;

// Source row of rank i, or -1 if rank i does not move.
__device__ __forceinline__ int source_row(const Params& p, const int32_t* idx, int i, int N) {
  const int n_keep = min(N, p.budget);
  if (i >= n_keep) return -1;
  const int src = idx[i];
  if (p.mode == CAOTE_COMPACT_SWAP_LAST && N - n_keep == 1) return -1;   // k_swap_last's job
  return src == i ? -1 : src;
}

// Evict-one sequences in SWAP_LAST mode: the kept list is 0..N-2 with one index missing;
// the last row drops into that hole.  One workgroup per (sequence, head); source and
// destination are different rows, so no staging is needed.
__global__ __launch_bounds__(kThreads) void k_swap_last(const Params p, int row_bytes) {
  const int bh = blockIdx.x, b = bh / p.Hkv, hk = bh % p.Hkv;
  const int N = seq_len(p, b);
  const int n_keep = min(N, p.budget);
  if (N - n_keep != 1) return;
  const int32_t* idx = p.kept + (int64_t)bh * p.budget;
  // The hole is the first rank whose index is not its own; ranks below it hold their own index,
  // ranks from it on hold index + 1, so two rounds of loads find it: the segment (one probe per
  // thread, at the end of its segment), then the rank inside the segment.
  __shared__ int s_seg, s_hole;
  if (threadIdx.x == 0) { s_seg = kThreads; s_hole = N - 1; }   // nothing missing: the last row goes
  __syncthreads();
  const int seg = (n_keep + kThreads - 1) / kThreads;
  {
    const int e = min(n_keep, (threadIdx.x + 1) * seg) - 1;     // last rank of this thread's segment
    if (threadIdx.x * seg < n_keep && idx[e] != e) atomicMin(&s_seg, (int)threadIdx.x);
  }
  __syncthreads();
  if (s_seg < kThreads) {
    const int i0 = s_seg * seg, i1 = min(n_keep, i0 + seg);
    for (int i = i0 + threadIdx.x; i < i1; i += kThreads)
      if (idx[i] != i) atomicMin(&s_hole, i);
  }
  __syncthreads();
  const int hole = s_hole;
  if (hole == N - 1) return;
  const int esz = p.dtype == CAOTE_F32 ? 4 : 2;
  char* Kb = reinterpret_cast<char*>(p.K) + ((int64_t)b * p.ksb + (int64_t)hk * p.ksh) * esz;
  char* Vb = reinterpret_cast<char*>(p.V) + ((int64_t)b * p.vsb + (int64_t)hk * p.vsh) * esz;
  const int64_t krow = p.ksn * esz, vrow = p.vsn * esz;
  const int cpr = row_bytes / 16;
  const int t = threadIdx.x;
  if (t < cpr)
    *reinterpret_cast<uint4*>(Kb + hole * krow + t * 16) = *reinterpret_cast<const uint4*>(Kb + (N - 1) * krow + t * 16);
  else if (t < 2 * cpr)
    *reinterpret_cast<uint4*>(Vb + hole * vrow + (t - cpr) * 16) =
        *reinterpret_cast<const uint4*>(Vb + (N - 1) * vrow + (t - cpr) * 16);
  else if (t == 2 * cpr && p.base)
    p.base[(int64_t)bh * p.cap + hole] = p.base[(int64_t)bh * p.cap + N - 1];
}

// dir 0: cache -> staging, dir 1: staging -> cache.
template <int DIR>
__global__ __launch_bounds__(kThreads) void k_move_rows(const Params p, int row_bytes) {
  const int bh = blockIdx.y, b = bh / p.Hkv, hk = bh % p.Hkv;
  const int N = seq_len(p, b);
  const int cpr = row_bytes / 16;                     // 16-byte chunks per row
  const int64_t id = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  const int i = (int)(id / cpr), ch = (int)(id % cpr);
  if (i >= p.budget) return;
  const int32_t* idx = p.kept + (int64_t)bh * p.budget;
  const int src = source_row(p, idx, i, N);
  if (src < 0) return;
  const bool direct = src >= min(N, p.budget);        // source row outside the destination range
  if (DIR == 0 && direct) return;

  const int esz = p.dtype == CAOTE_F32 ? 4 : 2;
  char* Kb = reinterpret_cast<char*>(p.K) + ((int64_t)b * p.ksb + (int64_t)hk * p.ksh) * esz;
  char* Vb = reinterpret_cast<char*>(p.V) + ((int64_t)b * p.vsb + (int64_t)hk * p.vsh) * esz;
  char* stK = reinterpret_cast<char*>(p.stage) + (int64_t)bh * p.budget * row_bytes;
  char* stV = stK + (int64_t)p.B * p.Hkv * p.budget * row_bytes;
  float* stB = reinterpret_cast<float*>(reinterpret_cast<char*>(p.stage) +
                                        2 * (int64_t)p.B * p.Hkv * p.budget * row_bytes) +
               (int64_t)bh * p.budget;
  const int64_t krow = p.ksn * esz, vrow = p.vsn * esz;
  // (both loads, and the accumulator's, before the first store: one round trip, not two)
  const bool acc = ch == 0 && p.base;
  if (DIR == 0) {
    const uint4 k4 = *reinterpret_cast<const uint4*>(Kb + src * krow + ch * 16);
    const uint4 v4 = *reinterpret_cast<const uint4*>(Vb + src * vrow + ch * 16);
    const float b1 = acc ? p.base[(int64_t)bh * p.cap + src] : 0.f;
    *reinterpret_cast<uint4*>(stK + (int64_t)i * row_bytes + ch * 16) = k4;
    *reinterpret_cast<uint4*>(stV + (int64_t)i * row_bytes + ch * 16) = v4;
    if (acc) stB[i] = b1;
  } else if (direct) {
    const uint4 k4 = *reinterpret_cast<const uint4*>(Kb + src * krow + ch * 16);
    const uint4 v4 = *reinterpret_cast<const uint4*>(Vb + src * vrow + ch * 16);
    const float b1 = acc ? p.base[(int64_t)bh * p.cap + src] : 0.f;
    *reinterpret_cast<uint4*>(Kb + i * krow + ch * 16) = k4;
    *reinterpret_cast<uint4*>(Vb + i * vrow + ch * 16) = v4;
    if (acc) p.base[(int64_t)bh * p.cap + i] = b1;
  } else {
    const uint4 k4 = *reinterpret_cast<const uint4*>(stK + (int64_t)i * row_bytes + ch * 16);
    const uint4 v4 = *reinterpret_cast<const uint4*>(stV + (int64_t)i * row_bytes + ch * 16);
    const float b1 = acc ? stB[i] : 0.f;
    *reinterpret_cast<uint4*>(Kb + i * krow + ch * 16) = k4;
    *reinterpret_cast<uint4*>(Vb + i * vrow + ch * 16) = v4;
    if (acc) p.base[(int64_t)bh * p.cap + i] = b1;
  }
}

// CAOTE_COMPACT_FILL: the kept rows below the new length stay, the kept rows from at or beyond
// it ("movers", ascending) drop into the positions below it that evicted rows leave free
// ("holes", ascending).  Sources and destinations are disjoint, so one kernel and no staging.
// The kept list is ascending: its first p entries are the rows that stay, and the q-th hole is
// q + #{i < p : idx[i] - i <= q} (idx[i] - i = holes below idx[i], non-decreasing in i).
// A workgroup takes kFillRows movers; the kept list sits in LDS for the count and the searches
// (budget <= CAOTE_FILL_MAX_BUDGET entries).
constexpr int kFillRows = 64;

__global__ __launch_bounds__(kThreads) void k_fill_holes(const Params p, int row_bytes) {
  const int bh = blockIdx.y, b = bh / p.Hkv, hk = bh % p.Hkv;
  const int N = seq_len(p, b);
  const int n_keep = min(N, p.budget);
  if (N <= n_keep) return;                             // nothing evicted
  const int q0 = blockIdx.x * kFillRows;
  if (q0 >= N - n_keep) return;                        // at most N - n_keep rows can move
  const int32_t* idx = p.kept + (int64_t)bh * p.budget;
  __shared__ int s_p;
  __shared__ int s_dst[kFillRows];
  __shared__ int s_idx[CAOTE_FILL_MAX_BUDGET];
  const int tid = threadIdx.x;
  // The whole kept list comes into LDS in one round of loads; p = number of its entries below
  // n_keep (it is ascending, so they are its first p).
  if (tid == 0) s_p = 0;
  __syncthreads();
  int below = 0;
  for (int i = tid; i < n_keep; i += kThreads) {
    const int v = idx[i];
    s_idx[i] = v;
    below += v < n_keep ? 1 : 0;
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) below += __shfl_xor(below, o, kWave);
  if ((tid & (kWave - 1)) == 0 && below) atomicAdd(&s_p, below);
  __syncthreads();
  const int np = s_p, m = n_keep - np;                 // rows that stay, rows that move
  if (q0 >= m) return;
  const int rows = min(kFillRows, m - q0);
  if (tid < rows) {
    const int q = q0 + tid;
    int lo = 0, hi = np;                               // count of i with s_idx[i] - i <= q
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (s_idx[mid] - mid <= q) lo = mid + 1; else hi = mid;
    }
    s_dst[tid] = q + lo;
  }
  __syncthreads();
  const int esz = p.dtype == CAOTE_F32 ? 4 : 2;
  char* Kb = reinterpret_cast<char*>(p.K) + ((int64_t)b * p.ksb + (int64_t)hk * p.ksh) * esz;
  char* Vb = reinterpret_cast<char*>(p.V) + ((int64_t)b * p.vsb + (int64_t)hk * p.vsh) * esz;
  const int64_t krow = p.ksn * esz, vrow = p.vsn * esz;
  const int cpr = row_bytes / 16;
  // four chunks per thread at a time, all their loads requested before the first store (the
  // compiler cannot know that sources and destinations are different rows)
  constexpr int kB = 4;
  for (int id0 = tid; id0 < rows * cpr; id0 += kB * kThreads) {
    uint4 kk[kB], vv[kB];
    float bb[kB];
    int dd[kB], cc[kB];
#pragma unroll
    for (int u = 0; u < kB; ++u) {
      const int id = id0 + u * kThreads;
      dd[u] = -1;
      if (id < rows * cpr) {
        const int r = id / cpr, ch = id % cpr;
        const int src = s_idx[np + q0 + r], dst = s_dst[r];
        if (src >= n_keep && src < N && dst < n_keep) {          // (a malformed list moves nothing out of bounds)
          dd[u] = dst; cc[u] = ch;
          kk[u] = *reinterpret_cast<const uint4*>(Kb + src * krow + ch * 16);
          vv[u] = *reinterpret_cast<const uint4*>(Vb + src * vrow + ch * 16);
          bb[u] = ch == 0 && p.base ? p.base[(int64_t)bh * p.cap + src] : 0.f;
        }
      }
    }
#pragma unroll
    for (int u = 0; u < kB; ++u) {
      if (dd[u] < 0) continue;
      *reinterpret_cast<uint4*>(Kb + dd[u] * krow + cc[u] * 16) = kk[u];
      *reinterpret_cast<uint4*>(Vb + dd[u] * vrow + cc[u] * 16) = vv[u];
      if (cc[u] == 0 && p.base) p.base[(int64_t)bh * p.cap + dd[u]] = bb[u];
    }
  }
}

// Block-wise prefill (Sec. 2): the new block's rows go behind the rows a sequence holds.
// One thread per 16-byte chunk of a new row; K and V in the same pass.
__global__ __launch_bounds__(kThreads) void k_append(const Params p, const char* k_new, const char* v_new,
                                                     int n_at, int n_new, int row_bytes) {
  const int bh = blockIdx.y, b = bh / p.Hkv, hk = bh % p.Hkv;
  const int cpr = row_bytes / 16;
  const int64_t id = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  const int i = (int)(id / cpr), ch = (int)(id % cpr);
  if (i >= n_new) return;
  int at = n_at;
  if (p.seq_lens) { at = p.seq_lens[b]; at = at < 0 ? 0 : at; }
  const int row = at + i;
  if (row >= p.cap) return;                           // does not fit: dropped
  const int esz = p.dtype == CAOTE_F32 ? 4 : 2;
  char* Kb = reinterpret_cast<char*>(p.K) + ((int64_t)b * p.ksb + (int64_t)hk * p.ksh) * esz;
  char* Vb = reinterpret_cast<char*>(p.V) + ((int64_t)b * p.vsb + (int64_t)hk * p.vsh) * esz;
  const int64_t src = ((int64_t)bh * n_new + i) * row_bytes + ch * 16;
  *reinterpret_cast<uint4*>(Kb + row * p.ksn * esz + ch * 16) = *reinterpret_cast<const uint4*>(k_new + src);
  *reinterpret_cast<uint4*>(Vb + row * p.vsn * esz + ch * 16) = *reinterpret_cast<const uint4*>(v_new + src);
  if (ch == 0 && p.base) p.base[(int64_t)bh * p.cap + row] = 0.f;
}

}  // namespace

hipError_t launch_append(const Params& p, const void* k_new, const void* v_new, int n_at, int n_new,
                         hipStream_t s) {
  const int row_bytes = p.D * (p.dtype == CAOTE_F32 ? 4 : 2);
  const int64_t chunks = (int64_t)n_new * (row_bytes / 16);
  const dim3 grid((unsigned)((chunks + kThreads - 1) / kThreads), p.B * p.Hkv);
  hipLaunchKernelGGL(k_append, grid, dim3(kThreads), 0, s, p, reinterpret_cast<const char*>(k_new),
                     reinterpret_cast<const char*>(v_new), n_at, n_new, row_bytes);
  return hipGetLastError();
}

hipError_t launch_compact(const Params& p, hipStream_t s, PhaseHook* hook) {
  const int row_bytes = p.D * (p.dtype == CAOTE_F32 ? 4 : 2);
  const int64_t chunks = (int64_t)p.budget * (row_bytes / 16);
  const dim3 grid((unsigned)((chunks + kThreads - 1) / kThreads), p.B * p.Hkv);
  if (p.mode == CAOTE_COMPACT_FILL) {
    // movers per (sequence, head): at most min(budget, cap - budget)
    const int most = p.budget < p.cap - p.budget ? p.budget : p.cap - p.budget;
    if (most <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_fill_holes, dim3((most + kFillRows - 1) / kFillRows, p.B * p.Hkv), dim3(kThreads), 0, s, p,
                       row_bytes);
    if (mark(hook, "compact_fill")) return hipGetLastError();
    return hipGetLastError();
  }
  if (p.mode == CAOTE_COMPACT_SWAP_LAST) {
    if (!p.select_swaps) {               // else the selection kernel has moved the row already
      hipLaunchKernelGGL(k_swap_last, dim3(p.B * p.Hkv), dim3(kThreads), 0, s, p, row_bytes);
      if (mark(hook, "compact_swap")) return hipGetLastError();
    }
    // with equal lengths and exactly one token over budget every sequence is an evict-one
    if (p.seq_lens == nullptr && p.cap - p.budget == 1) return hipGetLastError();
  }
  hipLaunchKernelGGL(k_move_rows<0>, grid, dim3(kThreads), 0, s, p, row_bytes);
  if (mark(hook, "compact_gather")) return hipGetLastError();
  hipLaunchKernelGGL(k_move_rows<1>, grid, dim3(kThreads), 0, s, p, row_bytes);
  if (mark(hook, "compact_scatter")) return hipGetLastError();
  return hipGetLastError();
}

}  // namespace caote
