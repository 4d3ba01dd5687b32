// Per-head top-`budget` selection (Sec. 2: the top-b tokens by score are retained).
//
// Scores are compared through their order-preserving 32-bit integer image, so the whole
// selection is integer work: exact, and independent of launch shape.  Equal scores at the
// threshold keep the lower indices.  Three short kernels, each with many workgroups per
// head (one workgroup streaming a whole head's scores is limited by the loads a single
// compute unit can keep in flight):
//   k_select_hist  4096-bin histogram of the top 12 key bits per head;
//   k_select_span  per span of 2048 tokens: walk the histogram from the top to the bin that
//                  holds the budget-th largest key, count the span's keys in higher bins
//                  and set the span's keys of that bin aside (its "candidates");
//   k_select_emit  per span: finish the radix search on the low 20 bits over the head's
//                  candidates (a few hundred keys, every span's workgroup repeats it),
//                  derive the span's output offset from the earlier spans' counts, and
//                  emit the span's survivors in ascending order by ballot and popcount.
#include "common.hpp"

namespace caote {
namespace {

constexpr int kT = 256;                   // threads per workgroup
constexpr int kW = kT / kWave;            // waves per workgroup
constexpr int kPer = kSelSpan / kT;       // tokens per thread in a span (8)
constexpr int kRows = kSelSpan / kW / kWave;   // 64-token rows per wave (8)
constexpr int kSmallCand = 128;           // candidate lists up to this length are ranked against each other
constexpr int kCandCap = 4096;            // candidate lists up to this length are searched in LDS
static_assert(kPer * kT == kSelSpan && kRows * kW * kWave == kSelSpan, "span geometry");
static_assert(kHistShift == 20, "the one-workgroup selection splits the open bits 10 + 10");

// Exclusive prefix sum of v over the 256 threads of the block, and the block total.
__device__ __forceinline__ int block_excl_scan(int v, int* wave_tot, int& total) {
  const int lane = threadIdx.x % kWave, wv = threadIdx.x / kWave;
  int inc = v;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const int up = __shfl_up(inc, o, kWave);
    if (lane >= o) inc += up;
  }
  __syncthreads();                        // wave_tot is reused by consecutive calls
  if (lane == kWave - 1) wave_tot[wv] = inc;
  __syncthreads();
  int before = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kW; ++w) {
    const int t = wave_tot[w];
    before += w < wv ? t : 0;
    tot += t;
  }
  total = tot;
  return before + inc - v;
}

__global__ __launch_bounds__(kT) void k_select_zero(const Params p) {
  uint32_t* hist = p.hist + (int64_t)blockIdx.x * kHistBins;
  for (int i = threadIdx.x; i < kHistBins; i += kT) hist[i] = 0u;
}

// 4096 tokens per workgroup: histogram in LDS first, then one global atomic per bin that
// the workgroup touched (scores of one head crowd into a few dozen bins, so adding token
// by token to global memory would serialise on those addresses).
__global__ __launch_bounds__(1024) void k_select_hist(const Params p) {
  const int bh = blockIdx.y, b = bh / p.Hkv;
  const int N = seq_len(p, b);
  const int tid = threadIdx.x;
  const int j0 = blockIdx.x * 4096;
  if (j0 >= N || N <= p.budget) return;
  __shared__ uint32_t lh[kHistBins];
#pragma unroll
  for (int u = 0; u < kHistBins / 1024; ++u) lh[tid + u * 1024] = 0u;
  __syncthreads();
  const float* sc = p.scores + (int64_t)bh * p.cap;
  uint32_t key[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int j = j0 + u * 1024 + tid;
    key[u] = j < N ? float_key(sc[j]) : 0u;
  }
#pragma unroll
  for (int u = 0; u < 4; ++u)
    if (j0 + u * 1024 + tid < N) atomicAdd(&lh[key[u] >> kHistShift], 1u);
  __syncthreads();
  uint32_t* hist = p.hist + (int64_t)bh * kHistBins;
#pragma unroll
  for (int u = 0; u < kHistBins / 1024; ++u) {
    const uint32_t c = lh[tid + u * 1024];
    if (c) atomicAdd(&hist[tid + u * 1024], c);
  }
}

// Keys of this wave's part of the span: row u = tokens s0 + wave*512 + u*64 + lane.
__device__ __forceinline__ void load_span_keys(const float* sc, int s0, int N, uint32_t (&key)[kRows],
                                               bool (&valid)[kRows]) {
  const int lane = threadIdx.x % kWave, wv = threadIdx.x / kWave;
#pragma unroll
  for (int u = 0; u < kRows; ++u) {
    const int j = s0 + (wv * kRows + u) * kWave + lane;
    valid[u] = j < N;
    key[u] = valid[u] ? float_key(sc[j]) : 0u;
  }
}

__global__ __launch_bounds__(kT) void k_select_span(const Params p) {
  const int bh = blockIdx.y, b = bh / p.Hkv;
  const int N = seq_len(p, b);
  const int s0 = blockIdx.x * kSelSpan;
  const int k = p.budget;
  if (s0 >= N || N <= k) return;          // nothing to evict: k_select_emit writes the identity
  const int tid = threadIdx.x, lane = tid % kWave;
  const float* sc = p.scores + (int64_t)bh * p.cap;
  __shared__ int wave_tot[kW];
  __shared__ uint32_t s_bin;
  __shared__ int s_krem, s_ncand, s_pos, s_hi;

  uint32_t key[kRows];
  bool valid[kRows];
  load_span_keys(sc, s0, N, key, valid);   // in flight during the histogram walk

  // ---- the histogram bin that holds the k-th largest key ----------------------------------
  {
    const uint32_t* gh = p.hist + (int64_t)bh * kHistBins;
    constexpr int BPT = kHistBins / kT;   // bins per thread, descending: a prefix scan over
    const int top = kHistBins - 1 - tid * BPT;   // threads walks down from the largest key
    int cnt[BPT], mine = 0;
#pragma unroll
    for (int i = 0; i < BPT; ++i) { cnt[i] = (int)gh[top - i]; mine += cnt[i]; }
    int total;
    int above = block_excl_scan(mine, wave_tot, total);
    if (tid == 0) { s_pos = 0; s_hi = 0; }
    if (above < k && k <= above + mine) {  // exactly one thread
#pragma unroll
      for (int i = 0; i < BPT; ++i) {
        if (above < k && k <= above + cnt[i]) {
          s_bin = (uint32_t)(top - i);
          s_krem = k - above;
          s_ncand = cnt[i];
        }
        above += cnt[i];
      }
    }
    __syncthreads();
  }
  const uint32_t bin = s_bin;
  // ---- this span: keys in higher bins are kept for sure, keys of the bin are set aside ------
  const uint64_t lt_mask = (1ull << lane) - 1ull;
  int w_hi = 0, w_c = 0;
#pragma unroll
  for (int u = 0; u < kRows; ++u) {
    w_hi += __popcll(__ballot(valid[u] && (key[u] >> kHistShift) > bin));
    w_c += __popcll(__ballot(valid[u] && (key[u] >> kHistShift) == bin));
  }
  int base = 0;
  if (lane == 0) {
    if (w_c) base = atomicAdd(&s_pos, w_c);      // order inside a span's list is irrelevant
    if (w_hi) atomicAdd(&s_hi, w_hi);
  }
  base = __shfl(base, 0, kWave);
  uint32_t* cand = p.sel_cand + (int64_t)bh * p.cap + s0;
#pragma unroll
  for (int u = 0; u < kRows; ++u) {
    const bool hit = valid[u] && (key[u] >> kHistShift) == bin;
    const uint64_t bal = __ballot(hit);
    if (hit) cand[base + __popcll(bal & lt_mask)] = key[u];
    base += __popcll(bal);
  }
  __syncthreads();
  if (tid == 0) {
    int32_t* rec = p.sel_rec + ((int64_t)bh * p.n_span + blockIdx.x) * 2;
    rec[0] = s_hi;
    rec[1] = s_pos;
    if (blockIdx.x == 0) {
      int32_t* head = p.sel_head + (int64_t)bh * 4;
      head[0] = (int32_t)bin; head[1] = s_krem; head[2] = s_ncand;
    }
  }
}

__global__ __launch_bounds__(kT) void k_select_emit(const Params p) {
  const int bh = blockIdx.y, b = bh / p.Hkv;
  const int N = seq_len(p, b);
  const int s0 = blockIdx.x * kSelSpan;
  const int k = p.budget;
  const int tid = threadIdx.x, lane = tid % kWave, wv = tid / kWave;
  int32_t* out = p.kept + (int64_t)bh * k;
  if (N <= k) {                           // nothing to evict: identity, -1 padded
    for (int i = s0 + tid; i < min(k, s0 + kSelSpan); i += kT) out[i] = i < N ? i : -1;
    return;
  }
  if (s0 >= N) return;
  const float* sc = p.scores + (int64_t)bh * p.cap;
  __shared__ int wave_tot[kW], wave_eq[kW], wave_keep[kW];
  __shared__ int hist[256];
  __shared__ int pre[kMaxSpans + 1];
  __shared__ uint32_t s_prefix;
  __shared__ int s_krem, s_off, s_ties;
  __shared__ __attribute__((aligned(16))) uint32_t cl[kCandCap];     // the head's candidates, if they fit

  uint32_t key[kRows];
  bool valid[kRows];
  load_span_keys(sc, s0, N, key, valid);   // in flight during the search below

  const int32_t* head = p.sel_head + (int64_t)bh * 4;
  const int32_t* rec = p.sel_rec + (int64_t)bh * p.n_span * 2;
  const uint32_t* cand = p.sel_cand + (int64_t)bh * p.cap;
  const int ns = (N + kSelSpan - 1) / kSelSpan;
  const int me = blockIdx.x;
  uint32_t prefix = (uint32_t)head[0] << kHistShift;   // key bits fixed so far
  int krem = head[1];                                  // rank still to locate inside the class

  // ---- candidate lists of all spans as one flat sequence: pre[s] = candidates before span s --
  int hi_before = 0;                      // keys of earlier spans in bins above the threshold bin
  {
    int run = 0;
    for (int sb = 0; sb < ns; sb += kT) {
      const int s = sb + tid;
      const int n = s < ns ? rec[s * 2 + 1] : 0;
      hi_before += s < me ? rec[s * 2] : 0;
      int total;
      const int ex = block_excl_scan(n, wave_tot, total);
      if (s < ns) pre[s] = run + ex;
      run += total;
    }
    if (tid == 0) pre[ns] = run;
    int total;
    block_excl_scan(hi_before, wave_tot, total);
    hi_before = total;
    __syncthreads();
  }
  const int ncand = pre[ns];
  // flat candidate i lives in the span s with pre[s] <= i < pre[s+1]
  auto cand_at = [&](int i) -> uint32_t {
    int lo = 0, hi = ns;                  // invariant: pre[lo] <= i < pre[hi]
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (pre[mid] <= i) lo = mid; else hi = mid;
    }
    return cand[lo * kSelSpan + (i - pre[lo])];
  };

  // The candidates come into LDS once, eight loads per thread in flight at a time (each is a
  // dependent search in `pre` plus a load: one by one they would cost a round trip apiece).
  const bool in_lds = ncand <= kCandCap;
  const int n_pad = ((ncand + 3) & ~3) - ncand;         // zero keys that fill the last uint4
  if (in_lds) {
    constexpr int kCB = 8;
    for (int i0 = 0; i0 < ncand; i0 += kCB * kT) {
      uint32_t c[kCB];
#pragma unroll
      for (int u = 0; u < kCB; ++u) {
        const int i = i0 + u * kT + tid;
        c[u] = i < ncand ? cand_at(i) : 0u;
      }
#pragma unroll
      for (int u = 0; u < kCB; ++u) {
        const int i = i0 + u * kT + tid;
        if (i < ncand) cl[i] = c[u];
      }
    }
    if (tid < n_pad) cl[ncand + tid] = 0u;
  }
  auto cand_of = [&](int i) -> uint32_t { return in_lds ? cl[i] : cand_at(i); };

  uint32_t theta;                         // key of the k-th largest score
  if (ncand <= kSmallCand) {
    // ---- few candidates: rank them against each other in LDS ------------------------------------
    // theta is the candidate with fewer than krem candidates above it and at least krem at or
    // above it; the same pass over the list gives the counts of the earlier spans.
    if (tid == 0) { s_prefix = prefix; s_krem = 0; }    // (no candidate: not reached, krem >= 1)
    __syncthreads();
    for (int i = tid; i < ncand; i += kT) {
      const uint32_t mine = cl[i];
      int gt = 0, ge = 0;
      for (int c = 0; c < ncand; c += 4) {
        const uint4 v = *reinterpret_cast<const uint4*>(&cl[c]);
        gt += (v.x > mine) + (v.y > mine) + (v.z > mine) + (v.w > mine);
        ge += (v.x >= mine) + (v.y >= mine) + (v.z >= mine) + (v.w >= mine);
      }
      if (mine == 0u) ge -= n_pad;        // the padding is no candidate
      if (gt < krem && krem <= ge) { s_prefix = mine; s_krem = krem - gt; }   // ties write the same
    }
    __syncthreads();
    theta = s_prefix;
    krem = s_krem;
    int gt = 0, eq = 0;
    for (int i = tid; i < pre[me]; i += kT) {
      gt += cl[i] > theta;
      eq += cl[i] == theta;
    }
    int total_gt, total_eq;
    block_excl_scan(gt, wave_tot, total_gt);
    block_excl_scan(eq, wave_tot, total_eq);
    if (tid == 0) {
      s_off = hi_before + total_gt + min(krem, total_eq);
      s_ties = max(0, krem - total_eq);
    }
    __syncthreads();
  } else {
    // ---- finish the radix search on the low 20 bits, over every span's candidates -----------
    __syncthreads();                        // the list is in LDS
    int shift = kHistShift;
    while (shift > 0) {
      const int bits = shift >= 8 ? 8 : shift;
      shift -= bits;
      const uint32_t himask = 0xffffffffu << (shift + bits);
      hist[tid] = 0;
      __syncthreads();
      for (int i = tid; i < ncand; i += kT) {
        const uint32_t ck = cand_of(i);
        if ((ck & himask) == prefix) atomicAdd(&hist[(ck >> shift) & ((1u << bits) - 1u)], 1);
      }
      __syncthreads();
      {                                     // walk down from the largest digit, in parallel
        const int nd = 1 << bits;
        const int mine = tid < nd ? hist[nd - 1 - tid] : 0;
        int total;
        const int above = block_excl_scan(mine, wave_tot, total);
        if (tid < nd && above < krem && krem <= above + mine) {   // exactly one thread
          s_prefix = prefix | ((uint32_t)(nd - 1 - tid) << shift);
          s_krem = krem - above;
        }
      }
      __syncthreads();
      prefix = s_prefix;
      krem = s_krem;
      __syncthreads();
    }
    // prefix = key of the k-th largest score; krem = how many of its ties are kept.
    theta = prefix;

    // ---- where this span's survivors start ---------------------------------------------------------
    // The earlier spans keep their keys in higher bins, their candidates above theta, and, since
    // ties go to the lowest indices, the first min(krem, ties before this span) ties.
    {
      int gt = 0, eq = 0;
      for (int i = tid; i < pre[me]; i += kT) {
        const uint32_t ck = cand_of(i);
        gt += ck > theta;
        eq += ck == theta;
      }
      int total_gt, total_eq;
      block_excl_scan(gt, wave_tot, total_gt);
      block_excl_scan(eq, wave_tot, total_eq);
      if (tid == 0) {
        s_off = hi_before + total_gt + min(krem, total_eq);
        s_ties = max(0, krem - total_eq);
      }
      __syncthreads();
    }
  }
  const int span_off = s_off;             // output position of this span's first survivor
  const int span_ties = s_ties;           // ties this span may still keep

  // ---- emit, ascending: each wave owns 512 consecutive tokens of the span -------------------
  const uint64_t lt_mask = (1ull << lane) - 1ull;
  int w_gt = 0, w_eq = 0;
#pragma unroll
  for (int u = 0; u < kRows; ++u) {
    w_gt += __popcll(__ballot(valid[u] && key[u] > theta));
    w_eq += __popcll(__ballot(valid[u] && key[u] == theta));
  }
  if (lane == 0) wave_eq[wv] = w_eq;
  __syncthreads();
  int eq_before = 0;
#pragma unroll
  for (int w = 0; w < kW; ++w) eq_before += w < wv ? wave_eq[w] : 0;
  int ties_left = max(0, min(w_eq, span_ties - eq_before));
  if (lane == 0) wave_keep[wv] = w_gt + ties_left;
  __syncthreads();
  int pos = span_off;
#pragma unroll
  for (int w = 0; w < kW; ++w) pos += w < wv ? wave_keep[w] : 0;
#pragma unroll
  for (int u = 0; u < kRows; ++u) {
    const bool gt = valid[u] && key[u] > theta, eq = valid[u] && key[u] == theta;
    const uint64_t eqm = __ballot(eq);
    const bool keep = gt || (eq && (int)__popcll(eqm & lt_mask) < ties_left);
    const uint64_t km = __ballot(keep);
    if (keep) out[pos + __popcll(km & lt_mask)] = s0 + (wv * kRows + u) * kWave + lane;
    pos += __popcll(km);
    ties_left -= min(ties_left, (int)__popcll(eqm));
  }
}


// ---------------------------------------------------------------------------------------------
// Caches of up to 4096 rows (decode at a 2k-4k budget, block-wise prefill): the whole selection
// of a head in ONE workgroup of 1024 threads, four consecutive tokens per thread, everything
// in registers and LDS.  Three dependent kernels cost about 5 us each at this size, whatever
// they do; one costs about 6.  In a fused evict-one call in swap-last mode the workgroup also
// moves the last row into the hole it has just chosen (it knows the hole).
// ---------------------------------------------------------------------------------------------
constexpr int kST = 1024;                 // threads
constexpr int kSW = kST / kWave;          // waves
constexpr int kSPer = 4;                  // tokens per thread
constexpr int kSmallCap = kST * kSPer;    // 4096
static_assert(kOneWgCap == 4 * kSmallCap, "one workgroup holds at most four rows of 4096 tokens per thread");

// Exclusive prefix sum over the 1024 threads, and the total.  wave_tot: kSW ints of LDS.
__device__ __forceinline__ int block_excl_scan_1024(int v, int* wave_tot, int& total) {
  const int lane = threadIdx.x % kWave, wv = threadIdx.x / kWave;
  int inc = v;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const int up = __shfl_up(inc, o, kWave);
    if (lane >= o) inc += up;
  }
  __syncthreads();                        // wave_tot is reused by consecutive calls
  if (lane == kWave - 1) wave_tot[wv] = inc;
  __syncthreads();
  int before = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kSW; ++w) {
    const int t = wave_tot[w];
    before += w < wv ? t : 0;
    tot += t;
  }
  total = tot;
  return before + inc - v;
}

// Evict-one in swap-last mode (fused call): the last row of K, V and the accumulator drops
// into the hole.  Called by all threads of the head's workgroup.
__device__ __forceinline__ void swap_last_row(const Params& p, int bh, int b, int hk, int hole, int N,
                                              int row_bytes) {
  const int tid = threadIdx.x;
  const int esz = p.dtype == CAOTE_F32 ? 4 : 2;
  char* Kb = reinterpret_cast<char*>(p.K) + ((int64_t)b * p.ksb + (int64_t)hk * p.ksh) * esz;
  char* Vb = reinterpret_cast<char*>(p.V) + ((int64_t)b * p.vsb + (int64_t)hk * p.vsh) * esz;
  const int64_t krow = p.ksn * esz, vrow = p.vsn * esz;
  const int cpr = row_bytes / 16;
  if (tid < cpr)
    *reinterpret_cast<uint4*>(Kb + hole * krow + tid * 16) = *reinterpret_cast<const uint4*>(Kb + (N - 1) * krow + tid * 16);
  else if (tid < 2 * cpr)
    *reinterpret_cast<uint4*>(Vb + hole * vrow + (tid - cpr) * 16) =
        *reinterpret_cast<const uint4*>(Vb + (N - 1) * vrow + (tid - cpr) * 16);
  else if (tid == 2 * cpr && p.base)        // (combine_in_select: the accumulator row as k_vside left it)
    p.base[(int64_t)bh * p.cap + hole] = (p.combine_in_select ? p.h : p.base)[(int64_t)bh * p.cap + N - 1];
}

// One token leaves (generation): the smallest key goes, among equal keys the highest index;
// no histogram, one reduction.  `best` packs a thread's candidates, key in the high word and
// ~index in the low word (the minimum over the head is the token to drop).  Writes the kept
// list and, in the fused call in swap-last mode, moves the last row into the hole.
__device__ __forceinline__ void evict_one(const Params& p, unsigned long long best, int bh, int b, int hk,
                                          int N, int row_bytes, unsigned long long* wave_min) {
  const int tid = threadIdx.x, k = p.budget;
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    const unsigned long long c = __shfl_xor(best, o, kWave);
    best = c < best ? c : best;
  }
  if ((tid & 63) == 0) wave_min[tid >> 6] = best;
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kSW; ++w) best = wave_min[w] < best ? wave_min[w] : best;
  const int hole = (int)~(uint32_t)best;
  int32_t* out = p.kept + (int64_t)bh * k;
  for (int i = tid; i < k; i += kST) out[i] = i < hole ? i : i + 1;
  if (p.select_swaps && p.mode == CAOTE_COMPACT_SWAP_LAST && hole != N - 1)
    swap_last_row(p, bh, b, hk, hole, N, row_bytes);
}
__device__ __forceinline__ unsigned long long pack_candidate(uint32_t key, int j) {
  return ((unsigned long long)key << 32) | (uint32_t)~(uint32_t)j;
}

// The score of token j: from memory or, in the fused call on a short cache, put together here
// from the column slices that k_vside left (and written out on the way).
__device__ __forceinline__ float score_at(const Params& p, const float* sc, int bh, int j, int N) {
  return p.combine_in_select ? combine_score(p, bh, j, N) : sc[j];
}

__global__ __launch_bounds__(kST) void k_select_small(const Params p, int row_bytes) {
  const int bh = blockIdx.x, b = bh / p.Hkv, hk = bh % p.Hkv;
  const int N = seq_len(p, b);
  const int k = p.budget;
  const int tid = threadIdx.x;
  int32_t* out = p.kept + (int64_t)bh * k;
  if (N <= k) {                           // nothing to evict: identity, -1 padded
    for (int i = tid; i < k; i += kST) out[i] = i < N ? i : -1;
    if (p.combine_in_select)              // the scores are still owed
      for (int j = tid; j < N; j += kST) combine_score(p, bh, j, N);
    return;
  }
  __shared__ int hist[kHistBins];
  __shared__ uint32_t cand[kSmallCap];
  __shared__ int wave_tot[kSW];
  __shared__ uint32_t s_prefix;
  __shared__ int s_bin, s_krem, s_hole;

  const float* sc = p.scores + (int64_t)bh * p.cap;
  const int j0 = tid * kSPer;             // this thread's tokens j0 .. j0+3
  uint32_t key[kSPer];
  bool valid[kSPer];
#pragma unroll
  for (int e = 0; e < kSPer; ++e) {
    valid[e] = j0 + e < N;
    key[e] = valid[e] ? float_key(score_at(p, sc, bh, j0 + e, N)) : 0u;
  }
  if (N - k == 1) {                       // one token leaves: no histogram
    __shared__ unsigned long long wave_min[kSW];
    unsigned long long best = ~0ull;
#pragma unroll
    for (int e = 0; e < kSPer; ++e)
      if (valid[e]) { const unsigned long long c = pack_candidate(key[e], j0 + e); best = c < best ? c : best; }
    evict_one(p, best, bh, b, hk, N, row_bytes, wave_min);
    return;
  }
#pragma unroll
  for (int u = 0; u < kHistBins / kST; ++u) hist[tid + u * kST] = 0;
  if (tid == 0) s_hole = -1;
  __syncthreads();
#pragma unroll
  for (int e = 0; e < kSPer; ++e)
    if (valid[e]) atomicAdd(&hist[key[e] >> kHistShift], 1);
  __syncthreads();
  // ---- the bin that holds the k-th largest key: threads walk down from the largest bin ------
  {
    constexpr int BPT = kHistBins / kST;
    const int top = kHistBins - 1 - tid * BPT;
    int cnt[BPT], mine = 0;
#pragma unroll
    for (int i = 0; i < BPT; ++i) { cnt[i] = hist[top - i]; mine += cnt[i]; }
    int total;
    int above = block_excl_scan_1024(mine, wave_tot, total);
    if (above < k && k <= above + mine) {  // exactly one thread
#pragma unroll
      for (int i = 0; i < BPT; ++i) {
        if (above < k && k <= above + cnt[i]) { s_bin = top - i; s_krem = k - above; }
        above += cnt[i];
      }
    }
    __syncthreads();
  }
  const uint32_t bin = (uint32_t)s_bin;
  int krem = s_krem;                      // rank still to locate inside the bin
  // ---- the bin's keys, as a list in LDS -----------------------------------------------------------
  int ncand;
  {
    int c = 0;
#pragma unroll
    for (int e = 0; e < kSPer; ++e) c += valid[e] && (key[e] >> kHistShift) == bin;
    int at = block_excl_scan_1024(c, wave_tot, ncand);
#pragma unroll
    for (int e = 0; e < kSPer; ++e)
      if (valid[e] && (key[e] >> kHistShift) == bin) cand[at++] = key[e];
    __syncthreads();
  }
  // ---- radix search on the low 20 bits over the list, 10 bits a pass: one bin per thread ------
  uint32_t prefix = bin << kHistShift;
  int shift = kHistShift;
  while (shift > 0) {
    const int bits = shift >= 10 ? 10 : shift;
    shift -= bits;
    const uint32_t himask = 0xffffffffu << (shift + bits);
    hist[tid] = 0;
    __syncthreads();
    for (int i = tid; i < ncand; i += kST) {
      const uint32_t ck = cand[i];
      if ((ck & himask) == prefix) atomicAdd(&hist[(ck >> shift) & ((1u << bits) - 1u)], 1);
    }
    __syncthreads();
    {
      const int nd = 1 << bits;
      const int mine = tid < nd ? hist[nd - 1 - tid] : 0;
      int total;
      const int above = block_excl_scan_1024(mine, wave_tot, total);
      if (tid < nd && above < krem && krem <= above + mine) {   // exactly one thread
        s_prefix = prefix | ((uint32_t)(nd - 1 - tid) << shift);
        s_krem = krem - above;
      }
    }
    __syncthreads();
    prefix = s_prefix;
    krem = s_krem;
    __syncthreads();
  }
  const uint32_t theta = prefix;          // key of the k-th largest score; krem of its ties are kept
  // ---- emit in ascending order: a token's rank = kept tokens before it ---------------------------
  int gt = 0, eq = 0;
#pragma unroll
  for (int e = 0; e < kSPer; ++e) { gt += valid[e] && key[e] > theta; eq += valid[e] && key[e] == theta; }
  int tot_gt, tot_eq;
  const int gt_before = block_excl_scan_1024(gt, wave_tot, tot_gt);
  const int eq_before = block_excl_scan_1024(eq, wave_tot, tot_eq);
  int pos = gt_before + min(eq_before, krem);
  int ties_left = max(0, krem - eq_before);
  int dropped = -1;                       // a token of this thread that is not kept
#pragma unroll
  for (int e = 0; e < kSPer; ++e) {
    bool keep = valid[e] && key[e] > theta;
    if (valid[e] && key[e] == theta && ties_left > 0) { keep = true; --ties_left; }
    if (keep) out[pos++] = j0 + e;
    else if (valid[e]) dropped = j0 + e;
  }
  // ---- evict-one in swap-last mode (fused call): the last row drops into the hole ----------------
  if (p.select_swaps && p.mode == CAOTE_COMPACT_SWAP_LAST && N - k == 1) {
    if (dropped >= 0) s_hole = dropped;    // exactly one token of the head is dropped
    __syncthreads();
    const int hole = s_hole;
    if (hole < 0 || hole == N - 1) return;
    swap_last_row(p, bh, b, hk, hole, N, row_bytes);
  }
}

// Caches of 4097 .. 16384 rows: still one workgroup per head, thread t holding four tokens of
// each of U rows of 4096.  The radix passes count straight from the registers, and the ranks
// for the ordered emit come from one scan over the per-thread counts in token order.  Beyond
// 16384 rows one compute unit cannot pull the scores in fast enough (measured at 32768: 26 us
// against 19 us) and the three multi-workgroup kernels take over.
template <int U>
__global__ __launch_bounds__(kST) void k_select_one(const Params p, int row_bytes) {
  const int bh = blockIdx.x, b = bh / p.Hkv, hk = bh % p.Hkv;
  const int N = seq_len(p, b);
  const int k = p.budget;
  const int tid = threadIdx.x;
  int32_t* out = p.kept + (int64_t)bh * k;
  if (N <= k) {                           // nothing to evict: identity, -1 padded
    for (int i = tid; i < k; i += kST) out[i] = i < N ? i : -1;
    if (p.combine_in_select)              // the scores are still owed
      for (int j = tid; j < N; j += kST) combine_score(p, bh, j, N);
    return;
  }
  __shared__ int hist[kHistBins];
  __shared__ uint32_t cnt[U * kST];       // per (row, thread): kept-for-sure << 16 | ties
  __shared__ int wave_tot[kSW];
  __shared__ uint32_t s_prefix;
  __shared__ int s_bin, s_krem, s_hole;

  const float* sc = p.scores + (int64_t)bh * p.cap;
  uint32_t key[U][kSPer];                 // thread t: tokens u * 4096 + 4 t .. + 3 of every row u
#pragma unroll
  for (int u = 0; u < U; ++u)
#pragma unroll
    for (int e = 0; e < kSPer; ++e) {
      const int j = u * kSmallCap + tid * kSPer + e;
      key[u][e] = j < N ? float_key(score_at(p, sc, bh, j, N)) : 0u;
    }
  if (N - k == 1) {                       // one token leaves: no histogram
    __shared__ unsigned long long wave_min[kSW];
    unsigned long long best = ~0ull;
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int e = 0; e < kSPer; ++e) {
        const int j = u * kSmallCap + tid * kSPer + e;
        if (j < N) { const unsigned long long c = pack_candidate(key[u][e], j); best = c < best ? c : best; }
      }
    evict_one(p, best, bh, b, hk, N, row_bytes, wave_min);
    return;
  }
#pragma unroll
  for (int u = 0; u < kHistBins / kST; ++u) hist[tid + u * kST] = 0;
  if (tid == 0) s_hole = -1;
  __syncthreads();
#pragma unroll
  for (int u = 0; u < U; ++u)
#pragma unroll
    for (int e = 0; e < kSPer; ++e)
      if (u * kSmallCap + tid * kSPer + e < N) atomicAdd(&hist[key[u][e] >> kHistShift], 1);
  __syncthreads();
  // ---- the bin that holds the k-th largest key: threads walk down from the largest bin ------
  {
    constexpr int BPT = kHistBins / kST;
    const int top = kHistBins - 1 - tid * BPT;
    int cnt[BPT], mine = 0;
#pragma unroll
    for (int i = 0; i < BPT; ++i) { cnt[i] = hist[top - i]; mine += cnt[i]; }
    int total;
    int above = block_excl_scan_1024(mine, wave_tot, total);
    if (above < k && k <= above + mine) {  // exactly one thread
#pragma unroll
      for (int i = 0; i < BPT; ++i) {
        if (above < k && k <= above + cnt[i]) { s_bin = top - i; s_krem = k - above; }
        above += cnt[i];
      }
    }
    __syncthreads();
  }
  const uint32_t bin = (uint32_t)s_bin;
  int krem = s_krem;                      // rank still to locate inside the bin
  // ---- radix search on the low 20 bits over the list, 10 bits a pass: one bin per thread ------
  uint32_t prefix = bin << kHistShift;
  int shift = kHistShift;
  while (shift > 0) {
    const int bits = shift >= 10 ? 10 : shift;
    shift -= bits;
    const uint32_t himask = 0xffffffffu << (shift + bits);
    hist[tid] = 0;
    __syncthreads();
#pragma unroll
    for (int u = 0; u < U; ++u)                         // straight from the registers: no list
#pragma unroll
      for (int e = 0; e < kSPer; ++e)
        if ((key[u][e] & himask) == prefix && u * kSmallCap + tid * kSPer + e < N)
          atomicAdd(&hist[(key[u][e] >> shift) & ((1u << bits) - 1u)], 1);
    __syncthreads();
    {
      const int nd = 1 << bits;
      const int mine = tid < nd ? hist[nd - 1 - tid] : 0;
      int total;
      const int above = block_excl_scan_1024(mine, wave_tot, total);
      if (tid < nd && above < krem && krem <= above + mine) {   // exactly one thread
        s_prefix = prefix | ((uint32_t)(nd - 1 - tid) << shift);
        s_krem = krem - above;
      }
    }
    __syncthreads();
    prefix = s_prefix;
    krem = s_krem;
    __syncthreads();
  }
  const uint32_t theta = prefix;          // key of the k-th largest score; krem of its ties are kept
  // ---- ranks: ONE scan over the U x 1024 per-thread counts in token order, "greater" and
  // "equal" packed into the halves of a word (greater < N <= 32768, equal <= 32768) ----------------
#pragma unroll
  for (int u = 0; u < U; ++u) {
    uint32_t c = 0;
#pragma unroll
    for (int e = 0; e < kSPer; ++e) {
      const bool v = u * kSmallCap + tid * kSPer + e < N;
      c += (v && key[u][e] > theta ? 0x10000u : 0u) + (v && key[u][e] == theta ? 1u : 0u);
    }
    cnt[u * kST + tid] = c;
  }
  __syncthreads();
  {
    uint32_t loc[U], sum = 0;             // entries tid * U .. + U - 1 of the row-major sequence
#pragma unroll
    for (int i = 0; i < U; ++i) { loc[i] = cnt[tid * U + i]; sum += loc[i]; }
    int total;
    uint32_t run = (uint32_t)block_excl_scan_1024((int)sum, wave_tot, total);
#pragma unroll
    for (int i = 0; i < U; ++i) { cnt[tid * U + i] = run; run += loc[i]; }
    __syncthreads();
  }
  int dropped = -1;                       // a token of this thread that is not kept
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const uint32_t before = cnt[u * kST + tid];
    const int gt_before = (int)(before >> 16), eq_before = (int)(before & 0xffffu);
    int pos = gt_before + min(eq_before, krem);
    int ties_left = max(0, krem - eq_before);
#pragma unroll
    for (int e = 0; e < kSPer; ++e) {
      const int j = u * kSmallCap + tid * kSPer + e;
      const bool v = j < N;
      bool keep = v && key[u][e] > theta;
      if (v && key[u][e] == theta && ties_left > 0) { keep = true; --ties_left; }
      if (keep) out[pos++] = j;
      else if (v) dropped = j;
    }
  }
  // ---- evict-one in swap-last mode (fused call): the last row drops into the hole ----------------
  if (p.select_swaps && p.mode == CAOTE_COMPACT_SWAP_LAST && N - k == 1) {
    if (dropped >= 0) s_hole = dropped;    // exactly one token of the head is dropped
    __syncthreads();
    const int hole = s_hole;
    if (hole < 0 || hole == N - 1) return;
    swap_last_row(p, bh, b, hk, hole, N, row_bytes);
  }
}

}  // namespace

hipError_t launch_select(const Params& p, hipStream_t s, PhaseHook* hook) {
  const int bh = p.B * p.Hkv;
  if (p.cap <= kOneWgCap) {
    const int row_bytes = p.D * (p.dtype == CAOTE_F32 ? 4 : 2);
    if (p.cap <= kSmallCap)          hipLaunchKernelGGL(k_select_small, dim3(bh), dim3(kST), 0, s, p, row_bytes);
    else if (p.cap <= 2 * kSmallCap) hipLaunchKernelGGL(k_select_one<2>, dim3(bh), dim3(kST), 0, s, p, row_bytes);
    else                             hipLaunchKernelGGL(k_select_one<4>, dim3(bh), dim3(kST), 0, s, p, row_bytes);
    if (mark(hook, "select")) return hipGetLastError();
    return hipGetLastError();
  }
  if (!p.hist_zeroed) hipLaunchKernelGGL(k_select_zero, dim3(bh), dim3(kT), 0, s, p);
  if (!p.hist_in_vscore) {               // else the scoring kernel has built the histogram
    hipLaunchKernelGGL(k_select_hist, dim3((p.cap + 4095) / 4096, bh), dim3(1024), 0, s, p);
    if (mark(hook, "select_hist")) return hipGetLastError();
  }
  hipLaunchKernelGGL(k_select_span, dim3(p.n_span, bh), dim3(kT), 0, s, p);
  if (mark(hook, "select_span")) return hipGetLastError();
  const int n_out = (max(p.cap, p.budget) + kSelSpan - 1) / kSelSpan;   // also pads past the cache
  hipLaunchKernelGGL(k_select_emit, dim3(n_out, bh), dim3(kT), 0, s, p);
  if (mark(hook, "select_emit")) return hipGetLastError();
  return hipGetLastError();
}

}  // namespace caote
