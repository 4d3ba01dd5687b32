// Per-head top-`budget` selection (Sec. 2: the top-b tokens by score are retained).
//
// Scores are compared through their order-preserving 32-bit integer image, so the whole
// selection is integer work: exact, and independent of launch shape.
//   1. a 4096-bin histogram of the top 12 key bits per head (k_select_hist);
//   2. one workgroup per head (k_select_main) walks the histogram from the top to the bin
//      that holds the budget-th largest score, gathers that bin's keys into LDS and
//      finishes the radix search on the remaining 20 bits there (three short passes);
//   3. the same workgroup emits the kept indices in ascending order: every wave owns a
//      contiguous span of the tokens and places its survivors by ballot and popcount.
// Equal scores at the threshold keep the lower indices.
// Each wave reads its span once, 64 tokens per load, and keeps the keys in registers
// (up to 32 loads in flight per lane) for both the gather and the emit.
#include "common.hpp"

namespace caote {
namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / kWave;
constexpr int kCandMax = 12288;          // keys of the threshold bin held in LDS
constexpr int kIterReg = 32;             // spans up to 32 x 64 tokens per wave stay in registers

// Exclusive prefix sum of v over the block (threads in order) and the block total.
__device__ __forceinline__ int block_excl_scan(int v, int* wave_tot, int& total) {
  const int lane = threadIdx.x % kWave, wv = threadIdx.x / kWave;
  int inc = v;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const int up = __shfl_up(inc, o, kWave);
    if (lane >= o) inc += up;
  }
  __syncthreads();                       // wave_tot is reused by consecutive calls
  if (lane == kWave - 1) wave_tot[wv] = inc;
  __syncthreads();
  int before = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) {
    const int t = wave_tot[w];
    before += w < wv ? t : 0;
    tot += t;
  }
  total = tot;
  return before + inc - v;
}

__global__ __launch_bounds__(256) void k_select_zero(const Params p) {
  uint32_t* hist = p.hist + (int64_t)blockIdx.x * kHistBins;
  for (int i = threadIdx.x; i < kHistBins; i += 256) hist[i] = 0u;
}

// 4096 tokens per workgroup: histogram in LDS first, then one global atomic per bin that
// the workgroup touched (scores of one head crowd into a few dozen bins, so adding token
// by token to global memory would serialise on those addresses).
__global__ __launch_bounds__(kSelThreads) void k_select_hist(const Params p) {
  const int bh = blockIdx.y, b = bh / p.Hkv;
  const int N = seq_len(p, b);
  const int tid = threadIdx.x;
  const int j0 = blockIdx.x * (4 * kSelThreads);
  if (j0 >= N) return;
  __shared__ uint32_t lh[kHistBins];
#pragma unroll
  for (int u = 0; u < kHistBins / kSelThreads; ++u) lh[tid + u * kSelThreads] = 0u;
  __syncthreads();
  const float* sc = p.scores + (int64_t)bh * p.cap;
  uint32_t key[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int j = j0 + u * kSelThreads + tid;
    key[u] = j < N ? float_key(sc[j]) : 0u;
  }
#pragma unroll
  for (int u = 0; u < 4; ++u)
    if (j0 + u * kSelThreads + tid < N) atomicAdd(&lh[key[u] >> kHistShift], 1u);
  __syncthreads();
  uint32_t* hist = p.hist + (int64_t)bh * kHistBins;
#pragma unroll
  for (int u = 0; u < kHistBins / kSelThreads; ++u) {
    const uint32_t c = lh[tid + u * kSelThreads];
    if (c) atomicAdd(&hist[tid + u * kSelThreads], c);
  }
}

// IN_REGS: every wave's span fits kIterReg loads per lane (N <= 32768).
template <bool IN_REGS>
__global__ __launch_bounds__(kSelThreads) void k_select_main(const Params p) {
  const int bh = blockIdx.x, b = bh / p.Hkv;
  const int N = seq_len(p, b);
  const int tid = threadIdx.x, lane = tid % kWave, wv = tid / kWave;
  const float* sc = p.scores + (int64_t)bh * p.cap;
  int32_t* out = p.kept + (int64_t)bh * p.budget;
  const int k = p.budget;

  if (N <= k) {                          // nothing to evict: identity, -1 padded
    for (int i = tid; i < k; i += kSelThreads) out[i] = i < N ? i : -1;
    return;
  }
  __shared__ int wave_tot[kSelWaves], wave_eq[kSelWaves], wave_keep[kSelWaves];
  __shared__ int hist[256];
  __shared__ uint32_t s_prefix;
  __shared__ int s_krem, s_ncand;
  extern __shared__ uint32_t cand[];     // [kCandMax]

  // Span of this wave: [s0, s1), read as `iters` rows of 64 consecutive tokens.
  const uint64_t lt_mask = (1ull << lane) - 1ull;
  const int span = ((N + kSelWaves - 1) / kSelWaves + kWave - 1) / kWave * kWave;
  const int s0 = min(N, wv * span), s1 = min(N, s0 + span);
  const int iters = span / kWave;
  uint32_t keys[IN_REGS ? kIterReg : 1];
  if (IN_REGS) {                         // all loads of the span in flight at once
#pragma unroll
    for (int it = 0; it < kIterReg; ++it) {
      const int j = s0 + it * kWave + lane;
      keys[it] = j < s1 ? float_key(sc[j]) : 0u;
    }
  }
  // Applies f(it, key, valid) to every row of the span, in order.
  auto for_span = [&](auto&& f) {
    if (IN_REGS) {
#pragma unroll
      for (int it = 0; it < kIterReg; ++it) f(it, keys[it], s0 + it * kWave + lane < s1);
    } else {
      for (int it0 = 0; it0 < iters; it0 += 8) {               // 8 loads in flight
        uint32_t kk[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int j = s0 + (it0 + u) * kWave + lane;
          kk[u] = j < s1 ? float_key(sc[j]) : 0u;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
          if (it0 + u < iters) f(it0 + u, kk[u], s0 + (it0 + u) * kWave + lane < s1);
      }
    }
  };

  // ---- 1. the histogram bin that holds the k-th largest key ----------------------------
  {
    const uint32_t* gh = p.hist + (int64_t)bh * kHistBins;
    constexpr int BPT = kHistBins / kSelThreads;            // bins per thread
    // thread t owns bins of descending value: reversed index so that a prefix scan over
    // threads is a walk down from the largest key
    const int top = kHistBins - 1 - tid * BPT;
    int cnt[BPT], mine = 0;
#pragma unroll
    for (int i = 0; i < BPT; ++i) { cnt[i] = (int)gh[top - i]; mine += cnt[i]; }
    int total;
    int above = block_excl_scan(mine, wave_tot, total);
    if (above < k && k <= above + mine) {                     // exactly one thread
#pragma unroll
      for (int i = 0; i < BPT; ++i) {
        if (above < k && k <= above + cnt[i]) {
          s_prefix = (uint32_t)(top - i) << kHistShift;
          s_krem = k - above;
          s_ncand = cnt[i];
        }
        above += cnt[i];
      }
    }
    __syncthreads();
  }
  uint32_t prefix = s_prefix;            // key bits fixed so far (high bits)
  int krem = s_krem;                     // rank still to locate inside the prefix class
  const int ncand = s_ncand;
  const bool in_lds = ncand <= kCandMax;
  __syncthreads();

  // ---- 2. finish the radix search on the low 20 bits ------------------------------------
  if (in_lds) {                          // gather the threshold bin's keys (order is irrelevant)
    if (tid == 0) s_ncand = 0;
    __syncthreads();
    const uint32_t bin = prefix >> kHistShift;
    int w_hits = 0;
    for_span([&](int, uint32_t key, bool valid) {
      w_hits += __popcll(__ballot(valid && (key >> kHistShift) == bin));
    });
    int base = 0;
    if (lane == 0 && w_hits) base = atomicAdd(&s_ncand, w_hits);   // one LDS atomic per wave
    base = __shfl(base, 0, kWave);
    for_span([&](int, uint32_t key, bool valid) {
      const bool hit = valid && (key >> kHistShift) == bin;
      const uint64_t bal = __ballot(hit);
      if (hit) cand[base + __popcll(bal & lt_mask)] = key;
      base += __popcll(bal);
    });
    __syncthreads();
  }
  const int n_src = in_lds ? ncand : N;
  int shift = kHistShift;
  while (shift > 0) {
    const int bits = shift >= 8 ? 8 : shift;
    shift -= bits;
    const uint32_t himask = 0xffffffffu << (shift + bits);
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    for (int j = tid; j < n_src; j += kSelThreads) {
      const uint32_t key = in_lds ? cand[j] : float_key(sc[j]);
      if ((key & himask) == prefix) atomicAdd(&hist[(key >> shift) & ((1u << bits) - 1u)], 1);
    }
    __syncthreads();
    {                                    // walk down from the largest digit, in parallel:
      const int nd = 1 << bits;          // thread t holds digit nd-1-t, a prefix scan counts
      const int mine = tid < nd ? hist[nd - 1 - tid] : 0;     // the keys in larger digits
      int total;
      const int above = block_excl_scan(mine, wave_tot, total);
      if (tid < nd && above < krem && krem <= above + mine) {  // exactly one thread
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
  const uint32_t theta = prefix;

  // ---- 3. emit, ascending -----------------------------------------------------------------
  int w_gt = 0, w_eq = 0;                // wave-uniform counts
  for_span([&](int, uint32_t key, bool valid) {
    w_gt += __popcll(__ballot(valid && key > theta));
    w_eq += __popcll(__ballot(valid && key == theta));
  });
  if (lane == 0) wave_eq[wv] = w_eq;
  __syncthreads();
  int eq_before = 0;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) eq_before += w < wv ? wave_eq[w] : 0;
  int ties_left = max(0, min(w_eq, krem - eq_before));        // ties this wave may keep
  if (lane == 0) wave_keep[wv] = w_gt + ties_left;
  __syncthreads();
  int pos = 0;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) pos += w < wv ? wave_keep[w] : 0;
  for_span([&](int it, uint32_t key, bool valid) {
    const bool gt = valid && key > theta, eq = valid && key == theta;
    const uint64_t eqm = __ballot(eq);
    const bool keep = gt || (eq && (int)__popcll(eqm & lt_mask) < ties_left);
    const uint64_t km = __ballot(keep);
    if (keep) out[pos + __popcll(km & lt_mask)] = s0 + it * kWave + lane;
    pos += __popcll(km);
    ties_left -= min(ties_left, (int)__popcll(eqm));
  });
}

}  // namespace

hipError_t launch_select(const Params& p, hipStream_t s, PhaseHook* hook) {
  const int bh = p.B * p.Hkv;
  if (!p.hist_zeroed) hipLaunchKernelGGL(k_select_zero, dim3(bh), dim3(256), 0, s, p);
  hipLaunchKernelGGL(k_select_hist, dim3((p.cap + 4 * kSelThreads - 1) / (4 * kSelThreads), bh),
                     dim3(kSelThreads), 0, s, p);
  mark(hook, "select_hist");
  const size_t lds = kCandMax * sizeof(uint32_t);
  if (p.cap <= kIterReg * kWave * kSelWaves)
    hipLaunchKernelGGL(k_select_main<true>, dim3(bh), dim3(kSelThreads), lds, s, p);
  else
    hipLaunchKernelGGL(k_select_main<false>, dim3(bh), dim3(kSelThreads), lds, s, p);
  mark(hook, "select");
  return hipGetLastError();
}

}  // namespace caote
