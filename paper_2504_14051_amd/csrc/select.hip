// Per-head top-`budget` selection (Sec. 2: the top-b tokens by score are retained).
//
// The k-th largest score is found by a most-significant-digit radix search on the
// order-preserving integer image of the floats (4 digits of 8 bits), then the kept
// indices are emitted in ascending order with a block-wide prefix scan.  Equal scores
// at the threshold keep the lower indices.  Integer work throughout: the result is
// exact and independent of launch shape.
#include "common.hpp"

namespace caote {
namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / kWave;

// Exclusive prefix count of `flag` over the block, plus the block total.
__device__ __forceinline__ int block_excl_count(bool flag, int* wave_tot, int& total) {
  const uint64_t bal = __ballot(flag);
  const int lane = threadIdx.x % kWave, wv = threadIdx.x / kWave;
  const int in_wave = __popcll(bal & ((1ull << lane) - 1ull));
  __syncthreads();                       // wave_tot is reused by consecutive calls
  if (lane == 0) wave_tot[wv] = __popcll(bal);
  __syncthreads();
  int before = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) {
    const int t = wave_tot[w];
    before += w < wv ? t : 0;
    tot += t;
  }
  total = tot;
  return before + in_wave;
}

__global__ __launch_bounds__(kSelThreads) void k_select_single(const Params p) {
  const int bh = blockIdx.x, b = bh / p.Hkv;
  const int N = seq_len(p, b);
  const float* sc = p.scores + (int64_t)bh * p.cap;
  int32_t* out = p.kept + (int64_t)bh * p.budget;
  const int k = p.budget;

  if (N <= k) {                          // nothing to evict: identity, -1 padded
    for (int i = threadIdx.x; i < k; i += kSelThreads) out[i] = i < N ? i : -1;
    return;
  }
  __shared__ int hist[256];
  __shared__ int wave_tot[kSelWaves];
  __shared__ uint32_t s_prefix;
  __shared__ int s_krem;

  uint32_t prefix = 0;                   // digits fixed so far (high bits)
  int krem = k;                          // rank still to locate inside the prefix class
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    const uint32_t himask = pass == 0 ? 0u : 0xffffffffu << (shift + 8);
    if (threadIdx.x < 256) hist[threadIdx.x] = 0;
    __syncthreads();
    for (int j = threadIdx.x; j < N; j += kSelThreads) {
      const uint32_t key = float_key(sc[j]);
      if ((key & himask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
    }
    __syncthreads();
    if (threadIdx.x == 0) {              // walk down from the largest digit
      int rem = krem, dgt = 255;
      for (; dgt > 0; --dgt) {
        if (hist[dgt] >= rem) break;
        rem -= hist[dgt];
      }
      s_prefix = prefix | ((uint32_t)dgt << shift);
      s_krem = rem;
    }
    __syncthreads();
    prefix = s_prefix;
    krem = s_krem;
    __syncthreads();
  }
  // prefix = key of the k-th largest score; krem = how many of its ties are kept.
  const uint32_t theta = prefix;
  int base_out = 0, ties_seen = 0;
  for (int j0 = 0; j0 < N; j0 += kSelThreads) {
    const int j = j0 + threadIdx.x;
    const uint32_t key = j < N ? float_key(sc[j]) : 0u;
    const bool gt = j < N && key > theta;
    const bool eq = j < N && key == theta;
    int eq_total, keep_total;
    const int eq_before = block_excl_count(eq, wave_tot, eq_total);
    const bool keep = gt || (eq && ties_seen + eq_before < krem);
    const int pos = block_excl_count(keep, wave_tot, keep_total);
    if (keep) out[base_out + pos] = j;
    base_out += keep_total;
    ties_seen += eq_total;
  }
}

}  // namespace

hipError_t launch_select(const Params& p, hipStream_t s, PhaseHook* hook) {
  hipLaunchKernelGGL(k_select_single, dim3(p.B * p.Hkv), dim3(kSelThreads), 0, s, p);
  mark(hook, "select");
  return hipGetLastError();
}

}  // namespace caote
