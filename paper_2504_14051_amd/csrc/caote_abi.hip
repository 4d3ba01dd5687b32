// C ABI of the CAOTE hot path: argument validation, workspace carving, launches.
// No allocation, no synchronisation, no state between calls.
#include <algorithm>
#include <math.h>
#include <mutex>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include "common.hpp"

using caote::Params;

namespace {

thread_local char g_err[512] = "";

caote_status fail(caote_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

caote_status check_layout(const caote_layout* L, int32_t budget, bool need_budget) {
  if (!L) return fail(CAOTE_EINVAL, "layout is NULL");
  if (L->batch < 1 || L->n_q_heads < 1 || L->n_kv_heads < 1)
    return fail(CAOTE_EINVAL, "batch, n_q_heads and n_kv_heads must be >= 1");
  if (L->n_q_heads % L->n_kv_heads != 0)
    return fail(CAOTE_EINVAL, "n_q_heads (%d) is not a multiple of n_kv_heads (%d)", L->n_q_heads,
                L->n_kv_heads);
  if (L->head_dim != 64 && L->head_dim != 128)
    return fail(CAOTE_EUNSUPPORTED, "head_dim %d: only 64 and 128 are supported", L->head_dim);
  if (L->window < 1) return fail(CAOTE_EINVAL, "window must be >= 1");
  if ((int64_t)L->window * (L->n_q_heads / L->n_kv_heads) > (1 << 20))
    return fail(CAOTE_EUNSUPPORTED, "more than 2^20 query rows per KV head");
  if (L->capacity < 1) return fail(CAOTE_EINVAL, "capacity must be >= 1");
  if (L->dtype != CAOTE_BF16 && L->dtype != CAOTE_F32) return fail(CAOTE_EINVAL, "unknown dtype %d", L->dtype);
  if (L->base < CAOTE_BASE_NONE || L->base > CAOTE_BASE_SNAPKV) return fail(CAOTE_EINVAL, "unknown base %d", L->base);
  if (L->variant != CAOTE_EXACT && L->variant != CAOTE_FAST) return fail(CAOTE_EINVAL, "unknown variant %d", L->variant);
  if (L->pool_kernel < 1 || L->pool_kernel % 2 == 0)
    return fail(CAOTE_EINVAL, "pool_kernel must be odd and >= 1 (got %d)", L->pool_kernel);
  if (L->n_protect_head < 0 || L->n_protect_tail < 0) return fail(CAOTE_EINVAL, "negative protected row count");
  if (!(L->softmax_scale == L->softmax_scale) || isinf(L->softmax_scale))
    return fail(CAOTE_EINVAL, "softmax_scale is not finite");
  if (!(L->softmax_scale > 0.f)) return fail(CAOTE_EINVAL, "softmax_scale must be > 0");
  if (L->window_in_cache && !L->seq_lens && L->capacity < L->window)
    return fail(CAOTE_EINVAL, "window (%d) exceeds the cache length (%d)", L->window, L->capacity);
  const int esz = L->dtype == CAOTE_F32 ? 4 : 2;
  const int64_t st[] = {L->k_stride_b, L->k_stride_h, L->k_stride_n, L->v_stride_b, L->v_stride_h,
                        L->v_stride_n, L->q_stride_b, L->q_stride_h, L->q_stride_w};
  for (int i = 0; i < 9; ++i) {
    if (st[i] < 0) return fail(CAOTE_EINVAL, "negative stride");
    if ((st[i] * esz) % 16 != 0) return fail(CAOTE_EINVAL, "strides must be multiples of 16 bytes");
  }
  if (L->k_stride_n < L->head_dim || L->v_stride_n < L->head_dim || L->q_stride_w < L->head_dim)
    return fail(CAOTE_EINVAL, "row stride smaller than head_dim");
  if (L->row_lse && ((uintptr_t)L->row_lse % sizeof(float)) != 0)
    return fail(CAOTE_EINVAL, "row_lse is not aligned to 4 bytes");
  if ((int64_t)L->batch * L->n_kv_heads > 65535)
    return fail(CAOTE_EUNSUPPORTED, "batch * n_kv_heads > 65535");
  if (need_budget && budget < 1) return fail(CAOTE_EINVAL, "budget must be >= 1");
  if (need_budget && L->capacity > caote::kSelSpan * caote::kMaxSpans)
    return fail(CAOTE_EUNSUPPORTED, "selection supports at most %d tokens per head",
                caote::kSelSpan * caote::kMaxSpans);
  return CAOTE_OK;
}

// Fills the launch geometry and the workspace offsets of `p`; returns bytes needed.
size_t plan(const caote_layout* L, int32_t budget, Params& p, char* ws) {
  memset(&p, 0, sizeof(p));
  p.seq_lens = L->seq_lens;
  p.lse_in = L->row_lse;
  p.B = L->batch; p.Hq = L->n_q_heads; p.Hkv = L->n_kv_heads; p.G = p.Hq / p.Hkv;
  p.D = L->head_dim; p.W = L->window; p.R = p.G * p.W; p.cap = L->capacity;
  p.ksb = L->k_stride_b; p.ksh = L->k_stride_h; p.ksn = L->k_stride_n;
  p.vsb = L->v_stride_b; p.vsh = L->v_stride_h; p.vsn = L->v_stride_n;
  p.qsb = L->q_stride_b; p.qsh = L->q_stride_h; p.qsw = L->q_stride_w;
  p.base_mode = L->base; p.pool = L->pool_kernel; p.wic = L->window_in_cache ? 1 : 0;
  p.ph = L->n_protect_head; p.pt = L->n_protect_tail; p.variant = L->variant; p.dtype = L->dtype;
  p.budget = budget;
  p.c2 = L->softmax_scale * 1.4426950408889634f;
  p.rcpW = 1.0f / (float)L->window;

  const int BH = p.B * p.Hkv;
  // Token chunk per workgroup: about `target` workgroups per launch, whole 64-key tiles.
  auto chunk_len = [&](int target, int lo, int hi) {
    int n = ceil_div(target, BH);
    n = n < 1 ? 1 : n;
    int len = (int)align_up((size_t)ceil_div(p.cap, n), 64);
    return len < lo ? lo : (len > hi ? hi : len);
  };
  p.use_mfma = p.dtype == CAOTE_BF16 && p.D == 128 && p.R > 16;
  p.small_r = !p.use_mfma && p.R <= 8;
  p.s_rows = p.R <= 4 ? 4 : 8;
  p.s_pitch = (int)align_up((size_t)p.cap, 4);
  if (p.use_mfma) {
    // equal lengths: one or two workgroups per compute unit, one round.  Ragged lengths (known
    // on the device only): splits of at least 2048 keys in about eight rounds, so that compute
    // units that drew short or empty splits take more of them (measured on 16 prompts of
    // 8k..32k tokens: 3 % faster than one round of 16384-key splits; shorter splits lose to
    // the set-up each workgroup pays)
    if (!p.seq_lens) p.split_len = chunk_len(p.R > 128 ? 256 : 512, 128, 1 << 20);
    else             p.split_len = chunk_len(8 * (p.R > 128 ? 256 : 512), 2048, 1 << 20);
  }
  else if (p.R <= 8)                                      // few rows: matrix cores (bf16, d 128) or vector ALUs
    p.split_len = p.dtype == CAOTE_BF16 && p.D == 128 ? chunk_len(768, 128, 8192) : chunk_len(2048, 128, 8192);
  else
    p.split_len = chunk_len(1024, 256, 8192);
  p.n_split = ceil_div(p.cap, p.split_len);
  // ragged lengths on the matrix-core path: equal shares of all heads' tiles per workgroup
  // (common.hpp, Params::dyn_split); a share is never shorter than 1/32 of a full cache, so a
  // head has at most 34 pieces
  p.dyn_split = (p.use_mfma && p.seq_lens && p.B <= caote::kDynMaxBatch) ? 1 : 0;
  if (p.dyn_split) {
    p.dyn_wgs = p.R > 128 ? 256 : 512;
    p.dyn_min_tiles = std::max(1, ceil_div(ceil_div(p.cap, 64), 32));
    p.n_split = std::min(ceil_div(p.cap, 64), 34);
    p.split_len = 64;      // (not used by the sweeps in this mode)
  }
  p.split_len0 = p.split_len; p.n_split0 = p.n_split; p.n_rg0 = 1;
  if (p.use_mfma) {
    // rows a workgroup of the matrix-core sweeps keeps in registers (see launch_score_mfma)
    const int nrb = ceil_div(p.R, 32), rows = nrb <= 2 ? 64 : (nrb <= 4 ? 128 : 256);
    const int n_rg = ceil_div(p.R, rows);
    if (n_rg > 1 && p.dyn_split) {
      p.n_rg0 = n_rg;    // (each row group runs the same shares)
    } else if (n_rg > 1) {      // several row groups: side by side in the first sweep instead of in turn
      const int want = std::max(1, (rows == 256 ? 256 : 512) / (BH * n_rg));
      p.split_len0 = std::max(128, (int)align_up((size_t)ceil_div(p.cap, want), 64));
      p.n_split0 = ceil_div(p.cap, p.split_len0);
      p.n_rg0 = n_rg;
    }
  }
  p.vchunk_len = caote::kVChunk;
  p.n_vchunk = ceil_div(p.cap, p.vchunk_len);
  p.vrep = ceil_div(p.cap, 128 * caote::kVChunk);      // at most 128 partial sums per head
  p.n_vsum = ceil_div(p.n_vchunk, p.vrep);
  p.Rp = (int)align_up((size_t)p.R, 32);
  p.halo = p.base_mode == CAOTE_BASE_SNAPKV ? p.pool / 2 : 0;
  p.fuse_v = p.use_mfma && p.halo <= 64;
  p.n_vpart = p.fuse_v ? p.n_split : p.n_vsum;
  // short caches whose value sweeps are not fused into the key sweep: V read once, rows held
  // in registers between their two uses
  // (k_vside addresses the rows of a head with 32-bit byte offsets)
  p.vside_cs = (p.dtype == CAOTE_BF16 && p.D == 128 && !p.fuse_v && (int64_t)p.cap * p.vsn * 2 < (1ll << 31))
                   ? caote::vside_column_split(p.cap) : 0;

  size_t off = 0;
  auto carve = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return ws ? ws + o : nullptr; };
  p.stats = (float*)carve((size_t)BH * std::max(p.n_split, p.n_split0) * p.Rp * 2 * sizeof(float));
  p.lse2 = (float*)carve((size_t)BH * p.Rp * sizeof(float));
  p.S = (float*)carve(p.small_r ? (size_t)BH * p.s_pitch * p.s_rows * sizeof(float) : 0);
  p.a = (float*)carve((size_t)BH * p.cap * sizeof(float));
  p.h = (float*)carve((size_t)BH * p.cap * sizeof(float));
  p.opart = (float*)carve((size_t)BH * p.n_vpart * p.D * sizeof(float));
  p.zpart = (float*)carve((size_t)BH * p.n_vpart * sizeof(float));
  p.osum = (float*)carve((size_t)BH * (caote::kMaxD + 1) * sizeof(float));
  p.hist = (uint32_t*)carve((size_t)BH * caote::kHistBins * sizeof(uint32_t));
  p.seg_tab = (caote::SegTab*)carve(p.dyn_split ? (size_t)BH * sizeof(caote::SegTab) : 0);
  p.wg_tab = (int32_t*)carve(p.dyn_split ? (size_t)p.dyn_wgs * sizeof(int32_t) : 0);
  p.seg_glob = (int32_t*)carve(p.dyn_split ? 64 : 0);
  p.n_span = ceil_div(p.cap, caote::kSelSpan);
  p.sel_cand = (uint32_t*)carve((size_t)BH * p.cap * sizeof(uint32_t));
  p.sel_rec = (int32_t*)carve((size_t)BH * p.n_span * 2 * sizeof(int32_t));
  p.sel_head = (int32_t*)carve((size_t)BH * 4 * sizeof(int32_t));
  const size_t row_bytes = (size_t)p.D * (p.dtype == CAOTE_F32 ? 4 : 2);
  const int bud = budget > 0 ? budget : 0;
  p.stage = carve((size_t)BH * bud * (2 * row_bytes + sizeof(float)));
  p.merge_in_vside = p.vside_cs && p.small_r;
  p.d2part = (float*)carve((size_t)p.vside_cs * BH * p.cap * sizeof(float));
  if (p.cap <= caote::kJointMaxCap) {
    p.j_slice = caote::joint_slice_len();
    p.j_c = ceil_div(p.cap, p.j_slice);
    p.j_part = (float*)carve((size_t)2 * BH * p.j_c * (4 + caote::kMaxD) * sizeof(float));
    p.j_u = (float*)carve((size_t)2 * BH * caote::kMaxD * sizeof(float));
    p.j_rest = (double*)carve((size_t)2 * BH * sizeof(double));
  }
  return off;
}

caote_status check_ws(const caote_layout* L, int32_t budget, void* ws, size_t ws_bytes, Params& p) {
  if (!ws) return fail(CAOTE_EWORKSPACE, "workspace is NULL");
  if (((uintptr_t)ws) % 256 != 0) return fail(CAOTE_EWORKSPACE, "workspace is not 256-byte aligned");
  const size_t need = plan(L, budget, p, (char*)ws);
  if (ws_bytes < need)
    return fail(CAOTE_EWORKSPACE, "workspace too small: %zu bytes given, %zu needed", ws_bytes, need);
  return CAOTE_OK;
}

// The kernels fetch rows of q, K and V in 16-byte pieces (DMA into LDS, uint4 loads): with the
// strides already multiples of 16 bytes, the base addresses have to be too.
caote_status check_aligned16(const void* q, const void* K, const void* V) {
  if ((((uintptr_t)q) | ((uintptr_t)K) | ((uintptr_t)V)) % 16 != 0)
    return fail(CAOTE_EINVAL, "q_window, K and V must be 16-byte aligned");
  return CAOTE_OK;
}

caote_status device_status(hipError_t e, const char* what) {
  if (e == hipSuccess) return CAOTE_OK;
  return fail(CAOTE_EDEVICE, "%s: %s", what, hipGetErrorString(e));
}

// Measurement aid: counts and names the kernels of one call and stops the call after the
// first `limit` of them.
struct PrefixHook final : caote::PhaseHook {
  const char* names[CAOTE_MAX_PHASES];
  int n = 0, limit;
  explicit PrefixHook(int lim) : limit(lim) {}
  bool mark(const char* name) override {
    if (n < CAOTE_MAX_PHASES) names[n] = name;
    ++n;
    return limit >= 0 && n >= limit;
  }
  bool full() const override { return limit >= 0 && n >= limit; }
};

caote_status do_score(Params& p, hipStream_t s, PrefixHook* hook = nullptr) {
  hipError_t e = p.use_mfma   ? caote::launch_score_mfma(p, s, hook)
                 : p.small_r  ? (p.dtype == CAOTE_BF16 && p.D == 128 ? caote::launch_score_few_mfma(p, s, hook)
                                                                    : caote::launch_score_small(p, s, hook))
                              : caote::launch_score_generic(p, s, hook);
  if (e != hipSuccess) return device_status(e, "score (key sweeps)");
  if (hook && hook->full()) return CAOTE_OK;
  return device_status(p.vside_cs ? caote::launch_value_side(p, s, hook) : caote::launch_value_passes(p, s, hook),
                       "score (value sweeps)");
}

thread_local const char* g_phase_names[CAOTE_MAX_PHASES] = {};

}  // namespace

// ---- scratch of the entry point that allocates nothing (caote_evict_static) ------------------
// The array lives in the device image: every GPU that loads the library holds its own copy at
// its own address.  In host code the name `scratch` is only a handle for hipGetSymbolAddress;
// the address kernels may use is what that call returns, looked up once per device.
static __device__ __align__(256) unsigned char scratch[CAOTE_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};   // per device: device address of `scratch`, once known

// Device address of the current device's copy of `scratch`.
caote_status static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return device_status(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return fail(CAOTE_EUNSUPPORTED, "device ordinal %d out of range", dev);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return device_status(e, "hipGetSymbolAddress(scratch)");
    if (!ptr || ((uintptr_t)ptr % 256) != 0)
      return fail(CAOTE_EDEVICE, "static scratch resolved to an unusable address %p", ptr);
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return CAOTE_OK;
}

}  // namespace

#pragma GCC visibility push(default)
extern "C" {

const char* caote_last_error(void) { return g_err; }

int32_t caote_version(void) { return 200; }

size_t caote_workspace_bytes(const caote_layout* layout, int32_t budget) {
  if (check_layout(layout, budget, false) != CAOTE_OK) return 0;
  Params p;
  return plan(layout, budget, p, nullptr);
}

caote_status caote_score(const void* q_window, const void* K, const void* V, float* base_score,
                         const caote_layout* layout, float* scores, void* workspace,
                         size_t workspace_bytes, void* hip_stream) {
  caote_status st = check_layout(layout, 0, false);
  if (st != CAOTE_OK) return st;
  if (!q_window || !K || !V || !scores) return fail(CAOTE_EINVAL, "q_window, K, V and scores must not be NULL");
  if ((st = check_aligned16(q_window, K, V)) != CAOTE_OK) return st;
  if (layout->base == CAOTE_BASE_H2O && !base_score)
    return fail(CAOTE_EINVAL, "CAOTE_BASE_H2O needs base_score (the accumulator)");
  Params p;
  st = check_ws(layout, 0, workspace, workspace_bytes, p);
  if (st != CAOTE_OK) return st;
  p.q = q_window; p.K = const_cast<void*>(K); p.V = const_cast<void*>(V);
  p.base = base_score; p.scores = scores;
  if (layout->base == CAOTE_BASE_H2O && !p.vside_cs) p.h = base_score;   // (k_vside keeps h apart)
  return do_score(p, (hipStream_t)hip_stream);
}

caote_status caote_select(const float* scores, const caote_layout* layout, int32_t budget,
                          int32_t* kept_idx, void* workspace, size_t workspace_bytes,
                          void* hip_stream) {
  caote_status st = check_layout(layout, budget, true);
  if (st != CAOTE_OK) return st;
  if (!scores || !kept_idx) return fail(CAOTE_EINVAL, "scores and kept_idx must not be NULL");
  Params p;
  st = check_ws(layout, budget, workspace, workspace_bytes, p);
  if (st != CAOTE_OK) return st;
  p.scores = const_cast<float*>(scores); p.kept = kept_idx;
  return device_status(caote::launch_select(p, (hipStream_t)hip_stream, nullptr), "select");
}

static caote_status check_mode(int32_t mode, int32_t budget) {
  if (mode != CAOTE_COMPACT_STABLE && mode != CAOTE_COMPACT_SWAP_LAST && mode != CAOTE_COMPACT_FILL)
    return fail(CAOTE_EINVAL, "unknown compaction mode %d", mode);
  if (mode == CAOTE_COMPACT_FILL && budget > CAOTE_FILL_MAX_BUDGET)
    return fail(CAOTE_EUNSUPPORTED, "CAOTE_COMPACT_FILL takes budgets up to %d (got %d)", CAOTE_FILL_MAX_BUDGET, budget);
  return CAOTE_OK;
}

caote_status caote_compact(void* K, void* V, float* base_score, const int32_t* kept_idx,
                           const caote_layout* layout, int32_t budget, int32_t mode,
                           void* workspace, size_t workspace_bytes, void* hip_stream) {
  caote_status st = check_layout(layout, budget, true);
  if (st != CAOTE_OK) return st;
  if (!K || !V || !kept_idx) return fail(CAOTE_EINVAL, "K, V and kept_idx must not be NULL");
  if ((st = check_aligned16(nullptr, K, V)) != CAOTE_OK) return st;
  if ((st = check_mode(mode, budget)) != CAOTE_OK) return st;
  Params p;
  st = check_ws(layout, budget, workspace, workspace_bytes, p);
  if (st != CAOTE_OK) return st;
  p.K = K; p.V = V; p.base = base_score; p.kept = const_cast<int32_t*>(kept_idx); p.mode = mode;
  return device_status(caote::launch_compact(p, (hipStream_t)hip_stream, nullptr), "compact");
}

caote_status caote_append(void* K, void* V, float* base_score, const void* k_new,
                          const void* v_new, const caote_layout* layout, int32_t n_at,
                          int32_t n_new, void* hip_stream) {
  caote_status st = check_layout(layout, 0, false);
  if (st != CAOTE_OK) return st;
  if (!K || !V || !k_new || !v_new) return fail(CAOTE_EINVAL, "K, V, k_new and v_new must not be NULL");
  if ((st = check_aligned16(nullptr, K, V)) != CAOTE_OK) return st;
  if (n_new < 0) return fail(CAOTE_EINVAL, "n_new must be >= 0");
  if (!layout->seq_lens && (n_at < 0 || (int64_t)n_at + n_new > layout->capacity))
    return fail(CAOTE_EINVAL, "rows [%d, %d) do not fit the capacity %d", n_at, n_at + n_new,
                layout->capacity);
  if (((uintptr_t)k_new | (uintptr_t)v_new) % 16 != 0)
    return fail(CAOTE_EINVAL, "k_new and v_new must be 16-byte aligned");
  if (n_new == 0) return CAOTE_OK;
  Params p;
  plan(layout, 0, p, nullptr);
  p.K = K; p.V = V; p.base = base_score;
  return device_status(caote::launch_append(p, k_new, v_new, n_at, n_new, (hipStream_t)hip_stream),
                       "append");
}

// Host-side argument checks of the fused calls (nothing is launched before they pass).
static caote_status check_evict_args(const void* q_window, const void* K, const void* V,
                                     const float* base_score, const caote_layout* layout,
                                     int32_t budget, int32_t mode, const float* scores,
                                     const int32_t* kept_idx, bool joint, const int32_t* evicted,
                                     const float* joint_error) {
  caote_status st = check_layout(layout, budget, true);
  if (st != CAOTE_OK) return st;
  if (joint) {
    if (layout->capacity > caote::kJointMaxCap)
      return fail(CAOTE_EUNSUPPORTED, "greedy joint eviction supports a capacity of at most %d rows (got %d)",
                  caote::kJointMaxCap, layout->capacity);
    if (layout->variant != CAOTE_EXACT)
      return fail(CAOTE_EUNSUPPORTED, "greedy joint eviction is defined for CAOTE_EXACT only");
    if ((int64_t)layout->n_protect_head + layout->n_protect_tail > budget)
      return fail(CAOTE_EINVAL, "budget (%d) is smaller than the number of protected rows", budget);
    if (layout->capacity > budget && (!evicted || !joint_error))
      return fail(CAOTE_EINVAL, "evicted and joint_error must not be NULL when capacity > budget");
  }
  if (!q_window || !K || !V || !scores || !kept_idx)
    return fail(CAOTE_EINVAL, "q_window, K, V, scores and kept_idx must not be NULL");
  if ((st = check_aligned16(q_window, K, V)) != CAOTE_OK) return st;
  if (layout->base == CAOTE_BASE_H2O && !base_score)
    return fail(CAOTE_EINVAL, "CAOTE_BASE_H2O needs base_score (the accumulator)");
  if ((st = check_mode(mode, budget)) != CAOTE_OK) return st;
  return CAOTE_OK;
}

// `joint`: selection by the greedy joint error (evicted / joint_error are its extra outputs).
static caote_status evict_impl(const void* q_window, void* K, void* V, float* base_score,
                               const caote_layout* layout, int32_t budget, int32_t mode,
                               float* scores, int32_t* kept_idx, void* workspace,
                               size_t workspace_bytes, hipStream_t s, PrefixHook* prefix,
                               bool joint = false, int32_t* evicted = nullptr,
                               float* joint_error = nullptr) {
  PrefixHook* hook = prefix;
  caote_status st = check_evict_args(q_window, K, V, base_score, layout, budget, mode, scores, kept_idx,
                                     joint, evicted, joint_error);
  if (st != CAOTE_OK) return st;
  Params p;
  st = check_ws(layout, budget, workspace, workspace_bytes, p);
  if (st != CAOTE_OK) return st;
  p.q = q_window; p.K = K; p.V = V; p.base = base_score; p.scores = scores; p.kept = kept_idx;
  p.mode = mode;
  // the merge of the row statistics (or, on the matrix-core path, the second sweep) clears
  // the selection's counters on its way
  p.hist_zeroed = ((!p.lse_in && !p.merge_in_vside) || p.use_mfma) ? 1 : 0;
  // up to 128 scoring workgroups per head add to the same few dozen bins: beyond that the
  // serialised device atomics outlast the kernel, and a histogram kernel of its own is faster
  p.hist_in_vscore = (p.cap > 16384 && p.cap <= 32768 && p.hist_zeroed) ? 1 : 0;
  p.select_swaps = p.cap <= caote::kOneWgCap ? 1 : 0;  // (the one-workgroup selections of launch_select)
  p.combine_in_select = (p.vside_cs && !joint) ? 1 : 0;   // (k_vside caches are short: one-workgroup selection)
  if (joint) p.hist_in_vscore = p.select_swaps = 0;
  if (layout->base == CAOTE_BASE_H2O && !p.vside_cs) p.h = base_score;
  st = do_score(p, s, hook);
  if (st != CAOTE_OK || (prefix && prefix->full())) return st;
  if (joint) {
    const int max_evict = p.cap > budget ? p.cap - budget : 0;
    st = device_status(caote::launch_select_joint(p, evicted, joint_error, max_evict, s, hook), "select (joint)");
  } else {
    st = device_status(caote::launch_select(p, s, hook), "select");
  }
  if (st != CAOTE_OK || (prefix && prefix->full())) return st;
  return device_status(caote::launch_compact(p, s, hook), "compact");
}

caote_status caote_evict(const void* q_window, void* K, void* V, float* base_score,
                         const caote_layout* layout, int32_t budget, int32_t mode, float* scores,
                         int32_t* kept_idx, void* workspace, size_t workspace_bytes,
                         void* hip_stream) {
  return evict_impl(q_window, K, V, base_score, layout, budget, mode, scores, kept_idx, workspace,
                    workspace_bytes, (hipStream_t)hip_stream, nullptr);
}

caote_status caote_evict_static(const void* q_window, void* K, void* V, float* base_score,
                                const caote_layout* layout, int32_t budget, int32_t mode,
                                float* scores, int32_t* kept_idx, void* hip_stream) {
  caote_status st = check_evict_args(q_window, K, V, base_score, layout, budget, mode, scores, kept_idx,
                                     false, nullptr, nullptr);
  if (st != CAOTE_OK) return st;
  Params probe;
  const size_t need = plan(layout, budget, probe, nullptr);
  if (need > (size_t)CAOTE_STATIC_SCRATCH_BYTES)
    return fail(CAOTE_EWORKSPACE,
                "this layout and budget need %zu bytes of scratch; the static array holds %zu "
                "(use caote_evict with a workspace of your own)", need, (size_t)CAOTE_STATIC_SCRATCH_BYTES);
  void* ws = nullptr;
  st = static_scratch(&ws);
  if (st != CAOTE_OK) return st;
  return evict_impl(q_window, K, V, base_score, layout, budget, mode, scores, kept_idx, ws,
                    (size_t)CAOTE_STATIC_SCRATCH_BYTES, (hipStream_t)hip_stream, nullptr);
}

caote_status caote_evict_joint(const void* q_window, void* K, void* V, float* base_score,
                               const caote_layout* layout, int32_t budget, int32_t mode,
                               float* scores, int32_t* kept_idx, int32_t* evicted,
                               float* joint_error, void* workspace, size_t workspace_bytes,
                               void* hip_stream) {
  return evict_impl(q_window, K, V, base_score, layout, budget, mode, scores, kept_idx, workspace,
                    workspace_bytes, (hipStream_t)hip_stream, nullptr, true, evicted, joint_error);
}

caote_status caote_evict_prefix(const void* q_window, void* K, void* V, float* base_score,
                                const caote_layout* layout, int32_t budget, int32_t mode,
                                float* scores, int32_t* kept_idx, void* workspace,
                                size_t workspace_bytes, void* hip_stream, int32_t n_kernels,
                                int32_t* n_launched) {
  PrefixHook hook(n_kernels);
  if (n_kernels == 0) {
    if (n_launched) *n_launched = 0;
    return CAOTE_OK;
  }
  caote_status st = evict_impl(q_window, K, V, base_score, layout, budget, mode, scores, kept_idx,
                               workspace, workspace_bytes, (hipStream_t)hip_stream, &hook);
  if (st != CAOTE_OK) return st;
  for (int i = 0; i < CAOTE_MAX_PHASES; ++i) g_phase_names[i] = i < hook.n ? hook.names[i] : nullptr;
  if (n_launched) *n_launched = hook.n;
  return CAOTE_OK;
}

caote_status caote_read_stream(const void* buf, size_t bytes, void* sink, void* hip_stream) {
  if (!buf || !sink) return fail(CAOTE_EINVAL, "buf and sink must not be NULL");
  if (((uintptr_t)buf % 16) != 0 || bytes % 16 != 0)
    return fail(CAOTE_EINVAL, "buf must be 16-byte aligned and bytes a multiple of 16");
  return device_status(caote::launch_read_stream(buf, bytes, sink, (hipStream_t)hip_stream), "read_stream");
}

caote_status caote_issue_probe(int32_t variant, int32_t iters, void* out, void* hip_stream) {
  if (!out) return fail(CAOTE_EINVAL, "out must not be NULL");
  if (variant < 0 || variant >= CAOTE_ISSUE_PROBE_VARIANTS) return fail(CAOTE_EINVAL, "unknown probe variant %d", variant);
  if (iters < 1 || iters > (1 << 20)) return fail(CAOTE_EINVAL, "iters must be in [1, 2^20]");
  return device_status(caote::launch_issue_probe(variant, iters, (float*)out, (hipStream_t)hip_stream), "issue_probe");
}

const char* caote_phase_name(int32_t i) {
  return i >= 0 && i < CAOTE_MAX_PHASES && g_phase_names[i] ? g_phase_names[i] : "";
}

}  // extern "C"
#pragma GCC visibility pop
