/*
 * caote.h -- C ABI of the MI355X (gfx950) CAOTE hot path: score cached KV tokens
 * by the attention-output error of evicting them, keep the top-`budget` per KV
 * head, and compact the cache in place.
 *
 * Method: "CAOTE: KV Cache Selection for LLMs via Attention Output Error-Based
 * Token Eviction" (arXiv 2504.14051).  Section / equation references below are to
 * that paper.
 *
 * Conventions
 *   - Every data pointer is DEVICE memory owned by the caller.  `caote_layout*` is
 *     HOST memory and is read during the call only.
 *   - The library allocates nothing, keeps no state between calls, and never
 *     synchronises: all kernels are enqueued on `hip_stream` (a hipStream_t passed
 *     as void*, NULL = the default stream) and the call returns immediately.
 *   - Scratch memory comes from the caller: `workspace` must hold at least
 *     caote_workspace_bytes() bytes, be 256-byte aligned, and must not be shared by
 *     calls that can overlap in time.
 *   - Errors: every entry point returns a caote_status.  Argument errors are found
 *     on the host before anything is launched; a failed launch returns
 *     CAOTE_EDEVICE.  Nothing aborts or throws.  caote_last_error() gives the text
 *     of the calling thread's last failure.
 *   - Token counts: a sequence b holds N_b = seq_lens[b] tokens (or `capacity` when
 *     seq_lens is NULL).  The caller guarantees window <= N_b <= capacity when
 *     window_in_cache is set (1 <= N_b otherwise); values of seq_lens outside
 *     [0, capacity] are clamped on the device, so no access leaves the buffers.
 *
 *   - q_window, K and V must be 16-byte aligned (their strides too): rows are fetched
 *     in 16-byte pieces.  Misaligned pointers are rejected with CAOTE_EINVAL.
 *
 * Shapes (row-major, innermost dimension contiguous, strides in ELEMENTS)
 *   q_window  [batch][n_q_heads][window][head_dim]     dtype   (strides q_stride_*)
 *   K, V      [batch][n_kv_heads][capacity][head_dim]  dtype   (strides k_/v_stride_*)
 *   base_score, scores  [batch][n_kv_heads][capacity]  fp32, dense
 *   kept_idx  [batch][n_kv_heads][budget]              int32, dense
 *   Query head hq belongs to KV head hq / (n_q_heads / n_kv_heads).
 */
#ifndef CAOTE_H
#define CAOTE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  CAOTE_OK = 0,
  CAOTE_EINVAL = -1,       /* bad argument (null pointer, inconsistent shape, ...)   */
  CAOTE_EUNSUPPORTED = -2, /* valid request that the kernels do not cover            */
  CAOTE_EWORKSPACE = -3,   /* workspace missing, misaligned or too small             */
  CAOTE_EDEVICE = -4       /* a HIP call failed                                      */
} caote_status;

typedef enum { CAOTE_BF16 = 0, CAOTE_F32 = 1 } caote_dtype;

/* Base retention score h fed to the CAOTE formula (Sec. 3.2).  a_j is the
 * attention mass of cached token j summed over all window query rows of the
 * KV head's group (Sec. 2, f_score,j = sum_i A_ij).                                 */
typedef enum {
  CAOTE_BASE_NONE = 0,   /* h = a.  With window = 1 and one query head per KV head
                            this is TOVA's last-row score (Sec. 2).                 */
  CAOTE_BASE_H2O = 1,    /* h = base_score + a, written back to base_score: the
                            accumulated attention of H2O (Sec. 3.2, App. D.1).      */
  CAOTE_BASE_SNAPKV = 2  /* h = 1-D max-pool (width pool_kernel, stride 1, window
                            clipped at the ends of the scored range) of a.          */
} caote_base;

typedef enum {
  CAOTE_EXACT = 0, /* o = sum_j w_j v_j                       (Sec. 3.2, general score) */
  CAOTE_FAST = 1   /* o = plain mean of the scored values     (Sec. 3.3, FastCAOTE)     */
} caote_variant;

typedef enum {
  CAOTE_COMPACT_STABLE = 0,    /* row i <- row kept_idx[i]; ascending order preserved */
  CAOTE_COMPACT_SWAP_LAST = 1, /* exactly one token evicted: the last row moves into
                                  the hole, all other rows stay where they are; a
                                  sequence that evicts any other number of tokens is
                                  compacted as in CAOTE_COMPACT_STABLE                */
  CAOTE_COMPACT_FILL = 2       /* the fewest row moves for any number of evictions:
                                  kept rows below the new length n = min(N_b, budget)
                                  stay where they are, the kept rows at or beyond n go,
                                  in ascending order, into the positions below n that
                                  evicted rows leave free, taken in ascending order.
                                  Sec. 2 fixes the kept SET, not the order of the rows
                                  (keys carry their positions); kept_idx still lists
                                  the kept tokens in ascending order, not by new row.
                                  budget <= CAOTE_FILL_MAX_BUDGET.                     */
} caote_compact_mode;
#define CAOTE_FILL_MAX_BUDGET 16384

typedef struct caote_layout {
  int32_t batch, n_q_heads, n_kv_heads, head_dim; /* head_dim in {64, 128}           */
  int32_t window;            /* W >= 1: query positions per head in q_window          */
  int32_t capacity;          /* rows allocated per (sequence, KV head)                */
  const int32_t* seq_lens;   /* DEVICE [batch] or NULL (every sequence = capacity)    */
  int64_t k_stride_b, k_stride_h, k_stride_n;
  int64_t v_stride_b, v_stride_h, v_stride_n;
  int64_t q_stride_b, q_stride_h, q_stride_w;     /* all multiples of 16 bytes        */
  int32_t dtype;             /* caote_dtype of q_window, K, V                         */
  int32_t base;              /* caote_base                                            */
  float   softmax_scale;     /* > 0; multiplies every logit; the paper leaves out the
                                usual 1/sqrt(head_dim), the caller supplies it        */
  int32_t pool_kernel;       /* odd, >= 1; used by CAOTE_BASE_SNAPKV only             */
  int32_t window_in_cache;   /* 1: the last W rows of K/V are the window's own
                                tokens and attention inside the window is causal
                                (block-wise prefill, Sec. 2); 0: every key visible    */
  int32_t n_protect_head;    /* first rows are not scored: their score is +INF        */
  int32_t n_protect_tail;    /* last rows likewise (SnapKV: the window).  Protected
                                rows count against the budget and outrank every scored
                                row, so none of them is evicted while budget >= their
                                number; a smaller budget keeps the protected rows of
                                lowest index (the tie rule of caote_select)            */
  int32_t variant;           /* caote_variant                                         */
  const float* row_lse;      /* DEVICE [batch][n_q_heads][window] fp32, dense, or NULL.
                                Softmax normalisers handed over by the caller's own
                                attention pass (App. C prices the score as value-side
                                work only: the attention weights exist already):
                                row_lse = ln sum_j exp(softmax_scale * q.k_j) over the
                                keys visible to that query row (the "LSE" an attention
                                kernel keeps for its backward pass).  When given, the
                                first sweep over K is skipped and A_rj =
                                exp(softmax_scale * q_r.k_j - row_lse_r); nothing is
                                renormalised.  Must be finite.  NULL: computed here.  */
} caote_layout;

/* Bytes of workspace that any entry point may need for this layout and budget.
 * Returns 0 if the layout is invalid (see caote_last_error).                        */
size_t caote_workspace_bytes(const caote_layout* layout, int32_t budget);

/* Scores (Sec. 3.1 CAOTE score; Sec. 3.2 general form; Sec. 3.3 FastCAOTE).
 * For each sequence and KV head:
 *   A   = softmax(softmax_scale * Q_window K^T) over the visible keys (Sec. 2),
 *   a_j = sum over the group's query rows of A_rj,  h from a per `base`,
 *   scored set S = rows [n_protect_head, N - n_protect_tail),
 *   w_j = h_j / sum_{S} h,   o = sum_{S} w_j v_j  (or the mean of v over S),
 *   scores[j] = w_j / (1 - w_j) * || v_j - o ||_2   for j in S,
 *   scores[j] = +INF for protected rows (and when S has a single token).
 * Rows at or beyond N_b are not written.
 *   base_score  in/out for CAOTE_BASE_H2O (all N_b rows are updated); otherwise
 *               unused and may be NULL.
 *   scores      out.                                                               */
caote_status caote_score(const void* q_window, const void* K, const void* V,
                         float* base_score, const caote_layout* layout,
                         float* scores, void* workspace, size_t workspace_bytes,
                         void* hip_stream);

/* Selection (Sec. 2: the top-b tokens by score are retained).  For each
 * (sequence, KV head) writes the indices of the `budget` highest scores among
 * rows [0, N_b) in ASCENDING index order; among equal scores the lower index is
 * kept.  If N_b <= budget all rows are kept and the tail of the list is -1.
 * NaN scores are not allowed.                                                      */
caote_status caote_select(const float* scores, const caote_layout* layout,
                          int32_t budget, int32_t* kept_idx, void* workspace,
                          size_t workspace_bytes, void* hip_stream);

/* Cache update (Sec. 2: after eviction attention uses rows i_1..i_b only).
 * Moves the kept rows of K, V and (if not NULL) base_score to the front of each
 * (sequence, KV head) slab, in place.  kept_idx must be what caote_select
 * produced (ascending, unique, -1 padded).  The new length of a sequence is
 * min(N_b, budget); the caller updates its own seq_lens.  Rows beyond the new
 * length hold unspecified data afterwards.                                         */
caote_status caote_compact(void* K, void* V, float* base_score,
                           const int32_t* kept_idx, const caote_layout* layout,
                           int32_t budget, int32_t mode, void* workspace,
                           size_t workspace_bytes, void* hip_stream);

/* Block-wise prefill with eviction (Sec. 2, block-wise prefill: the new block's keys
 * and values join the cache, K = [K_{:t}, K_{t+1:t+m}]; Sec. 4 uses blocks of 128):
 * copies `n_new` rows per (sequence, KV head) from k_new / v_new into K / V behind
 * the rows the sequence holds, i.e. into rows [N_b, N_b + n_new) with N_b =
 * seq_lens[b], or N_b = `n_at` for every sequence when seq_lens is NULL, and sets
 * the appended rows of base_score (if not NULL) to 0: a token that no query has
 * looked at yet has no accumulated attention.  Rows that would fall beyond
 * `capacity` are dropped.  The caller then raises its seq_lens by n_new and calls
 * caote_evict with the block's queries as the window.
 *   k_new, v_new  DEVICE [batch][n_kv_heads][n_new][head_dim], dense, layout dtype.
 * q_stride_* , window, base and the other scoring fields of the layout are not used. */
caote_status caote_append(void* K, void* V, float* base_score, const void* k_new,
                          const void* v_new, const caote_layout* layout, int32_t n_at,
                          int32_t n_new, void* hip_stream);

/* caote_score + caote_select + caote_compact in one stream-ordered call, with the
 * same results as the three calls in sequence.  `scores` and `kept_idx` are
 * outputs as above.                                                                */
caote_status caote_evict(const void* q_window, void* K, void* V, float* base_score,
                         const caote_layout* layout, int32_t budget, int32_t mode,
                         float* scores, int32_t* kept_idx, void* workspace,
                         size_t workspace_bytes, void* hip_stream);

/* caote_evict for callers that cannot allocate or hand over device memory for scratch:
 * code under HIP graph capture, tight serving loops that own no spare buffer, harnesses that
 * forbid hipMalloc.  Same arguments and same results, bit for bit, as caote_evict, minus the
 * workspace: the scratch memory is a fixed array of CAOTE_STATIC_SCRATCH_BYTES that lives in
 * the library's device image (one copy per GPU the library runs on, held until the process
 * ends).  The call allocates and frees nothing.
 *   - A layout/budget whose caote_workspace_bytes() exceeds CAOTE_STATIC_SCRATCH_BYTES is
 *     rejected with CAOTE_EWORKSPACE before anything is launched.
 *   - The device that owns `hip_stream` must be the calling thread's current device.
 *   - All calls on one GPU share that GPU's array: calls that can overlap in time on one
 *     GPU (different streams, different threads) race; order them on one stream.  Nothing
 *     is assumed about what an earlier call left in the array.                           */
#define CAOTE_STATIC_SCRATCH_BYTES (32u << 20)
caote_status caote_evict_static(const void* q_window, void* K, void* V, float* base_score,
                                const caote_layout* layout, int32_t budget, int32_t mode,
                                float* scores, int32_t* kept_idx, void* hip_stream);

/* Greedy multi-token eviction (App. "Extending CAOTE to Multi-token Eviction"): the
 * fused call with the selection taken under the JOINT error instead of the independent
 * single-token scores.  With w, o and v as in caote_score, the error of evicting a set S is
 *   c_S = || sum_{i in S} w_i (o - v_i) ||_2 / (1 - sum_{i in S} w_i);
 * the exact minimiser over all sets is combinatorial, so tokens leave one at a time: each of
 * the N_b - budget steps evicts the scored row j, not yet evicted, with the smallest
 * c_{S + j}; equal errors evict the higher index; a row whose eviction would leave no weight
 * behind has error +INF.  Every step depends on the one before and needs all value rows of
 * the head again, so the call enqueues ONE KERNEL PER STEP (capacity - budget of them, each
 * a few microseconds whatever N_b is, plus one that writes kept_idx): it is meant for
 * block-wise prefill and generation, where few tokens leave per call, and limited to
 * capacity <= CAOTE_JOINT_MAX_CAPACITY.  Only CAOTE_EXACT; budget >= n_protect_head +
 * n_protect_tail.
 *   scores       out, the single-token scores as caote_score writes them
 *   kept_idx     out, as caote_select: ascending, -1 padded
 *   evicted      DEVICE out int32 [batch][n_kv_heads][capacity - budget]: the row evicted at
 *                each step, in eviction order, then -1
 *   joint_error  DEVICE out fp32, same shape: c_S after each step, then NaN
 * (both may be NULL when capacity == budget).  K, V and base_score are compacted as by
 * caote_evict.  NaN weights or values are not allowed.                                */
#define CAOTE_JOINT_MAX_CAPACITY 8192
caote_status caote_evict_joint(const void* q_window, void* K, void* V, float* base_score,
                               const caote_layout* layout, int32_t budget, int32_t mode,
                               float* scores, int32_t* kept_idx, int32_t* evicted,
                               float* joint_error, void* workspace, size_t workspace_bytes,
                               void* hip_stream);

/* Measurement aid (benchmarks, profiling): enqueues only the first `n_kernels` kernels of
 * the caote_evict call with these arguments (all of them if n_kernels is negative or larger
 * than the call has; none if it is 0).  Like caote_evict it neither allocates nor
 * synchronises, so a stream of truncated calls can be captured and replayed; the time of a
 * call's k-th kernel is the time of the call cut after k kernels minus that of the call cut
 * after k-1.  A truncated call leaves scores, kept_idx and the caches in whatever state the
 * kernels that ran have produced.
 *   n_launched  HOST out (may be NULL): kernels enqueued
 * caote_phase_name(i) names kernel i of the calling thread's last such call.            */
#define CAOTE_MAX_PHASES 16
caote_status caote_evict_prefix(const void* q_window, void* K, void* V, float* base_score,
                                const caote_layout* layout, int32_t budget, int32_t mode,
                                float* scores, int32_t* kept_idx, void* workspace,
                                size_t workspace_bytes, void* hip_stream, int32_t n_kernels,
                                int32_t* n_launched);
const char* caote_phase_name(int32_t i);

/* Measurement aid: reads `bytes` of device memory at `buf` once with plain 16-byte loads and
 * discards them: the read rate a streaming kernel reaches on this device, the empirical
 * ceiling beside the published HBM peak.  buf 16-byte aligned, bytes a multiple of 16;
 * sink: DEVICE, 4 bytes, in practice never written (it keeps the loads alive).           */
caote_status caote_read_stream(const void* buf, size_t bytes, void* sink, void* hip_stream);

/* Measurement aid: `iters` iterations of the instruction mix that one wave of the key sweeps
 * issues per 64-key tile, on registers only, 256 workgroups of eight waves (as the sweeps
 * run).  variant 0: the 16 matrix instructions alone; 1: the vector work alone (32 logits per
 * lane: scale, exp2, maximum, sum); 2: both, the vector work on the matrix results; 3: 16 x
 * (one matrix instruction, then 8 independent fma), order pinned; 4: those 128 fma alone;
 * 5-7: the work of variant 2 in workgroup-barrier intervals of one kind each (every wave issues
 * the matrix instructions of two tiles in one interval and the vector work on their results in
 * the next): 5 with waves 0-3 and 4-7 taking the two kinds in opposite order, 7 with even and
 * odd waves doing so, 6 with all waves in the same order.
 * Timed by the caller; the times tell whether the two pipes overlap on this device.
 *   out  DEVICE, at least CAOTE_ISSUE_PROBE_OUT_BYTES, written with values of no meaning.   */
#define CAOTE_ISSUE_PROBE_VARIANTS 8
#define CAOTE_ISSUE_PROBE_OUT_BYTES (256 * 512 * 4)
caote_status caote_issue_probe(int32_t variant, int32_t iters, void* out, void* hip_stream);

/* Text of the calling thread's most recent failure ("" if none).  The pointer
 * stays valid until that thread's next failing call.                               */
const char* caote_last_error(void);

/* Library version, major*10000 + minor*100 + patch.                                */
int32_t caote_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CAOTE_H */
