/*
 * xkv.h - C ABI of libxkv: the decode hot path of XKV (arXiv 2412.05896,
 * "Personalized KV Cache Memory Reduction for Long-Context LLM Inference") on
 * one AMD MI355X (gfx950).
 *
 * The library keeps a ragged KV cache in which every layer (and sequence) has
 * its own token budget, and provides
 *   - xkv_allocate_budgets      host solver for the per-layer cache sizes
 *   - xkv_decode_attend_score   one decode step of attention over the cache
 *                               that also accumulates every cached token's
 *                               attention probability into its importance
 *   - xkv_evict_compact         keep the top-budget tokens per (layer, KV
 *                               head) and compact K, V, score, pos in place
 *   - xkv_decode_step           the two above as one call
 *   - xkv_prefill_evict         fill the cache from a dense prompt, keeping per
 *                               (layer, KV head) the tokens the observation
 *                               window attends to most (xkv_prefill_evict_lse:
 *                               with the window rows' softmax normalisers given)
 *   - xkv_window_importance, xkv_cache_importance, xkv_allocate_budgets_device,
 *     xkv_average_allocations   the per-layer score vectors and the allocation
 *                               on the device, for budgets that follow the task
 *   - xkv_repack                move the live tokens into arenas of other
 *                               capacities
 *
 * Conventions for every call
 *   - Pointers marked HOST are ordinary host memory, pointers marked DEVICE
 *     are device memory of the current HIP device.  All are owned by the
 *     caller; the library allocates no device memory and frees nothing.
 *     Scratch comes in through `workspace` (xkv_workspace_bytes), a DEVICE
 *     buffer aligned to 256 bytes.
 *   - Device work is enqueued on `hip_stream` (a hipStream_t, NULL = default
 *     stream) and the call returns without waiting.  The host `len` table is
 *     updated at enqueue time: lengths never depend on data.
 *   - Argument errors are detected before anything is enqueued and leave all
 *     state untouched.  No call throws, aborts or synchronises the device.
 *   - Calls on one cache must be ordered by the caller (same stream).
 *   - The library keeps a little process-wide state (xkv_configure,
 *     xkv_profile_*, cached device properties of the first device used): calls
 *     from several host threads must be serialised by the caller, and one
 *     process drives one GPU.
 */
#ifndef XKV_H
#define XKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t xkv_status;

enum {
  XKV_OK = 0,
  XKV_ERR_INVALID_ARG = -1, /* NULL, bad range, bad value */
  XKV_ERR_INFEASIBLE = -2,  /* allocator constraints cannot be met */
  XKV_ERR_CAPACITY = -3,    /* a stream or the workspace is too small */
  XKV_ERR_UNSUPPORTED = -4, /* head_dim / dtype / group size not built */
  XKV_ERR_DEVICE = -5       /* a HIP launch failed */
};

enum { XKV_F32 = 0, XKV_BF16 = 1 };

enum {
  XKV_ALLOC_TOTAL_SIZE = 0, /* Eq. 17: maximise R_avg s.t. sum n_i = total */
  XKV_ALLOC_TARGET_RAVG = 1 /* Eq. 18: minimise sum n_i s.t. R_avg >= target */
};

/* Human-readable name of a status code (static string, never NULL). */
const char* xkv_status_string(xkv_status s);

/*
 * Adaptive allocation (Alg. 1; objectives Eq. 17 and Eq. 18; retention ratio
 * Eq. 4).  Host only, touches no device.
 *
 *   w[l]          HOST, len[l] non-negative finite floats: the attention-score
 *                 distribution vector of layer l, in any order; not modified
 *   mode          XKV_ALLOC_TOTAL_SIZE: budgets sum to total_size exactly and
 *                 maximise R_avg = (1/L) sum_l Sum(TopK(n_l, w_l)) / Sum(w_l).
 *                 XKV_ALLOC_TARGET_RAVG: the greedy stops as soon as
 *                 R_avg >= target_ravg (a fraction in [0,1]); total_size is
 *                 ignored.
 *   min_budget    HOST [n_layers] floors, NULL = 0
 *   max_budget    HOST [n_layers] caps, NULL = len (values above len[l] are
 *                 clamped to len[l])
 *   budgets_out   HOST [n_layers]
 *   ravg_out      HOST, R_avg of the result as a fraction; may be NULL
 *
 * Equal contributions go to the lower layer index, so the result is unique.
 * A layer whose w sums to zero contributes 0 per token.
 * Errors: INVALID_ARG (NULL, n_layers <= 0, negative len, NaN/Inf/negative w,
 * bad mode, target outside [0,1]); INFEASIBLE (min > max, sum(min) >
 * total_size, total_size > sum(max)).
 */
xkv_status xkv_allocate_budgets(int32_t n_layers, const float* const* w, const int64_t* len,
                                int32_t mode, int64_t total_size, double target_ravg,
                                const int64_t* min_budget, const int64_t* max_budget,
                                int64_t* budgets_out, double* ravg_out);

/*
 * Sampling-based overhead reduction (Sec. 4.3): the allocation list for a new
 * task of a known type, from the lists that the allocator produced on sampled
 * tasks of that type.  Host only.
 *
 *   lists        HOST [n_samples][n_layers], each >= 0, not all zero
 *   total_size   tokens to hand out; the per-layer averages are scaled so that
 *                they sum to it: x_l = total_size * sum_s lists[s][l] / sum of
 *                all entries (exact rational arithmetic)
 *   budgets_out  HOST [n_layers]: floor(x_l), plus one for the layers with the
 *                largest fractional parts until the total is met (equal parts:
 *                lower layer first).  With bounds, the list is then clamped and
 *                single tokens go to the layer furthest below its x_l that is
 *                under its cap, or leave the one furthest above that is over its
 *                floor (equal distances: lower layer), until the total is met.
 * Errors: INVALID_ARG, INFEASIBLE (min > max, total outside [sum min, sum max]).
 */
xkv_status xkv_average_allocations(int32_t n_samples, int32_t n_layers, const int64_t* lists,
                                   int64_t total_size, const int64_t* min_budget,
                                   const int64_t* max_budget, int64_t* budgets_out);

/*
 * Device form of the allocation (Alg. 1; Eq. 17 and Eq. 18), for score vectors
 * that already live on the device, such as the w_out of xkv_window_importance.
 * XKV_ALLOC_TOTAL_SIZE gives the same result as xkv_allocate_budgets whenever no
 * two layers have contributions that agree to the last bit at the threshold (the
 * layer sums are added in a different order, which can move such a tie); the
 * retained importance R_avg of the result is the optimum in every case.
 * XKV_ALLOC_TARGET_RAVG bisects the total-size solver for the smallest total whose
 * R_avg reaches target_ravg (all tokens if none does); where R_avg of a total
 * equals the target to within rounding, that total may differ from the host
 * version's by the tokens whose contributions fall inside that rounding.
 *
 *   w             DEVICE fp32: layer l's len values start at w + l * layer_stride
 *                 (layer_stride >= len); non-negative and finite (not checked:
 *                 the call does not read w on the host)
 *   min_budget, max_budget, budgets_out, ravg_out   HOST, as above
 *   workspace     DEVICE, 256-byte aligned, xkv_allocate_device_workspace_bytes
 *
 * Unlike the other device calls this one returns host results: it waits for
 * hip_stream (once per round of bound fixing, usually one or two rounds; the
 * target mode solves about log2(total tokens) total-size problems).
 * Supported: n_layers <= 256.  Errors: INVALID_ARG, INFEASIBLE, UNSUPPORTED,
 * CAPACITY, DEVICE.
 */
xkv_status xkv_allocate_device_workspace_bytes(int32_t n_layers, int64_t len, size_t* bytes_out);
xkv_status xkv_allocate_budgets_device(int32_t n_layers, const float* w, int64_t len,
                                       int64_t layer_stride, int32_t mode, int64_t total_size,
                                       double target_ravg, const int64_t* min_budget,
                                       const int64_t* max_budget, int64_t* budgets_out,
                                       double* ravg_out, void* workspace, size_t workspace_bytes,
                                       void* hip_stream);

/*
 * The ragged cache.  Region (l, b) holds n_kv_heads streams, one per KV head,
 * each with room for cap[l*batch+b] tokens ("slots") of which the first
 * len[l*batch+b] are live; all heads of a region have the same length.
 * Stream (l, b, h) starts at slot  S = region_off[l*batch+b] + h*cap[l*batch+b]:
 *   its K rows are k[(S + j)*head_dim .. +head_dim), likewise v;
 *   score[S + j] is the token's accumulated attention mass (fp32);
 *   pos[S + j]   is the token's original position in the sequence.
 * Rows are contiguous [slot][head_dim]; k and v must be 16-byte aligned.
 * The order of slots inside a stream carries no meaning (attention does not
 * depend on it); pos travels with each row.
 */
typedef struct {
  int32_t n_layers, batch, n_q_heads, n_kv_heads, head_dim;
  int32_t dtype;             /* XKV_F32 or XKV_BF16: element type of k, v, q */
  int64_t arena_slots;       /* slots in each of k, v, score, pos (for bounds checks) */
  void* k;                   /* DEVICE [arena_slots][head_dim] */
  void* v;                   /* DEVICE [arena_slots][head_dim] */
  float* score;              /* DEVICE [arena_slots] */
  int32_t* pos;              /* DEVICE [arena_slots] */
  const int64_t* region_off; /* HOST [n_layers*batch], in slots */
  const int32_t* cap;        /* HOST [n_layers*batch] */
  int32_t* len;              /* HOST [n_layers*batch], updated by the library */
} xkv_cache;

/*
 * Bytes of device workspace that any later call on at most
 * max_layers_per_call layers of this cache can need, whatever the lengths
 * (computed from cap, not len).  Errors: INVALID_ARG, UNSUPPORTED.
 */
xkv_status xkv_workspace_bytes(const xkv_cache* cache, int32_t max_layers_per_call,
                               size_t* bytes_out);

/*
 * One decode step over layers [layer_begin, layer_end)  (Eq. 1 and Eq. 2; the
 * generation phase of Sec. 4.1; scoring = the Select and Merge steps of Eq. 3 /
 * Alg. 2 with the decode query as the observation row and a sum as the merge).
 *
 * For every (l, b, h): if k_new/v_new are given, the new token's rows are
 * appended at slot len (score 0, pos = pos_new[b]) and len grows by one; then
 * for each of the G = n_q_heads/n_kv_heads query heads g of KV head h
 *     p_j   = softmax_j( scale * q_g . K_j )      over all len live slots
 *     out_g = sum_j p_j V_j
 * and score[j] += sum_g p_j.  Products of stored elements are exact and sums
 * are fp32, with one exception: for bf16 caches with head_dim 128 and G >= 4 the
 * output sum runs on the matrix cores, where each unnormalised probability
 * enters as the sum of two bf16 numbers (its rounded value and the rounded
 * remainder): a relative error below 2^-16 per term of out.  The scores do not
 * take that route.
 *
 *   q        DEVICE [layers][batch][n_q_heads][head_dim], cache dtype; query
 *            head hq reads KV head hq / G
 *   k_new, v_new  DEVICE [layers][batch][n_kv_heads][head_dim]; both NULL = no
 *            append
 *   pos_new  HOST [batch]; ignored without append
 *   softmax_scale  0 = 1/sqrt(head_dim)
 *   out      DEVICE [layers][batch][n_q_heads][head_dim] fp32.  A stream with
 *            no live slot gives a zero row.
 *
 * Supported: head_dim 64 or 128, G in {1, 2, 4, 8}; streams of up to 12288 / G
 * strips (strips are 256 to 4096 slots: 786 432 slots at G = 8 in the worst
 * case), beyond which the call returns UNSUPPORTED.
 * Errors: INVALID_ARG, UNSUPPORTED, CAPACITY (len + 1 > cap on append, or the
 * workspace is too small), DEVICE.  Results are bit-reproducible: no atomics.
 */
xkv_status xkv_decode_attend_score(xkv_cache* cache, int32_t layer_begin, int32_t layer_end,
                                   const void* q, const void* k_new, const void* v_new,
                                   const int32_t* pos_new, float softmax_scale, float* out,
                                   void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * xkv_decode_attend_score for callers that cannot allocate device memory or hand
 * over a workspace: code running under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments without the workspace, same
 * kernels (the streaming kernel plus the finalize kernel; never the fused
 * launch) and bit-identical results; the strip records live in a fixed array of
 * XKV_NOALLOC_SCRATCH_BYTES inside the library's device image, which every GPU
 * the library runs on holds until the process ends.  The call makes no hipMalloc,
 * hipFree or other allocating device call.  (The first call on a device looks up
 * the array's device address; make that call outside stream capture.)
 *
 * Limit: the call's strip records must fit the array; roughly 2 G bytes (bf16
 * caches) or 4 G bytes (fp32 caches) per live token per KV head plus 1 KiB per
 * strip (the 32k-context benchmark step of 6.7 M token-heads at G = 1 takes
 * 15 MB of the 32 MiB).  Beyond it the call returns
 * XKV_ERR_CAPACITY and does nothing.  Nothing in the array needs clearing between
 * calls (every record is written before it is read), but all calls on one GPU
 * share it: calls that overlap on one GPU (different streams, or several host
 * threads) race, and the caller must order them.
 * Errors: as xkv_decode_attend_score; DEVICE also when the array's address cannot
 * be resolved.
 */
#define XKV_NOALLOC_SCRATCH_BYTES (32u << 20)
xkv_status xkv_decode_attend_score_noalloc(xkv_cache* cache, int32_t layer_begin, int32_t layer_end,
                                           const void* q, const void* k_new, const void* v_new,
                                           const int32_t* pos_new, float softmax_scale, float* out,
                                           void* hip_stream);

/*
 * Eviction of layers [layer_begin, layer_end)  (Alg. 2 steps 4-7: Pooling,
 * TopK, EvictByIndex on K and V).
 *
 * For every (l, b, h) with n = len and k' = min(budgets[(l-layer_begin)*batch+b], n):
 *   key_j = score_j, or for pool_size > 1 the fp32 sum, added left to right,
 *           of score over the window of pool_size slots centred on j (zeros
 *           outside the stream);
 *   tokens whose pos is among the n_protect highest positions of the stream
 *           (pos >= 1 + max pos - n_protect) are never evicted;
 *   the k' tokens with the largest key are kept, equal keys by lower slot;
 *   kept tokens at slots >= k' are moved, in ascending order, into the
 *           evicted slots < k', in ascending order (K, V, score and pos move
 *           together; nothing else moves); len becomes k'.
 *
 *   budgets       HOST [layers][batch], each >= 0 and >= n_protect
 *   pool_size     odd, >= 1
 *   kept_idx_out  DEVICE [arena_slots] or NULL: entry S + s (s < k') receives
 *                 the slot, before the call, of the token now at slot s
 *
 * budget >= len is not an error: nothing moves and kept_idx is the identity.
 * Scores are expected to be non-negative and not NaN (they are sums of
 * probabilities); otherwise the selection is unspecified.
 * Errors: INVALID_ARG, CAPACITY (workspace too small), DEVICE.
 */
xkv_status xkv_evict_compact(xkv_cache* cache, int32_t layer_begin, int32_t layer_end,
                             const int32_t* budgets, int32_t pool_size, int32_t n_protect,
                             int32_t* kept_idx_out, void* workspace, size_t workspace_bytes,
                             void* hip_stream);

/*
 * One decode step of layers [layer_begin, layer_end): xkv_decode_attend_score
 * followed by xkv_evict_compact with the same arguments, as one call (Sec. 4.1,
 * generation phase: every new token is appended, attended to and scored, and the
 * cache is cut back to its budget; Eq. 1-3, Alg. 2 steps 4-7).  The cache, out
 * and kept_idx_out end up exactly as after the two calls (scores, kept indices
 * and moved rows bit for bit; out up to the order of its fp32 sums).
 *
 * In the steady state of decoding (every stream of the call evicts at most 8
 * tokens, at most 1 with pooling or protected tokens, and a query group the
 * split-K kernels serve without the matrix cores)
 * the eviction runs inside the kernel that updates the scores, on the scores it
 * has just computed: one launch less, no key workspace and, without pooling and
 * protected tokens, no second pass over the scores.  Any other call runs the two
 * calls' kernels one after the other.
 *
 *   arguments   as for xkv_decode_attend_score and xkv_evict_compact; budgets apply
 *               to the lengths after the append; workspace at least
 *               xkv_workspace_bytes
 * Errors: those of the two calls, all detected before anything is enqueued.
 */
xkv_status xkv_decode_step(xkv_cache* cache, int32_t layer_begin, int32_t layer_end, const void* q,
                           const void* k_new, const void* v_new, const int32_t* pos_new,
                           float softmax_scale, float* out, const int32_t* budgets, int32_t pool_size,
                           int32_t n_protect, int32_t* kept_idx_out, void* workspace,
                           size_t workspace_bytes, void* hip_stream);

/*
 * Moves the live tokens of layers [layer_begin, layer_end) of `src` into `dst`, a
 * cache of the same shape (layers, batch, heads, head_dim, dtype) with arenas and
 * stream capacities of its own: slot j < len of every stream (l, b, h) of src goes
 * to slot j of the same stream of dst (K row, V row, score, pos), and dst's len
 * becomes src's.  This is how the ragged layout follows the allocation list of
 * Alg. 1: after the first eviction has cut every layer to its budget, the
 * prompt-sized arena is left for one whose streams hold budget + a few slots.
 * One launch per 1024 regions on hip_stream, geometry in the kernel arguments;
 * src is not modified.
 * Errors: INVALID_ARG (shapes differ, or the arenas of src and dst overlap),
 * CAPACITY (a stream of dst is shorter than its length in src; nothing is
 * enqueued), DEVICE.
 */
xkv_status xkv_repack(const xkv_cache* src, xkv_cache* dst, int32_t layer_begin, int32_t layer_end,
                      void* hip_stream);

/*
 * Eviction of the prefill phase for layers [layer_begin, layer_end): Alg. 2 as
 * written (attention weights of the observation window, Select, Merge, Pooling,
 * TopK, EvictByIndex; Eq. 3 and the attention processing module of Sec. 4.1),
 * from a dense prompt into the ragged cache.
 *
 * For every (l, b, h), with tc = t - ows candidates and k' = min(budget, t):
 *   window row r (prompt position tc + r) of each of the G query heads of KV
 *     head h attends causally to positions 0 .. tc + r:
 *     p_rj = softmax_j( scale * q_r . K_j ) over those positions;
 *   w_j = sum over the G heads and the ows rows of p_rj (fp32), for all j < t:
 *     the mean the paper merges with, times the constant ows;
 *   key_j, j < tc = w_j, or for pool_size > 1 the fp32 sum, added left to right,
 *     of w over the window of pool_size candidates centred on j (zeros outside
 *     [0, tc): nothing of the observation window enters a key);
 *   kept = the k' - ows candidates with the largest key (equal keys by lower
 *     position) and the ows window positions;
 *   slot s < k' of the stream receives the s-th kept position j, in ascending
 *     order: its K and V rows, score = w_j (not pooled), pos = j.  len becomes
 *     k'; what the region held before is overwritten.
 *
 *   q_win    DEVICE [layers][batch][n_q_heads][ows][head_dim], cache dtype
 *   k_src, v_src  DEVICE [layers][batch][n_kv_heads][t][head_dim], cache dtype;
 *            must not overlap the cache
 *   t        rows per stream of k_src / v_src / w_out: the longest prompt of the batch
 *   t_per_seq  HOST [batch] or NULL: the prompt length t_b of every sequence,
 *            ows <= t_b <= t (rows at or beyond t_b are never read, and their
 *            w_out entries are not written); NULL = all prompts have t tokens.
 *            Wherever t appears above, sequence b uses t_b.  1 <= ows <= t
 *   budgets  HOST [layers][batch], each >= ows
 *   softmax_scale  0 = 1/sqrt(head_dim)
 *   w_out    DEVICE [layers][batch][n_kv_heads][t] fp32 or NULL: receives w
 *   workspace  at least xkv_prefill_workspace_bytes
 *
 * Supported: ows * G <= 64, t - ows <= 262144, batch <= 256 when t_per_seq is given.  Errors: INVALID_ARG, UNSUPPORTED,
 * CAPACITY (k' > cap or the workspace is too small), DEVICE.  Bit-reproducible.
 *
 * A call with few, long streams (more than 8192 candidates each, and no more
 * (8192-candidate chunk, stream) pairs than the GPU has compute units) runs TopK
 * as one launch whose workgroups wait for each other between the digits of the
 * radix select.  The waits are bounded (XKV_CFG_FUSED_SPIN_LIMIT, at most 2^16
 * polls); they complete whenever the launch is resident, which one workgroup per
 * compute unit is on an otherwise idle GPU.  Should one run out, the
 * regions of the streams concerned keep what they held before the call (their
 * len is still set to k'), the other streams are complete, and
 * xkv_fused_status reports it.
 */
xkv_status xkv_prefill_workspace_bytes(const xkv_cache* cache, int32_t max_layers_per_call,
                                       int32_t t, int32_t ows, size_t* bytes_out);
xkv_status xkv_prefill_evict(xkv_cache* cache, int32_t layer_begin, int32_t layer_end,
                             const void* q_win, const void* k_src, const void* v_src, int32_t t,
                             const int32_t* t_per_seq, int32_t ows, int32_t pool_size,
                             const int32_t* budgets,
                             float softmax_scale, float* w_out, void* workspace,
                             size_t workspace_bytes, void* hip_stream);

/*
 * xkv_prefill_evict for a caller that already holds the softmax normalisers of the
 * observation window's rows (Eq. 2): an attention forward pass over the prompt
 * leaves, for every query row, the logarithm of its row sum; Alg. 2 takes the
 * window's attention weights from that pass.  With them given the statistics pass
 * over K is not needed and K is read once.
 *
 *   lse_win  DEVICE [layers][batch][n_q_heads][ows] fp32, natural logarithm:
 *            lse = ln sum_{j <= tc + r} exp(scale * q_r . K_j) for window row r
 *            (its causal range, sequence b's own t_b), the same scale as
 *            softmax_scale
 *
 * Everything else as xkv_prefill_evict, with p_rj = exp(scale * q_r . K_j - lse):
 * the result is that of xkv_prefill_evict up to rounding when lse_win holds the
 * rows' true normalisers, and whatever the formula gives otherwise (the library
 * cannot check them).  Both dtypes; same workspace size.
 * Errors: as xkv_prefill_evict; INVALID_ARG for a NULL or misaligned lse_win.
 */
xkv_status xkv_prefill_evict_lse(xkv_cache* cache, int32_t layer_begin, int32_t layer_end,
                                 const void* q_win, const void* k_src, const void* v_src, int32_t t,
                                 const int32_t* t_per_seq, int32_t ows, int32_t pool_size,
                                 const int32_t* budgets, float softmax_scale, const float* lse_win,
                                 float* w_out, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The attention processing module of the mini-prefill (Sec. 4.1, Eq. 3) for
 * layers [layer_begin, layer_end) of a cache geometry: the attention score
 * distribution vector of every (layer, sequence), ready for the allocator.
 *
 *   w_out[l][b][j], j < t - ows  =  pooled_j( sum over the KV heads h of w^h ),
 * with w^h the window mass of xkv_prefill_evict for stream (l, b, h); the heads
 * are added in index order in fp32, and pooling is the same left-to-right window
 * sum over the candidate vector (zeros outside).  Only K is read; the cache's
 * arenas are not touched (only its shape fields are used).
 *
 *   q_win, k_src, t, t_per_seq, ows, pool_size, softmax_scale   as for xkv_prefill_evict
 *   w_out      DEVICE [layers][batch][t - ows] fp32 (sequence b: the first t_b - ows entries)
 *   workspace  at least xkv_prefill_workspace_bytes
 * Errors: INVALID_ARG, UNSUPPORTED, CAPACITY, DEVICE.
 */
xkv_status xkv_window_importance(const xkv_cache* cache, int32_t layer_begin, int32_t layer_end,
                                 const void* q_win, const void* k_src, int32_t t,
                                 const int32_t* t_per_seq, int32_t ows, int32_t pool_size, float softmax_scale, float* w_out,
                                 void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * xkv_window_importance with the window rows' normalisers given (lse_win as for
 * xkv_prefill_evict_lse): K is read once.
 * Errors: as xkv_window_importance; INVALID_ARG for a NULL or misaligned lse_win.
 */
xkv_status xkv_window_importance_lse(const xkv_cache* cache, int32_t layer_begin, int32_t layer_end,
                                     const void* q_win, const void* k_src, int32_t t,
                                     const int32_t* t_per_seq, int32_t ows, int32_t pool_size,
                                     float softmax_scale, const float* lse_win, float* w_out,
                                     void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The attention score distribution vector of every (layer, sequence) of layers
 * [layer_begin, layer_end) taken from the cache itself, so that the allocation
 * (Alg. 1) can be run again during generation (the allocation is meant to follow
 * the task, Sec. 2; Alg. 1 takes one vector per layer, Sec. 4.1).  After per-head
 * eviction the KV heads of a layer hold different tokens, so the vector is
 * indexed by original position:
 *
 *   w_out[l][b][p], p < n_pos  =  sum over the KV heads h, in index order, fp32,
 *       of score[j] of the live slot j of stream (l, b, h) with pos[j] = p,
 *       over the heads that hold such a slot; 0 where none does.
 *
 * Positions are expected to be distinct within a stream (they are original token
 * positions); live slots whose pos lies outside [0, n_pos) are left out.  The
 * result feeds xkv_allocate_budgets_device (per sequence b: w = w_out + b * n_pos,
 * layer_stride = batch * n_pos, len = n_pos); the new budgets take effect through
 * xkv_repack (if a layer is to grow) and xkv_evict_compact.
 *
 *   w_out   DEVICE [layers][batch][n_pos] fp32, fully written (zero-filled)
 * No workspace; one launch per 1024 regions on hip_stream; bit-reproducible.
 * Errors: INVALID_ARG (NULL, n_pos < 1), DEVICE.
 */
xkv_status xkv_cache_importance(const xkv_cache* cache, int32_t layer_begin, int32_t layer_end,
                                int32_t n_pos, float* w_out, void* hip_stream);

/*
 * Process-wide options, for tests and benchmarks.
 *   XKV_CFG_ATTEND_PATH  how xkv_decode_attend_score runs: 0 = the library's
 *       choice (default; at present the two kernels); 1 = a streaming kernel plus
 *       a finalize kernel; 2 = one fused cooperative launch that keeps the logits
 *       in LDS, or XKV_ERR_UNSUPPORTED when the call does not fit the chip at once.
 *   XKV_CFG_FUSED_SPIN_LIMIT  polls of the fused launch's grid-wide wait before a
 *       workgroup gives up (0 .. 2^30; -1 = the default, 2^24, several hundred
 *       milliseconds).  For tests of the give-up path: with 0 every workgroup but
 *       the last to arrive gives up at once, and the kernel still ends normally.
 *       The waits of xkv_prefill_evict's one-launch TopK take the same limit,
 *       capped at 2^16 (their polls are slower); with 0 they give up unpolled.
 * Errors: INVALID_ARG for an unknown key or value.
 */
enum { XKV_CFG_ATTEND_PATH = 1, XKV_CFG_FUSED_SPIN_LIMIT = 2 };
xkv_status xkv_configure(int32_t key, int64_t value);

/*
 * How a caller learns that a fused launch (XKV_CFG_ATTEND_PATH = 2) gave up.
 * The fused kernel's workgroups meet once at a grid-wide wait; it completes
 * whenever all workgroups are resident, which the library ensures by sizing the
 * grid from the occupancy query.  Should a workgroup nevertheless exhaust its
 * polls, it raises a flag in the workspace; every workgroup that finds the flag up
 * after the wait skips the merge: the out rows of the streams it worked on become
 * NaN, and their scores and the pos of their appended tokens are not written (the
 * appended K/V rows are in place and len has grown).  The remaining rows are
 * complete.
 *
 * xkv_fused_status waits for the stream of the most recent call of this process
 * that launched a kernel with such waits (a fused xkv_decode_attend_score, or an
 * xkv_prefill_evict whose TopK ran as one launch) and stores 1 in gave_up_out if
 * any of its launches raised the flag, else 0 (also 0 if there was no such call).
 * Call it before that call's workspace is used again or freed.
 * Errors: INVALID_ARG, DEVICE.
 */
xkv_status xkv_fused_status(int32_t* gave_up_out);

/*
 * Per-kernel timing for benchmarks.  While enabled, the device calls above record
 * HIP events around their dominant kernel (the K/V streaming kernel of
 * xkv_decode_attend_score, kernel index 0, the selection kernel of
 * xkv_evict_compact, kernel index 1, the first K pass of xkv_prefill_evict,
 * kernel index 2, and the kernel of xkv_decode_step that updates the scores and
 * evicts, kernel index 3: it is recorded only when the step took that kernel) on
 * the stream they launch on.
 * xkv_profile_read waits for those events, returns the number of launches and
 * their summed duration in milliseconds since the last xkv_profile_enable(1),
 * and keeps them until the next enable.  Off by default; not for use under
 * stream capture.
 */
xkv_status xkv_profile_enable(int32_t on);
xkv_status xkv_profile_read(int32_t kernel_index, int64_t* launches_out, double* total_ms_out);

/*
 * Measurement helper, no part of the method: one launch of a kernel that only
 * reads `bytes` (rounded down to a multiple of 128 KiB) of the DEVICE buffer,
 * in the shape of the attention kernels' K/V read (256-thread workgroups, 128 KiB
 * each, 16-byte loads), with non-temporal loads or ordinary ones, and writes
 * store_floats_per_workgroup floats per workgroup to the DEVICE array `sink`
 * (which must hold that many floats per 128 KiB read, and at least one) with
 * store_policy 0 = ordinary stores, 1 = non-temporal stores, 2 = the stores the
 * library uses for its workspace (system scope, written through).  The buffer
 * should not consist of words whose XOR is 0x9e3779b9.
 * The caller times it.  Errors: INVALID_ARG, DEVICE.
 */
xkv_status xkv_probe_stream_read(const void* buffer, size_t bytes, int32_t non_temporal,
                                 int32_t store_floats_per_workgroup, int32_t store_policy,
                                 float* sink, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* XKV_H */
