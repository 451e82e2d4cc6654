/*
 * laq.h -- C ABI of the LAQ re-eviction hot path for AMD MI355X (gfx950).
 *
 * The library implements the second-round eviction of Lookahead Q-Cache
 * (paper Sec. 4.3 "KV-Cache Re-eviction", Eq. 4): the cached lookahead queries
 * (the Q-cache of Sec. 4.2) act as the observation window; their attention to
 * every cached key is summed, the ranking is cut at the budget B, and the
 * surviving key/value rows form the cache that decoding continues on.
 *
 * Terms used below
 *   instance   one (sequence, layer) pair; all instances of a call share a shape
 *   Hq, Hkv    query heads / KV heads, G = Hq / Hkv consecutive query heads per KV head
 *   L          rows of K (and V) per KV head handed in; the last W rows are the
 *              window tokens themselves, P = L - W is the prefix that is ranked
 *   W          cached window queries per query head; query w stands at position
 *              P + w and sees keys j <= P + w
 *   Bk         min(budget, L): rows kept per KV head, window included
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller; tensors are dense,
 *     row-major, innermost dimension contiguous (k and v may instead carry the strides of
 *     laq_shape).  `budget` is a HOST array.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     only enqueue work on it and return; the caller synchronises.
 *   - The device that owns the tensors must be the current device of the calling thread
 *     (hipSetDevice): kernels are launched on the current device.
 *   - The library allocates and frees no device memory and keeps no device state between
 *     calls; scratch memory comes in through `ws` (laq_workspace_bytes).  On the host it keeps,
 *     per device, what laq_init() looks up (kernel attributes, how many workgroups the device
 *     holds at once); a scoring call on a device that laq_init() has not seen does that lookup
 *     itself, before it enqueues anything.
 *     Calls that may run at the same time (different streams) need a workspace each; calls
 *     on one stream may share one.
 *   - Errors are reported by the return value (LAQ_OK = 0, negative otherwise), never
 *     by exception or abort.  Arguments are validated before anything is enqueued, so
 *     a call that returns LAQ_ERR_INVALID / _UNSUPPORTED / _WORKSPACE has done nothing.
 *     LAQ_ERR_DEVICE reports a failed launch (hipGetLastError).
 *   - Results are a pure function of the inputs (no floating-point atomics; two runs
 *     give identical bits).
 */
#ifndef LAQ_H
#define LAQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { LAQ_F32 = 0, LAQ_BF16 = 1 } laq_dtype;

/* Sequence pooling of the raw scores: the maximum (default) or the average that Sec. 5.1
 * names for the observation-window baseline used as stage-1 eviction (Sec. 4.2). */
typedef enum { LAQ_POOL_MAX = 0, LAQ_POOL_AVG = 1 } laq_pool_mode;

enum {
  LAQ_OK = 0,
  LAQ_ERR_INVALID = -1,     /* null pointer, bad shape, budget < W, even pool kernel ... */
  LAQ_ERR_UNSUPPORTED = -2, /* valid request outside what the kernels cover (see each call) */
  LAQ_ERR_WORKSPACE = -3,   /* ws is NULL or smaller than laq_workspace_bytes() */
  LAQ_ERR_DEVICE = -4,      /* a HIP call (launch, attribute query, copy) failed */
  LAQ_ERR_TIMEOUT = -5      /* laq_workspace_status: a kernel gave up a wait, the results are invalid */
};

/* Shape shared by all instances of one call. */
typedef struct laq_shape {
  int32_t n_inst;  /* >= 1: sequences x layers */
  int32_t Hq;      /* query heads, multiple of Hkv */
  int32_t Hkv;     /* KV heads */
  int32_t d;       /* head size, multiple of 8, <= 256 */
  int32_t L;       /* key rows per KV head */
  int32_t W;       /* observation-window queries per query head, >= 1 */
  int32_t dtype;   /* laq_dtype of q_win, k, v, k_out, v_out */
  float scale;     /* logit scale; <= 0 selects 1/sqrt(d) */
  /*
   * General observation window (Sec. 4.3, Eq. 5: local window queries joined with the
   * lookahead Q-cache).  Both fields are optional; a zeroed q_pos with keep = -1 is the
   * trailing-window layout in which the W queries belong to the last W keys.
   *   q_pos  HOST array [W] or NULL.  q_pos[w] >= 0 is the position of query w in the key
   *          sequence: it attends to keys j <= q_pos[w]; a lookahead query, generated after
   *          the prompt, has q_pos[w] >= L-1 and sees every key.  NULL: q_pos[w] = L-W+w
   *          (needs W <= L).  At most 512 entries (LAQ_ERR_UNSUPPORTED beyond).
   *   keep   number of trailing keys that are always retained and take no part in ranking
   *          and pooling (the local window's own tokens), 0 <= keep <= L; negative: W
   *          (needs W <= L).  Every budget must be >= keep.
   */
  const int32_t *q_pos;
  int32_t keep;
  /*
   * laq_pool_mode of every pool_kernel > 1 below (0 = LAQ_POOL_MAX).  LAQ_POOL_AVG replaces
   * the window maximum by (sum of raw[g,i], |i-j| <= (p-1)/2, 0 <= i < P) / p, i.e. the window
   * mean with zeros outside the prefix, summed in fp32 in ascending i.
   */
  int32_t pool_mode;
  /*
   * Layout of k and v as laq_score, laq_compact and laq_evict read them: distances, in elements,
   * between instances, KV heads and consecutive key rows; the d elements of a row are always
   * contiguous.  All zero: the dense [n_inst, Hkv, L, d] of the conventions above.  A token-major
   * cache [n_inst, L, Hkv, d] is {L*Hkv*d, d, Hkv*d}.  Each stride is a multiple of 16 bytes,
   * kv_stride_row >= d, v has the strides of k, and rows must not overlap (not checked).  Outputs
   * (scores, idx, k_out, v_out) keep their layouts.
   */
  int64_t kv_stride_inst;
  int64_t kv_stride_head;
  int64_t kv_stride_row;
  /*
   * Paged cache (optional; all zero: none).  With a block table, k and v are pools of blocks of
   * block_rows key rows each, as serving engines keep the caches of many sequences (Sec. 4.3's
   * re-eviction then reads the prefill cache through the table and writes a packed one):
   *   block_table      DEVICE array int32 [n_inst, ceil(L / block_rows)], dense.  Key row j of instance i
   *                    is row j % block_rows of block block_table[i][j / block_rows]; instances may
   *                    share blocks.  Block numbers are not checked: each must name a block of the pool.
   *   block_rows       rows per block: a multiple of 256, the unit of the scoring kernels
   *   kv_stride_block  distance between blocks of the pool, in elements (a multiple of 16 bytes)
   * kv_stride_head and kv_stride_row then describe the inside of a block (both zero: the dense block
   * [Hkv, block_rows, d]; a token-major block [block_rows, Hkv, d] is {d, Hkv*d}); kv_stride_inst is
   * not used.  laq_score, laq_compact and laq_evict read paged caches, with the same choice of
   * scoring kernels as for dense ones.
   */
  const int32_t *block_table;
  int32_t block_rows;
  int64_t kv_stride_block;
  /*
   * Which scoring kernels to take where more than one applies (laq_score_choice; 0 = LAQ_CHOOSE_AUTO:
   * the single-read kernel for at most 64 score rows per KV head from 128 MiB of keys per call on,
   * otherwise the two streaming passes, whose launches cost less and which are the faster ones with
   * more rows).  A choice that does not apply to the shape is ignored; laq_score_kernel()
   * tells what a call will run.
   */
  int32_t score_choice;
} laq_shape;

/*
 * One-time set-up for the current device: sets the attributes of the scoring kernels and asks the
 * runtime how many of their workgroups the device holds at once (the persistent kernels of Sec. 4.3's
 * scoring step are launched with exactly that many).  Optional: the first scoring call on a device
 * does the same.  Call it first if that call is to be recorded by a stream capture, which must not
 * contain such queries.  Idempotent, thread-safe.  LAQ_OK or LAQ_ERR_DEVICE.
 */
int laq_init(void);

/*
 * Bytes of device scratch that laq_score / laq_evict need for this shape (0 on a bad shape): the
 * per-chunk softmax statistics and row constants of the key-axis softmax (Sec. 4.3, Eq. 4 taken on
 * attention scores), a raw-score plane in front of the pooling, the hand-over plane between scoring
 * and selection, and the exchange memory of the single-read kernel.  Depends on n_inst, Hq, Hkv, L,
 * W only.
 */
size_t laq_workspace_bytes(const laq_shape *shape);

/*
 * Whether the last scoring call that used this workspace completed all its waits.  The single-read
 * scoring kernel lets the workgroups that share a KV head exchange their softmax statistics while
 * it runs; each of those waits is bounded, and a kernel that gives one up (which needs the device
 * to withhold part of a cooperative launch for about a second) finishes with invalid scores and
 * leaves a mark in the workspace.  Synchronises `stream`, reads the mark: LAQ_OK, LAQ_ERR_TIMEOUT,
 * or an argument / device error.  For callers that want the proof; results of a call that has
 * completed on an otherwise healthy device need no check.
 */
int laq_workspace_status(const laq_shape *shape, const void *ws, size_t ws_bytes, void *stream);

/*
 * Importance scores (Eq. 4's sum over the Q-cache, taken on attention scores).
 *   q_win  [n_inst, Hq, W, d]   observation-window queries (Q-cache, local window, or both); always
 *                               dense (no strides)
 *   k      [n_inst, Hkv, L, d]  key cache.  Read once where a team of workgroups keeps a head's
 *                               unnormalised probabilities on chip until the softmax denominators
 *                               are known: bf16, d = 128, at most 128 score rows G * W per KV
 *                               head, L up to 1024 / 512 / 256 keys (for at most 32 / 64 / 128
 *                               score rows) x the workgroups the device holds, 512 on an MI355X.
 *                               The library takes that kernel by itself with at most 64 score
 *                               rows and at least 128 MiB of keys in the call, where it is the
 *                               faster one; shape.score_choice asks for it or against it.
 *                               Otherwise K is streamed twice (laq_score_kernel() says which).
 *                               The single-read kernel is started with a cooperative launch,
 *                               which keeps a team of workgroups on the device together; with
 *                               LAQ_COOPERATIVE_LAUNCH=0 in the environment (read at the first
 *                               such call) it is an ordinary launch of the same grid, for
 *                               profilers that cannot follow cooperative launches -- then
 *                               other work on the device can make the call end in LAQ_ERR_TIMEOUT.
 *   scores [n_inst, Hkv, L]     fp32 out.  For each KV head g and key j:
 *            raw[g,j] = sum over the G heads of the group and the W queries of
 *                       softmax_j(scale * <q, k_j>) restricted to j <= P + w.
 *          With pool_kernel == 1 scores = raw.  With an odd pool_kernel p > 1 the prefix
 *          columns hold max(raw[g,i] : |i-j| <= (p-1)/2, 0 <= i < P) (the sequence pooling
 *          of the observation-window procedure, Sec. 2.1 / 5.1) and the W window columns
 *          keep raw (LAQ_POOL_AVG: the window mean instead, see laq_shape).  The raw scores
 *          do not depend on pool_kernel and both places pool with the same arithmetic, so
 *          laq_score(p) + laq_select(1) and laq_score(1) + laq_select(p) give the same indices.
 *   ws / ws_bytes  device scratch of at least laq_workspace_bytes(shape)
 * Supported: dtype BF16 or F32; any Hq/Hkv/W/L within the limits of laq_shape;
 * pool_kernel odd, 1 <= pool_kernel <= 63.  BF16 with d = 64 or 128 and W <= 512 runs on the
 * matrix cores; everything else runs on a vector-ALU path with the same results to within the
 * rounding of its fp32 sums, several times slower per key.  q_win, k and scores must be 16-byte
 * aligned.
 */
int laq_score(const laq_shape *shape, const void *q_win, const void *k, int pool_kernel,
              float *scores, void *ws, size_t ws_bytes, void *stream);

/*
 * Per-KV-head selection ("ArgSort(...)[:B]" of Eq. 4) under a per-instance budget.
 *   scores [n_inst, Hkv, L] fp32, non-negative (as laq_score writes them)
 *   budget [n_inst] HOST array, budget[i] >= W.  Bk(i) = min(budget[i], L).
 *   pool_kernel  odd >= 1; p > 1 applies the pooling described above (shape->pool_mode) to
 *                the prefix columns before ranking (use 1 if laq_score already pooled)
 *   idx    int32 out, packed: instance i starts at element sum_{i'<i} Hkv * Bk(i') and
 *          holds [Hkv, Bk(i)].  Each row: the Bk - W prefix positions with the largest
 *          pooled score (ties to the lower position), ascending, then P .. L-1.
 * budget[i] >= L keeps every row.  Uses no workspace.
 */
int laq_select(const laq_shape *shape, const float *scores, const int32_t *budget,
               int pool_kernel, int32_t *idx, void *stream);

/*
 * Score-free stage-1 eviction in the StreamingLLM form (Sec. 2.1; Sec. 4.2 allows it as the
 * low-budget eviction that precedes the lookahead decoding): every KV head keeps the first
 * n_sink positions and the most recent ones.
 *   budget [n_inst] HOST array, budget[i] >= 1.  Bk(i) = min(budget[i], L).
 *   n_sink >= 0.  s = min(n_sink, Bk): a row is 0 .. s-1 followed by L-(Bk-s) .. L-1.
 *   idx    int32 out, packed exactly as laq_select packs it (feed it to laq_compact with a
 *          shape whose keep is 0).
 * Takes plain sizes: n_inst, Hkv, L >= 1, Hkv <= 65535.  Uses no workspace.
 */
int laq_select_sink_recent(int32_t n_inst, int32_t Hkv, int32_t L, const int32_t *budget,
                           int32_t n_sink, int32_t *idx, void *stream);

/*
 * Which kernels laq_score (and laq_evict) take for this shape on the current device, for callers
 * that account for memory traffic (Sec. 4.3's scoring reads K once or twice accordingly):
 * LAQ_KERNEL_VECTOR (vector-ALU path, K streamed twice), LAQ_KERNEL_TWO_PASS (matrix cores, K
 * streamed twice) or LAQ_KERNEL_SINGLE_READ (matrix cores, K read once); a negative error code
 * for an invalid shape.  The strides, the block table and the score_choice of `shape` are taken
 * into account like laq_score does.  Launches nothing.
 */
enum { LAQ_KERNEL_VECTOR = 0, LAQ_KERNEL_TWO_PASS = 1, LAQ_KERNEL_SINGLE_READ = 2 };
typedef enum { LAQ_CHOOSE_AUTO = 0, LAQ_CHOOSE_TWO_PASS = 1, LAQ_CHOOSE_SINGLE_READ = 2 } laq_score_choice;
int laq_score_kernel(const laq_shape *shape);

/*
 * Recall of one selection against another (Sec. 3, Eq. 1-3): with M_gold the positions selected
 * by one set of queries (the response tokens') and M_pred those selected by another (an
 * observation window's), Recall = |M_pred ∩ M_gold| / |M_gold| per KV head.
 *   idx_pred, budget_pred   a packed index list and the HOST budget array it was made with
 *   idx_gold, budget_gold   the same for the reference selection; budgets >= 1
 *   Both lists as laq_select / laq_select_sink_recent write them: every row ascending, no
 *   repeats (rows that are not ascending give an undefined count, nothing else).
 *   overlap  int32 out [n_inst, Hkv]: size of the intersection
 *   recall   fp32 out [n_inst, Hkv], may be NULL: overlap / min(budget_gold[i], L)
 * Takes plain sizes: n_inst, Hkv, L >= 1, Hkv <= 65535.  Uses no workspace.
 */
int laq_recall(int32_t n_inst, int32_t Hkv, int32_t L, const int32_t *idx_pred,
               const int32_t *budget_pred, const int32_t *idx_gold, const int32_t *budget_gold,
               int32_t *overlap, float *recall, void *stream);

/*
 * Cache compaction (Sec. 4.3: the cache is re-evicted to the given budget; decoding continues on
 * what is left): gather the retained rows.
 *   k, v         [n_inst, Hkv, L, d]; v (and v_out) may be NULL to compact K only
 *   idx, budget  as written by / passed to laq_select
 *   k_out, v_out packed like idx: instance i starts at row sum_{i'<i} Hkv * Bk(i') and
 *                holds [Hkv, Bk(i), d]; bit copies of the selected rows
 * Indices must lie in [0, L); out-of-range entries are skipped (row left untouched).  k, v, k_out,
 * v_out must be 16-byte aligned.
 */
int laq_compact(const laq_shape *shape, const void *k, const void *v, const int32_t *idx,
                const int32_t *budget, void *k_out, void *v_out, void *stream);

/*
 * The whole path of Sec. 4.3 on one stream: laq_score(pool_kernel) + laq_select(1) + laq_compact;
 * outputs identical to those of the three calls.  `scores` may be NULL: the pooled scores are then
 * handed from scoring to selection through the workspace and not returned; otherwise it is left
 * holding them.
 */
int laq_evict(const laq_shape *shape, const void *q_win, const void *k, const void *v,
              const int32_t *budget, int pool_kernel, float *scores, int32_t *idx,
              void *k_out, void *v_out, void *ws, size_t ws_bytes, void *stream);

/*
 * laq_evict for callers that cannot allocate device memory (code under stream capture, tight
 * serving loops, harnesses that forbid it): the same path, same outputs bit for bit, with the
 * workspace taken from an array of LAQ_STATIC_SCRATCH_BYTES that is part of the library's code
 * object (every device the library runs on holds one until the process ends).  It calls no
 * allocating routine.  A shape whose laq_workspace_bytes() exceeds LAQ_STATIC_SCRATCH_BYTES is
 * rejected with LAQ_ERR_WORKSPACE before anything is enqueued (16 MiB covers e.g. three layers of 8
 * KV heads x 32768 keys with 128 score rows each, the usual one-layer-at-a-time call many times
 * over).  All calls on one device share the array and nothing in it survives a call: calls that
 * overlap on one device (different streams) race; calls on one stream are fine.  The first call on
 * a device (or laq_init) looks the array's address up; call laq_init() before a capture.
 */
#define LAQ_STATIC_SCRATCH_BYTES (16u << 20)
int laq_evict_static(const laq_shape *shape, const void *q_win, const void *k, const void *v,
                     const int32_t *budget, int pool_kernel, float *scores, int32_t *idx,
                     void *k_out, void *v_out, void *stream);

/*
 * Q-cache capture (Sec. 4.2: the lookahead decoding keeps its query states): store the queries of
 * lookahead step t into the Q-cache that laq_score later reads as q_win.
 *   q_step  [n_inst, Hq, d]     queries of the step, dtype shape->dtype
 *   t       0 <= t < shape->W   slot of the step
 *   q_cache [n_inst, Hq, W, d]  rows [.., t, :] are overwritten, the others left alone
 * Reads n_inst, Hq, d, W, dtype of the shape (the remaining fields must still be valid).
 */
int laq_qcache_store(const laq_shape *shape, const void *q_step, int32_t t, void *q_cache,
                     void *stream);

/*
 * Decoding on the compacted cache (Sec. 4.3: after the re-eviction, generation continues as
 * standard autoregressive decoding): attention of one new token per instance over the retained
 * rows, out[h] = softmax_j(scale * <q[h], K'[h/G, j]>) V'[h/G], no mask (every retained key
 * precedes the new token).
 *   q          [n_inst, Hq, d]  dtype shape->dtype
 *   k_c, v_c   packed as laq_compact writes them: instance i holds [Hkv, Bk(i), d]
 *   budget     HOST array [n_inst], >= 1; Bk(i) = min(budget[i], L)
 *   out        fp32 [n_inst, Hq, d]
 *   ws / ws_bytes  optional device scratch (ws may be NULL).  With at least
 *              laq_decode_workspace_bytes(shape, budget) bytes, a call with few instances and
 *              heads spreads every cache of more than 512 rows over several workgroups and
 *              merges their partial results; LAQ_ERR_WORKSPACE if ws is given but too small.
 *              Without it every cache is read by one workgroup.
 * Reads n_inst, Hq, Hkv, d, L, dtype, scale of the shape.  Partial sums are merged in a fixed
 * order: two runs of the same call give identical bits (with and without ws the last bits of
 * `out` may differ, the order of the sums being different).
 */
size_t laq_decode_workspace_bytes(const laq_shape *shape, const int32_t *budget);
int laq_decode_attention(const laq_shape *shape, const void *q, const void *k_c, const void *v_c,
                         const int32_t *budget, float *out, void *ws, size_t ws_bytes, void *stream);

/* Static description of an error code (never NULL; "unknown error" for a code that is none of the above). */
const char *laq_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* LAQ_H */
