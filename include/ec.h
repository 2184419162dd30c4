/*
 * libelastic_cache -- C ABI of the Elastic Cache hot path on AMD MI355X (gfx950).
 *
 * The library implements, as hand-written HIP kernels, the per-layer KV-cache
 * compression of the paper's instruction-encoding stage and the attention +
 * fixed-point elimination of its output-generation stage (Sec. 3.3 "One
 * Sequence, Two Policies"; Alg. 1).
 *
 * Conventions common to every entry point
 *  - Pointers named below as DEVICE point to memory of the current HIP device,
 *    owned by the caller for the whole call and until the stream has drained.
 *    The library allocates nothing and frees nothing; scratch comes from the
 *    caller's workspace `ws` (size from ec_workspace_bytes), except in
 *    ec_decode_score_step_static, which uses an array built into the library.
 *  - All tensors are dense, row-major, in the element type `dt` unless a C type
 *    is given.  Prompt tensors are [B,H,T,D] (sequence on axis 2, as Alg. 1
 *    reads it), caches are [B,H,cap,D].  Positions are 0-based.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Work is enqueued asynchronously; no call synchronises with the device.
 *  - Every entry point returns an ec_status.  Arguments are validated on the
 *    host before anything is launched: on EC_EINVAL / EC_EUNSUPPORTED /
 *    EC_EWORKSPACE nothing was enqueued.  EC_EDEVICE reports a HIP launch error.
 *  - G is the number of score groups per layer: G = 1 is the paper's layer-wise
 *    policy (all heads of a layer share anchor positions, Sec. 3.3), G = H the
 *    head-wise variant of the ablation (Table 3c).
 *  - Supported: D in {64,128}; dt in {EC_F32, EC_BF16}; multi-head attention
 *    with as many key/value heads as query heads.
 */
#ifndef EC_H_
#define EC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    EC_OK = 0,
    EC_EINVAL = 1,       /* bad shape, NULL required pointer, index out of range   */
    EC_EUNSUPPORTED = 2, /* valid request the kernels do not cover (D, dtype, ...) */
    EC_EWORKSPACE = 3,   /* ws NULL or smaller than ec_workspace_bytes             */
    EC_EDEVICE = 4       /* HIP runtime reported an error at launch                */
} ec_status;

typedef enum { EC_F32 = 0, EC_BF16 = 1 } ec_dtype;

typedef enum {
    EC_FN_PREFILL_SCORE = 0,
    EC_FN_SELECT_ANCHORS = 1,
    EC_FN_MERGE_COMPACT = 2,
    EC_FN_DECODE_STEP = 3,
    EC_FN_DECODE_SCORE_STEP = 4,
    EC_FN_EVICT_MIN = 5
} ec_fn;

/* Budget rule of the retention test (Sec. 3.3 Output Generation; Alg. 1). */
typedef enum {
    EC_BUDGET_RATIO = 0, /* keep ceil(gamma * n) rows: Alg. 1's int(seq_len - n(1-r)) >= 1 test */
    EC_BUDGET_FIXED = 1  /* keep a constant number of rows                                  */
} ec_budget_mode;

/* Truncation location of the fixed-point elimination (Sec. 3.3; Sec. 4.1). */
typedef enum {
    EC_TRUNC_RECENT = 0, /* `recent` rows before the newest one (25 in Sec. 4.1) */
    EC_TRUNC_ABS = 1     /* absolute location N_tl                              */
} ec_trunc_mode;

/* What ec_merge_compact stores for an anchor (Sec. 3.3 "Cache Eviction v.s. Cache Merging"; Table 3b). */
typedef enum {
    EC_MERGE_MEAN = 0, /* the paper's method: mean of the anchor's bucket (Eq. 3)            */
    EC_MERGE_EVICT = 1 /* eviction-only ablation: the anchor's own row, the rest is dropped  */
} ec_merge_mode;

/* Human-readable name of a status code.  Host, pure. */
const char* ec_status_string(int status);

/*
 * Bytes of workspace the given entry point needs for these shapes.  Host, pure.
 * For EC_FN_DECODE_STEP and EC_FN_DECODE_SCORE_STEP pass T = cap.  Returns 0 for entry points that need none
 * and (size_t)-1 for unsupported shapes.
 */
size_t ec_workspace_bytes(int fn, int B, int H, int T, int D, int dt);

/*
 * Instruction-encoding attention with importance scores (Sec. 3.3, Eq. 1 and the
 * definition of I_n that follows it).  For every (b,h):
 *     A     = row-softmax over n <= m of scale * <q_m, k_n>      (T x T, never stored)
 *     out_m = sum_n A_mn v_n,   lse_m = log sum_{n<=m} exp(scale <q_m,k_n>)
 *     I_n   = sum_{m>=n} A_mn                                    (column mass)
 * score[b,g,n] = I_n of head g when G == H, or the mean of I_n over the H heads
 * when G == 1 (the paper's layer-wise metric).  scale = 1 gives Eq. 1 literally;
 * models use 1/sqrt(D).  scale must be finite and > 0 (else EC_EINVAL).
 *   q,k,v  DEVICE [B,H,T,D] dt, read only
 *   out    DEVICE [B,H,T,D] dt, written; may be NULL (attention output not wanted)
 *   lse    DEVICE [B,H,T] float, written; may be NULL (kept in ws instead)
 *   score  DEVICE [B,G,T] float, written
 *   ws     DEVICE scratch, ec_workspace_bytes(EC_FN_PREFILL_SCORE, B,H,T,D,dt)
 * bf16 inputs are multiplied on the matrix cores with fp32 accumulation; fp32
 * inputs use fp32 arithmetic throughout.  Results are deterministic.
 */
int ec_prefill_score(const void* q, const void* k, const void* v, void* out, float* lse,
                     float* score, int B, int H, int G, int T, int D, int dt, float scale,
                     void* ws, size_t ws_bytes, void* stream);

/*
 * Instruction encoding of a later chunk over an existing compressed cache (Sec. 3.3: the compression is
 * applied to all concatenated inputs, chat history included; Alg. 1's multi-token branch entered with a
 * non-empty past, where the attention matrix is gen_len x seq_len).  For every head, k and v hold the P
 * rows of the compressed cache followed by the T_new rows of the chunk, in a buffer whose heads are
 * kv_rows rows apart (kv_rows >= P + T_new; rows beyond P + T_new are never read).  Query m of the chunk
 * (0-based) attends rows n <= P + m:
 *     A     = row-softmax over n <= P + m of scale * <q_m, k_n>      (T_new x (P + T_new), never stored)
 *     out_m, lse_m as in ec_prefill_score
 *     I_n   = sum over m >= max(0, n - P) of A_mn, for every row n of [cache | chunk]
 * The scores are this pass's column sums (Alg. 1 assigns its score buffer in this branch, it does not
 * accumulate over passes).  score[b,g,n] is I_n of head g (G == H) or the head mean (G == 1).
 *   q      DEVICE [B,H,T_new,D] dt, read only
 *   k,v    DEVICE [B,H,kv_rows,D] dt, read only
 *   out    DEVICE [B,H,T_new,D] dt, written; may be NULL
 *   lse    DEVICE [B,H,T_new] float, written; may be NULL
 *   score  DEVICE [B,G,P+T_new] float, written
 *   ws     DEVICE scratch, ec_workspace_bytes(EC_FN_PREFILL_SCORE, B,H, P+T_new, D,dt)
 * P = 0 and kv_rows = T_new is ec_prefill_score itself; T_new = 1 is one generation step's attention.
 * Anchors are then chosen with ec_select_anchors over the P + T_new rows and the rows merged with
 * ec_remerge_compact.
 */
int ec_chunk_score(const void* q, const void* k, const void* v, void* out, float* lse, float* score,
                   int B, int H, int G, int T_new, int P, int kv_rows, int D, int dt, float scale,
                   void* ws, size_t ws_bytes, void* stream);

/*
 * A "Mean" importance metric in the sense of the ablation on the importance metric (Table 3d), from the
 * "Sum" the scoring calls emit.  The paper names the metric but prints no formula for it; the definition
 * here is this library's own reading: every score is divided, in place, by the number of queries that can
 * see its row.
 * After ec_prefill_score pass T_new = T, P = 0 (row n is seen by T - n queries); after ec_chunk_score pass
 * its T_new and P (row n is seen by T_new - max(0, n - P) queries).
 *   score  DEVICE [B,G,P+T_new] float, updated in place
 */
int ec_importance_mean(float* score, int B, int G, int T_new, int P, void* stream);

/*
 * Anchor selection (Sec. 3.3: the N_I positions of largest importance, listed in
 * ascending position; Sec. 4.1: the first and the most recent token are protected).
 * For every (b,g): positions 0..protect_first-1 and T-protect_last..T-1 are
 * always selected; of the others the n_anchor - protect_first - protect_last
 * with the largest score are selected, equal scores going to the lower position.
 * Scores are compared as fp32 values (-0 == +0); NaN is outside the domain.
 *   score       DEVICE [B,G,T] float, read only
 *   anchor_idx  DEVICE [B,G,n_anchor] int32, written, strictly ascending
 * Requires 1 <= n_anchor <= T <= 65536, protect_first + protect_last <= n_anchor.
 * N_I = ceil(gamma*T) is the caller's to compute (Alg. 1's del_num rounding).
 */
int ec_select_anchors(const float* score, int B, int G, int T, int n_anchor, int protect_first,
                      int protect_last, int32_t* anchor_idx, void* ws, size_t ws_bytes,
                      void* stream);

/*
 * Bucket division, cache merging and compaction (Sec. 3.3, Eq. 2 and Eq. 3;
 * Alg. 1's Nearest / scatter_reduce / gather).  With anchors t_0 < ... < t_{n-1}
 * bucket j holds positions floor((t_{j-1}+t_j)/2)+1 .. floor((t_j+t_{j+1})/2), the
 * first bucket starting at 0 and the last ending at T-1 (every position goes to
 * its nearest anchor, ties to the earlier one).  For every head, cache row j is
 * the mean of the K (resp. V) rows of bucket j, accumulated in fp32 and rounded
 * once (to nearest even) to dt: in ascending position for buckets of up to 128
 * rows, as interleaved partial sums added in a fixed order for longer ones
 * (results are deterministic either way).
 *   k,v              DEVICE [B,H,T,D] dt, read only
 *   anchor_idx       DEVICE [B,G,n_anchor] int32 ascending, read only
 *   k_cache,v_cache  DEVICE [B,H,cap,D] dt; rows 0..n_anchor-1 written, rest untouched
 *   counts           DEVICE [B,G,n_anchor] int32 bucket sizes, written; may be NULL
 *   assign           DEVICE [B,G,T] int32 bucket number of every position; may be NULL
 *   pos              DEVICE [B,G,cap] int32; entries 0..n_anchor-1 = anchor positions;
 *                    may be NULL
 * merge_mode EC_MERGE_EVICT (the "Cache Eviction" row of Table 3b) copies the anchor rows bit for
 * bit instead; counts are then 1 and assign is -1 for every dropped position.
 * Requires 1 <= n_anchor <= min(T, cap).  Anchors that are not strictly ascending
 * inside [0,T) give unspecified cache contents (no out-of-bounds access).
 */
int ec_merge_compact(const void* k, const void* v, const int32_t* anchor_idx, int B, int H, int G,
                     int T, int D, int n_anchor, int dt, int merge_mode, void* k_cache, void* v_cache,
                     int cap, int32_t* counts, int32_t* assign, int32_t* pos, void* stream);

/*
 * ec_merge_compact for rows that may already be merged (Sec. 3.3, Eq. 2 and Eq. 3 applied again to
 * [compressed cache | new chunk]; Alg. 1 runs the same gather / scatter_reduce / gather on whatever the
 * cache holds).  Buckets are formed over ROW INDICES 0..L-1 of the source buffer exactly as in
 * ec_merge_compact.  Differences:
 *   src_rows   rows between the heads of k and v (>= L): the source may be a cache buffer with spare rows
 *   weights    DEVICE [B,G,L] int32 or NULL.  NULL: every row weighs 1 -- the plain mean of Alg. 1, which
 *              for rows that are themselves means is a mean of means.  Given (an extension beside the
 *              paper): row t weighs weights[t] >= 1 (values below 1 are taken as 1), the number of
 *              original tokens it stands for; cache row j = sum w_t x_t / sum w_t over bucket j, which is
 *              the mean of the original tokens, and counts[j] = sum w_t.  Ignored by EC_MERGE_EVICT.
 *   src_pos    DEVICE [B,G,L] int32 or NULL: original position of every source row; pos[j] is then
 *              src_pos[anchor_j] instead of anchor_j
 * k_cache / v_cache must not be k / v, and pos must not overlap src_pos (rows are written while others
 * are still being read).
 * Everything else is as in ec_merge_compact, which is this call with src_rows = T and both NULL.
 */
int ec_remerge_compact(const void* k, const void* v, int src_rows, const int32_t* weights,
                       const int32_t* src_pos, const int32_t* anchor_idx, int B, int H, int G, int L,
                       int D, int n_anchor, int dt, int merge_mode, void* k_cache, void* v_cache, int cap,
                       int32_t* counts, int32_t* assign, int32_t* pos, void* stream);

/*
 * Retention test and truncation location of the fixed-point elimination
 * (Sec. 3.3 Output Generation; Alg. 1's del_num and fix_idx; Sec. 4.1: recent
 * distance 25).  Host, pure integer arithmetic.
 *   n_seen            tokens seen so far, including the one just appended
 *   len_after_append  cache rows including the new one
 *   gamma_num/den     retention ratio gamma as an exact fraction
 *   budget_mode       EC_BUDGET_RATIO: evict iff len_after_append > ceil(gamma*n_seen)
 *                     EC_BUDGET_FIXED: evict iff len_after_append > fixed_len
 *   trunc_mode        EC_TRUNC_RECENT: idx = len_after_append - 1 - recent
 *                     EC_TRUNC_ABS:    idx = n_tl
 *   protect_first     rows below this index are never evicted (idx is raised to it)
 * Returns the row to evict, or -1 for none (also when the only candidate would
 * be the newest row), or -2 on invalid arguments.
 */
int ec_evict_index(int64_t n_seen, int len_after_append, int gamma_num, int gamma_den,
                   int budget_mode, int fixed_len, int trunc_mode, int recent, int n_tl,
                   int protect_first);

/*
 * One output-generation step of one layer over the compressed cache (Sec. 3.1
 * Output Generation; Sec. 3.3 fixed-point elimination; Alg. 1's last branch).
 * For every (b,h), in this order:
 *   1. row cache_len of k_cache/v_cache <- k_new/v_new        (pos <- new_pos)
 *   2. out = softmax_j(scale * <q, k_cache_j>) . v_cache over rows 0..cache_len
 *      (plain softmax; merged rows carry no count weights)
 *   3. if evict_idx >= 0, row evict_idx is removed and the rows behind it move
 *      up by one (Alg. 1's cat of the two sides); the cache then holds
 *      cache_len rows, else cache_len + 1.
 *   q,k_new,v_new     DEVICE [B,H,D] dt, read only
 *   k_cache,v_cache   DEVICE [B,H,cap,D] dt, updated in place
 *   pos               DEVICE [B,G,cap] int32 original position of every row, updated
 *                     like the cache; may be NULL
 *   out               DEVICE [B,H,D] dt, written
 *   ws                DEVICE scratch, optional: ec_workspace_bytes(EC_FN_DECODE_STEP, B,H,cap,D,dt)
 *                     bytes, which is 0 for the launch shape the library picks itself (one workgroup
 *                     streams a whole (batch, head); nothing is staged), so ws may be NULL.  A shape
 *                     that divides a (batch, head) over several workgroups, whose partial results
 *                     meet in ws and are merged by a second launch on the same stream, exists and is
 *                     reached through ec_decode_step_shaped; it measured slower at every workload.
 * Requires 0 <= cache_len < cap, -1 <= evict_idx <= cache_len and a finite scale > 0.  Dot
 * products and the softmax are evaluated in fp32.
 */
int ec_decode_step(const void* q, const void* k_new, const void* v_new, void* k_cache,
                   void* v_cache, int32_t* pos, int B, int H, int G, int D, int cap, int cache_len,
                   int evict_idx, int32_t new_pos, float scale, int dt, void* out, void* ws,
                   size_t ws_bytes, void* stream);

/*
 * ec_decode_step with an explicit launch shape, for tests and tuning sweeps (the library reads no
 * environment variable and keeps no state: a shape other than its own choice is requested here).
 *   waves   wavefronts per workgroup (0 = the library's choice)
 *   unroll  16-byte loads of K and of V each lane keeps in flight (0 = the library's choice)
 *   splits  workgroups per (batch, head): 0 = the library's choice, 1 = one workgroup and no
 *           workspace, n > 1 = n workgroups plus the merging launch; ws must then hold
 *           4 * B * H * n * (D + 2) bytes, else EC_EWORKSPACE
 * Combinations the library has no kernel for return EC_EINVAL.  Everything else as ec_decode_step.
 */
int ec_decode_step_shaped(const void* q, const void* k_new, const void* v_new, void* k_cache,
                          void* v_cache, int32_t* pos, int B, int H, int G, int D, int cap,
                          int cache_len, int evict_idx, int32_t new_pos, float scale, int dt, void* out,
                          void* ws, size_t ws_bytes, int waves, int unroll, int splits, void* stream);

/*
 * Ragged batches: the same four steps for a batch whose sequences differ in length (what a serving
 * loop hands over; the paper's Alg. 1 treats one sequence, so each batch element simply follows it with
 * its own numbers).  All tensors keep the padded shapes of the dense calls -- prompt tensors
 * [B,H,T_max,D], scores [B,G,T_max], anchors and counts [B,G,n_max], caches [B,H,cap,D] -- and the
 * per-sequence numbers are DEVICE int32 arrays of B entries, so a generation loop never has to
 * synchronise with the host:
 *   seq_len[b]      positions of batch element b (clamped into 0..T_max; 0 = nothing is done for b)
 *   n_anchor_b[b]   anchors of b (clamped into 0..min(seq_len[b], n_max))
 *   cache_len_b[b]  rows its cache holds before the step (clamped into 0..cap-1)
 *   evict_idx_b[b]  row to remove after the step or -1 (clamped into -1..cache_len_b[b]); NULL = none
 *   new_pos_b[b]    original position of the appended row (required when pos is given)
 * For batch element b every result equals the dense call on that element alone with T = seq_len[b]
 * (resp. n_anchor = n_anchor_b[b], cache_len = cache_len_b[b], ...).  Entries of the padded outputs beyond a
 * sequence's own length (out, lse and score rows >= seq_len[b], anchors >= n_anchor_b[b], ...) are
 * unspecified; padding rows of the inputs are never read.  protect_first / protect_last are common to the
 * batch and are cut to n_anchor_b[b] where a sequence has fewer anchors.
 */
int ec_prefill_score_varlen(const void* q, const void* k, const void* v, void* out, float* lse,
                            float* score, const int32_t* seq_len, int B, int H, int G, int T_max, int D,
                            int dt, float scale, void* ws, size_t ws_bytes, void* stream);
int ec_select_anchors_varlen(const float* score, const int32_t* seq_len, const int32_t* n_anchor_b, int B,
                             int G, int T_max, int n_max, int protect_first, int protect_last,
                             int32_t* anchor_idx, void* ws, size_t ws_bytes, void* stream);
int ec_merge_compact_varlen(const void* k, const void* v, const int32_t* anchor_idx, const int32_t* seq_len,
                            const int32_t* n_anchor_b, int B, int H, int G, int T_max, int D, int n_max,
                            int dt, int merge_mode, void* k_cache, void* v_cache, int cap, int32_t* counts,
                            int32_t* assign, int32_t* pos, void* stream);
int ec_decode_step_varlen(const void* q, const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                          int32_t* pos, const int32_t* cache_len_b, const int32_t* evict_idx_b,
                          const int32_t* new_pos_b, int B, int H, int G, int D, int cap, float scale, int dt,
                          void* out, void* ws, size_t ws_bytes, void* stream);

/*
 * ec_evict_index for every sequence of a ragged batch, on the device (Alg. 1's del_num and fix_idx; Sec. 4.1's
 * recent distance), so that a generation loop -- for instance one captured HIP graph replayed per token --
 * needs no host arithmetic.  Call it once before every layer walk of a generated token; all arrays are
 * DEVICE int32 [B] and are updated in place:
 *   1. if pending_b[b] is set, the step prepared by the previous call has run: cache_len_b[b] grows by one
 *      unless that step removed a row (evict_idx_b[b] >= 0); pending_b[b] is cleared
 *   2. unless flush_only: n_seen_b[b] += 1; evict_idx_b[b] = ec_evict_index(n_seen_b[b], cache_len_b[b] + 1, ...)
 *      with the budget / truncation arguments given here; new_pos_b[b] = n_seen_b[b] - 1; pending_b[b] = 1
 * cache_len_b, evict_idx_b and new_pos_b are then what ec_decode_step_varlen takes for every layer of this
 * token.  pending_b starts as zeros; call once more with flush_only = 1 after the last token so that
 * cache_len_b holds the final lengths.
 */
int ec_retention_step_varlen(int32_t* n_seen_b, int32_t* cache_len_b, int32_t* evict_idx_b,
                             int32_t* new_pos_b, int32_t* pending_b, int B, int gamma_num, int gamma_den,
                             int budget_mode, int fixed_len, int trunc_mode, int recent, int n_tl,
                             int protect_first, int flush_only, void* stream);

/*
 * The "Frequency" discard policy of the generation stage -- the Frequency Cache of Sec. 4.1 Baselines that
 * the ablation of Table 3a ("Discard Position") compares the fixed-point elimination with: every cached
 * row carries the attention mass it has received, every generated token adds its attention row to it,
 * and when a row has to go the row of least mass goes.  Two calls per generated token:
 *
 * ec_decode_score_step = steps 1 and 2 of ec_decode_step (append, attend; no removal) plus
 *     freq[b,g,j] += p_j for rows j < cache_len,   freq[b,g,cache_len] = p_{cache_len}
 * where p is this step's softmax row of head g (G == H) or its mean over the heads, added in ascending head
 * order (G == 1, the layer-wise metric of Sec. 3.3).  The new row's mass starts at what its own query
 * gives it (the paper does not say where it starts).
 *   freq   DEVICE [B,G,cap] float, updated in place (a compressed prompt's rows start at values of the
 *          caller's choice, e.g. the importance scores of their anchors)
 *   ws     DEVICE scratch, ec_workspace_bytes(EC_FN_DECODE_SCORE_STEP, B,H,cap,D,dt)
 * All other arguments as in ec_decode_step.  The cache then holds cache_len + 1 rows.
 */
int ec_decode_score_step(const void* q, const void* k_new, const void* v_new, void* k_cache,
                         void* v_cache, int32_t* pos, float* freq, int B, int H, int G, int D, int cap,
                         int cache_len, int32_t new_pos, float scale, int dt, void* out, void* ws,
                         size_t ws_bytes, void* stream);

/*
 * ec_decode_score_step for callers that cannot provide device scratch of their own and must not allocate:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments minus
 * the workspace; the scratch (every row's score and the softmax statistics, 4*B*H*(cap+2) bytes rounded up
 * to 256-byte blocks) lives in an array built into the library, 4 MiB per GPU the library runs on, held
 * until the process ends.  Shapes that need more return EC_EWORKSPACE and launch nothing.  The call
 * allocates and frees nothing.  The array's device address is looked up on the first call on each device
 * (make that call outside a stream capture).  All calls on one GPU share the array: calls that overlap in
 * time on one GPU (different streams, or threads) race; calls on one stream are ordered and safe.  Nothing
 * in the array needs to start at zero: every word read is written earlier in the same call.
 */
int ec_decode_score_step_static(const void* q, const void* k_new, const void* v_new, void* k_cache,
                                void* v_cache, int32_t* pos, float* freq, int B, int H, int G, int D, int cap,
                                int cache_len, int32_t new_pos, float scale, int dt, void* out, void* stream);

/*
 * ec_evict_min removes, for every (b,g), the row of least mass among rows protect_first ..
 * len-1-protect_recent (masses compared as fp32 values, -0 == +0, the lowest index among equals; NaN is
 * outside the domain) from k_cache, v_cache, pos and freq; the rows behind it move up by one, so the cache
 * then holds len - 1 rows.  Whether a row has to go is the caller's retention test (ec_evict_index >= 0).
 *   k_cache,v_cache  DEVICE [B,H,cap,D] dt, updated in place
 *   pos              DEVICE [B,G,cap] int32, updated; may be NULL
 *   freq             DEVICE [B,G,cap] float, updated
 *   victim           DEVICE [B,G] int32, written: the index removed
 * Requires 1 <= len <= cap and protect_first + protect_recent < len.  The victim differs between batch
 * elements (and heads when G == H), but every (b,h) loses exactly one row, so len stays common.
 */
int ec_evict_min(void* k_cache, void* v_cache, int32_t* pos, float* freq, int B, int H, int G, int D,
                 int cap, int len, int protect_first, int protect_recent, int dt, int32_t* victim,
                 void* stream);

#ifdef __cplusplus
}
#endif
#endif /* EC_H_ */
