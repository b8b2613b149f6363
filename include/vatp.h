/*
 * vatp.h -- C ABI of the MI355X (gfx950) value-aware token pruning library.
 *
 * The library scores the tokens of a per-head KV cache by accumulated attention
 * (paper Eq. 2) times the l1 norm of the token's value vector (Eq. 4), keeps a fixed
 * budget of rows per head -- a forced prefix of F "attention sink" rows, a window of the
 * R most recent rows and the most important of the rest -- and compacts the surviving
 * K/V rows (Methodology section; Implementation Details appendix; Fig. 2).
 *
 * Conventions shared by every call
 *   - Plain C types only.  Pointers named in UPPER CASE or documented "device" are device
 *     pointers owned by the caller; `len`, `budget`, `new_pos` are HOST arrays.  The
 *     library never allocates or frees device memory.
 *   - Layout is head-major: a cache tensor is [batch, n_heads, cap, head_dim] contiguous,
 *     per-row scalars (S, nrm, pos) are [batch, n_heads, cap].  Heads keep different
 *     tokens after pruning, so every (batch, head) unit owns `cap` rows of its own.
 *     Rows [0, len[b]) of a unit are valid; the others are never read.
 *     len and budget are per sequence; heads that need row counts or budgets of their own
 *     (non-uniform budgets, Implementation Details appendix) are passed as sequences:
 *     [batch, n_heads, ...] with n_heads = 1 and batch = sequences * heads (<= VATP_MAX_BATCH) is the same memory.
 *   - dtype covers Q, K, V and the caches; S and nrm are always float32, pos int32.
 *   - Calls enqueue work on `hip_stream` (a hipStream_t passed as void*, NULL = the null
 *     stream) and return without synchronising.  Errors that can be seen before launch
 *     are returned at once and nothing is enqueued; launch failures give VATP_E_DEVICE.
 *   - A context serves one stream at a time: calls that share a context must be
 *     stream-ordered with respect to each other.
 *   - Inputs must be finite.  A NaN or infinity in Q, K or V gives unspecified scores
 *     (never an out-of-bounds access).
 */
#ifndef VATP_H
#define VATP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define VATP_MAX_BATCH 256         /* sequences per call                                  */
#define VATP_MAX_UNITS 16384       /* batch * n_heads * max(q_per_kv, 1) per call         */
#define VATP_MAX_GROUP 16          /* query heads per K/V head (grouped-query attention)  */
#define VATP_MAX_CAP   4194304     /* rows per (batch, head) unit: cap and cap_out        */
#define VATP_STATIC_SCRATCH_BYTES 16777216   /* scratch of vatp_decode_prune_step_static, per GPU */

typedef struct vatp_ctx vatp_ctx;  /* opaque */

typedef enum {
    VATP_OK = 0,
    VATP_E_NULL = -1,        /* a required pointer is NULL                                 */
    VATP_E_SHAPE = -2,       /* batch / heads / head_dim / cap / len / norm out of range   */
    VATP_E_DTYPE = -3,       /* dtype is neither VATP_F32 nor VATP_BF16                    */
    VATP_E_BUDGET = -4,      /* budget[b] < n_sink + recent, survivors exceed cap_out (or  */
                             /* cap_hist), or a fused step would have to remove two rows  */
    VATP_E_WORKSPACE = -5,   /* workspace missing, too small or not 256-byte aligned       */
    VATP_E_DEVICE = -6       /* HIP reported an error (no device, launch failure), or the  */
                             /* context's device is not the current one                    */
} vatp_status;

enum { VATP_F32 = 0, VATP_BF16 = 1 };
enum { VATP_NORM_L1 = 0, VATP_NORM_L2 = 1, VATP_NORM_LINF = 2, VATP_NORM_NONE = 3 };
enum { VATP_CALL_PREFILL_SCORE = 0, VATP_CALL_DECODE_STEP = 1, VATP_CALL_SELECT_COMPACT = 2,
       VATP_CALL_DECODE_ATTEND_STEP = 3, VATP_CALL_DECODE_PRUNE_STEP = 4,
       VATP_CALL_PREFILL_SCORE_WINDOW = 5 };

typedef struct {
    int32_t batch;          /* 1 .. VATP_MAX_BATCH                                         */
    int32_t n_heads;        /* >= 1, batch * n_heads <= VATP_MAX_UNITS                     */
    int32_t head_dim;       /* 64 or 128                                                   */
    int32_t dtype;          /* VATP_F32 or VATP_BF16                                       */
    int32_t n_sink;         /* F: rows [0,F) are always kept (Attention Sink Tokens par.)  */
    int32_t recent;         /* R: the last R rows are always kept (local window, App. A)   */
    int32_t cap;            /* rows allocated per (batch, head) unit in the input buffers, */
                            /*   1 .. VATP_MAX_CAP                                         */
    int32_t cap_out;        /* same for the *_out buffers of vatp_select_compact; 0 = cap  */
    float   scale;          /* logit scale c; 0 selects 1/sqrt(head_dim)                   */
    const int32_t *len;     /* HOST [batch]: valid rows per sequence, same for all heads   */
    const int32_t *budget;  /* HOST [batch]: B, rows kept per head (F and R included).     */
                            /*   read by the calls that prune (vatp_select_compact*,       */
                            /*   vatp_decode_prune_step*); may be NULL elsewhere           */
    int32_t norm;           /* value-row norm of Eq. 4: VATP_NORM_L1 (0, the paper's choice), */
                            /*   VATP_NORM_L2 or VATP_NORM_LINF (the ablation of Table 2), or  */
                            /*   VATP_NORM_NONE: nrm = 1, the attention-only baseline (H2O)    */
    int32_t q_per_kv;       /* g: query heads per K/V head, 0 or 1 .. VATP_MAX_GROUP (0 = 1).  */
                            /*   g > 1 is grouped-query attention: see the note below          */
} vatp_params;

/*
 * Grouped-query attention (Limitations section, paragraph on GQA: the group-wise averaged
 * attention score as the token score).  With g = q_per_kv > 1, n_heads counts the K/V heads --
 * the caches, S, nrm, pos, budgets and kept sets are per K/V head as before -- and every tensor
 * of queries, and what is computed per query head, has n_heads * g heads: Q
 * [batch, n_heads * g, cap, head_dim], q [batch, n_heads * g, head_dim], lse
 * [batch, n_heads * g, cap], out [batch, n_heads * g, head_dim]; query head h * g + r belongs
 * to K/V head h.  Each query head has its own softmax over the rows of its K/V head (Eq. 1);
 * the score of a row is the mean over the group of what the g heads give it,
 *     S[i] = (1/g) sum_r sum_j a_i^{j,r}   (prompt),     S[i] += (1/g) sum_r a_i^r   (decode),
 * and Eq. 4 multiplies it by the norm of the shared value row.  Supported by
 * every call that takes queries (vatp_select_compact* involve none).  With a history window
 * (Eq. 3) the window runs over the group-averaged weights, and hist holds their means.
 */

/* Creates a context for HIP device `device` (host memory only; it also looks up the address of the
 * library's static scratch array on that device, making the device current for the lookup and
 * restoring the caller's device afterwards).  The device must be the
 * current HIP device whenever a call that takes the context is made: a call made while
 * another device is current returns VATP_E_DEVICE and enqueues nothing. */
vatp_status vatp_create(vatp_ctx **ctx, int device);
void        vatp_destroy(vatp_ctx *ctx);
const char *vatp_strerror(vatp_status st);

/*
 * Checks `p` for call `which_call` (a VATP_CALL_* value) exactly as that call does before
 * it launches anything; touches no device.  For the decode calls, len[b] + 1 <= cap is
 * required (room for the appended row).
 */
vatp_status vatp_validate(const vatp_params *p, int which_call);

/* Bytes of device workspace call `which_call` needs for `p` (0 on invalid params).
 * `ctx` may be NULL.  The workspace must be 256-byte aligned; its contents on entry do
 * not matter and are undefined on return. */
size_t vatp_workspace_bytes(const vatp_ctx *ctx, const vatp_params *p, int which_call);

/*
 * Prompt pass (Eq. 1 and Eq. 2 with t = len-1; Eq. 4's norm).
 * For every unit:  S[i]   = sum_{j=i}^{len-1} softmax_{i'<=j}(c <q_j, k_i'>)[i]
 *                  nrm[i] = |V[i]|_1 (or the norm `norm` selects)  for i < len[b].
 * Q, K, V: device [batch, n_heads, cap, head_dim] (dtype).  S, nrm: device float32
 * [batch, n_heads, cap], written for rows < len[b] only.  Nothing is pruned here.
 */
vatp_status vatp_prefill_score(vatp_ctx *ctx, const vatp_params *p,
                               const void *Q, const void *K, const void *V,
                               float *S, float *nrm,
                               void *ws, size_t ws_bytes, void *hip_stream);

/*
 * The same prompt pass when the row log-sum-exp of the causal softmax is already known, as a
 * fused attention kernel returns it: lse[j] = ln sum_{i<=j} exp(c <q_j, k_i>), device float32
 * [batch, n_heads, cap], rows < len[b].  The row-statistics pass is skipped (half of the
 * matrix work of Eq. 1/2); S and nrm are as above.  lse must be finite for rows < len[b].
 */
vatp_status vatp_prefill_score_lse(vatp_ctx *ctx, const vatp_params *p,
                                   const void *Q, const void *K, const void *V, const float *lse,
                                   float *S, float *nrm,
                                   void *ws, size_t ws_bytes, void *hip_stream);

/*
 * One decode step (Eq. 2 taken incrementally; order of operations as in Fig. 2).
 * For every unit with n0 = len[b] rows: the new token's k, v are stored as row n0 of the
 * K, V caches, nrm[n0] = |v| (same norm), pos[n0] = new_pos[b]; the new query attends over the
 * n0 + 1 rows and S[r] += a_r for r <= n0 (row n0 starts from 0).  The caller then uses
 * len[b] + 1.  q, k, v: device [batch, n_heads, head_dim] (dtype).  K, V, S, nrm, pos:
 * device caches, updated in place.  pos may be NULL (then new_pos may be NULL too).
 * new_pos: HOST [batch].
 */
vatp_status vatp_decode_step(vatp_ctx *ctx, const vatp_params *p,
                             const void *q, const void *k, const void *v,
                             void *K, void *V, float *S, float *nrm, int32_t *pos,
                             const int32_t *new_pos,
                             void *ws, size_t ws_bytes, void *hip_stream);

/*
 * vatp_decode_step that also returns the attention output of the new token (Eq. 1),
 *     out[x] = sum_{r<=n0} a_r V[r][x],
 * from the same pass over the cache (the probabilities are already there; this adds one read
 * of the V rows).  out: device float32 [batch, n_heads, head_dim].  Workspace size:
 * vatp_workspace_bytes(..., VATP_CALL_DECODE_ATTEND_STEP).
 */
vatp_status vatp_decode_attend_step(vatp_ctx *ctx, const vatp_params *p,
                                    const void *q, const void *k, const void *v,
                                    void *K, void *V, float *S, float *nrm, int32_t *pos,
                                    const int32_t *new_pos, float *out,
                                    void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Budgeted selection and compaction (Eq. 4; forced prefix, budget and local window from
 * the Attention Sink Tokens paragraph and the Implementation Details appendix).
 * For every unit with n = len[b] rows and B = budget[b]:
 *   n <= B : all rows survive (identity copy);
 *   else   : rows [0,F) and [n-R,n) survive, and of rows [F,n-R) the B-F-R with the
 *            largest I = S*nrm (float32 product; equal I: the lower row index wins).
 * The min(n,B) survivors are written, in ascending source-row order, to rows
 * [0, min(n,B)) of K_out, V_out ([batch, n_heads, cap_out, head_dim]) and S_out, nrm_out,
 * pos_out ([batch, n_heads, cap_out]); kept_idx ([batch, n_heads, cap_out], int32)
 * receives the source row of each survivor.  Out-of-place: no *_out buffer may alias an
 * input.  pos / pos_out may both be NULL.  The caller then uses len[b] = min(n, B).
 */
vatp_status vatp_select_compact(vatp_ctx *ctx, const vatp_params *p,
                                const void *K, const void *V, const float *S,
                                const float *nrm, const int32_t *pos,
                                void *K_out, void *V_out, float *S_out, float *nrm_out,
                                int32_t *pos_out, int32_t *kept_idx,
                                void *ws, size_t ws_bytes, void *hip_stream);

/*
 * The steady state of generation in one call: vatp_decode_step (or vatp_decode_attend_step
 * when out is not NULL) followed by vatp_select_compact, for caches that hold at most
 * budget[b] rows before the step, so that at most one row per head leaves (Fig. 2: the new
 * token is added, the least important unprotected one removed; Eq. 2 incrementally, Eq. 4).
 * The results are bit-identical to the two separate calls; one launch (many heads of at most 1024
 * rows) or two instead of three, and the rows that both cache sets already share are not copied again.
 *
 * The caller keeps two cache sets and alternates them: (K, V, S, nrm, pos) is the current set
 * with len[b] rows, (K_out, V_out, S_out, nrm_out, pos_out) the other one.  The call appends the
 * new row to K, V, nrm, pos (as vatp_decode_step does; S is only read), and makes the *_out set
 * the pruned state with min(len[b] + 1, budget[b]) rows, which is the current set of the next
 * call.  synced_in / synced_out: two distinct device int32 arrays [batch * n_heads].
 * synced_in[u] is the number of leading rows of K_out, V_out, nrm_out, pos_out that already
 * equal the leading rows of K, V, nrm, pos: 0 before the first call (or whenever the other set
 * was written by anything but this call), afterwards the array the previous call returned in
 * synced_out -- the caller swaps the two arrays together with the cache sets and must leave
 * the other set untouched in between.  synced_out[u] receives the row removed from head u
 * (len[b] + 1 if none), which is that count for the next call.  Rows from
 * min(synced_in[u], synced_out[u]) on are rewritten; S_out is rewritten in full.
 * kept_idx ([batch, n_heads, cap_out], may be NULL) receives the source row of each survivor,
 * out (device float32 [batch, n_heads, head_dim], may be NULL) the attention output.
 * Requires len[b] <= budget[b] (VATP_E_BUDGET otherwise) and len[b] + 1 <= cap.
 * Workspace size: vatp_workspace_bytes(..., VATP_CALL_DECODE_PRUNE_STEP).  new_pos: HOST.
 */
vatp_status vatp_decode_prune_step(vatp_ctx *ctx, const vatp_params *p,
                                   const void *q, const void *k, const void *v,
                                   void *K, void *V, const float *S, float *nrm, int32_t *pos,
                                   const int32_t *new_pos,
                                   void *K_out, void *V_out, float *S_out, float *nrm_out,
                                   int32_t *pos_out, int32_t *kept_idx,
                                   const int32_t *synced_in, int32_t *synced_out, float *out,
                                   void *ws, size_t ws_bytes, void *hip_stream);

/*
 * vatp_decode_prune_step for callers that cannot allocate device memory and have no workspace to
 * hand over: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, same results bit for bit, but no ws / ws_bytes: the step's scratch (logits, per-chunk
 * softmax statistics, partial attention outputs) lives in a static device array of
 * VATP_STATIC_SCRATCH_BYTES (16 MiB) that every GPU the library runs on holds until the process ends.
 * The call allocates and frees nothing.  It returns VATP_E_WORKSPACE, and enqueues nothing, when
 * vatp_workspace_bytes(ctx, p, VATP_CALL_DECODE_PRUNE_STEP) exceeds VATP_STATIC_SCRATCH_BYTES (16 MiB
 * cover a layer of 512 heads with 2458-row caches).  All calls on one GPU, from any context,
 * share that GPU's array: calls that overlap in time on one GPU (different streams) race; calls ordered
 * by one stream do not.  Nothing in the array has to start at zero: every call writes what it reads.
 */
vatp_status vatp_decode_prune_step_static(vatp_ctx *ctx, const vatp_params *p,
                                          const void *q, const void *k, const void *v,
                                          void *K, void *V, const float *S, float *nrm, int32_t *pos,
                                          const int32_t *new_pos,
                                          void *K_out, void *V_out, float *S_out, float *nrm_out,
                                          int32_t *pos_out, int32_t *kept_idx,
                                          const int32_t *synced_in, int32_t *synced_out, float *out,
                                          void *hip_stream);

/*
 * History-window scores (Eq. 3: S_k^t = sum of a_k^j over the last w+1 steps j only, the score
 * of the paper's "Scissorhands w/ VATP" variant).  Three calls mirror the three phases.
 *
 * vatp_prefill_score_window: as vatp_prefill_score with S_i = sum_{j >= max(len-1-w, i)} a_i^j
 * (only the prompt's last w+1 query rows are evaluated, a (w+1) x len band instead of the
 * triangle).  hist (device float32 [batch, n_heads, w+1, cap], may be NULL) receives those
 * attention rows, a_i^j at row j - max(len-1-w, 0), column i, for i <= j; other entries are left
 * undefined.  Workspace size: vatp_workspace_bytes(..., VATP_CALL_PREFILL_SCORE_WINDOW).
 *
 * vatp_select_compact_window: vatp_select_compact of the prompt (hist: what the call above
 * left), after which hist_out (device
 * float32 [batch, n_heads, w+2, cap_hist], cap_hist >= min(len, budget)) holds the history of
 * the survivors as a ring (query j in row j mod (w+2)), column o for survivor o, hid_out ([batch, n_heads, cap_out] int32) is set to
 * o and free_out ([batch * n_heads] int32) to the survivor count.  S_lo_out (device float32
 * [batch, n_heads, cap_out]) receives the low-order part of every survivor's score (see below).
 *
 * vatp_decode_prune_step_window: vatp_decode_prune_step with S_new = S + a^t - a^(t-w-1),
 * t = new_pos[b] (HOST, required: the index of the new token in its sequence, counted on from
 * the prompt).  Every cached row owns one history column for its lifetime: hid / hid_out are
 * per-row int32 like pos / pos_out and move with the rows; the appended row takes column
 * free_in[u], and free_out[u] receives the column the evicted row gave up (or the next fresh
 * one while the cache still grows); free_in / free_out are distinct device arrays
 * [batch * n_heads] that the caller swaps like synced_in / synced_out.  hist is updated in
 * place: ring row t mod (w+2) is written, row (t+1) mod (w+2) read.  cap_hist >= budget[b] + 1.
 * The score of a row is carried as the unevaluated sum of two floats, S (what the selection
 * sees) and a low-order part S_lo / S_lo_out (device float32, per row like S / S_out, moving with
 * the rows; distinct arrays that alternate with the cache sets): a weight is added when it enters
 * the window and the same float is subtracted when it leaves, each time by an error-free
 * transformation, so the error of a score stays relative to the score itself (about 2^-47 of the
 * running sum per step) however large the score once was and however many steps have passed.
 */
vatp_status vatp_prefill_score_window(vatp_ctx *ctx, const vatp_params *p,
                                      const void *Q, const void *K, const void *V, int32_t window,
                                      float *S, float *nrm, float *hist,
                                      void *ws, size_t ws_bytes, void *hip_stream);

vatp_status vatp_select_compact_window(vatp_ctx *ctx, const vatp_params *p,
                                       const void *K, const void *V, const float *S,
                                       const float *nrm, const int32_t *pos, const float *hist,
                                       int32_t window,
                                       void *K_out, void *V_out, float *S_out, float *nrm_out,
                                       int32_t *pos_out, int32_t *kept_idx, float *hist_out,
                                       int32_t cap_hist, int32_t *hid_out, int32_t *free_out,
                                       float *S_lo_out,
                                       void *ws, size_t ws_bytes, void *hip_stream);

vatp_status vatp_decode_prune_step_window(vatp_ctx *ctx, const vatp_params *p,
                                          const void *q, const void *k, const void *v,
                                          void *K, void *V, const float *S, float *nrm,
                                          int32_t *pos, int32_t *hid, const int32_t *new_pos,
                                          void *K_out, void *V_out, float *S_out, float *nrm_out,
                                          int32_t *pos_out, int32_t *hid_out, int32_t *kept_idx,
                                          const int32_t *synced_in, int32_t *synced_out,
                                          const int32_t *free_in, int32_t *free_out,
                                          float *hist, const float *S_lo, float *S_lo_out,
                                          int32_t window, int32_t cap_hist, float *out,
                                          void *ws, size_t ws_bytes, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* VATP_H */
