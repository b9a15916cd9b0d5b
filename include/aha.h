/*
 * aha.h -- C ABI of the AhaKV eviction hot path for AMD MI355X (gfx950).
 *
 * The four operations follow the paper's problem statement (Alg. 1): per
 * layer, per head, Q, K, V in R^{n x d}; a total cache budget B made of a
 * recent budget B_r and a selected budget B_s = B - B_r; an observation
 * window of the r most recent query rows.
 *
 * General rules for every entry point
 *   - All tensor arguments are DEVICE pointers owned by the caller.  The
 *     library never allocates or frees device memory, never synchronises and
 *     keeps no pointer after the call returns.  Scratch memory is the
 *     caller's `workspace` (device memory, 256-byte aligned, at least
 *     aha_workspace_bytes() bytes, contents arbitrary on entry and exit).
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     Calls only enqueue work on it.  Two calls that share a workspace or a
 *     cache must be ordered by the caller (same stream, or events).
 *   - Token positions are 0-indexed; query row i attends keys 0..i.
 *   - Element strides (batch, head, token) are given in ELEMENTS; the
 *     head_dim axis is contiguous.  Rows must be 16-byte aligned (base
 *     pointers 16-byte aligned, strides multiples of 8 elements for bf16 and
 *     4 for fp32).
 *   - Return value: AHA_OK or a negative status.  All argument, size and
 *     workspace checks happen on the host before anything is launched: with
 *     AHA_ERR_INVALID_ARG, AHA_ERR_UNSUPPORTED or AHA_ERR_WORKSPACE nothing has
 *     been enqueued.  AHA_ERR_HIP reports that the HIP runtime refused a
 *     launch; earlier launches of the same call may already be enqueued and
 *     the outputs are then undefined.
 *     aha_last_error() returns a thread-local, human readable reason.
 *   - No C++ exception crosses this boundary.
 */
#ifndef AHA_H_
#define AHA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    AHA_OK = 0,
    AHA_ERR_INVALID_ARG = -1, /* a null pointer, an impossible size or stride */
    AHA_ERR_UNSUPPORTED = -2, /* legal but not built: head_dim, dtype, sizes */
    AHA_ERR_WORKSPACE = -3,   /* workspace null, misaligned or too small */
    AHA_ERR_HIP = -4          /* the HIP runtime refused a launch */
};

enum { AHA_F32 = 0, AHA_BF16 = 1 };
enum { AHA_SCALE_FIXED = 0, AHA_SCALE_ADAPTIVE = 1 };

/*
 * Problem description shared by the four operations.
 *
 *  window       r, the number of most recent query rows whose attention
 *               rows are accumulated (Sec. 4.1, Recent Accumulation).
 *               window == seq_len gives the plain accumulated attention
 *               score (the H2O score of Sec. 4.1).
 *  budget       B, total retained tokens per (batch, KV head); it is also k
 *               in the adaptive scale.  1 <= budget <= seq_len.
 *  recent       B_r, most recent tokens that are always retained;
 *               0 <= recent <= budget.
 *  scale_mode   AHA_SCALE_FIXED: softmax(fixed_scale * q.k).  1/sqrt(d)
 *               gives the standard attention row.
 *               AHA_SCALE_ADAPTIVE: step-gain softmax of Sec. 4.2 with
 *               lambda_i = sqrt(2 ln(c_i / budget) / d), c_i = number of keys
 *               the row normalises over, the logarithm clamped at 0 and the
 *               result floored at lambda_floor (lambda_floor < 0 means
 *               1/sqrt(d)).  lambda replaces 1/sqrt(d); it multiplies the raw
 *               dot product in fp32.
 *  value_prior  non-zero: scores are multiplied by gamma_bar of Sec. 4.3,
 *               gamma = average pool over tokens (odd width pool_kernel,
 *               stride 1, edge-truncated mean) of ||V_j||^2, divided by its
 *               maximum over the sequence of that (batch, KV head).  If every
 *               value row of a head is zero the quotient is undefined and
 *               gamma_bar is taken as 1 (the scores stay unrefined).
 *  n_q_heads    must be a multiple of n_kv_heads; the score of a KV head is
 *               the sum over the query heads that share it.
 *  score_pool   smoothing of the scores before the selection (caption of the
 *               method's overview figure): aha_select_topk ranks the
 *               candidates by the average pool of the scores over tokens
 *               (odd width score_pool, stride 1, edge-truncated mean over all
 *               seq_len tokens, formed in fp32 left to right).  0 or 1: off.
 *               The scores themselves, and with them the running scores that
 *               aha_compact_kv seeds, are not changed.
 *  sink         the first `sink` tokens are always retained, like the `recent`
 *               last ones (the static policy of the related work, which keeps
 *               the beginning tokens and the most recent ones, as a mode of
 *               this selection): aha_select_topk fills the remaining
 *               budget - sink - recent places by score, aha_decode_step never
 *               evicts a position < sink.  budget = sink + recent is the
 *               static policy itself.  0: off.
 *  decode_value_prior  the value prior of Sec. 4.3 inside the generation loop:
 *               aha_decode_step multiplies what it adds to the running score
 *               of slot s by ||v_cache[s]||^2 / max over the live slots (no
 *               average pool: neighbouring slots are not neighbouring tokens;
 *               all-zero values: factor 1).  0: the loop as the algorithm
 *               prints it.
 */
typedef struct aha_params {
    int32_t batch;        /* batch * n_kv_heads <= 65535 */
    int32_t n_q_heads;
    int32_t n_kv_heads;
    int32_t head_dim;     /* 64 or 128 */
    int32_t seq_len;      /* n (prefill), 1..2^30 ; ignored by aha_decode_step */
    int32_t window;       /* r, 1..seq_len */
    int32_t budget;       /* B, <= 2^30 */
    int32_t recent;       /* B_r */
    int32_t dtype;        /* AHA_F32 | AHA_BF16: element type of Q, K, V, caches, out */
    int32_t scale_mode;   /* AHA_SCALE_FIXED | AHA_SCALE_ADAPTIVE */
    float fixed_scale;    /* >= 0 */
    float lambda_floor;   /* see above */
    int32_t value_prior;  /* 0 | 1 */
    int32_t pool_kernel;  /* odd, 1..255 */
    int64_t q_stride[3];  /* elements: batch, head, token (prefill Q) */
    int64_t k_stride[3];  /* elements: batch, head, token (prefill K) */
    int64_t v_stride[3];  /* elements: batch, head, token (prefill V) */
    int32_t score_pool;   /* 0 | odd, 1..255; used by aha_select_topk (and the workspace size) */
    int32_t sink;         /* >= 0, sink + recent <= budget: first tokens always retained */
    int32_t decode_value_prior; /* 0 | 1: aha_decode_step refines what it adds to the scores */
    int32_t reserved;     /* must be 0 */
} aha_params;

/*
 * Bytes of workspace that any of the calls below needs for `p` (the maximum
 * over the four operations, a multiple of 256).  With p->seq_len == 0 only
 * aha_decode_step is counted and the prefill fields are not looked at (for a
 * caller that holds a compact cache and no prompt).
 */
int32_t aha_workspace_bytes(const aha_params *p, size_t *out_bytes);

/*
 * Prefill eviction scores (Alg. 1 Prefill, score lines; Sec. 4.1 - 4.3).
 *
 *   scores[b, h, j] = gamma_bar[b, h, j] *
 *        sum_{g in group(h)} sum_{i = n-r}^{n-1} softmax_{j' <= i}(s_i * Q_i . K_j')_j
 *
 *  q       [batch, n_q_heads, seq_len, head_dim] by q_stride; only the last
 *          `window` rows of each head are read.
 *  k, v    [batch, n_kv_heads, seq_len, head_dim] by k_stride / v_stride.
 *  scores  out, fp32, dense [batch, n_kv_heads, seq_len].
 * The probability matrix is never written to memory: one pass over the keys
 * finds each row's maximum and log-sum-exp, a second pass recomputes the
 * logits and accumulates the column sums.
 */
int32_t aha_prefill_scores(const aha_params *p, const void *q, const void *k,
                           const void *v, float *scores, void *workspace,
                           size_t workspace_bytes, void *stream);

/*
 * Prefill eviction scores beside an attention forward pass that has already
 * normalised the observed rows (appendix on compatibility with
 * FlashAttention: the score is an extra product of a forward pass, which keeps
 * the logarithm of every row's softmax denominator).  Same result and
 * arguments as aha_prefill_scores, except that the row-statistics pass is
 * skipped and
 *
 *  lse     fp32 dense [batch, n_q_heads, window]: for window row ii (query
 *          position seq_len - window + ii) the natural logarithm of
 *          sum_{j <= i} exp(s_i * Q_i . K_j), s_i being the scale that
 *          p->scale_mode gives that row - with AHA_SCALE_FIXED and
 *          fixed_scale = 1/sqrt(d) this is the forward pass's log-sum-exp.
 *
 * The probabilities are formed as exp(s_i * Q_i . K_j - lse_i): a normaliser
 * that does not belong to the row scales that row's contribution and is not
 * detected.  The stage events of aha_profile_events are recorded as for
 * aha_prefill_scores (events[1] and [2] then bracket nothing).
 */
int32_t aha_prefill_scores_lse(const aha_params *p, const void *q, const void *k,
                               const void *v, const float *lse, float *scores,
                               void *workspace, size_t workspace_bytes, void *stream);

/*
 * Prefill eviction scores accumulated over query rows that the caller chose
 * (Limitations: the recent rows are not the only possible choice of the
 * constant number of accumulators; the same number of rows may be selected by
 * a Top-k strategy - the criterion is the caller's, e.g. the rows of lowest
 * entropy from aha_prefill_row_stats).  Same result and arguments as
 * aha_prefill_scores, except that the `window` accumulated rows of query head
 * (b, hq) are the positions
 *
 *  rows    int32 dense [batch, n_q_heads, window], each in [0, seq_len)
 *          (positions outside are clamped to the sequence; a position listed
 *          twice is accumulated twice).
 *
 * The row at position i attends keys j <= i with the scale of a row over
 * i + 1 keys.  bf16: n_q_heads / n_kv_heads * window must not exceed 256
 * (AHA_ERR_UNSUPPORTED otherwise).
 */
int32_t aha_prefill_scores_rows(const aha_params *p, const void *q, const void *k,
                                const void *v, const int32_t *rows, float *scores,
                                void *workspace, size_t workspace_bytes, void *stream);

/*
 * Attention output of the observed rows, beside which the score is computed
 * (appendix on compatibility with FlashAttention; Alg. 1 Prefill forms both
 * from the logits A = Q K^T / sqrt(d)):
 *
 *   out[b, h, ii, :] = sum_{j <= i} softmax_j(Q_i . K_j / sqrt(d)) V_j,
 *                      i = seq_len - window + ii,
 *
 * always with the standard scale, whatever p->scale_mode says.
 *
 *  q, k, v  as in aha_prefill_scores.
 *  out      element type p->dtype, dense [batch, n_q_heads, window, head_dim].
 *  lse      out, fp32 dense [batch, n_q_heads, window] or NULL: natural log of
 *           sum_{j <= i} exp(Q_i . K_j / sqrt(d)): with scale_mode FIXED and
 *           fixed_scale = 1/sqrt(d), what aha_prefill_scores_lse takes - the two
 *           calls then give output and scores with one pass over the keys each.
 *  workspace  at least aha_window_attention_workspace_bytes() bytes (its own
 *           size query: the partial outputs of the key ranges, which
 *           aha_workspace_bytes does not count; 0 for fp32).
 * bf16 runs on the matrix cores (one flash-style pass); fp32 is a plain kernel
 * for small problems.
 */
int32_t aha_window_attention_workspace_bytes(const aha_params *p, size_t *out_bytes);
int32_t aha_prefill_window_attention(const aha_params *p, const void *q, const void *k,
                                     const void *v, void *out, float *lse,
                                     void *workspace, size_t workspace_bytes,
                                     void *stream);

/*
 * Statistics of the observed rows (Sec. 4.2: the information entropy of an
 * attention row, H_i = - sum_{j <= i} a_ij ln a_ij, whose expectation the
 * adaptive scale is derived from), by the row-statistics pass alone:
 *
 *  lse      out, fp32 dense [batch, n_q_heads, window] or NULL: natural
 *           logarithm of sum_{j <= i} exp(s_i * Q_i . K_j) of window row ii
 *           (query position seq_len - window + ii), s_i the scale that
 *           p->scale_mode gives the row: what aha_prefill_scores_lse takes.
 *  entropy  out, fp32 dense [batch, n_q_heads, window] or NULL: H_i in nats of
 *           the row softmax_{j <= i}(s_i * Q_i . K_j).
 * At least one of the two must be given.  window == seq_len gives the curve
 * over all positions.  v, value_prior and pool_kernel are not used.
 */
int32_t aha_prefill_row_stats(const aha_params *p, const void *q, const void *k,
                              float *lse, float *entropy, void *workspace,
                              size_t workspace_bytes, void *stream);

/*
 * Selection (Alg. 1: recent set, TopK, union).
 *
 *  scores  fp32 [batch, n_kv_heads, seq_len], non-negative and finite.
 *  idx     out, int32 dense [batch, n_kv_heads, budget], ascending token
 *          positions: the first `sink` positions, the budget - sink - recent
 *          highest-scoring tokens among sink <= position < seq_len - recent
 *          (ties: lower position wins), and the `recent` last positions.
 * With p->score_pool > 1 the candidates are ranked by their pooled scores,
 * which are written to the workspace first (batch * n_kv_heads * seq_len
 * floats; aha_workspace_bytes accounts for them); otherwise the workspace is
 * not used and may be null.
 */
int32_t aha_select_topk(const aha_params *p, const float *scores, int32_t *idx,
                        void *workspace, size_t workspace_bytes, void *stream);

/*
 * Compaction (Alg. 1 Generation: K_S, V_S, F_0 = refined prefill score).
 * Of `p` only the shape, dtype, budget and the K / V strides are used.
 *
 *  k, v         as in aha_prefill_scores.
 *  scores, idx  as produced by the two calls above.
 *  k_cache, v_cache  out, element type p->dtype, dense
 *               [batch, n_kv_heads, cache_slots, head_dim]; cache_slots >=
 *               budget + 1.  Slot s < budget receives row idx[s]; the other
 *               slots are zero-filled.
 *  scores_c     out, fp32 dense [batch, n_kv_heads, cache_slots]: running
 *               score F of each slot (0 for empty slots).
 *  pos_c        out, int32 dense [batch, n_kv_heads, cache_slots]: token
 *               position of each slot, -1 for an empty slot.
 *  free_slot    out, int32 [batch, n_kv_heads]: the slot the next generated
 *               token will occupy (= budget).
 */
int32_t aha_compact_kv(const aha_params *p, const void *k, const void *v,
                       const float *scores, const int32_t *idx, void *k_cache,
                       void *v_cache, float *scores_c, int32_t *pos_c,
                       int32_t *free_slot, int32_t cache_slots, void *stream);

/*
 * One generation step with running eviction (Alg. 1 Generation, loop body),
 * for every (batch, KV head), in place on the compact cache:
 *   1. k_new / v_new are written to slot free_slot, score 0, position
 *      logical_pos - 1;
 *   2. w_s = q . k_cache[s] over the budget + 1 live slots (slots 0..budget);
 *   3. out = sum_s softmax_s(w_s / sqrt(d)) v_cache[s]   (the attention output);
 *   4. scores_c[s] += sum_{g in group} softmax_s(scale * w_s), with the scale
 *      of p->scale_mode evaluated at c = logical_pos;
 *      (with p->decode_value_prior, times the value prior of the slot);
 *   5. slots whose position >= logical_pos - recent or < p->sink are
 *      protected; of the others the one with the smallest score is evicted
 *      (ties: the highest position): pos_c = -1 there and free_slot points to it.
 *
 *  q_new        [batch, n_q_heads, head_dim] dense, p->dtype.
 *  k_new, v_new [batch, n_kv_heads, head_dim] dense, p->dtype.
 *  logical_pos  number of tokens seen so far including the new one.
 *  out          [batch, n_q_heads, head_dim] dense, p->dtype.
 * p->seq_len, window, value_prior, pool_kernel and the strides are ignored.
 * Exactly budget + 1 slots must be live on entry (budget occupied + the free
 * one), which aha_compact_kv and every previous step guarantee.
 * The dots of a head's live slots are kept in on-chip memory: with fewer than
 * 128 (batch, KV head) problems the slots are split over up to 64 workgroups
 * (group * slots-per-split * 4 + 16 * group * head_dim bytes each, at most
 * 64 KiB), otherwise one workgroup holds 8 * group * (budget + 1) bytes (at
 * most 150 KiB); larger budgets return AHA_ERR_UNSUPPORTED.
 */
int32_t aha_decode_step(const aha_params *p, const void *q_new, const void *k_new,
                        const void *v_new, void *k_cache, void *v_cache,
                        float *scores_c, int32_t *pos_c, int32_t *free_slot,
                        int32_t cache_slots, int32_t logical_pos, void *out,
                        void *workspace, size_t workspace_bytes, void *stream);

/*
 * aha_decode_step for callers that cannot allocate or carry a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, result and errors as aha_decode_step, without
 * the workspace: the scratch of the few-heads path lives in a buffer built
 * into the library (4 MiB per GPU, held until the process ends).  The call
 * allocates and frees nothing.  A shape whose scratch (aha_workspace_bytes
 * with seq_len = 0) exceeds 4 MiB returns AHA_ERR_UNSUPPORTED before anything
 * is launched - e.g. 8 KV heads x 4 query heads x budget 2048 needs 0.8 MiB.
 * All calls on one GPU share the buffer: two calls that may overlap in time
 * (different streams, different threads) race and must be ordered by the
 * caller.  The buffer keeps the previous call's contents; the kernels read
 * nothing from it that the same call has not written.
 */
int32_t aha_decode_step_static(const aha_params *p, const void *q_new, const void *k_new,
                               const void *v_new, void *k_cache, void *v_cache,
                               float *scores_c, int32_t *pos_c, int32_t *free_slot,
                               int32_t cache_slots, int32_t logical_pos, void *out,
                               void *stream);

/*
 * Optional stage timing for aha_prefill_scores (Sec. 4.1 - 4.3 are computed by
 * three launches: value prior, row statistics, column sums).  `events` is an
 * array of `count` caller-created hipEvent_t handles (HOST array, copied by
 * the call); while set, aha_prefill_scores on this thread records events[0]
 * before its first launch and events[1], [2], [3] after the value-prior,
 * row-statistics and column-sum launches, on the call's stream.  count must
 * be 0 (with events NULL: switch off) or 4.  The library neither creates,
 * waits on nor destroys the events.
 */
int32_t aha_profile_events(void *const *events, int32_t count);

/* Thread-local description of the last error returned on this thread. */
const char *aha_last_error(void);

/* Library version string, e.g. "aha-gfx950 0.1". */
const char *aha_version(void);

#ifdef __cplusplus
}
#endif
#endif /* AHA_H_ */
