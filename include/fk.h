/*
 * fk — budgeted KV-cache decoding with learned eviction (ForesightKV generation path)
 * for AMD MI355X (gfx950).  C ABI; every kernel behind it is hand-written HIP.
 *
 * The path (Section 3.1 of the paper, "Dynamic KV Cache Eviction During Long-Context
 * Generation"): the cache holds at most B + L pairs per (sequence, KV head).  Every
 * decode step appends the new pair (fk_append) and attends over the retained pairs
 * (fk_decode_attn).  After every L steps the retained pairs are scored by an MLP
 * (fk_score_kv), the L newest plus the B - L most important others are selected
 * (fk_select_keep) and the cache is compacted back to B entries (fk_compact).
 *
 * Memory layout (row major, all DEVICE memory owned by the caller):
 *   K, V   [batch][n_kv_heads][capacity][head_dim]   dtype (fp32 or bf16)
 *   pos    [batch][n_kv_heads][capacity]             int32 absolute position of each slot
 *   len    [batch][n_kv_heads]                       int32 retained count of each row
 * A (sequence, KV head) pair is called a row; row index r = b * n_kv_heads + h.  Slots
 * 0 .. len[r]-1 of a row are live.  Every row carries its own count (each KV head keeps its own
 * retained set); under one budget for all heads the counts of a sequence are equal.
 * Precondition kept by fk_append and fk_compact: along the live slots of a row the
 * positions are strictly increasing, so slot order is position order.
 *
 * Conventions:
 *   - descriptor structs are HOST memory, read during the call only;
 *   - all other pointers are DEVICE pointers, 16-byte aligned, owned by the caller;
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream); every call
 *     only enqueues work on it and returns; nothing is allocated.  The only state the library keeps is per
 *     device and invisible to results: flags "this kernel's dynamic-LDS limit has been raised" and, for
 *     fk_decode_step_static, the address of its fixed scratch array;
 *   - errors are return codes; arguments are validated on the host before any launch;
 *   - `max_len` is a host-side upper bound on every len[r] at the time the kernels run
 *     (pass `capacity` when unknown); it only sizes the launch.  Every call stays correct when a row is longer
 *     than max_len (the last workgroup of the row runs on to the row's end: slower, same results).
 *   - supported: head_dim 64 or 128; dtype fp32 or bf16; n_q_heads a multiple of
 *     n_kv_heads with group size <= 8; capacity < 2^24.
 */
#ifndef FK_H
#define FK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FK_OK = 0,
    FK_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, inconsistent sizes */
    FK_ERR_UNSUPPORTED = 2, /* shape or dtype outside the supported set */
    FK_ERR_WORKSPACE = 3,   /* workspace missing or too small */
    FK_ERR_LAUNCH = 4       /* the HIP runtime refused a launch */
} fk_status;

typedef enum { FK_F32 = 0, FK_BF16 = 1 } fk_dtype;

typedef struct {
    int32_t batch;      /* sequences */
    int32_t n_q_heads;  /* query heads per sequence */
    int32_t n_kv_heads; /* KV heads per sequence; group size g = n_q_heads / n_kv_heads */
    int32_t head_dim;   /* D */
    int32_t capacity;   /* slots per row, >= B + L */
    int32_t dtype;      /* fk_dtype of q, K, V, out and of the scorer's W1 */
    int32_t flags;      /* FK_CACHE_* bits, 0 by default */
} fk_cache_desc;

/* The cache is not expected to sit in the GPU's caches when a call starts (one layer of a deep stack whose
 * layers are visited in turn): attention streams K and V with non-temporal loads whatever their size.  Without
 * the flag that is done from 352 MB of K + V per call on, below which a cache re-read every step stays in the
 * Infinity Cache, and rows may be cut into more splits (size the workspace with the same descriptor).  A hint:
 * results are the same up to the order of the floating-point merges. */
#define FK_CACHE_COLD 1

/* Scoring model of one layer (Appendix B.1): phi = gelu(x W1 + b1) W2 + b2, x = concat(k, v). */
typedef struct {
    const void *w1;   /* device [n_sets][2*head_dim][hidden], cache dtype */
    const float *b1;  /* device [n_sets][hidden] */
    const float *w2;  /* device [n_sets][hidden] */
    const float *b2;  /* device [n_sets] */
    int32_t hidden;   /* H; bf16: multiple of 8 with H'*(2*head_dim+8)*2 + 8*H' <= 160 KiB of LDS, H' = H rounded up to 32 */
    int32_t per_head; /* 1: n_sets = n_kv_heads, one model per KV head; 0: one shared model */
    int32_t skip_len; /* rows with len[r] <= skip_len are skipped, their scores not written (pass the budget:
                         rows at or under budget are not pruned and need no scores); 0 scores every row */
} fk_scorer;

const char *fk_status_string(fk_status s);

/* Names the build: "fk <version> gfx950". */
const char *fk_version(void);

/*
 * Section 3.1 (a generated token joins the cache): for every sequence b and KV head h write
 * k_new[b][h][:], v_new[b][h][:] and pos_new[b] into slot len[r] of row r = (b, h), then
 * len[r] += 1.  k_new, v_new: [batch][n_kv_heads][head_dim] dtype; pos_new: [batch] int32.
 * A row whose len[r] == capacity is left unchanged (nothing is written past the row).
 */
fk_status fk_append(const fk_cache_desc *desc, void *K, void *V, int32_t *pos, int32_t *len,
                    const void *k_new, const void *v_new, const int32_t *pos_new, void *stream);

/*
 * Bytes of device workspace fk_decode_attn / fk_decode_step need (0 on bad args).  The size does
 * not depend on max_len, so one workspace serves every call on this descriptor.  The workspace
 * starts with per-row arrival counters: the caller zero-fills it ONCE after allocating it; every call
 * leaves the counters at zero again.  Calls sharing a workspace must not overlap in time.
 */
size_t fk_decode_attn_workspace(const fk_cache_desc *desc, int32_t max_len);

/*
 * Appendix A, "Problem Setup" (attention over the retained set, renormalised softmax):
 *   out[b][hq][:] = sum_{i < len[b][hq/g]} softmax_i(softmax_scale * <q[b][hq], K[b][hq/g][i]>) V[b][hq/g][i]
 * q, out: [batch][n_q_heads][head_dim] dtype; accumulation in fp32 (bf16 with head_dim 128: the
 * softmax weights are rounded to bf16 before the P.V contraction and normalised by the sum of the
 * rounded weights).  Query heads of a row with len == 0 get zeros.  workspace: >= fk_decode_attn_workspace(desc, max_len) bytes, zero-filled
 * once by the caller (see above); FK_ERR_WORKSPACE if missing or too small.  One launch.
 */
fk_status fk_decode_attn(const fk_cache_desc *desc, const void *q, const void *K, const void *V,
                         const int32_t *len, int32_t max_len, float softmax_scale, void *out,
                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * One decode step in ONE launch: fk_append followed by fk_decode_attn (Section 3.1 for the append,
 * Appendix A "Problem Setup" for the attention), with the same arguments and results as the two
 * calls in that order; the new pair takes part in the attention.  max_len bounds len[r] + 1.
 */
fk_status fk_decode_step(const fk_cache_desc *desc, const void *q, void *K, void *V, int32_t *pos,
                         int32_t *len, const void *k_new, const void *v_new, const int32_t *pos_new,
                         int32_t max_len, float softmax_scale, void *out, void *workspace,
                         size_t workspace_bytes, void *stream);

/*
 * fk_decode_step for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): same arguments and results as fk_decode_step without the workspace,
 * which is a fixed FK_STATIC_SCRATCH_BYTES array inside the library's device image (each GPU the library runs on
 * holds its own copy until the process ends).  FK_ERR_WORKSPACE when fk_decode_attn_workspace(desc, max_len)
 * exceeds FK_STATIC_SCRATCH_BYTES (about batch * n_kv_heads * splits * g * (head_dim + 2) * 4 bytes; the Qwen3-4B
 * layer shape at batch 16 needs 0.8 MB); FK_ERR_LAUNCH if the array's address cannot be resolved.  Nothing is
 * allocated or freed, by this call or by anything it calls.  The first call on a device looks the array up and
 * clears it with a small kernel on `stream` (make that call outside a graph capture); every call leaves the
 * counters in it at zero for the next one.  All calls on one GPU share the array: calls that overlap in time
 * on one GPU (two streams, two threads) race, the caller must serialise them.
 */
#define FK_STATIC_SCRATCH_BYTES (8u << 20)
fk_status fk_decode_step_static(const fk_cache_desc *desc, const void *q, void *K, void *V, int32_t *pos,
                                int32_t *len, const void *k_new, const void *v_new, const int32_t *pos_new,
                                int32_t max_len, float softmax_scale, void *out, void *stream);

/*
 * Section 3.1 (the L generation steps between two eviction events): n_steps consecutive fk_decode_step calls
 * enqueued by one call, step t on q_seq[t], k_seq[t], v_seq[t], pos_seq[t] with its output in out_seq[t] and
 * max_len = min(max_len_first + t, capacity); max_len_first bounds len[r] + 1 at the first step.
 *   q_seq, out_seq [n_steps][batch][n_q_heads][head_dim], k_seq, v_seq [n_steps][batch][n_kv_heads][head_dim]
 *   dtype; pos_seq [n_steps][batch] int32.
 * Results are those of the n_steps single calls; the host returns to its caller once per window instead
 * of once per step.  n_steps == 0 is a no-op.  On an error the steps before it stay enqueued.
 */
fk_status fk_decode_window(const fk_cache_desc *desc, const void *q_seq, void *K, void *V, int32_t *pos,
                           int32_t *len, const void *k_seq, const void *v_seq, const int32_t *pos_seq,
                           int32_t n_steps, int32_t max_len_first, float softmax_scale, void *out_seq,
                           void *workspace, size_t workspace_bytes, void *stream);

/*
 * Section 3.1 Eq. 1 and Appendix B.1 (importance score of every retained pair, features
 * restricted to the key and value vectors):
 *   scores[b][h][i] = sum_j gelu(sum_f x_f W1[f][j] + b1[j]) W2[j] + b2,  x = [K[b][h][i], V[b][h][i]]
 * for i < len[r]; gelu is the exact erf form; fp32 accumulation (bf16: MFMA).  scores:
 * [batch][n_kv_heads][capacity] fp32; slots >= len[r] are not written.
 */
fk_status fk_score_kv(const fk_cache_desc *desc, const void *K, const void *V, const int32_t *len,
                      int32_t max_len, const fk_scorer *scorer, float *scores, void *stream);

/*
 * Section 3.1 (keep the most recent L pairs, prune the others to the B - L most important;
 * deterministic Top-K form).  For every row with len[r] > budget: keep the last
 * `protect_recent` live slots and, of the other len[r] - protect_recent, the
 * budget - protect_recent best under the total order (score descending, then slot
 * ascending = position ascending).  -0 equals +0; NaN ranks below -inf.  The kept slot
 * indices are written ascending to keep_idx[b][h][0 .. budget-1].  Rows with
 * len[r] <= budget get the identity keep_idx[j] = j for all j < budget (nothing to prune; fk_compact moves nothing).
 * keep_idx: [batch][n_kv_heads][budget] int32.  pos may be NULL: it is not read, slot order
 * stands for position order (see the precondition above).
 * Requires 0 <= protect_recent <= budget <= capacity.
 */
fk_status fk_select_keep(const fk_cache_desc *desc, const float *scores, const int32_t *pos,
                         const int32_t *len, int32_t max_len, int32_t budget,
                         int32_t protect_recent, int32_t *keep_idx, void *stream);

/*
 * fk_select_keep for few, long rows (Section 4.3: one-shot compression of a long prompt before
 * decoding; the same selection rule, applied once to rows far over budget).  Same arguments,
 * same result bit for bit.  With at most 64 rows of max_len >= 16384 a row is cut into chunks that
 * are selected by one workgroup each, and a second launch selects among the chunks' survivors (a
 * pair among the row's best budget - protect_recent is among its chunk's best under the same total
 * order); otherwise this is fk_select_keep.  workspace: caller-owned device scratch of at least
 * fk_select_keep_workspace(desc, max_len, budget, protect_recent) bytes (0 when rows are not split;
 * then workspace may be NULL), contents undefined before and after; FK_ERR_WORKSPACE if too small.
 */
size_t fk_select_keep_workspace(const fk_cache_desc *desc, int32_t max_len, int32_t budget,
                                int32_t protect_recent);
fk_status fk_select_keep_ws(const fk_cache_desc *desc, const float *scores, const int32_t *pos,
                            const int32_t *len, int32_t max_len, int32_t budget,
                            int32_t protect_recent, int32_t *keep_idx, void *workspace,
                            size_t workspace_bytes, void *stream);

/*
 * Section 3.1 Eq. 2 and Appendix B.2 (Top-K multinomial eviction, the paper's inference policy).
 * For every row with len[r] > budget, E = len[r] - budget pairs go: the last `protect_recent` live
 * slots are kept; of the others, the max(n_candidates, E) lowest-ranked under (score descending,
 * slot ascending) are candidates (the paper uses 2E), the rest are kept; E candidates are drawn
 * without replacement with probabilities softmax(-score), in Gumbel-top-k form: the caller supplies
 * noise[b][h][i] (iid Gumbel(0,1) for the paper's law; fp32, [batch][n_kv_heads][capacity]) and the
 * E candidates with the smallest fp32 value of scores - noise are evicted, ties evicting the higher
 * slot first.  noise == 0 or n_candidates <= E gives fk_select_keep's result.  Output, rows at or
 * under budget, pos and the special values are as for fk_select_keep.  capacity <= 131072
 * (FK_ERR_UNSUPPORTED above).
 */
fk_status fk_select_keep_sampled(const fk_cache_desc *desc, const float *scores, const float *noise,
                                 const int32_t *pos, const int32_t *len, int32_t max_len,
                                 int32_t budget, int32_t protect_recent, int32_t n_candidates,
                                 int32_t *keep_idx, void *stream);

/*
 * Section 1 / 3.1 (evicted pairs are discarded for good; stable in-place form): for every row
 * with len[r] > budget, slot j of K, V and pos receives the former contents of slot
 * keep_idx[b][h][j], j = 0 .. budget-1 (bit copies; keep_idx ascending with keep_idx[j] >= j,
 * as fk_select_keep writes it), then len[r] = budget.  Rows with len[r] <= budget are untouched.
 * What moves is read from keep_idx alone (one launch, the length is clamped in the same kernel): every row of
 * keep_idx must be written in full, rows at or under budget with the identity or with entries outside
 * [0, capacity) (both move nothing; fk_select_keep and fk_select_keep_sampled write the identity).
 */
fk_status fk_compact(const fk_cache_desc *desc, void *K, void *V, int32_t *pos, int32_t *len,
                     const int32_t *keep_idx, int32_t budget, void *stream);

/*
 * ---- Attention features of the scoring model (Appendix B.1) ----
 *
 * Beside k and v the scorer sees, for every retained pair and every query head of its group, six sums of
 * the attention weights the pair received: over the last 8, 16 and 32 queries of the current chunk of L
 * steps, over the whole chunk so far (wL), and the sums carried over the earlier chunks, plain (cum)
 * and decayed by 0.9 per chunk (dec).  Device state, owned by the caller, zero-filled at the start:
 *   feat [batch][n_kv_heads][6][capacity][GP] fp32, GP = 4 if g <= 4 else 8 (heads >= g hold zeros),
 *   planes in the order w8, w16, w32, wL, cum, dec; cum and dec hold the state BEFORE the current chunk.
 * The scorer's feature vector of a pair is a[head * 6 + plane] with cum + wL and 0.9 dec + wL in the
 * last two planes, so W1 has 2 * head_dim + 6 g rows: k, v, then a.
 */

/* Bytes of workspace fk_decode_step_feat needs (0 on bad args); no initialisation required. */
size_t fk_decode_step_feat_workspace(const fk_cache_desc *desc);

/*
 * fk_decode_step that also accounts the step's attention weights (softmax over the retained set
 * including the new pair, fp32 weights from the unrounded exponentials) in `feat`: the slot of the
 * new pair restarts all six planes from zero, then every live slot i gains p[hq][i] in wL and in each
 * window plane w with chunk_pos >= chunk_len - w.  chunk_pos = 0 .. chunk_len - 1 counts the steps since
 * the last eviction event, chunk_len = L.  One launch, one workgroup per row.  The workspace holds the
 * step's logits; calls sharing it must not overlap in time.
 */
fk_status fk_decode_step_feat(const fk_cache_desc *desc, const void *q, void *K, void *V, int32_t *pos,
                              int32_t *len, const void *k_new, const void *v_new,
                              const int32_t *pos_new, int32_t max_len, float softmax_scale, float *feat,
                              int32_t chunk_pos, int32_t chunk_len, void *out, void *workspace,
                              size_t workspace_bytes, void *stream);

/*
 * Appendix B.1 (the queries of one chunk): n_steps consecutive fk_decode_step_feat calls enqueued by one
 * call, step t at chunk position chunk_pos_first + t, on q_seq[t], k_seq[t], v_seq[t], pos_seq[t] with its
 * output in out_seq[t] and max_len = min(max_len_first + t, capacity).  Layouts as for fk_decode_window;
 * the window must end inside the chunk (chunk_pos_first + n_steps <= chunk_len).  Results are those of
 * the n_steps single calls.
 */
fk_status fk_decode_window_feat(const fk_cache_desc *desc, const void *q_seq, void *K, void *V, int32_t *pos,
                                int32_t *len, const void *k_seq, const void *v_seq, const int32_t *pos_seq,
                                int32_t n_steps, int32_t max_len_first, float softmax_scale, float *feat,
                                int32_t chunk_pos_first, int32_t chunk_len, void *out_seq, void *workspace,
                                size_t workspace_bytes, void *stream);

/*
 * fk_score_kv on x = concat(k, v, a) (Section 3.1 Eq. 1 with the attention features of Appendix
 * B.1).  scorer->w1 is [n_sets][2*head_dim + 6 g][hidden]; the fp32 features enter the contraction as
 * a bf16 head plus a bf16 remainder (16 significant bits; fp32 caches: plain fp32).  bf16: FK_ERR_UNSUPPORTED
 * unless hidden is a multiple of 8 and H' * (2*head_dim + roundup(6 g, 16) + 8) * 2 + 8 * H' <= 160 KiB (H' = hidden rounded up to 32).
 */
fk_status fk_score_kv_feat(const fk_cache_desc *desc, const void *K, const void *V, const float *feat,
                           const int32_t *len, int32_t max_len, const fk_scorer *scorer, float *scores,
                           void *stream);

/*
 * fk_compact that also closes the chunk of the features: for every row and live slot cum += wL,
 * dec = 0.9 dec + wL, the planes w8, w16, w32, wL restart from zero, and rows over budget move the
 * features of slot keep_idx[j] to slot j together with K, V and pos.  Other arguments and results as
 * fk_compact.
 */
fk_status fk_compact_feat(const fk_cache_desc *desc, void *K, void *V, int32_t *pos, float *feat,
                          int32_t *len, const int32_t *keep_idx, int32_t budget, void *stream);

/*
 * ---- Golden Eviction label builder (Section 3.2 Eq. 3-5; training-side, outside the decode loop) ----
 *
 * Input: the attention matrices of the query heads of one layer on a full trace of T tokens,
 *   A [n_q_heads][T][ld] dtype (fp32 or bf16), row = query position, column = key position (0-based),
 *   ld >= T elements per row with ld % 8 == 0; precondition A[h][q][i] == 0 for i > q (causal).
 * With budget B and eviction length L (L <= B) the queries from B + L on form M = ceil((T - B)/L) - 1
 * blocks; block t = 1 .. M holds queries B + tL .. min(B + (t+1)L, T) - 1, the last one counted as L
 * queries (zero padded).
 */

/* M for a trace of T tokens; -1 on bad arguments. */
int32_t fk_golden_steps(int32_t T, int32_t budget, int32_t interval);

/*
 * Eq. 3-4 and the first half of Eq. 5:
 *   block_scores[h'][t-1][i] = 1/(g L) sum_{h in group h'} sum_{q in block t} A[h][q][i]     (average pooling)
 *   alpha[h'][t-1][i]        = max_{t <= j <= M} block_scores[h'][j-1][i]                    (future score)
 * both [n_kv_heads][M][T] fp32, fp32 accumulation; nothing is written when M == 0.
 */
fk_status fk_golden_scores(const void *A, int32_t dtype, int32_t n_q_heads, int32_t n_kv_heads, int32_t T,
                           int64_t ld, int32_t budget, int32_t interval, float *block_scores,
                           float *alpha, void *stream);

/*
 * Second half of Eq. 5 as an eviction trace under the protocol of Section 3.1: before step 1 the cache
 * holds positions 0 .. B + L - 1; step t keeps the L newest (B + tL - L .. B + tL - 1) and, of the other B
 * it holds, the B - L with the largest alpha[h'][t-1][.] (ties: the lower position); then positions
 * B + tL .. B + (t+1)L - 1 join.  kept [n_kv_heads][M][B] int32: the positions retained after step t,
 * ascending.  -0 equals +0 and NaN ranks lowest, as in fk_select_keep.  B + L <= 12288
 * (FK_ERR_UNSUPPORTED above).
 */
fk_status fk_golden_trace(const float *alpha, int32_t n_kv_heads, int32_t T, int32_t budget,
                          int32_t interval, int32_t *kept, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* FK_H */
