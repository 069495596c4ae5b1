/*
 * h2o.h — C ABI of the MI355X (gfx950) H2O attention hot path.
 *
 * H2O ("Heavy-Hitter Oracle", arXiv 2306.14048) keeps a KV cache of fixed size
 * k = heavy + recent per attention head.  At every generation step the new
 * token attends to the k cached tokens and to itself (Definition 2.2: softmax
 * restricted to the tokens in the cache), the step's probabilities are added to
 * one accumulated score per cached token (Algorithm 2, accumulate line), and
 * the cached token with the smallest accumulated score outside the `recent`
 * most recent ones is evicted (Definition 4.3 with F_score = sum of accumulated
 * scores; budget split of Sec. 5.1 / App. A) and its storage is overwritten in
 * place by the new token's key/value (Sec. 4.2 "Implementation details": no
 * swap, fill directly).  The prompt phase seeds the scores with the column sums
 * of the prompt's causal softmax matrix and keeps `heavy` best + `recent` last
 * tokens (App. A, pseudocode commentary).  Heads are independent.
 *
 * Conventions
 *   - every pointer named dev/Q/K/V/q/k_new/v_new/out/colsum/acc/pos/workspace
 *     is a DEVICE pointer owned by the caller; the library never allocates or
 *     frees device memory and never synchronises: all work is enqueued on the
 *     `hip_stream` argument (a hipStream_t passed as void*, NULL = default
 *     stream) and the call returns at once;
 *   - the only thing the library owns is the small host-side handle
 *     `h2o_cache`, created by h2o_cache_init and released by h2o_cache_destroy;
 *   - device pointers must be 16-byte aligned;
 *   - layouts are contiguous, last index fastest:
 *       prompt  Q, K, V        [batch, heads, n, head_dim]     (cfg.dtype)
 *       step    q, k_new, v_new, out  [batch, heads, head_dim] (cfg.dtype)
 *       cache   K, V           [batch, heads, k, head_dim]     (cfg.dtype)
 *               acc            [batch, heads, k]  float  accumulated scores
 *               pos            [batch, heads, k]  int32  token position held
 *                                                  by the slot, -1 = free
 *     Which slot holds which token is an implementation detail: only the set
 *     of positions is meaningful.
 *     With cfg.kv_bits = 4 the cached K and V are stored as 4-bit codes instead
 *     (see h2o_config); everything the caller passes in stays in cfg.dtype.
 *   - positions count tokens from 0; `t` = number of tokens seen so far is the
 *     same for all heads (prompts are padded to one length, Sec. 5.3) and is
 *     tracked on the host handle;
 *   - every function returns an h2o_status (0 = success, negative = error);
 *     on error nothing has been enqueued unless stated otherwise.
 */
#ifndef H2O_H
#define H2O_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum h2o_status {
    H2O_OK = 0,
    H2O_EINVAL = -1,        /* null pointer, non-positive size, misaligned pointer */
    H2O_EUNSUPPORTED = -2,  /* head_dim not in {64, 128}, budget or prompt too large */
    H2O_ENOMEM = -3,        /* caller-provided buffer too small */
    H2O_ESTATE = -4,        /* call not legal in the cache's current state */
    H2O_EHIP = -5,          /* the HIP runtime reported an error */
    H2O_ESCRATCH = -6       /* request needs more than the library's built-in scratch */
} h2o_status;

typedef enum h2o_dtype { H2O_F32 = 0, H2O_F16 = 1, H2O_BF16 = 2 } h2o_dtype;

/* What ranks a cached token when one has to be evicted (and when the prompt is
 * compressed).  H2O_RANK_ACCUMULATED is the method (Algorithm 2: the accumulated
 * attention score).  H2O_RANK_AVERAGED divides that score by the number of
 * queries that have scored the token (its own included), the variant the paper
 * reports trying against the bias towards old tokens (App. B, "Previous
 * Attempts"); only the ranking changes, the stored scores stay accumulated. */
typedef enum h2o_rank { H2O_RANK_ACCUMULATED = 0, H2O_RANK_AVERAGED = 1 } h2o_rank;

/*
 * What the eviction may not touch.  H2O_PROTECT_RECENT is the method: the last
 * `recent` positions (Sec. 5.1 budget split, App. A).  The other two put a
 * sparse-attention pattern in the window's place, the combination the paper
 * evaluates in Sec. 5.2 ("Enhancing Baseline Techniques", Table 2) without giving
 * a rule; the reading taken: the positions the pattern lets the current query (at
 * position t) attend to are protected, every other cached token competes on its
 * score as before.  For a token at position p:
 *     H2O_PROTECT_STRIDED  t - p < recent  or  (t - p) mod stride == 0
 *     H2O_PROTECT_FIXED    p div stride == t div stride  or  p mod stride >= stride - recent
 * (`recent` is then the width of the local band / the number of summary columns
 * per block; the cache still holds heavy + recent tokens).  If the pattern covers
 * every cached token, protection is void for that eviction: the smallest
 * (rank value, position) among the cached tokens goes (the new token itself is
 * always kept in these two modes).  The prompt compression evicts by the same
 * rule, one token at a time with the last prompt token as the query: it keeps
 * what the pattern covers plus the best of the rest up to the budget, or, if the
 * pattern covers more than the budget, the best of what it covers.
 */
typedef enum h2o_protect {
    H2O_PROTECT_RECENT = 0, H2O_PROTECT_STRIDED = 1, H2O_PROTECT_FIXED = 2
} h2o_protect;

/* Largest supported budget (heavy + recent) and prompt length. */
#define H2O_MAX_BUDGET 4096
#define H2O_MAX_PROMPT 65536

/*
 * 4-bit cache storage (Sec. 5.4, "compatible with quantization"; App. on the
 * throughput of H2O combined with quantisation).  The paper names the
 * group-wise min-max quantiser of the serving system it builds on and prints
 * no formula; the published one is used.  Along head_dim, per group of
 * H2O_Q4_GROUP consecutive elements of a row:
 *     mn = min, mx = max, scale = (mx - mn) / 15,
 *     code_i = clamp(round_half_even((x_i - mn) / scale), 0, 15)   (scale = 0: 0),
 *     stored value = mn + code_i * scale,
 * every operation being one binary32 operation.  A row is quantised when it
 * enters the cache: the rows kept by the prompt compression, and the new token
 * after its own generation step (in that step it attends to itself with its
 * unquantised key and value).  Scores, ranking and eviction are unchanged.
 * A stored K (or V) row is head_dim/2 bytes of codes (element e in bits
 * 4*(e%8) .. 4*(e%8)+3 of the little-endian 32-bit word e/8) followed by
 * head_dim/64 pairs of floats (scale, min), padded to a multiple of 16 bytes:
 * H2O_Q4_ROW_BYTES(head_dim) = 80 for 128, 48 for 64 (against 256 and 128 bytes
 * of a 16-bit row).  Limits: heavy + recent <= H2O_Q4_MAX_BUDGET; no chunked
 * prompt processing (h2o_prefill_chunk) on such a cache.
 */
#define H2O_Q4_GROUP 64
#define H2O_Q4_ROW_BYTES(head_dim) ((head_dim) / 2 + 16)
#define H2O_Q4_MAX_BUDGET 2048

typedef struct h2o_config {
    int32_t batch;      /* B  >= 1 */
    int32_t heads;      /* Hh >= 1 */
    int32_t head_dim;   /* d: 64 or 128 */
    int32_t heavy;      /* H >= 0, heavy-hitter share of the budget */
    int32_t recent;     /* R >= 0, recent-window share; H + R >= 1 */
    int32_t dtype;      /* h2o_dtype of Q/K/V/q/k/v/out and of the cached K/V */
    float scale;        /* logit scale; 0 selects 1/sqrt(head_dim) */
    int32_t rank;       /* h2o_rank; 0 = the method's accumulated score */
    int32_t kv_bits;    /* cached K/V storage: 0 = elements of `dtype`, 4 = 4-bit codes */
    int32_t protect;    /* h2o_protect; 0 = the method's recent window */
    int32_t stride;     /* period of the strided / fixed pattern (>= 1); ignored for protect = 0 */
} h2o_config;

typedef struct h2o_cache h2o_cache;   /* opaque host-side handle */

/* Device bytes needed for one cache: K | V | acc | pos, each 256-byte aligned.
 * Returns 0 for an invalid configuration. */
size_t h2o_cache_bytes(const h2o_config *cfg);

/* Device bytes of scratch the prompt phase needs for a prompt of n tokens
 * (row log-sum-exps and column sums, float [batch, heads, n] each).
 * Returns 0 for invalid arguments. */
size_t h2o_prefill_workspace_bytes(const h2o_config *cfg, int32_t n);

/*
 * Creates a handle over caller-owned device memory `dev_mem` of `bytes` bytes
 * (>= h2o_cache_bytes) and enqueues the fill that marks every slot free
 * (pos = -1, acc = 0).  The cache starts empty with t = 0.
 * This is the fixed-size, preallocated cache of App. A ("implementation details":
 * the storage is allocated once at k = heavy + recent entries per head and never
 * grows or moves; an evicted entry is overwritten in place, Sec. 4.2).
 * Errors: EINVAL, EUNSUPPORTED, ENOMEM (bytes too small), EHIP.
 */
int h2o_cache_init(const h2o_config *cfg, void *dev_mem, size_t bytes,
                   void *hip_stream, h2o_cache **out);

/* Marks every slot free again and sets t = 0 (enqueued on the stream). */
int h2o_cache_reset(h2o_cache *cache, void *hip_stream);

/* Releases the host handle only (device memory stays the caller's). */
void h2o_cache_destroy(h2o_cache *cache);

/*
 * Prompt scoring (exact generative process, App. D "Eviction policy"; scores as
 * in Algorithm 2's accumulate line): for every head
 *     S_ij = scale * <Q_i, K_j>  (j <= i),   P = row-softmax(S),
 *     colsum_j = sum_{i >= j} P_ij.
 * Two MFMA passes: row log-sum-exp, then exp(S - LSE) reduced over rows.
 *   Q, K        [batch, heads, n, head_dim] in cfg->dtype
 *   workspace   >= h2o_prefill_workspace_bytes(cfg, n)
 *   colsum_out  float [batch, heads, n]
 * Needs no cache.  Errors: EINVAL, EUNSUPPORTED (n > H2O_MAX_PROMPT), ENOMEM, EHIP.
 */
int h2o_prefill_colsum(const h2o_config *cfg, const void *Q, const void *K,
                       int32_t n, void *workspace, size_t ws_bytes,
                       float *colsum_out, void *hip_stream);

/*
 * Prompt compression (App. A: keep K heavy hitters and K recent tokens, or all
 * tokens if the prompt is not longer than that): given a score per prompt token, keep the last
 * `recent` tokens and the `heavy` highest-scoring older ones (all n tokens if
 * n <= heavy + recent; equal scores: the higher position is kept; with
 * H2O_RANK_AVERAGED the older tokens are ranked by score[j] / (n - j)), copy their
 * K/V rows into slots in ascending position order, set acc/pos, mark the rest
 * free, and set t = n.  The cache must be empty (fresh or reset).
 * The compression itself orders any finite scores correctly (negative ones and
 * signed zeros included); generation steps that follow need them non-negative.
 *   K, V    [batch, heads, n, head_dim];   score  float [batch, heads, n]
 * Errors: EINVAL, EUNSUPPORTED, ESTATE (cache not empty), EHIP.
 */
int h2o_prefill_select(h2o_cache *cache, const void *K, const void *V,
                       const float *score, int32_t n, void *hip_stream);

/*
 * The whole prompt phase: h2o_prefill_colsum followed by h2o_prefill_select on
 * the sums.  `colsum_out` (nullable) additionally receives the column sums.
 * Q is only used for scoring; V only for the copy into the cache.
 */
int h2o_prefill_scores(h2o_cache *cache, const void *Q, const void *K,
                       const void *V, int32_t n, void *workspace,
                       size_t ws_bytes, float *colsum_out, void *hip_stream);

/*
 * h2o_prefill_scores for callers that cannot allocate or bring a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid allocation.
 * Same arguments minus the workspace, same results; the row statistics and column
 * sums live in a fixed array of H2O_NOALLOC_SCRATCH_BYTES bytes inside the
 * library's device image (one copy per GPU, held until the process ends), so the
 * call allocates nothing, on the device or through any library.
 *   limit   h2o_prefill_workspace_bytes(cfg, n) <= H2O_NOALLOC_SCRATCH_BYTES, i.e.
 *           batch * heads * n <= 2 097 152 (rounded to 256 bytes per array);
 *           beyond it the call returns H2O_ESCRATCH and enqueues nothing
 *   sharing every call on a GPU uses that GPU's one array: calls that overlap in
 *           time on one GPU (different streams) race; calls on one stream do not.
 *           The array keeps the previous call's contents; nothing in it needs to
 *           start at zero.
 * The device current at the call must be the one the cache lives on (as for every
 * entry point that launches).  Errors: as h2o_prefill_scores, and ESCRATCH.
 */
#define H2O_NOALLOC_SCRATCH_BYTES (16u << 20)
int h2o_prefill_scores_noalloc(h2o_cache *cache, const void *Q, const void *K,
                               const void *V, int32_t n, float *colsum_out,
                               void *hip_stream);

/* Device bytes of scratch h2o_prefill_chunk needs for chunks of up to m tokens
 * (cache + chunk as one candidate list: K and V rows, old scores, positions,
 * column sums, row statistics, slot order; with_output != 0: also the transposed
 * V the attention output needs).  Returns 0 for invalid arguments, when heavy + recent
 * + m exceeds H2O_MAX_PROMPT, and for with_output on a binary32 configuration. */
size_t h2o_prefill_chunk_workspace_bytes(const h2o_config *cfg, int32_t m, int32_t with_output);

/*
 * The next m prompt tokens as one chunk: prompt processing with bounded memory.
 * The paper gives the two ends of the range: token-by-token eviction over the
 * whole sequence (Algorithm 1) and full attention over the prompt followed by
 * one compression (App. A).  Here every token of the chunk attends to the
 * tokens in the cache and, causally, to the chunk's own tokens (nothing is
 * evicted inside a chunk); the column sums of these m softmax rows are added to
 * the accumulated scores (Algorithm 2's accumulate line; binary32 add of the
 * binary32 column sum); then cache + chunk are compressed to the budget by the
 * prompt rule of h2o_prefill_select (last `recent` positions, `heavy` best older
 * ones).  m = 1 is the update h2o_decode_step makes to the cache; one
 * chunk holding the whole prompt on an empty cache is h2o_prefill_scores.
 *   Q, K, V   [batch, heads, m, head_dim] in cfg.dtype
 *   workspace >= h2o_prefill_chunk_workspace_bytes(cfg, m, out != NULL)
 *   out       NULL, or [batch, heads, m, head_dim] in cfg.dtype: the attention
 *             output of the chunk's tokens (sum over cached and chunk tokens of
 *             probability times value), which makes the call a layer's complete
 *             attention for the chunk; 16-bit element types only
 * May follow generation steps (a further prompt after some generated tokens):
 * the cached tokens are taken in position order whichever slots they sit in;
 * afterwards they sit in slots in ascending position order.
 * Then t becomes t + m.  Errors: EINVAL, EUNSUPPORTED (4-bit cache; out on a
 * binary32 configuration), ENOMEM, EHIP.
 */
int h2o_prefill_chunk(h2o_cache *cache, const void *Q, const void *K, const void *V,
                      int32_t m, void *workspace, size_t ws_bytes, void *out, void *hip_stream);

/*
 * Device bytes of scratch h2o_prefill_attention / h2o_prefill_attention_scores
 * need for a prompt of n tokens (a transposed copy of V padded to whole tiles,
 * then the scratch of h2o_prefill_workspace_bytes).  Returns 0 for invalid
 * arguments and for H2O_F32 (16-bit element types only).
 */
size_t h2o_prefill_attention_workspace_bytes(const h2o_config *cfg, int32_t n);

/*
 * Attention over the prompt (the prompt phase runs with the full cache, App. A
 * generation commentary; exact process of App. D): for every head
 *     out_i = sum_{j <= i} softmax_j(scale * <Q_i, K_j>) V_j,
 * one flash-style MFMA kernel (online softmax, fp32 accumulation, the
 * probabilities rounded to cfg->dtype for the second product).  The row
 * log-sum-exps it produces are what the column-sum pass needs, so a layer that
 * calls this gets the H2O scores for one extra matrix pass
 * (h2o_prefill_attention_scores) instead of two.
 *   Q, K, V   [batch, heads, n, head_dim] in cfg->dtype (H2O_F16 or H2O_BF16)
 *   out       [batch, heads, n, head_dim] in cfg->dtype
 *   lse_out   nullable, float [batch, heads, n]: log sum_j exp(scale * <Q_i, K_j>)
 *   workspace >= h2o_prefill_attention_workspace_bytes(cfg, n)
 * Needs no cache.  Errors: EINVAL, EUNSUPPORTED (H2O_F32, n > H2O_MAX_PROMPT),
 * ENOMEM, EHIP.
 */
int h2o_prefill_attention(const h2o_config *cfg, const void *Q, const void *K,
                          const void *V, int32_t n, void *workspace,
                          size_t ws_bytes, void *out, float *lse_out,
                          void *hip_stream);

/*
 * The whole prompt phase of an H2O attention layer: h2o_prefill_attention, the
 * column sums of the same softmax matrix from its row statistics (Algorithm 2's
 * accumulate line over the prompt rows), and h2o_prefill_select on the sums.
 * `colsum_out` (nullable) additionally receives the column sums.  The cache
 * must be empty.  Errors: those of the three calls.
 */
int h2o_prefill_attention_scores(h2o_cache *cache, const void *Q, const void *K,
                                 const void *V, int32_t n, void *workspace,
                                 size_t ws_bytes, void *out, float *colsum_out,
                                 void *hip_stream);

/*
 * One generation step for the token at position t, one fused kernel launch
 * (Definition 2.2, Algorithm 2, App. A decode commentary), per head:
 *   1. logits  s_j = scale * <q, K[slot j]> for every occupied slot, and
 *      s_self = scale * <q, k_new>;
 *   2. p = softmax over the occupied slots and the token itself;
 *   3. out = sum_j p_j V[slot j] + p_self * v_new;
 *   4. acc[j] += p_j (binary32 add of the binary32-rounded probability);
 *   5. if a slot is free the new token takes the lowest-indexed free slot;
 *      otherwise the occupied slot with the smallest (rank value, pos) among
 *      those with pos <= t - recent (for the pattern modes of h2o_protect: among
 *      those the pattern does not cover) is evicted, the rank value being acc or,
 *      for H2O_RANK_AVERAGED, the binary32 quotient acc / (t - pos + 1) (with recent == 0 the new token,
 *      scored p_self, competes and may itself be dropped);
 *   6. the chosen slot gets K = k_new, V = v_new, acc = p_self, pos = t.
 * Then t becomes t + 1.  The cache is read exactly once.
 * The position t and the number of occupied slots min(t, k) are tracked on the
 * host handle and passed to the kernel as launch arguments (they are the same
 * for all heads).  A captured HIP graph therefore replays exactly the steps it
 * captured, at the positions they had at capture: replaying it makes sense from
 * the same starting state only (e.g. reset + prompt + steps captured together);
 * it cannot be replayed to generate further tokens.
 * Errors: EINVAL, EHIP.
 */
int h2o_decode_step(h2o_cache *cache, const void *q, const void *k_new,
                    const void *v_new, void *out, void *hip_stream);

/* Copies pos / acc (each [batch, heads, k], device pointers, either may be
 * NULL) out of the cache, ordered after earlier work on the stream. */
int h2o_cache_snapshot(const h2o_cache *cache, int32_t *pos_out, float *acc_out,
                       void *hip_stream);

/*
 * Loads a complete cache state (checkpoint restore; also how tests start a
 * generation from a state computed elsewhere): K, V [batch, heads, k, head_dim]
 * (with kv_bits = 4: [batch, heads, k, H2O_Q4_ROW_BYTES] bytes in the stored
 * layout), acc, pos [batch, heads, k] are copied in and t is set to `tokens_seen`.
 * Requirements on the state, for every head (what the library's own calls leave
 * behind, and what every later call relies on without checking):
 *   - the occupied slots are exactly the prefix [0, min(tokens_seen, k)): slots
 *     fill in index order and are only ever overwritten in place, so a hole
 *     (pos = -1 below that bound) or an occupied slot above it cannot arise, and
 *     a step would attend to whatever the hole's rows hold;
 *   - every other slot has pos = -1;
 *   - occupied positions lie in [0, tokens_seen) and are distinct;
 *   - scores are finite and not negative (they are sums of probabilities; the
 *     eviction order of later steps is only defined for such values).
 * None of this is checked here (the data is on the device and the call does not
 * synchronise); h2o_cache_validate checks all of it on the device.
 * Errors: EINVAL, EHIP.
 */
int h2o_cache_restore(h2o_cache *cache, const void *K, const void *V,
                      const float *acc, const int32_t *pos,
                      int32_t tokens_seen, void *hip_stream);

/*
 * Checks the bookkeeping of every head against the requirements listed at
 * h2o_cache_restore (one small kernel, enqueued on the stream): flags_out
 * [batch, heads] (device, int32) receives 0 for a consistent head, else the sum of
 *     H2O_BAD_HOLE       1  a free slot below min(t, k)
 *     H2O_BAD_BEYOND     2  an occupied slot from min(t, k) on
 *     H2O_BAD_RANGE      4  a position outside [0, t)
 *     H2O_BAD_DUPLICATE  8  one position in two slots
 *     H2O_BAD_SCORE     16  a negative, infinite or NaN score
 * The caller reads the flags after synchronising (the Python binding's
 * H2OCache.restore(validate=True) does, and raises).  Intended after
 * h2o_cache_restore of a state from outside; states the library produced
 * itself pass.  Errors: EINVAL, EHIP.
 */
#define H2O_BAD_HOLE 1
#define H2O_BAD_BEYOND 2
#define H2O_BAD_RANGE 4
#define H2O_BAD_DUPLICATE 8
#define H2O_BAD_SCORE 16
int h2o_cache_validate(const h2o_cache *cache, int32_t *flags_out, void *hip_stream);

/*
 * Positions "rolled" into the cache (Sec. 5.4 Q1 and the appendix comparing with
 * StreamingLLM: inputs of unbounded length are handled with positions assigned
 * inside the cache instead of positions in the text): rolled_out[batch, heads, k]
 * (device, int32) receives for every occupied slot the rank of its token among
 * the head's cached tokens in position order (0 = oldest), -1 for a free slot.
 * What is done with them (positional encodings) lies outside this library.
 * Errors: EINVAL, EHIP.
 */
int h2o_cache_rolled_positions(const h2o_cache *cache, int32_t *rolled_out, void *hip_stream);

/* Number of tokens seen so far (prompt length + steps), or H2O_EINVAL. */
int h2o_cache_tokens_seen(const h2o_cache *cache);

/* Device addresses of the cache's four regions inside the caller's memory
 * (any output pointer may be NULL). */
int h2o_cache_regions(const h2o_cache *cache, void **K, void **V, float **acc,
                      int32_t **pos);

/* Static description of a status code. */
const char *h2o_status_str(int status);

#ifdef __cplusplus
}
#endif
#endif /* H2O_H */
