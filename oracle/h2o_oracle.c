/*
 * CPU oracle for the H2O (Heavy-Hitter Oracle) attention path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, fp64 statement of
 * what the method computes.  It shares no code with the HIP library, is never
 * linked into it and is never called by it; only the test-suite, the smoke
 * check and the benchmark's cpu_baseline leg use it.
 *
 * One object models ONE head (one (batch, head) pair); heads are independent
 * (the paper keeps/evicts per head and per layer, related-work comparison with
 * cross-head accumulation).  The object is position-indexed: it remembers every
 * token's key/value ever seen, a resident flag per position and one accumulated
 * score per position.  There are no slots and nothing is ever compacted, so a
 * reader can check each step against the paper by eye:
 *
 *   prefill  : exact / full-knowledge generative process (Sec. "Eviction
 *              Policy", definition "generative process with full knowledge"):
 *              o_i = softmax over K_{<=i}; accumulated scores are the column
 *              sums of those rows (Algorithm 2, the accumulate line); then the
 *              one-shot compression of App. A "System details/Pseudocode":
 *              keep `recent` last tokens plus the `heavy` best-scoring older
 *              ones, or everything if the prompt fits in the budget.
 *   decode   : Definition 2.2 (generative process with eviction policy):
 *              softmax restricted to the resident set (the "minus indicator"
 *              term removes exp(0) of the zeroed rows), with the new token
 *              attending to itself as in the exact process (o_{1,1} = 1);
 *              Algorithm 2: accumulate, then evict
 *              u = argmax_v F_score(G \ {v}), F_score = sum of accumulated
 *              scores, i.e. the member with the smallest accumulated score,
 *              restricted to tokens outside the recent window (Sec. 5.1
 *              budget split, App. A).
 *
 * Readings taken where the paper is silent (all restated in the design notes):
 *   - logits are scale * <q, k>; the paper's exp(QK^T) is scale = 1;
 *   - after the step for position t the recent window is {t-R+1..t}
 *     (it contains the new token); eviction candidates are resident
 *     positions <= t-R; with R = 0 the new token is itself a candidate;
 *   - ties: the smallest (score, position) pair is evicted;
 *   - while fewer than `budget` tokens are stored nothing is evicted;
 *   - `score_f32` != 0: accumulated scores are STORED in binary32 (the
 *     precision the workload definitions give for scores): each step's
 *     probability is rounded to binary32 and added in binary32; prefill column
 *     sums are accumulated in fp64 and rounded once when stored.  With
 *     `score_f32` == 0 everything stays fp64.  All other arithmetic is fp64.
 *
 *   - `policy` 1 (h2o_oracle_set_policy) ranks tokens by the AVERAGED score
 *     instead of the accumulated one: accumulated score divided by the number
 *     of queries that have scored the token (the variant App. B "Previous
 *     Attempts" reports trying against the bias towards old tokens).  Only the
 *     ranking changes; the stored scores stay the accumulated ones.  In
 *     `score_f32` mode the quotient is a binary32 division.
 *
 *   - chunked prompt processing (h2o_oracle_prefill_chunk): the paper gives the
 *     two ends, token-by-token eviction over the whole sequence (Algorithm 1)
 *     and one-shot compression after full attention over the prompt (App. A).
 *     A chunk of m tokens is the step in between: every token of the chunk
 *     attends to the tokens in the cache and, causally, to the chunk's own
 *     tokens (nothing is evicted inside a chunk); the chunk's probabilities
 *     are added to the scores (Algorithm 2's accumulate line); then cache plus
 *     chunk is compressed by the prompt rule.  m = 1 is the generation step,
 *     one chunk holding the whole prompt is the one-shot prompt phase.
 *
 *   - `kv_bits` 4 (h2o_oracle_set_kv_bits): cached keys and values are STORED
 *     as group-wise 4-bit codes (Sec. 5.4 "compatible with quantization",
 *     App. "Throughput improvement ... combining with quantization": the
 *     group-wise min-max quantisation of the serving system the paper builds
 *     on; the paper gives no formula, this is the published one).  Along the
 *     head dimension, per group of g consecutive elements:
 *         mn = min, mx = max, scale = (mx - mn) / 15,
 *         code_i = clamp(round_half_even((x_i - mn) / scale), 0, 15),
 *         stored value = mn + code_i * scale      (scale = 0: code 0, value mn).
 *     The code decision is an integer decided by floating point, so its
 *     precision is fixed: every operation above is one binary32 operation on
 *     binary32 inputs (cache element types convert exactly).  A row is
 *     quantised when it ENTERS the cache: the kept rows after a prompt phase,
 *     and the new token after its own generation step, in which it still
 *     attends to itself with its unquantised key and value.  Scores and
 *     eviction are untouched.  Chunked prompt processing is not defined with
 *     quantised storage here (returns -1).
 *
 *   - `protect` 1 / 2 (h2o_oracle_set_protect): what the eviction may not touch
 *     is given by a sparse-attention pattern instead of "the last `recent`
 *     positions" (Sec. 5.2 "Enhancing Baseline Techniques", Table 2: strided and
 *     fixed Sparse Transformer patterns combined with heavy hitters).  The
 *     paper prints accuracies only and no rule; the reading taken: the
 *     positions the pattern lets the current query attend to are PROTECTED,
 *     everything else in the cache competes on its accumulated score as
 *     before.  With the query at position t and a token at position p:
 *         strided: t - p < recent   or   (t - p) mod stride == 0
 *         fixed:   p div stride == t div stride   or   p mod stride >= stride - recent
 *     (`recent` is the width of the local band / of a block's summary
 *     columns).  If the pattern covers every cached token, protection is void
 *     for that eviction: the smallest (score, position) among all cached
 *     tokens other than the new one goes.  The cache size stays heavy + recent.
 *     The prompt phase evicts one token at a time by the same rule, with the
 *     last prompt token as the query, until the budget is met.
 *
 * Pins (tests/test_oracle_pins.py): brute-force set-function evaluation on tiny
 * inputs, reduction to textbook causal softmax attention when the budget
 * covers the sequence, harmonic-number closed form for equal logits, sliding
 * window for heavy = 0, mass conservation, set-size/window invariants.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct h2o_oracle {
    int d;              /* head dimension */
    int heavy;          /* H: heavy-hitter part of the budget */
    int recent;         /* R: recent-window part of the budget */
    int budget;         /* k = H + R */
    double scale;       /* logit scale */
    int score_f32;      /* store accumulated scores in binary32 */
    int policy;         /* 0: rank by accumulated score, 1: by averaged score */
    int protect;        /* 0: last `recent` positions, 1: strided pattern, 2: fixed pattern */
    int stride;         /* period of the strided / fixed pattern */
    int cap;            /* maximum number of tokens this object can see */
    int t;              /* tokens seen so far == position of the next token */
    int n_resident;
    double *K;          /* [cap][d] every key ever seen */
    double *V;          /* [cap][d] every value ever seen */
    double *acc;        /* [cap] accumulated attention score per position */
    unsigned char *resident; /* [cap] 1 if the token is in the cache */
    double evicted_mass;     /* sum of acc[] over evicted tokens at eviction time */
    double queries;          /* number of softmax rows accumulated so far */
    double *s;          /* [cap] scratch: logits */
    double *p;          /* [cap] scratch: probabilities */
    int kv_bits;        /* 0: rows stored as given; 4: group-wise 4-bit codes */
    int group;          /* elements per quantisation group */
    unsigned char *quantised; /* [cap] row has been replaced by its stored value */
    unsigned char *Kcode, *Vcode;   /* [cap][d] codes 0..15 */
    float *Kpar, *Vpar;             /* [cap][d/group][2] (scale, min) */
} h2o_oracle;

h2o_oracle *h2o_oracle_new(int d, int heavy, int recent, double scale,
                           int score_f32, int cap)
{
    if (d <= 0 || heavy < 0 || recent < 0 || heavy + recent < 1 || cap <= 0)
        return NULL;
    h2o_oracle *o = (h2o_oracle *)calloc(1, sizeof(*o));
    if (!o) return NULL;
    o->d = d; o->heavy = heavy; o->recent = recent; o->budget = heavy + recent;
    o->scale = scale; o->score_f32 = score_f32; o->cap = cap;
    o->K = (double *)calloc((size_t)cap * d, sizeof(double));
    o->V = (double *)calloc((size_t)cap * d, sizeof(double));
    o->acc = (double *)calloc(cap, sizeof(double));
    o->resident = (unsigned char *)calloc(cap, 1);
    o->s = (double *)calloc(cap, sizeof(double));
    o->p = (double *)calloc(cap, sizeof(double));
    if (!o->K || !o->V || !o->acc || !o->resident || !o->s || !o->p) {
        free(o->K); free(o->V); free(o->acc); free(o->resident);
        free(o->s); free(o->p); free(o);
        return NULL;
    }
    return o;
}

void h2o_oracle_free(h2o_oracle *o)
{
    if (!o) return;
    free(o->K); free(o->V); free(o->acc); free(o->resident);
    free(o->s); free(o->p);
    free(o->quantised); free(o->Kcode); free(o->Vcode); free(o->Kpar); free(o->Vpar);
    free(o);
}

/* Store cached rows as 4-bit codes in groups of `group` elements (bits = 4), or
 * as given (bits = 0).  Only on an object that has seen no token. */
int h2o_oracle_set_kv_bits(h2o_oracle *o, int bits, int group)
{
    if (!o || o->t != 0 || (bits != 0 && bits != 4)) return -1;
    if (bits == 4 && (group < 1 || o->d % group != 0)) return -1;
    o->kv_bits = bits;
    if (bits == 0) return 0;
    o->group = group;
    const size_t cap = (size_t)o->cap, ng = (size_t)(o->d / group);
    if (!o->quantised) {
        o->quantised = (unsigned char *)calloc(cap, 1);
        o->Kcode = (unsigned char *)calloc(cap * o->d, 1);
        o->Vcode = (unsigned char *)calloc(cap * o->d, 1);
        o->Kpar = (float *)calloc(cap * ng * 2, sizeof(float));
        o->Vpar = (float *)calloc(cap * ng * 2, sizeof(float));
    }
    return (o->quantised && o->Kcode && o->Vcode && o->Kpar && o->Vpar) ? 0 : -1;
}

/* One group of g elements: codes, (scale, min), and the stored values written
 * back over x.  Every step is a single binary32 operation (the volatiles keep
 * the compiler from contracting or widening them). */
static void quantise_group(double *x, int g, unsigned char *code, float *par)
{
    volatile float mn = (float)x[0], mx = (float)x[0];
    for (int i = 1; i < g; ++i) {
        const float v = (float)x[i];
        if (v < mn) mn = v;
        if (v > mx) mx = v;
    }
    volatile float range = mx - mn;
    volatile float scale = range / 15.0f;
    par[0] = scale; par[1] = mn;
    for (int i = 0; i < g; ++i) {
        float c = 0.0f;
        if (scale > 0.0f) {
            volatile float dist = (float)x[i] - mn;
            volatile float steps = dist / scale;
            c = rintf(steps);                 /* default rounding mode: half to even */
            if (c < 0.0f) c = 0.0f;
            if (c > 15.0f) c = 15.0f;
        }
        code[i] = (unsigned char)c;
        x[i] = (double)mn + (double)c * (double)scale;
    }
}

/* Replace the key and value rows of `pos` by what the quantised cache holds. */
static void store_row(h2o_oracle *o, int pos)
{
    if (o->kv_bits != 4 || o->quantised[pos]) return;
    const int d = o->d, g = o->group, ng = d / g;
    for (int b = 0; b < ng; ++b) {
        const size_t e = (size_t)pos * d + (size_t)b * g, q = ((size_t)pos * ng + b) * 2;
        quantise_group(o->K + e, g, o->Kcode + e, o->Kpar + q);
        quantise_group(o->V + e, g, o->Vcode + e, o->Vpar + q);
    }
    o->quantised[pos] = 1;
}

static void store_resident_rows(h2o_oracle *o, int first, int end)
{
    for (int j = first; j < end; ++j)
        if (o->resident[j]) store_row(o, j);
}

/* Add one probability to a stored score, in the storage precision. */
static double add_score(const h2o_oracle *o, double stored, double prob)
{
    if (o->score_f32) {
        volatile float a = (float)stored;
        volatile float b = (float)prob;
        volatile float r = a + b;
        return (double)r;
    }
    return stored + prob;
}

static double dot(const double *a, const double *b, int d)
{
    double acc = 0.0;
    for (int c = 0; c < d; ++c) acc += a[c] * b[c];
    return acc;
}

/* Select what ranks a token for eviction (0 accumulated, 1 averaged score). */
int h2o_oracle_set_policy(h2o_oracle *o, int policy)
{
    if (!o || (policy != 0 && policy != 1)) return -1;
    o->policy = policy;
    return 0;
}

/* The value that ranks position `pos` once the query at position `last_q` has
 * been accumulated: its accumulated score, or that score divided by the
 * number of queries that have scored it (pos .. last_q, itself included). */
static double rank_score(const h2o_oracle *o, int pos, int last_q)
{
    if (o->policy == 0) return o->acc[pos];
    const double cnt = (double)(last_q - pos + 1);
    if (o->score_f32) {
        volatile float a = (float)o->acc[pos];
        volatile float c = (float)cnt;
        volatile float r = a / c;
        return (double)r;
    }
    return o->acc[pos] / cnt;
}

/* Is (score a, position pa) strictly before (score b, position pb) in the
 * eviction order: lower score first, equal scores -> lower position first. */
static int evict_before(double a, int pa, double b, int pb)
{
    return (a < b) || (a == b && pa < pb);
}

/* Select what the eviction may not touch (0 recent window, 1 strided, 2 fixed
 * sparse pattern of the given period). */
int h2o_oracle_set_protect(h2o_oracle *o, int mode, int stride)
{
    if (!o || mode < 0 || mode > 2 || (mode != 0 && stride < 1)) return -1;
    o->protect = mode;
    o->stride = mode ? stride : 0;
    return 0;
}

/* Does the protection rule cover the token at position p when the latest query
 * sits at position t (p <= t)? */
static int is_protected(const h2o_oracle *o, int p, int t)
{
    switch (o->protect) {
    case 1:  return (t - p) < o->recent || (t - p) % o->stride == 0;
    case 2:  return p / o->stride == t / o->stride || p % o->stride >= o->stride - o->recent;
    default: return p > t - o->recent;
    }
}

/*
 * Pattern-protected eviction of ONE token after the query at position last_q:
 * the smallest (rank value, position) among the cached tokens the pattern does
 * not cover; if it covers them all, among all cached tokens except `exempt`
 * (the token that has just arrived; -1: nobody).  Reports the number of
 * candidates and the two lowest rank values like the generation step does.
 */
static int evict_one_protected(h2o_oracle *o, int last_q, int exempt, int *n_cand,
                               double *lowest, double *second)
{
    int u = -1, cnt = 0;
    double lo = INFINITY, se = INFINITY;
    for (int pass = 0; pass < 2 && u < 0; ++pass) {
        cnt = 0;
        for (int j = 0; j <= last_q; ++j) {
            if (!o->resident[j]) continue;
            if (pass == 0 ? is_protected(o, j, last_q) : j == exempt) continue;
            ++cnt;
            const double rj = rank_score(o, j, last_q);
            if (u < 0 || evict_before(rj, j, lo, u)) { se = lo; lo = rj; u = j; }
            else if (rj < se) se = rj;
        }
    }
    if (u >= 0) {
        o->resident[u] = 0;
        o->evicted_mass += o->acc[u];
        --o->n_resident;
    }
    if (n_cand) *n_cand = cnt;
    if (lowest) *lowest = lo;
    if (second) *second = se;
    return u;
}

/*
 * One-shot compression of a prompt of n tokens whose scores are in acc[0..n):
 * if the prompt fits in the budget keep everything; otherwise keep the last
 * `recent` tokens and, among the older ones, evict the smallest
 * (score, position) repeatedly until `heavy` of them remain (App. A's prompt
 * rule: the best-scoring tokens plus the most recent ones are what the prompt
 * phase hands on; written as repeated single evictions so that it is the same
 * rule the generation steps use).
 */
static void compress_prompt(h2o_oracle *o, int n)
{
    for (int j = 0; j < n; ++j) o->resident[j] = 1;
    o->n_resident = n;
    o->t = n;
    if (n <= o->budget) return;
    if (o->protect != 0) {
        /* pattern-protected: one eviction at a time, the last prompt token is the query */
        while (o->n_resident > o->budget) evict_one_protected(o, n - 1, -1, NULL, NULL, NULL);
        return;
    }
    const int first_recent = n - o->recent;   /* window = [n-R, n) */
    int older = first_recent;                 /* resident tokens outside it */
    while (older > o->heavy) {
        int u = -1;
        for (int j = 0; j < first_recent; ++j) {
            if (!o->resident[j]) continue;
            if (u < 0 || evict_before(rank_score(o, j, n - 1), j, rank_score(o, u, n - 1), u)) u = j;
        }
        o->resident[u] = 0;
        o->evicted_mass += o->acc[u];
        --older; --o->n_resident;
    }
}

/*
 * Prompt phase.  Q, K, V are [n][d] row-major fp64.
 *   colsum_out (nullable, [n]): full column sums of the causal softmax matrix
 *       in fp64, before any rounding and before compression.
 *   attn_out   (nullable, [n][d]): row i = sum_j p_ij V_j (full attention).
 * Returns 0, or -1 on bad arguments / state (object must be empty).
 */
int h2o_oracle_prefill(h2o_oracle *o, const double *Q, const double *K,
                       const double *V, int n, double *colsum_out,
                       double *attn_out)
{
    if (!o || !Q || !K || !V || n <= 0 || n > o->cap || o->t != 0) return -1;
    const int d = o->d;
    memcpy(o->K, K, (size_t)n * d * sizeof(double));
    memcpy(o->V, V, (size_t)n * d * sizeof(double));
    for (int j = 0; j < n; ++j) o->acc[j] = 0.0;

    /* Full-knowledge process: row i attends to keys 0..i (itself included). */
    for (int i = 0; i < n; ++i) {
        const double *qi = Q + (size_t)i * d;
        double m = -INFINITY;
        for (int j = 0; j <= i; ++j) {
            o->s[j] = o->scale * dot(qi, K + (size_t)j * d, d);
            if (o->s[j] > m) m = o->s[j];
        }
        double D = 0.0;
        for (int j = 0; j <= i; ++j) { o->p[j] = exp(o->s[j] - m); D += o->p[j]; }
        for (int j = 0; j <= i; ++j) {
            o->p[j] /= D;
            o->acc[j] += o->p[j];               /* column sum, fp64 */
        }
        if (attn_out) {
            double *oi = attn_out + (size_t)i * d;
            for (int c = 0; c < d; ++c) oi[c] = 0.0;
            for (int j = 0; j <= i; ++j) {
                const double *vj = V + (size_t)j * d;
                for (int c = 0; c < d; ++c) oi[c] += o->p[j] * vj[c];
            }
        }
    }
    o->queries = (double)n;
    if (colsum_out) memcpy(colsum_out, o->acc, (size_t)n * sizeof(double));
    if (o->score_f32)
        for (int j = 0; j < n; ++j) o->acc[j] = (double)(float)o->acc[j];

    compress_prompt(o, n);
    store_resident_rows(o, 0, n);
    return 0;
}

/*
 * The next m prompt tokens as one chunk (positions t .. t+m-1).  Q, K, V are
 * [m][d].  Token t+i attends to the resident tokens and to the chunk's tokens
 * t .. t+i; the column sums of these m softmax rows are added to the stored
 * scores (in binary32 storage: each column's chunk sum is rounded to binary32
 * and added in binary32); all chunk tokens become resident; if more than
 * `budget` tokens are resident the `recent` last positions stay and, among the
 * older resident ones, the smallest (rank value, position) is evicted
 * repeatedly until `heavy` of them remain.
 *   colsum_out (nullable, [t+m]): the chunk's column sums in fp64 by POSITION
 *       (zero for positions that were not attended to)
 *   attn_out   (nullable, [m][d]): attention output of every chunk token
 * Returns 0, or -1 on bad arguments / capacity.
 */
int h2o_oracle_prefill_chunk(h2o_oracle *o, const double *Q, const double *K,
                             const double *V, int m, double *colsum_out,
                             double *attn_out)
{
    if (!o || !Q || !K || !V || m <= 0 || o->t + m > o->cap || o->kv_bits != 0) return -1;
    const int d = o->d, t0 = o->t, t1 = o->t + m;
    memcpy(o->K + (size_t)t0 * d, K, (size_t)m * d * sizeof(double));
    memcpy(o->V + (size_t)t0 * d, V, (size_t)m * d * sizeof(double));
    double *chunk = (double *)calloc((size_t)t1, sizeof(double));
    if (!chunk) return -1;
    for (int j = t0; j < t1; ++j) { o->acc[j] = 0.0; o->resident[j] = 0; }

    for (int i = 0; i < m; ++i) {
        const int pi = t0 + i;                    /* position of this query */
        const double *qi = Q + (size_t)i * d;
        /* visible: resident tokens (all older than the chunk) and chunk tokens <= pi */
        double mx = -INFINITY;
        for (int j = 0; j <= pi; ++j) {
            if (j < t0 && !o->resident[j]) continue;
            o->s[j] = o->scale * dot(qi, o->K + (size_t)j * d, d);
            if (o->s[j] > mx) mx = o->s[j];
        }
        double D = 0.0;
        for (int j = 0; j <= pi; ++j) {
            if (j < t0 && !o->resident[j]) continue;
            o->p[j] = exp(o->s[j] - mx); D += o->p[j];
        }
        if (attn_out) for (int c = 0; c < d; ++c) attn_out[(size_t)i * d + c] = 0.0;
        for (int j = 0; j <= pi; ++j) {
            if (j < t0 && !o->resident[j]) continue;
            o->p[j] /= D;
            chunk[j] += o->p[j];
            if (attn_out) {
                const double *vj = o->V + (size_t)j * d;
                for (int c = 0; c < d; ++c) attn_out[(size_t)i * d + c] += o->p[j] * vj[c];
            }
        }
    }
    o->queries += (double)m;
    if (colsum_out) memcpy(colsum_out, chunk, (size_t)t1 * sizeof(double));
    for (int j = 0; j < t1; ++j) {
        if (j < t0 && !o->resident[j]) continue;
        o->acc[j] = add_score(o, o->acc[j], chunk[j]);
    }
    free(chunk);
    for (int j = t0; j < t1; ++j) o->resident[j] = 1;
    o->n_resident += m;
    o->t = t1;

    if (o->protect != 0) {
        while (o->n_resident > o->budget) evict_one_protected(o, t1 - 1, -1, NULL, NULL, NULL);
    } else if (o->n_resident > o->budget) {
        const int first_recent = t1 - o->recent;  /* window = [t1-R, t1) */
        int older = 0;
        for (int j = 0; j < first_recent; ++j) older += o->resident[j];
        while (older > o->heavy) {
            int u = -1;
            for (int j = 0; j < first_recent; ++j) {
                if (!o->resident[j]) continue;
                if (u < 0 || evict_before(rank_score(o, j, t1 - 1), j, rank_score(o, u, t1 - 1), u)) u = j;
            }
            o->resident[u] = 0;
            o->evicted_mass += o->acc[u];
            --older; --o->n_resident;
        }
    }
    return 0;
}

/*
 * Same compression as the tail of h2o_oracle_prefill, but with externally
 * supplied scores: loads n tokens (K, V, score[j]) into an empty object and
 * keeps the recent window plus the `heavy` best older tokens.  `queries` is
 * the number of softmax rows the scores stand for (n after a prompt).
 */
int h2o_oracle_load_and_select(h2o_oracle *o, const double *K, const double *V,
                               const double *score, int n)
{
    if (!o || !K || !V || !score || n <= 0 || n > o->cap || o->t != 0) return -1;
    const int d = o->d;
    memcpy(o->K, K, (size_t)n * d * sizeof(double));
    memcpy(o->V, V, (size_t)n * d * sizeof(double));
    for (int j = 0; j < n; ++j) {
        o->acc[j] = o->score_f32 ? (double)(float)score[j] : score[j];
    }
    o->queries = (double)n;
    compress_prompt(o, n);
    store_resident_rows(o, 0, n);
    return 0;
}

/*
 * One generation step for the token at position t = tokens seen so far.
 *   q, k_new, v_new : [d] fp64
 *   out             : [d] attention output for this token
 *   info[0] = evicted position (-1: nothing evicted)
 *   info[1] = number of eviction candidates
 *   low[0]  = lowest candidate score, low[1] = second lowest (+inf if none)
 *   p_self_out (nullable) = probability the token gave itself
 * Returns 0, or -1 on bad arguments / capacity exhausted.
 */
int h2o_oracle_decode(h2o_oracle *o, const double *q, const double *k_new,
                      const double *v_new, double *out, int *info, double *low,
                      double *p_self_out)
{
    if (!o || !q || !k_new || !v_new || !out || o->t >= o->cap) return -1;
    const int d = o->d, t = o->t;
    memcpy(o->K + (size_t)t * d, k_new, (size_t)d * sizeof(double));
    memcpy(o->V + (size_t)t * d, v_new, (size_t)d * sizeof(double));
    o->acc[t] = 0.0;
    o->resident[t] = 1;                 /* G = S_{t-1} U {t} */
    ++o->n_resident;

    /* softmax over G only */
    double m = -INFINITY;
    for (int j = 0; j <= t; ++j) {
        if (!o->resident[j]) continue;
        o->s[j] = o->scale * dot(q, o->K + (size_t)j * d, d);
        if (o->s[j] > m) m = o->s[j];
    }
    double D = 0.0;
    for (int j = 0; j <= t; ++j)
        if (o->resident[j]) { o->p[j] = exp(o->s[j] - m); D += o->p[j]; }
    for (int c = 0; c < d; ++c) out[c] = 0.0;
    for (int j = 0; j <= t; ++j) {
        if (!o->resident[j]) continue;
        o->p[j] /= D;
        const double *vj = o->V + (size_t)j * d;
        for (int c = 0; c < d; ++c) out[c] += o->p[j] * vj[c];
        o->acc[j] = add_score(o, o->acc[j], o->p[j]);   /* accumulate */
    }
    o->queries += 1.0;
    if (p_self_out) *p_self_out = o->p[t];

    int evicted = -1, n_cand = 0;
    double lowest = INFINITY, second = INFINITY;
    if (o->protect != 0) {
        if (o->n_resident > o->budget)
            evicted = evict_one_protected(o, t, t, &n_cand, &lowest, &second);
    } else if (o->n_resident > o->budget) {
        /* candidates: resident positions outside the window {t-R+1..t} */
        const int last_cand = t - o->recent;
        for (int j = 0; j <= last_cand; ++j) {
            if (!o->resident[j]) continue;
            ++n_cand;
            const double rj = rank_score(o, j, t);
            if (evicted < 0 || evict_before(rj, j, lowest, evicted)) {
                second = lowest; lowest = rj; evicted = j;
            } else if (rj < second) {
                second = rj;
            }
        }
        if (evicted >= 0) {
            o->resident[evicted] = 0;
            o->evicted_mass += o->acc[evicted];
            --o->n_resident;
        }
    }
    if (info) { info[0] = evicted; info[1] = n_cand; }
    if (low) { low[0] = lowest; low[1] = second; }
    o->t = t + 1;
    if (o->resident[t]) store_row(o, t);    /* the token enters the cache now */
    return 0;
}

/* Undo the eviction of `restore_pos` and evict `evict_pos` instead (used only
 * when a checked implementation legitimately broke a near-tie the other way). */
int h2o_oracle_resync(h2o_oracle *o, int restore_pos, int evict_pos)
{
    if (!o || restore_pos < 0 || restore_pos >= o->t || evict_pos < 0 ||
        evict_pos >= o->t) return -1;
    if (o->resident[restore_pos] || !o->resident[evict_pos]) return -1;
    o->resident[restore_pos] = 1; o->evicted_mass -= o->acc[restore_pos];
    o->resident[evict_pos] = 0;   o->evicted_mass += o->acc[evict_pos];
    store_row(o, restore_pos);
    return 0;
}

/* ---- read-only accessors ---- */
int h2o_oracle_tokens_seen(const h2o_oracle *o) { return o->t; }
int h2o_oracle_num_resident(const h2o_oracle *o) { return o->n_resident; }
double h2o_oracle_evicted_mass(const h2o_oracle *o) { return o->evicted_mass; }
double h2o_oracle_queries(const h2o_oracle *o) { return o->queries; }
int h2o_oracle_is_resident(const h2o_oracle *o, int pos)
{ return (pos >= 0 && pos < o->t) ? o->resident[pos] : 0; }
double h2o_oracle_score(const h2o_oracle *o, int pos)
{ return (pos >= 0 && pos < o->t) ? o->acc[pos] : NAN; }

/* Resident positions in ascending order with their scores; returns the count.
 * pos_out/score_out must hold at least `budget` (or t, if smaller) entries. */
int h2o_oracle_resident(const h2o_oracle *o, int *pos_out, double *score_out)
{
    int c = 0;
    for (int j = 0; j < o->t; ++j) {
        if (!o->resident[j]) continue;
        if (pos_out) pos_out[c] = j;
        if (score_out) score_out[c] = o->acc[j];
        ++c;
    }
    return c;
}

/* The 4-bit codes ([d] each, one per byte) and the (scale, min) pairs
 * ([d/group][2] each) a quantised cache holds for resident position `pos`. */
int h2o_oracle_token_codes(const h2o_oracle *o, int pos, unsigned char *kcode,
                           float *kpar, unsigned char *vcode, float *vpar)
{
    if (!o || o->kv_bits != 4 || pos < 0 || pos >= o->t || !o->quantised[pos]) return -1;
    const size_t d = (size_t)o->d, np = (size_t)(o->d / o->group) * 2;
    if (kcode) memcpy(kcode, o->Kcode + pos * d, d);
    if (vcode) memcpy(vcode, o->Vcode + pos * d, d);
    if (kpar) memcpy(kpar, o->Kpar + pos * np, np * sizeof(float));
    if (vpar) memcpy(vpar, o->Vpar + pos * np, np * sizeof(float));
    return 0;
}

/* Key/value history row (what a cache slot holding `pos` must contain). */
int h2o_oracle_token_kv(const h2o_oracle *o, int pos, double *k_out, double *v_out)
{
    if (pos < 0 || pos >= o->t) return -1;
    if (k_out) memcpy(k_out, o->K + (size_t)pos * o->d, (size_t)o->d * sizeof(double));
    if (v_out) memcpy(v_out, o->V + (size_t)pos * o->d, (size_t)o->d * sizeof(double));
    return 0;
}
