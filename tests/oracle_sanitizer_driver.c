/*
 * Exercises every entry point of the CPU oracle on small random inputs; built
 * with -fsanitize=address,undefined by tests/test_oracle_sanitizers.py so that
 * out-of-bounds accesses, leaks and undefined arithmetic in the checker itself
 * (test infrastructure, but everything else is judged against it) fail loudly.
 */
#include <stdio.h>
#include <stdlib.h>
#include "../oracle/h2o_oracle.c"

static double rnd(unsigned *s)
{
    *s = *s * 1664525u + 1013904223u;
    return ((double)(*s >> 8) / 8388608.0) - 1.0;          /* [-1, 1), multiples of 2^-23: exact in binary32 */
}

static void fill(double *x, int n, unsigned *s) { for (int i = 0; i < n; ++i) x[i] = 2.0 * rnd(s); }

static int run(int d, int heavy, int recent, int n, int T, int f32, int policy, int bits, int group)
{
    unsigned seed = 12345u + (unsigned)(d * 31 + heavy * 7 + recent * 3 + n + T + f32 + policy + bits);
    const int cap = n + 3 * T + 64;
    h2o_oracle *o = h2o_oracle_new(d, heavy, recent, 0.3, f32, cap);
    if (!o) return 1;
    if (h2o_oracle_set_policy(o, policy) != 0) return 2;
    if (h2o_oracle_set_kv_bits(o, bits, group) != 0) return 3;
    double *Q = malloc(sizeof(double) * (size_t)cap * d), *K = malloc(sizeof(double) * (size_t)cap * d);
    double *V = malloc(sizeof(double) * (size_t)cap * d), *out = malloc(sizeof(double) * (size_t)cap * d);
    double *col = malloc(sizeof(double) * (size_t)cap);
    fill(Q, cap * d, &seed); fill(K, cap * d, &seed); fill(V, cap * d, &seed);
    int rc = 0, info[2]; double low[2], ps;
    if (n > 0 && h2o_oracle_prefill(o, Q, K, V, n, col, out) != 0) rc = 4;
    for (int s = 0; s < T && !rc; ++s) {
        const size_t off = (size_t)(n + s) * d;
        if (h2o_oracle_decode(o, Q + off, K + off, V + off, out, info, low, &ps) != 0) rc = 5;
    }
    if (!rc && bits == 0) {                                 /* a further prompt in two chunks, then steps */
        const size_t off = (size_t)(n + T) * d;
        const int m1 = T / 2 + 1, m2 = T - m1 + 3;
        if (h2o_oracle_prefill_chunk(o, Q + off, K + off, V + off, m1, col, out) != 0) rc = 6;
        if (!rc && h2o_oracle_prefill_chunk(o, Q + off + (size_t)m1 * d, K + off + (size_t)m1 * d,
                                            V + off + (size_t)m1 * d, m2, col, NULL) != 0) rc = 7;
        for (int s = 0; s < 5 && !rc; ++s)
            if (h2o_oracle_decode(o, Q, K, V, out, info, low, NULL) != 0) rc = 8;
    }
    if (!rc) {
        int *pos = malloc(sizeof(int) * (size_t)(heavy + recent + 1));
        double *sc = malloc(sizeof(double) * (size_t)(heavy + recent + 1));
        const int c = h2o_oracle_resident(o, pos, sc);
        if (c != h2o_oracle_num_resident(o) || c > heavy + recent) rc = 9;
        unsigned char *kc = malloc((size_t)d), *vc = malloc((size_t)d);
        float *kp = malloc(sizeof(float) * 2 * (size_t)d), *vp = malloc(sizeof(float) * 2 * (size_t)d);
        for (int i = 0; i < c && !rc; ++i) {
            if (h2o_oracle_token_kv(o, pos[i], out, out + d) != 0) rc = 10;
            if (bits == 4 && h2o_oracle_token_codes(o, pos[i], kc, kp, vc, vp) != 0) rc = 11;
            if (!h2o_oracle_is_resident(o, pos[i]) || !(h2o_oracle_score(o, pos[i]) >= 0.0)) rc = 12;
        }
        if (!rc && c >= 2 && info[0] >= 0 && !h2o_oracle_is_resident(o, info[0]))
            if (h2o_oracle_resync(o, info[0], pos[0]) != 0) rc = 13;
        free(pos); free(sc); free(kc); free(vc); free(kp); free(vp);
    }
    /* a second object fed by externally supplied scores */
    if (!rc && n > 0) {
        h2o_oracle *p = h2o_oracle_new(d, heavy, recent, 0.3, f32, cap);
        h2o_oracle_set_kv_bits(p, bits, group);
        for (int j = 0; j < n; ++j) col[j] = 1.0 + rnd(&seed);
        if (h2o_oracle_load_and_select(p, K, V, col, n) != 0) rc = 14;
        h2o_oracle_free(p);
    }
    free(Q); free(K); free(V); free(out); free(col);
    h2o_oracle_free(o);
    return rc;
}

int main(void)
{
    static const int cfg[][9] = {
        /* d heavy recent  n   T f32 policy bits group */
        {8, 2, 2, 12, 20, 0, 0, 0, 4}, {8, 3, 0, 10, 15, 1, 0, 0, 4}, {8, 0, 3, 0, 25, 1, 1, 0, 4},
        {16, 4, 4, 40, 30, 1, 0, 4, 8}, {64, 1, 1, 5, 9, 0, 1, 4, 64}, {8, 5, 5, 3, 4, 0, 0, 4, 4},
        {128, 6, 6, 30, 12, 1, 0, 4, 64}, {4, 1, 0, 1, 6, 1, 0, 0, 4},
    };
    for (unsigned i = 0; i < sizeof(cfg) / sizeof(cfg[0]); ++i) {
        const int rc = run(cfg[i][0], cfg[i][1], cfg[i][2], cfg[i][3], cfg[i][4], cfg[i][5], cfg[i][6],
                           cfg[i][7], cfg[i][8]);
        if (rc) { printf("configuration %u failed at step %d\n", i, rc); return 1; }
    }
    /* rejected arguments must not touch memory */
    if (h2o_oracle_new(0, 1, 1, 1.0, 0, 8) || h2o_oracle_new(8, 0, 0, 1.0, 0, 8)) return 2;
    puts("oracle clean under the sanitizers");
    return 0;
}
