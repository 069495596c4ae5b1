/*
 * A plain C99 caller of the H2O library: proof that the boundary is a C ABI
 * (no C++ or Python needed).  Test infrastructure, built by tests/test_c_caller.py
 * with gcc and linked against libh2o_hip.so (and the HIP runtime for device memory).
 *
 *   c_caller host   walks the host-side argument checks; needs no GPU
 *   c_caller gpu    cache init -> prompt phase -> 4 generation steps -> snapshot on
 *                   device 0, then checks what holds for any input: positions in
 *                   range and distinct, the recent window resident, scores between 0
 *                   and the number of queries a token has seen, finite outputs, and
 *                   a consistent report from h2o_cache_validate
 *
 * Exit status 0 and a last line "host ok" / "gpu ok" on success.
 */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <hip/hip_runtime_api.h>

#include "h2o.h"

#define CHECK(cond)                                                                   \
    do {                                                                              \
        if (!(cond)) {                                                                \
            fprintf(stderr, "c_caller: check failed at line %d: %s\n", __LINE__, #cond); \
            return 1;                                                                 \
        }                                                                             \
    } while (0)

static h2o_config config(int batch, int heads, int d, int heavy, int recent, int dtype)
{
    h2o_config c;
    memset(&c, 0, sizeof c);
    c.batch = batch; c.heads = heads; c.head_dim = d; c.heavy = heavy; c.recent = recent;
    c.dtype = dtype;
    return c;
}

static int host_checks(void)
{
    h2o_config ok = config(16, 32, 128, 205, 205, H2O_F16);
    const size_t kv = (size_t)16 * 32 * 410 * 128 * 2, meta = (size_t)16 * 32 * 410 * 4;
    CHECK(h2o_cache_bytes(&ok) == 2 * kv + 2 * meta);
    CHECK(h2o_prefill_workspace_bytes(&ok, 2048) == (size_t)2 * 16 * 32 * 2048 * 4);
    CHECK(h2o_cache_bytes(NULL) == 0);
    h2o_config bad = config(1, 1, 96, 4, 4, H2O_F16);          /* head_dim not 64 / 128 */
    CHECK(h2o_cache_bytes(&bad) == 0);
    bad = config(1, 1, 128, 0, 0, H2O_F16);                    /* empty budget */
    CHECK(h2o_cache_bytes(&bad) == 0);
    bad = config(1, 1, 128, 4000, 4000, H2O_F16);              /* budget above the maximum */
    CHECK(h2o_cache_bytes(&bad) == 0);
    CHECK(h2o_prefill_workspace_bytes(&ok, 0) == 0);
    CHECK(h2o_prefill_workspace_bytes(&ok, H2O_MAX_PROMPT + 1) == 0);

    h2o_cache *cache = (h2o_cache *)&ok;                       /* must come back NULL */
    CHECK(h2o_cache_init(&ok, NULL, 1, NULL, &cache) == H2O_EINVAL);
    CHECK(cache == NULL);
    CHECK(h2o_cache_init(NULL, (void *)256, 1, NULL, &cache) == H2O_EINVAL);
    bad = config(1, 1, 96, 4, 4, H2O_F16);
    CHECK(h2o_cache_init(&bad, (void *)256, 1 << 20, NULL, &cache) == H2O_EUNSUPPORTED);
    CHECK(h2o_cache_init(&ok, (void *)264, 1 << 20, NULL, &cache) == H2O_EINVAL);   /* misaligned */
    CHECK(h2o_cache_init(&ok, (void *)256, 1024, NULL, &cache) == H2O_ENOMEM);      /* too small */
    CHECK(h2o_cache_reset(NULL, NULL) == H2O_EINVAL);
    CHECK(h2o_decode_step(NULL, NULL, NULL, NULL, NULL, NULL) == H2O_EINVAL);
    CHECK(h2o_prefill_scores(NULL, NULL, NULL, NULL, 8, NULL, 0, NULL, NULL) == H2O_EINVAL);
    CHECK(h2o_prefill_scores_noalloc(NULL, NULL, NULL, NULL, 8, NULL, NULL) == H2O_EINVAL);
    CHECK(h2o_prefill_colsum(&ok, NULL, NULL, 8, NULL, 0, NULL, NULL) == H2O_EINVAL);
    CHECK(h2o_cache_snapshot(NULL, NULL, NULL, NULL) == H2O_EINVAL);
    CHECK(h2o_cache_validate(NULL, NULL, NULL) == H2O_EINVAL);
    CHECK(h2o_cache_tokens_seen(NULL) == H2O_EINVAL);
    h2o_cache_destroy(NULL);                                   /* a no-op */
    CHECK(strcmp(h2o_status_str(H2O_OK), "ok") == 0);
    CHECK(strstr(h2o_status_str(H2O_ESCRATCH), "scratch") != NULL);
    CHECK(strlen(h2o_status_str(-99)) > 0);
    puts("host ok");
    return 0;
}

/* deterministic pseudo-random numbers in (-1, 1): inputs only, no method arithmetic */
static unsigned lcg_state = 20230614u;
static float next_unit(void)
{
    lcg_state = lcg_state * 1664525u + 1013904223u;
    return (float)((lcg_state >> 8) & 0xffff) / 32768.0f - 1.0f;
}
static void fill(float *x, size_t count, float amp)
{
    for (size_t i = 0; i < count; ++i) x[i] = amp * next_unit();
}

#define HIP(call) CHECK((call) == hipSuccess)

static int gpu_run(void)
{
    enum { B = 2, HH = 3, D = 64, N = 200, HEAVY = 12, RECENT = 10, K = HEAVY + RECENT, T = 4 };
    const int heads = B * HH;
    h2o_config cfg = config(B, HH, D, HEAVY, RECENT, H2O_F32);
    const size_t cache_bytes = h2o_cache_bytes(&cfg), ws_bytes = h2o_prefill_workspace_bytes(&cfg, N);
    CHECK(cache_bytes > 0 && ws_bytes > 0);
    const size_t prompt = (size_t)heads * N * D, step = (size_t)heads * D;

    float *hQ = malloc(prompt * 4), *hK = malloc(prompt * 4), *hV = malloc(prompt * 4);
    float *hs = malloc(3 * T * step * 4), *hout = malloc(T * step * 4);
    float *hacc = malloc((size_t)heads * K * 4);
    int32_t *hpos = malloc((size_t)heads * K * 4), *hflags = malloc((size_t)heads * 4);
    CHECK(hQ && hK && hV && hs && hout && hacc && hpos && hflags);
    fill(hQ, prompt, 1.0f); fill(hK, prompt, 1.5f); fill(hV, prompt, 1.0f); fill(hs, 3 * T * step, 1.0f);

    HIP(hipSetDevice(0));
    void *dmem, *dws, *dQ, *dK, *dV, *ds, *dout, *dacc, *dpos, *dflags;
    HIP(hipMalloc(&dmem, cache_bytes)); HIP(hipMalloc(&dws, ws_bytes));
    HIP(hipMalloc(&dQ, prompt * 4)); HIP(hipMalloc(&dK, prompt * 4)); HIP(hipMalloc(&dV, prompt * 4));
    HIP(hipMalloc(&ds, 3 * T * step * 4)); HIP(hipMalloc(&dout, T * step * 4));
    HIP(hipMalloc(&dacc, (size_t)heads * K * 4)); HIP(hipMalloc(&dpos, (size_t)heads * K * 4));
    HIP(hipMalloc(&dflags, (size_t)heads * 4));
    HIP(hipMemcpy(dQ, hQ, prompt * 4, hipMemcpyHostToDevice));
    HIP(hipMemcpy(dK, hK, prompt * 4, hipMemcpyHostToDevice));
    HIP(hipMemcpy(dV, hV, prompt * 4, hipMemcpyHostToDevice));
    HIP(hipMemcpy(ds, hs, 3 * T * step * 4, hipMemcpyHostToDevice));
    hipStream_t st;
    HIP(hipStreamCreate(&st));

    h2o_cache *cache = NULL;
    CHECK(h2o_cache_init(&cfg, dmem, cache_bytes, st, &cache) == H2O_OK && cache);
    CHECK(h2o_decode_step(cache, ds, ds, ds, (char *)dout + 4, st) == H2O_EINVAL);   /* misaligned */
    CHECK(h2o_prefill_scores(cache, dQ, dK, dV, N, dws, ws_bytes / 2, NULL, st) == H2O_ENOMEM);
    CHECK(h2o_prefill_scores(cache, dQ, dK, dV, N, dws, ws_bytes, NULL, st) == H2O_OK);
    CHECK(h2o_prefill_scores(cache, dQ, dK, dV, N, dws, ws_bytes, NULL, st) == H2O_ESTATE);
    CHECK(h2o_cache_tokens_seen(cache) == N);
    for (int s = 0; s < T; ++s) {
        const float *q = (const float *)ds + (size_t)(3 * s) * step;
        CHECK(h2o_decode_step(cache, q, q + step, q + 2 * step, (float *)dout + (size_t)s * step, st) == H2O_OK);
    }
    CHECK(h2o_cache_tokens_seen(cache) == N + T);
    CHECK(h2o_cache_snapshot(cache, dpos, dacc, st) == H2O_OK);
    CHECK(h2o_cache_validate(cache, dflags, st) == H2O_OK);
    HIP(hipStreamSynchronize(st));
    HIP(hipMemcpy(hpos, dpos, (size_t)heads * K * 4, hipMemcpyDeviceToHost));
    HIP(hipMemcpy(hacc, dacc, (size_t)heads * K * 4, hipMemcpyDeviceToHost));
    HIP(hipMemcpy(hout, dout, T * step * 4, hipMemcpyDeviceToHost));
    HIP(hipMemcpy(hflags, dflags, (size_t)heads * 4, hipMemcpyDeviceToHost));

    const int t = N + T;
    for (int h = 0; h < heads; ++h) {
        CHECK(hflags[h] == 0);
        int in_window = 0;
        double mass = 0.0;
        for (int s = 0; s < K; ++s) {
            const int p = hpos[h * K + s];
            const float a = hacc[h * K + s];
            CHECK(p >= 0 && p < t);
            for (int j = 0; j < s; ++j) CHECK(hpos[h * K + j] != p);
            if (p >= t - RECENT) ++in_window;
            CHECK(a >= 0.0f && a <= (float)(t - p) * 1.00001f);   /* at most 1 per query seen */
            mass += a;
        }
        CHECK(in_window == RECENT);
        CHECK(mass <= t * 1.00001);
    }
    for (size_t i = 0; i < T * step; ++i) CHECK(isfinite(hout[i]) && fabsf(hout[i]) <= 1.0f);   /* |V| < 1 */

    h2o_cache_destroy(cache);
    HIP(hipStreamDestroy(st));
    hipFree(dmem); hipFree(dws); hipFree(dQ); hipFree(dK); hipFree(dV); hipFree(ds); hipFree(dout);
    hipFree(dacc); hipFree(dpos); hipFree(dflags);
    free(hQ); free(hK); free(hV); free(hs); free(hout); free(hacc); free(hpos); free(hflags);
    puts("gpu ok");
    return 0;
}

int main(int argc, char **argv)
{
    if (argc == 2 && strcmp(argv[1], "host") == 0) return host_checks();
    if (argc == 2 && strcmp(argv[1], "gpu") == 0) return gpu_run();
    fprintf(stderr, "usage: c_caller host|gpu\n");
    return 2;
}
