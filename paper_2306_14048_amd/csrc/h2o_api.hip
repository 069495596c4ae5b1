// C ABI of the H2O hot path (declarations and contracts: include/h2o.h).
// Host-side only: argument validation, carving the caller's device memory into
// the four cache regions, state tracking (tokens seen), kernel launches.
#include <mutex>
#include <new>
#include "h2o_internal.h"

// Scratch of h2o_prefill_scores_noalloc: row statistics and column sums of one
// prompt phase.  Every GPU the library runs on holds its own copy of this array
// (at its own address) until the process ends.  In host code the array's name is
// only a handle for hipGetSymbolAddress; the device address it yields is what
// kernels and copies are given.
static __device__ __align__(256) unsigned char scratch[H2O_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
std::mutex scratch_mu;
void *scratch_ptr[MAX_DEVICES];      // device address of `scratch` per device, once resolved

// Address of the current device's copy of `scratch` (resolved on first use on that
// device; h2o_cache_init does it, so later calls only read the table).
int scratch_of_current_device(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return H2O_EHIP;
    if (dev < 0 || dev >= MAX_DEVICES) return H2O_EUNSUPPORTED;
    std::lock_guard<std::mutex> guard(scratch_mu);
    if (!scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return H2O_EHIP;
        scratch_ptr[dev] = p;
    }
    *out = scratch_ptr[dev];
    return H2O_OK;
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_config(const h2o_config *c)
{
    if (!c) return H2O_EINVAL;
    if (c->batch < 1 || c->heads < 1 || c->heavy < 0 || c->recent < 0) return H2O_EINVAL;
    if ((int64_t)c->heavy + c->recent < 1) return H2O_EINVAL;
    if (c->dtype != H2O_F32 && c->dtype != H2O_F16 && c->dtype != H2O_BF16) return H2O_EINVAL;
    if (!(c->scale >= 0.0f) || !(c->scale < 3.0e38f)) return H2O_EINVAL;
    if (c->rank != H2O_RANK_ACCUMULATED && c->rank != H2O_RANK_AVERAGED) return H2O_EINVAL;
    if (c->head_dim != 64 && c->head_dim != 128) return H2O_EUNSUPPORTED;
    if ((int64_t)c->heavy + c->recent > H2O_MAX_BUDGET) return H2O_EUNSUPPORTED;
    if ((int64_t)c->batch * c->heads > (1 << 24)) return H2O_EUNSUPPORTED;
    if (c->kv_bits != 0 && c->kv_bits != 4) return H2O_EINVAL;
    if (c->protect != H2O_PROTECT_RECENT && c->protect != H2O_PROTECT_STRIDED &&
        c->protect != H2O_PROTECT_FIXED)
        return H2O_EINVAL;
    if (c->protect != H2O_PROTECT_RECENT && (c->stride < 1 || c->stride > (1 << 30))) return H2O_EINVAL;
    if (c->kv_bits == 4 && (int64_t)c->heavy + c->recent > H2O_Q4_MAX_BUDGET) return H2O_EUNSUPPORTED;
    return H2O_OK;
}

struct Layout { size_t kv, acc_off, pos_off, total; };

Layout layout_of(const h2o_config &c)
{
    const size_t heads = (size_t)c.batch * c.heads, k = (size_t)c.heavy + c.recent;
    Layout l;
    l.kv = align_up(heads * k * h2o_row_bytes(c), 256);
    l.acc_off = 2 * l.kv;
    l.pos_off = l.acc_off + align_up(heads * k * sizeof(float), 256);
    l.total = l.pos_off + align_up(heads * k * sizeof(int32_t), 256);
    return l;
}

inline int hip_rc(hipError_t e) { return e == hipSuccess ? H2O_OK : H2O_EHIP; }

}  // namespace

extern "C" {
#pragma GCC visibility push(default)

size_t h2o_cache_bytes(const h2o_config *cfg)
{
    if (check_config(cfg) != H2O_OK) return 0;
    return layout_of(*cfg).total;
}

size_t h2o_prefill_workspace_bytes(const h2o_config *cfg, int32_t n)
{
    if (check_config(cfg) != H2O_OK || n < 1 || n > H2O_MAX_PROMPT) return 0;
    const size_t heads = (size_t)cfg->batch * cfg->heads;
    return 2 * align_up(heads * (size_t)n * sizeof(float), 256);
}

int h2o_cache_init(const h2o_config *cfg, void *dev_mem, size_t bytes, void *hip_stream,
                   h2o_cache **out)
{
    if (out) *out = nullptr;
    const int rc = check_config(cfg);
    if (rc != H2O_OK) return rc;
    if (!dev_mem || !out || !aligned16(dev_mem)) return H2O_EINVAL;
    const Layout l = layout_of(*cfg);
    if (bytes < l.total) return H2O_ENOMEM;
    h2o_cache *c = new (std::nothrow) h2o_cache;
    if (!c) return H2O_ENOMEM;
    {
        // resolve this device's built-in scratch now: the call that uses it may run
        // where nothing may be looked up any more (stream capture)
        void *unused = nullptr;
        const int src = scratch_of_current_device(&unused);
        if (src == H2O_EHIP) { delete c; return H2O_EHIP; }
    }
    c->cfg = *cfg;
    c->scale = h2o_scale_of(*cfg);
    c->k = cfg->heavy + cfg->recent;
    c->esize = h2o_esize(cfg->dtype);
    c->rowb = h2o_row_bytes(*cfg);
    c->t = 0;
    c->sorted = true;
    char *base = static_cast<char *>(dev_mem);
    c->K = base;
    c->V = base + l.kv;
    c->acc = reinterpret_cast<float *>(base + l.acc_off);
    c->pos = reinterpret_cast<int32_t *>(base + l.pos_off);
    c->kv_bytes = (size_t)cfg->batch * cfg->heads * c->k * c->rowb;
    const hipError_t e = h2o_launch_mark_free(*c, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) { delete c; return H2O_EHIP; }
    *out = c;
    return H2O_OK;
}

int h2o_cache_reset(h2o_cache *cache, void *hip_stream)
{
    if (!cache) return H2O_EINVAL;
    const hipError_t e = h2o_launch_mark_free(*cache, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return H2O_EHIP;
    cache->t = 0;
    cache->sorted = true;
    return H2O_OK;
}

void h2o_cache_destroy(h2o_cache *cache) { delete cache; }

int h2o_prefill_colsum(const h2o_config *cfg, const void *Q, const void *K, int32_t n,
                       void *workspace, size_t ws_bytes, float *colsum_out, void *hip_stream)
{
    const int rc = check_config(cfg);
    if (rc != H2O_OK) return rc;
    if (!Q || !K || !workspace || !colsum_out || n < 1) return H2O_EINVAL;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(workspace) || !aligned16(colsum_out))
        return H2O_EINVAL;
    if (n > H2O_MAX_PROMPT) return H2O_EUNSUPPORTED;
    if (ws_bytes < h2o_prefill_workspace_bytes(cfg, n)) return H2O_ENOMEM;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    float *lse = static_cast<float *>(workspace);
    const double scale = h2o_scale_of(*cfg);
    hipError_t e = h2o_launch_prefill_lse(*cfg, scale, Q, K, n, n, lse, st);
    if (e != hipSuccess) return H2O_EHIP;
    e = h2o_launch_prefill_colsum(*cfg, scale, Q, K, n, n, lse, colsum_out, st);
    return hip_rc(e);
}

int h2o_prefill_select(h2o_cache *cache, const void *K, const void *V, const float *score,
                       int32_t n, void *hip_stream)
{
    if (!cache || !K || !V || !score || n < 1) return H2O_EINVAL;
    if (!aligned16(K) || !aligned16(V) || !aligned16(score)) return H2O_EINVAL;
    if (n > H2O_MAX_PROMPT) return H2O_EUNSUPPORTED;
    if (cache->t != 0) return H2O_ESTATE;
    const hipError_t e =
        h2o_launch_select_gather(*cache, K, V, score, nullptr, nullptr, n, n,
                                 static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return H2O_EHIP;
    cache->t = n;
    cache->sorted = true;
    return H2O_OK;
}

int h2o_prefill_scores(h2o_cache *cache, const void *Q, const void *K, const void *V, int32_t n,
                       void *workspace, size_t ws_bytes, float *colsum_out, void *hip_stream)
{
    if (!cache || !V) return H2O_EINVAL;
    if (cache->t != 0) return H2O_ESTATE;
    if (n < 1) return H2O_EINVAL;
    if (n > H2O_MAX_PROMPT) return H2O_EUNSUPPORTED;
    const size_t need = h2o_prefill_workspace_bytes(&cache->cfg, n);
    if (!workspace || ws_bytes < need) return workspace ? H2O_ENOMEM : H2O_EINVAL;
    // second half of the workspace holds the sums unless the caller wants them
    float *sums = colsum_out ? colsum_out
                             : reinterpret_cast<float *>(static_cast<char *>(workspace) + need / 2);
    int rc = h2o_prefill_colsum(&cache->cfg, Q, K, n, workspace, ws_bytes, sums, hip_stream);
    if (rc != H2O_OK) return rc;
    return h2o_prefill_select(cache, K, V, sums, n, hip_stream);
}

int h2o_prefill_scores_noalloc(h2o_cache *cache, const void *Q, const void *K, const void *V,
                               int32_t n, float *colsum_out, void *hip_stream)
{
    if (!cache || !V) return H2O_EINVAL;
    if (cache->t != 0) return H2O_ESTATE;
    if (n < 1) return H2O_EINVAL;
    if (n > H2O_MAX_PROMPT) return H2O_EUNSUPPORTED;
    const size_t need = h2o_prefill_workspace_bytes(&cache->cfg, n);
    if (need == 0) return H2O_EUNSUPPORTED;
    if (need > H2O_NOALLOC_SCRATCH_BYTES) return H2O_ESCRATCH;
    void *ws = nullptr;
    const int rc = scratch_of_current_device(&ws);
    if (rc != H2O_OK) return rc;
    // nothing in the scratch has to start at zero: both passes write every word
    // they later read
    return h2o_prefill_scores(cache, Q, K, V, n, ws, H2O_NOALLOC_SCRATCH_BYTES, colsum_out, hip_stream);
}

size_t h2o_prefill_attention_workspace_bytes(const h2o_config *cfg, int32_t n)
{
    if (check_config(cfg) != H2O_OK || n < 1 || n > H2O_MAX_PROMPT) return 0;
    if (cfg->dtype == H2O_F32) return 0;
    return align_up(h2o_attn_vt_bytes(*cfg, n), 256) + h2o_prefill_workspace_bytes(cfg, n);
}

int h2o_prefill_attention(const h2o_config *cfg, const void *Q, const void *K, const void *V,
                          int32_t n, void *workspace, size_t ws_bytes, void *out, float *lse_out,
                          void *hip_stream)
{
    const int rc = check_config(cfg);
    if (rc != H2O_OK) return rc;
    if (!Q || !K || !V || !workspace || !out || n < 1) return H2O_EINVAL;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(workspace) ||
        !aligned16(out) || !aligned16(lse_out))
        return H2O_EINVAL;
    if (n > H2O_MAX_PROMPT || cfg->dtype == H2O_F32) return H2O_EUNSUPPORTED;
    if (ws_bytes < h2o_prefill_attention_workspace_bytes(cfg, n)) return H2O_ENOMEM;
    char *ws = static_cast<char *>(workspace);
    float *lse2 = reinterpret_cast<float *>(ws + align_up(h2o_attn_vt_bytes(*cfg, n), 256));
    return hip_rc(h2o_launch_prefill_attention(*cfg, h2o_scale_of(*cfg), Q, K, V, n, n, ws, lse2,
                                               lse_out, out, static_cast<hipStream_t>(hip_stream)));
}

int h2o_prefill_attention_scores(h2o_cache *cache, const void *Q, const void *K, const void *V,
                                 int32_t n, void *workspace, size_t ws_bytes, void *out,
                                 float *colsum_out, void *hip_stream)
{
    if (!cache || !aligned16(colsum_out)) return H2O_EINVAL;
    if (cache->t != 0) return H2O_ESTATE;
    const h2o_config *cfg = &cache->cfg;
    int rc = h2o_prefill_attention(cfg, Q, K, V, n, workspace, ws_bytes, out, nullptr, hip_stream);
    if (rc != H2O_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    char *ws = static_cast<char *>(workspace);
    const size_t half = h2o_prefill_workspace_bytes(cfg, n) / 2;
    float *lse2 = reinterpret_cast<float *>(ws + align_up(h2o_attn_vt_bytes(*cfg, n), 256));
    float *sums = colsum_out ? colsum_out : reinterpret_cast<float *>(reinterpret_cast<char *>(lse2) + half);
    const hipError_t e = h2o_launch_prefill_colsum(*cfg, h2o_scale_of(*cfg), Q, K, n, n, lse2, sums, st);
    if (e != hipSuccess) return H2O_EHIP;
    return h2o_prefill_select(cache, K, V, sums, n, hip_stream);
}

size_t h2o_prefill_chunk_workspace_bytes(const h2o_config *cfg, int32_t m, int32_t with_output)
{
    if (check_config(cfg) != H2O_OK || m < 1 || cfg->kv_bits != 0) return 0;
    if (with_output && cfg->dtype == H2O_F32) return 0;
    const size_t k = (size_t)cfg->heavy + cfg->recent;
    if (k + (size_t)m > H2O_MAX_PROMPT) return 0;
    const size_t heads = (size_t)cfg->batch * cfg->heads, ncat = k + m;
    const size_t rows = align_up(heads * ncat * cfg->head_dim * h2o_esize(cfg->dtype), 256);
    const size_t vec = align_up(heads * ncat * sizeof(float), 256);
    // K and V of cache + chunk, old scores, positions, column sums, row statistics,
    // the slots in position order (+ the transposed V of cache + chunk when the
    // attention output is wanted)
    return 2 * rows + 3 * vec + align_up(heads * (size_t)m * sizeof(float), 256) +
           align_up(heads * k * sizeof(int32_t), 256) +
           (with_output ? align_up(h2o_attn_vt_bytes(*cfg, (int)ncat), 256) : 0);
}

int h2o_prefill_chunk(h2o_cache *cache, const void *Q, const void *K, const void *V, int32_t m,
                      void *workspace, size_t ws_bytes, void *out, void *hip_stream)
{
    if (!cache || !Q || !K || !V || !workspace || m < 1) return H2O_EINVAL;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(workspace) || !aligned16(out))
        return H2O_EINVAL;
    if (cache->cfg.kv_bits != 0) return H2O_EUNSUPPORTED;   // cached rows would have to be dequantised
    if (out && cache->cfg.dtype == H2O_F32) return H2O_EUNSUPPORTED;
    const h2o_config &cfg = cache->cfg;
    const int occ = cache->t < cache->k ? cache->t : cache->k;
    if ((int64_t)cache->k + m > H2O_MAX_PROMPT || (int64_t)cache->t + m >= 0x7ffffff0) return H2O_EUNSUPPORTED;
    if (ws_bytes < h2o_prefill_chunk_workspace_bytes(&cfg, m, out != nullptr)) return H2O_ENOMEM;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const size_t heads = (size_t)cfg.batch * cfg.heads, ncat_max = (size_t)cache->k + m;
    const size_t rows = align_up(heads * ncat_max * cfg.head_dim * cache->esize, 256);
    const size_t vec = align_up(heads * ncat_max * sizeof(float), 256);
    char *ws = static_cast<char *>(workspace);
    char *Kcat = ws, *Vcat = ws + rows;
    float *base = reinterpret_cast<float *>(ws + 2 * rows);
    int32_t *pos_cat = reinterpret_cast<int32_t *>(ws + 2 * rows + vec);
    float *colsum = reinterpret_cast<float *>(ws + 2 * rows + 2 * vec);
    float *lse = reinterpret_cast<float *>(ws + 2 * rows + 3 * vec);
    int32_t *order = reinterpret_cast<int32_t *>(ws + 2 * rows + 3 * vec +
                                                 align_up(heads * (size_t)m * sizeof(float), 256));
    char *vt = reinterpret_cast<char *>(order) + align_up(heads * (size_t)cache->k * sizeof(int32_t), 256);
    const int ncat = occ + m;
    const double scale = h2o_scale_of(cfg);
    // after generation steps have evicted, the slots are first put in position order
    hipError_t e = h2o_launch_concat(*cache, K, V, m, occ, cache->sorted ? nullptr : order, Kcat, Vcat,
                                     base, pos_cat, st);
    if (e != hipSuccess) return H2O_EHIP;
    // row statistics: a by-product of the attention output when that is wanted
    e = out ? h2o_launch_prefill_attention(cfg, scale, Q, Kcat, Vcat, m, ncat, vt, lse, nullptr, out, st)
            : h2o_launch_prefill_lse(cfg, scale, Q, Kcat, m, ncat, lse, st);
    if (e != hipSuccess) return H2O_EHIP;
    e = h2o_launch_prefill_colsum(cfg, scale, Q, Kcat, m, ncat, lse, colsum, st);
    if (e != hipSuccess) return H2O_EHIP;
    e = h2o_launch_select_gather(*cache, Kcat, Vcat, colsum, base, pos_cat, ncat, cache->t + m, st);
    if (e != hipSuccess) return H2O_EHIP;
    cache->t += m;
    cache->sorted = true;
    return H2O_OK;
}

int h2o_decode_step(h2o_cache *cache, const void *q, const void *k_new, const void *v_new,
                    void *out, void *hip_stream)
{
    if (!cache || !q || !k_new || !v_new || !out) return H2O_EINVAL;
    if (!aligned16(q) || !aligned16(k_new) || !aligned16(v_new) || !aligned16(out))
        return H2O_EINVAL;
    if (cache->t >= 0x7ffffff0) return H2O_EUNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const hipError_t e = cache->cfg.kv_bits == 4 ? h2o_launch_decode_q4(*cache, q, k_new, v_new, out, st)
                                                 : h2o_launch_decode(*cache, q, k_new, v_new, out, st);
    if (e != hipSuccess) return H2O_EHIP;
    // free slots fill in index order (positions stay ascending); an eviction
    // overwrites a slot in the middle
    if (cache->t >= cache->k) cache->sorted = false;
    cache->t += 1;
    return H2O_OK;
}

int h2o_cache_snapshot(const h2o_cache *cache, int32_t *pos_out, float *acc_out, void *hip_stream)
{
    if (!cache) return H2O_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const size_t cnt = (size_t)cache->cfg.batch * cache->cfg.heads * cache->k;
    if (pos_out &&
        hipMemcpyAsync(pos_out, cache->pos, cnt * sizeof(int32_t), hipMemcpyDeviceToDevice, st) != hipSuccess)
        return H2O_EHIP;
    if (acc_out &&
        hipMemcpyAsync(acc_out, cache->acc, cnt * sizeof(float), hipMemcpyDeviceToDevice, st) != hipSuccess)
        return H2O_EHIP;
    return H2O_OK;
}

int h2o_cache_restore(h2o_cache *cache, const void *K, const void *V, const float *acc,
                      const int32_t *pos, int32_t tokens_seen, void *hip_stream)
{
    if (!cache || !K || !V || !acc || !pos || tokens_seen < 0) return H2O_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const size_t cnt = (size_t)cache->cfg.batch * cache->cfg.heads * cache->k;
    if (hipMemcpyAsync(cache->K, K, cache->kv_bytes, hipMemcpyDeviceToDevice, st) != hipSuccess ||
        hipMemcpyAsync(cache->V, V, cache->kv_bytes, hipMemcpyDeviceToDevice, st) != hipSuccess ||
        hipMemcpyAsync(cache->acc, acc, cnt * sizeof(float), hipMemcpyDeviceToDevice, st) != hipSuccess ||
        hipMemcpyAsync(cache->pos, pos, cnt * sizeof(int32_t), hipMemcpyDeviceToDevice, st) != hipSuccess)
        return H2O_EHIP;
    cache->t = tokens_seen;
    cache->sorted = false;      // not known
    return H2O_OK;
}

int h2o_cache_validate(const h2o_cache *cache, int32_t *flags_out, void *hip_stream)
{
    if (!cache || !flags_out) return H2O_EINVAL;
    return hip_rc(h2o_launch_validate(*cache, flags_out, static_cast<hipStream_t>(hip_stream)));
}

int h2o_cache_rolled_positions(const h2o_cache *cache, int32_t *rolled_out, void *hip_stream)
{
    if (!cache || !rolled_out) return H2O_EINVAL;
    return hip_rc(h2o_launch_rolled_positions(*cache, rolled_out, static_cast<hipStream_t>(hip_stream)));
}

int h2o_cache_tokens_seen(const h2o_cache *cache) { return cache ? cache->t : H2O_EINVAL; }

int h2o_cache_regions(const h2o_cache *cache, void **K, void **V, float **acc, int32_t **pos)
{
    if (!cache) return H2O_EINVAL;
    if (K) *K = cache->K;
    if (V) *V = cache->V;
    if (acc) *acc = cache->acc;
    if (pos) *pos = cache->pos;
    return H2O_OK;
}

const char *h2o_status_str(int status)
{
    switch (status) {
    case H2O_OK: return "ok";
    case H2O_EINVAL: return "invalid argument";
    case H2O_EUNSUPPORTED: return "unsupported configuration";
    case H2O_ENOMEM: return "caller buffer too small";
    case H2O_ESTATE: return "call not legal in this cache state";
    case H2O_EHIP: return "HIP runtime error";
    case H2O_ESCRATCH: return "request exceeds the library's built-in scratch";
    default: return "unknown status";
    }
}

#pragma GCC visibility pop
}  // extern "C"
