// Internal declarations shared by the translation units of the HIP library.
// Not part of the public ABI (see include/h2o.h for that).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "h2o.h"

struct h2o_cache {
    h2o_config cfg;
    double scale;      // logit scale actually used (cfg.scale, or 1/sqrt(d) in double)
    int k;             // heavy + recent
    int esize;         // bytes per element of Q/K/V/q/k/v/out
    int rowb;          // bytes of one cached K (or V) row as stored
    int t;             // tokens seen so far
    bool sorted;       // occupied slots hold ascending positions (true until a step evicts)
    char *K;           // [B*Hh][k][d]
    char *V;           // [B*Hh][k][d]
    float *acc;        // [B*Hh][k]
    int32_t *pos;      // [B*Hh][k]
    size_t kv_bytes;   // bytes of the K (= V) region
};

static inline int h2o_esize(int dtype) { return dtype == H2O_F32 ? 4 : 2; }
static inline int h2o_row_bytes(const h2o_config &c)
{
    return c.kv_bits == 4 ? H2O_Q4_ROW_BYTES(c.head_dim) : c.head_dim * h2o_esize(c.dtype);
}
static inline double h2o_scale_of(const h2o_config &c)
{
    return c.scale != 0.0f ? (double)c.scale : 1.0 / sqrt((double)c.head_dim);
}

// ---- kernel launchers (each enqueues on `st` and returns hipGetLastError()) ----
hipError_t h2o_launch_mark_free(const h2o_cache &c, hipStream_t st);
hipError_t h2o_launch_decode(const h2o_cache &c, const void *q, const void *k_new,
                             const void *v_new, void *out, hipStream_t st);
// the same step over a cache that stores 4-bit codes
hipError_t h2o_launch_decode_q4(const h2o_cache &c, const void *q, const void *k_new,
                                const void *v_new, void *out, hipStream_t st);
// prompt scoring: the nq queries (rows of Q) are the last nq positions of the nk
// keys; lse [B*Hh][nq] = log2 of the row normalisers, colsum [B*Hh][nk]
hipError_t h2o_launch_prefill_lse(const h2o_config &cfg, double scale, const void *Q,
                                  const void *K, int nq, int nk, float *lse, hipStream_t st);
hipError_t h2o_launch_prefill_colsum(const h2o_config &cfg, double scale, const void *Q,
                                     const void *K, int nq, int nk, const float *lse,
                                     float *colsum, hipStream_t st);
// causal attention of nq queries (the last nq of nk key positions) over nk keys: V
// ([nk][d] per head) is transposed into `vt` (h2o_attn_vt_bytes(cfg, nk) bytes),
// `lse2` receives log2 of every row's normaliser of exp2(scale*log2(e)*<q,k>),
// `lse_nat` (nullable) the natural-log row log-sum-exp; 16-bit element types only
size_t h2o_attn_vt_bytes(const h2o_config &cfg, int nk);
hipError_t h2o_launch_prefill_attention(const h2o_config &cfg, double scale, const void *Q,
                                        const void *K, const void *V, int nq, int nk, void *vt,
                                        float *lse2, float *lse_nat, void *out, hipStream_t st);
// compression of n candidates per head (entry j: position pos_in[j] or j, score
// base[j] + score[j] or score[j]) into the cache; t_new = tokens seen afterwards
hipError_t h2o_launch_select_gather(const h2o_cache &c, const void *K, const void *V,
                                    const float *score, const float *base, const int32_t *pos_in,
                                    int n, int t_new, hipStream_t st);
// the n_occ cached tokens in position order followed by the m chunk tokens as one
// candidate list; `order` (heads * k ints of scratch) is needed when the slots are
// not in position order, nullptr when they are
hipError_t h2o_launch_concat(const h2o_cache &c, const void *Kn, const void *Vn, int m, int n_occ,
                             int32_t *order, void *Kcat, void *Vcat, float *base, int32_t *pos_cat,
                             hipStream_t st);

// rolled[B*Hh][k]: rank of every occupied slot's token among the cached tokens by position
hipError_t h2o_launch_rolled_positions(const h2o_cache &c, int32_t *rolled, hipStream_t st);

// flags[B*Hh]: 0 for a head whose bookkeeping is consistent, else a bit mask (h2o.h)
hipError_t h2o_launch_validate(const h2o_cache &c, int32_t *flags, hipStream_t st);

// ---- element types ----------------------------------------------------------
// Raw storage views: f32 -> float, f16 -> _Float16, bf16 -> uint16_t bit pattern.
template <int DT> struct Elem;
template <> struct Elem<H2O_F32> {
    using T = float;
    static constexpr int EPL = 4;   // elements per 16-byte lane load
    __device__ static inline float to_f(T v) { return v; }
    __device__ static inline T from_f(float v) { return v; }
};
template <> struct Elem<H2O_F16> {
    using T = _Float16;
    static constexpr int EPL = 8;
    __device__ static inline float to_f(T v) { return (float)v; }
    __device__ static inline T from_f(float v) { return (T)v; }   // round-to-nearest-even
};
template <> struct Elem<H2O_BF16> {
    using T = uint16_t;
    static constexpr int EPL = 8;
    __device__ static inline float to_f(T v) { return __uint_as_float(((uint32_t)v) << 16); }
    __device__ static inline T from_f(float v)
    {
        uint32_t u = __float_as_uint(v);
        if ((u & 0x7fffffffu) > 0x7f800000u) return (T)((u >> 16) | 0x40u);   // NaN stays NaN
        u += 0x7fffu + ((u >> 16) & 1u);                                      // nearest-even
        return (T)(u >> 16);
    }
};
