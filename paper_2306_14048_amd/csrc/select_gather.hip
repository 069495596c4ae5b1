// Prompt compression for H2O on gfx950: given one score per prompt token, keep
// the `recent` last tokens plus the `heavy` best-scoring older ones (or all n
// tokens when n fits in the budget) and copy their key/value rows into the
// cache slots in ascending position order (App. A: the prompt phase returns the
// heavy hitters and the recent tokens, or everything for a short prompt).
//
// Selecting the `heavy` largest under the order (score, then position) is the
// same as repeatedly evicting the smallest (score, position) pair, the rule the
// generation steps use.  One workgroup per head: an exact 4x8-bit radix select
// on the order-preserving integer image of the scores finds the threshold, the
// positions of equal-score tokens break the tie at the threshold, a block scan
// assigns slots, then all threads copy rows with 128-bit accesses.
#include "wave_ops.h"

namespace {

constexpr int SG_NT = 512;
constexpr int SG_NW = SG_NT / 64;

__device__ inline unsigned order_key(float x)
{
    const unsigned u = __float_as_uint(x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);   // monotone in x
}

// Exclusive prefix sum of one int per thread over the workgroup; `total`
// receives the sum.  `scratch` holds SG_NW + 1 ints.
__device__ inline int block_exclusive_scan(int v, int *scratch, int &total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int y = __shfl_up(inc, o, 64);
        if (lane >= o) inc += y;
    }
    __syncthreads();                       // scratch may still be read from a previous scan
    if (lane == 63) scratch[wave] = inc;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < SG_NW; ++w) {
        const int s = scratch[w];
        if (w < wave) base += s;
        tot += s;
    }
    total = tot;
    return base + inc - v;
}

// Entry j of a head's n candidates is the token at position pos_in[j] (ascending;
// pos_in == nullptr: position j) with score base[j] + score[j] (base == nullptr:
// score[j]); t_new = number of tokens seen once these are stored.
// QDT < 0: the cache stores rows as they are (ROWB bytes each).  QDT = an element
// type: the cache stores 4-bit codes and the kept rows (ROWB bytes of QDT
// elements) are quantised on their way in.  PAT: built for a sparse-attention
// pattern as the protected set (the recent-window build carries none of that code).
template <int ROWB, int QDT, bool PAT>
__global__ __launch_bounds__(SG_NT) void select_gather_kernel(
    const char *__restrict__ Kp, const char *__restrict__ Vp, const float *__restrict__ score,
    const float *__restrict__ base, const int32_t *__restrict__ pos_in, int n, int t_new,
    char *__restrict__ Kc, char *__restrict__ Vc, float *__restrict__ acc_g,
    int32_t *__restrict__ pos_g, int k, int heavy, int recent, int rank, int protect, int stride)
{
    extern __shared__ __align__(16) unsigned char smem[];
    int *sel_l = reinterpret_cast<int *>(smem);        // [k] slot -> prompt position
    __shared__ unsigned hist[256];
    __shared__ unsigned sh_prefix, sh_need;
    __shared__ int scan_l[SG_NW + 1];

    const int head = blockIdx.x, tid = threadIdx.x;
    const float *sc_in = score + (size_t)head * n;
    const float *bs = base ? base + (size_t)head * n : nullptr;
    const int32_t *pin = pos_in ? pos_in + (size_t)head * n : nullptr;
    const size_t hoff = (size_t)head * k;
    // the score of entry j as it will be stored, and its position
    auto sc_of = [&](int j) { return bs ? bs[j] + sc_in[j] : sc_in[j]; };
    auto pos_of = [&](int j) { return pin ? pin[j] : j; };

    // what ranks an older token: its score, or (averaged ranking) its score over
    // the n - j prompt queries that scored it
    auto ranked = [&](float v, int j) {
        return rank == H2O_RANK_AVERAGED ? __fdiv_rn(v, (float)(t_new - pos_of(j))) : v;
    };

    for (int s = tid; s < k; s += SG_NT) sel_l[s] = -1;

    if (n <= k) {
        __syncthreads();
        for (int s = tid; s < n; s += SG_NT) sel_l[s] = s;
    } else {
        // Which entries compete.  With the recent window (protect 0) the candidates are
        // the entries in front of the last `recent` positions; positions ascend, so they
        // are a prefix [0, older) and `heavy` of them are kept.  With a sparse-attention
        // pattern as the protected set, the entries the pattern covers for the last
        // query (position t_new - 1) are kept and the best of the others fill the budget;
        // should it cover more than the budget, the covered entries compete for all
        // k slots and the others are dropped (the rule "evict one at a time, protection
        // void once everything left is covered", in one shot).
        int older = n - recent;
        bool overflow = false;
        int want = heavy;                              // candidates to keep
        auto covered = [&](int j) { return is_protected(pos_of(j), t_new - 1, recent, protect, stride); };
        if constexpr (PAT) {
            int cnt = 0;
            for (int j = tid; j < n; j += SG_NT) cnt += covered(j);
            int total;
            block_exclusive_scan(cnt, scan_l, total);
            overflow = total > k;
            want = overflow ? k : k - total;
            __syncthreads();
        } else if (pin) {
            int cnt = 0;
            for (int j = tid; j < n; j += SG_NT) cnt += pin[j] < t_new - recent;
            int total;
            block_exclusive_scan(cnt, scan_l, total);
            older = total;
            __syncthreads();
        }
        auto is_cand = [&](int j) {
            if constexpr (PAT) return covered(j) == overflow;
            else return j < older;
        };
        auto always = [&](int j) {
            if constexpr (PAT) return !overflow && covered(j);
            else return j >= older;
        };
        const int cand_end = PAT ? n : older;          // candidates lie in [0, cand_end)
        unsigned thr = 0, need = 0;                    // keep keys > thr, and `need` of those == thr
        if (want > 0) {
            // radix select: the want-th largest key among the candidates (there are more
            // than `want` of them: n exceeds the budget)
            unsigned prefix = 0, mask = 0;
            need = (unsigned)want;
            for (int shift = 24; shift >= 0; shift -= 8) {
                for (int b = tid; b < 256; b += SG_NT) hist[b] = 0;
                __syncthreads();
                for (int j = tid; j < cand_end; j += SG_NT) {
                    if (!is_cand(j)) continue;
                    const unsigned key = order_key(ranked(sc_of(j), j));
                    if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
                }
                __syncthreads();
                // the bin in which the count from the top reaches `need`: thread r looks
                // at bin 255 - r, the scan gives it the count of all higher bins
                {
                    const int bin = 255 - tid;
                    const int cnt = tid < 256 ? (int)hist[bin] : 0;
                    int total;
                    const int above = block_exclusive_scan(cnt, scan_l, total);
                    if (tid < 256 && (unsigned)above < need && (unsigned)(above + cnt) >= need) {
                        sh_prefix = prefix | ((unsigned)bin << shift);
                        sh_need = need - (unsigned)above;   // still needed inside that bin
                    }
                }
                __syncthreads();
                prefix = sh_prefix;
                need = sh_need;
                mask |= 255u << shift;
                __syncthreads();
            }
            thr = prefix;
        }
        // each thread owns a contiguous run of positions so that ranks follow position order
        const int per = (n + SG_NT - 1) / SG_NT;
        const int j0 = min(n, tid * per), j1 = min(n, j0 + per);
        int eq_cnt = 0;
        if (want > 0)
            for (int j = j0; j < min(j1, cand_end); ++j)
                eq_cnt += is_cand(j) && order_key(ranked(sc_of(j), j)) == thr;
        int eq_total;
        int eq_before = block_exclusive_scan(eq_cnt, scan_l, eq_total);
        // among equal scores the higher positions are kept: the last `need` of them
        const int eq_first_kept = eq_total - (int)need;
        auto kept = [&](int j, int &e) {
            if (always(j)) return true;
            if (want <= 0 || !is_cand(j)) return false;
            const unsigned key = order_key(ranked(sc_of(j), j));
            if (key > thr) return true;
            if (key == thr) { const bool keep = e >= eq_first_kept; ++e; return keep; }
            return false;
        };
        int keep_cnt = 0;
        {
            int e = eq_before;
            for (int j = j0; j < j1; ++j) keep_cnt += kept(j, e);
        }
        int kept_total;
        int slot = block_exclusive_scan(keep_cnt, scan_l, kept_total);
        {
            int e = eq_before;
            for (int j = j0; j < j1; ++j)
                if (kept(j, e)) { if (slot < k) sel_l[slot] = j; ++slot; }
        }
    }
    __syncthreads();

    // bookkeeping of every slot
    for (int s = tid; s < k; s += SG_NT) {
        const int j = sel_l[s];
        pos_g[hoff + s] = j >= 0 ? pos_of(j) : -1;
        acc_g[hoff + s] = j >= 0 ? sc_of(j) : 0.f;
    }
    if constexpr (QDT >= 0) {
        // quantising gather: D/8 lanes per row, 8 elements each; an aligned group of 8
        // lanes is one group of 64 elements
        using T = typename Elem<QDT>::T;
        constexpr int D = ROWB / (int)sizeof(T);
        constexpr int QL = D / 8;
        constexpr int CODEB = D / 2;
        constexpr unsigned QROWB = H2O_Q4_ROW_BYTES(D);
        constexpr int RPR = SG_NT / QL;              // rows per round
        const int l = tid % QL, rsub = tid / QL;
        const size_t pbase = (size_t)head * n * ROWB;
        typedef float f32x2 __attribute__((ext_vector_type(2)));
        // every lane runs every round (the reductions inside the quantiser span lanes)
        for (int s0 = 0; s0 < k; s0 += RPR) {
            const int s = s0 + rsub;
            const int j = s < k ? sel_l[s] : -1;
            const size_t off = pbase + (size_t)max(j, 0) * ROWB;
            float kx[8], vx[8];
            load8<QDT>(reinterpret_cast<const T *>(Kp + off) + l * 8, kx);
            load8<QDT>(reinterpret_cast<const T *>(Vp + off) + l * 8, vx);
            float ks, km, vs, vm;
            const unsigned kw = q4_quantise8(kx, ks, km);
            const unsigned vw = q4_quantise8(vx, vs, vm);
            if (j >= 0) {
                char *kr = Kc + (hoff + s) * QROWB, *vr = Vc + (hoff + s) * QROWB;
                *reinterpret_cast<unsigned *>(kr + l * 4) = kw;
                *reinterpret_cast<unsigned *>(vr + l * 4) = vw;
                if ((l & 7) == 0) {
                    *reinterpret_cast<f32x2 *>(kr + CODEB + (l / 8) * 8) = f32x2{ks, km};
                    *reinterpret_cast<f32x2 *>(vr + CODEB + (l / 8) * 8) = f32x2{vs, vm};
                }
            }
        }
        return;
    }
    // gather rows: LPR lanes copy one row of ROWB bytes
    constexpr int LPR = ROWB / 16;
    constexpr int ROWS_PER_ROUND = SG_NT / LPR;
    const int li = tid % LPR, rsub = tid / LPR;
    const size_t pbase = (size_t)head * n * ROWB;
    // four rows per thread in flight (unconditional loads of a clamped row, so that
    // the requests of a batch leave back to back)
    constexpr int UNR = 4;
    for (int s0 = rsub; s0 < k; s0 += UNR * ROWS_PER_ROUND) {
        int j[UNR];
        uint4 kv[UNR], vv[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int s = s0 + u * ROWS_PER_ROUND;
            j[u] = s < k ? sel_l[s] : -1;
            const size_t off = pbase + (size_t)max(j[u], 0) * ROWB + li * 16;
            kv[u] = *reinterpret_cast<const uint4 *>(Kp + off);
            vv[u] = *reinterpret_cast<const uint4 *>(Vp + off);
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int s = s0 + u * ROWS_PER_ROUND;
            if (j[u] >= 0) {
                *reinterpret_cast<uint4 *>(Kc + (hoff + s) * ROWB + li * 16) = kv[u];
                *reinterpret_cast<uint4 *>(Vc + (hoff + s) * ROWB + li * 16) = vv[u];
            }
        }
    }
}

__global__ void mark_free_kernel(float *__restrict__ acc, int32_t *__restrict__ pos, size_t count)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) { acc[i] = 0.f; pos[i] = -1; }
}

// Slot 0 of every head is what a step on an empty cache reads in place of the
// rows that do not exist yet (with weight zero): it must hold finite numbers.
__global__ void zero_first_rows_kernel(char *__restrict__ K, char *__restrict__ V, int k, int rowb)
{
    const size_t base = (size_t)blockIdx.x * k * rowb;
    for (int b = threadIdx.x * 4; b < rowb; b += blockDim.x * 4) {
        *reinterpret_cast<unsigned *>(K + base + b) = 0u;
        *reinterpret_cast<unsigned *>(V + base + b) = 0u;
    }
}

}  // namespace

hipError_t h2o_launch_mark_free(const h2o_cache &c, hipStream_t st)
{
    const size_t count = (size_t)c.cfg.batch * c.cfg.heads * c.k;
    const unsigned blocks = (unsigned)((count + 255) / 256);
    hipLaunchKernelGGL(mark_free_kernel, dim3(blocks), dim3(256), 0, st, c.acc, c.pos, count);
    hipLaunchKernelGGL(zero_first_rows_kernel, dim3(c.cfg.batch * c.cfg.heads), dim3(64), 0, st,
                       c.K, c.V, c.k, c.rowb);
    return hipGetLastError();
}

hipError_t h2o_launch_select_gather(const h2o_cache &c, const void *K, const void *V,
                                    const float *score, const float *base, const int32_t *pos_in,
                                    int n, int t_new, hipStream_t st)
{
    const int heads = c.cfg.batch * c.cfg.heads;
    const int rowb = c.cfg.head_dim * c.esize;
    const size_t smem = (size_t)c.k * sizeof(int);
    const char *Kp = static_cast<const char *>(K), *Vp = static_cast<const char *>(V);
#define H2O_SG_ARGS                                                                             \
    dim3(heads), dim3(SG_NT), smem, st, Kp, Vp, score, base, pos_in, n, t_new, c.K, c.V, c.acc,     \
        c.pos, c.k, c.cfg.heavy, c.cfg.recent, c.cfg.rank, c.cfg.protect, c.cfg.stride
#define H2O_SG(RB, QDT)                                                                         \
    do {                                                                                        \
        if (c.cfg.protect == H2O_PROTECT_RECENT)                                                \
            hipLaunchKernelGGL((select_gather_kernel<RB, QDT, false>), H2O_SG_ARGS);            \
        else                                                                                    \
            hipLaunchKernelGGL((select_gather_kernel<RB, QDT, true>), H2O_SG_ARGS);             \
    } while (0)
    if (c.cfg.kv_bits == 4) {
        const int d = c.cfg.head_dim;
        switch (c.cfg.dtype) {
        case H2O_F32: if (d == 64) H2O_SG(256, H2O_F32); else H2O_SG(512, H2O_F32); break;
        case H2O_F16: if (d == 64) H2O_SG(128, H2O_F16); else H2O_SG(256, H2O_F16); break;
        default: if (d == 64) H2O_SG(128, H2O_BF16); else H2O_SG(256, H2O_BF16); break;
        }
        return hipGetLastError();
    }
    switch (rowb) {
    case 128: H2O_SG(128, -1); break;
    case 256: H2O_SG(256, -1); break;
    case 512: H2O_SG(512, -1); break;
    default: return hipErrorInvalidValue;
    }
#undef H2O_SG
#undef H2O_SG_ARGS
    return hipGetLastError();
}

// ---- cache + chunk -> one candidate list per head ---------------------------------
//
// Chunked prompt processing treats the n_occ cached tokens (slots in ascending
// position order) followed by the m tokens of the chunk as one sequence of
// ncat = n_occ + m candidates: their K/V rows, the scores they already have
// (zero for the chunk) and their positions are laid out contiguously per head.
// `order` (nullable): order[head][r] = the slot that holds the r-th cached token in
// position order; nullptr = the slots already are in that order.
template <int ROWB>
__global__ __launch_bounds__(256) void concat_kernel(
    const char *__restrict__ Kc, const char *__restrict__ Vc, const float *__restrict__ acc_g,
    const int32_t *__restrict__ pos_g, const int32_t *__restrict__ order, const char *__restrict__ Kn,
    const char *__restrict__ Vn, int k, int n_occ, int m, int t, int blocks_per_head,
    char *__restrict__ Kcat, char *__restrict__ Vcat, float *__restrict__ base,
    int32_t *__restrict__ pos_cat)
{
    constexpr int LPR = ROWB / 16;
    const int head = blockIdx.x / blocks_per_head, ncat = n_occ + m;
    const int row = (blockIdx.x % blocks_per_head) * (256 / LPR) + threadIdx.x / LPR, li = threadIdx.x % LPR;
    if (row >= ncat) return;
    const bool cached = row < n_occ;
    const int slot = cached ? (order ? order[(size_t)head * k + row] : row) : 0;
    const char *ks = cached ? Kc + ((size_t)head * k + slot) * ROWB : Kn + ((size_t)head * m + (row - n_occ)) * ROWB;
    const char *vs = cached ? Vc + ((size_t)head * k + slot) * ROWB : Vn + ((size_t)head * m + (row - n_occ)) * ROWB;
    const size_t o = ((size_t)head * ncat + row) * ROWB + li * 16;
    *reinterpret_cast<uint4 *>(Kcat + o) = *reinterpret_cast<const uint4 *>(ks + li * 16);
    *reinterpret_cast<uint4 *>(Vcat + o) = *reinterpret_cast<const uint4 *>(vs + li * 16);
    if (li == 0) {
        base[(size_t)head * ncat + row] = cached ? acc_g[(size_t)head * k + slot] : 0.f;
        pos_cat[(size_t)head * ncat + row] = cached ? pos_g[(size_t)head * k + slot] : t + (row - n_occ);
    }
}

// Generation steps overwrite evicted slots in place, so slot order stops following
// position order.  order[head][r] = slot of the r-th smallest position among the
// n_occ occupied slots (the first n_occ), by counting: positions are distinct.
__global__ __launch_bounds__(256) void order_slots_kernel(const int32_t *__restrict__ pos_g, int k,
                                                          int n_occ, int32_t *__restrict__ order)
{
    extern __shared__ int32_t pos_l[];
    const size_t hoff = (size_t)blockIdx.x * k;
    for (int s = threadIdx.x; s < n_occ; s += 256) pos_l[s] = pos_g[hoff + s];
    __syncthreads();
    for (int s = threadIdx.x; s < n_occ; s += 256) {
        const int p = pos_l[s];
        int rank = 0;
        for (int j = 0; j < n_occ; ++j) rank += pos_l[j] < p;
        order[hoff + rank] = s;
    }
}

// rolled[head][slot] = how many cached tokens have a smaller position (-1 for a free slot)
__global__ __launch_bounds__(256) void rolled_positions_kernel(const int32_t *__restrict__ pos_g, int k,
                                                               int n_occ, int32_t *__restrict__ rolled)
{
    extern __shared__ int32_t pos_l[];
    const size_t hoff = (size_t)blockIdx.x * k;
    for (int s = threadIdx.x; s < n_occ; s += 256) pos_l[s] = pos_g[hoff + s];
    __syncthreads();
    for (int s = threadIdx.x; s < k; s += 256) {
        int rank = -1;
        if (s < n_occ) {
            const int p = pos_l[s];
            rank = 0;
            for (int j = 0; j < n_occ; ++j) rank += pos_l[j] < p;
        }
        rolled[hoff + s] = rank;
    }
}

hipError_t h2o_launch_rolled_positions(const h2o_cache &c, int32_t *rolled, hipStream_t st)
{
    const int n_occ = c.t < c.k ? c.t : c.k;
    hipLaunchKernelGGL(rolled_positions_kernel, dim3(c.cfg.batch * c.cfg.heads), dim3(256),
                       (size_t)(n_occ > 0 ? n_occ : 1) * sizeof(int32_t), st, c.pos, c.k, n_occ, rolled);
    return hipGetLastError();
}

// flags[head] = bit mask of what is wrong with the head's bookkeeping (0 = consistent):
//   1  a slot below n_occ is free (the occupied slots are not the prefix [0, n_occ))
//   2  a slot from n_occ on is occupied
//   4  a position outside [0, t)
//   8  two slots hold the same position
//  16  a score that is negative (sign bit set), infinite or NaN
__global__ __launch_bounds__(256) void validate_kernel(const int32_t *__restrict__ pos_g,
                                                       const float *__restrict__ acc_g, int k, int n_occ,
                                                       int t, int32_t *__restrict__ flags)
{
    extern __shared__ int32_t pos_l[];
    __shared__ int bad;
    const size_t hoff = (size_t)blockIdx.x * k;
    if (threadIdx.x == 0) bad = 0;
    for (int s = threadIdx.x; s < k; s += 256) pos_l[s] = pos_g[hoff + s];
    __syncthreads();
    int mine = 0;
    for (int s = threadIdx.x; s < k; s += 256) {
        const int p = pos_l[s];
        if (s < n_occ) {
            if (p < 0) mine |= 1;
            else if (p >= t) mine |= 4;
            const unsigned a = __float_as_uint(acc_g[hoff + s]);
            if (a >= 0x7f800000u) mine |= 16;          // sign bit, infinity or NaN
            if (p >= 0)
                for (int j = 0; j < s; ++j) mine |= (pos_l[j] == p) ? 8 : 0;
        } else if (p != -1) {
            mine |= 2;
        }
    }
    if (mine) atomicOr(&bad, mine);                    // LDS atomic
    __syncthreads();
    if (threadIdx.x == 0) flags[blockIdx.x] = bad;
}

hipError_t h2o_launch_validate(const h2o_cache &c, int32_t *flags, hipStream_t st)
{
    const int n_occ = c.t < c.k ? c.t : c.k;
    hipLaunchKernelGGL(validate_kernel, dim3(c.cfg.batch * c.cfg.heads), dim3(256),
                       (size_t)c.k * sizeof(int32_t), st, c.pos, c.acc, c.k, n_occ, c.t, flags);
    return hipGetLastError();
}

hipError_t h2o_launch_concat(const h2o_cache &c, const void *Kn, const void *Vn, int m, int n_occ,
                             int32_t *order, void *Kcat, void *Vcat, float *base, int32_t *pos_cat,
                             hipStream_t st)
{
    const int heads = c.cfg.batch * c.cfg.heads;
    const int rowb = c.cfg.head_dim * c.esize;
    const int ncat = n_occ + m;
    if (order && n_occ > 0) {
        hipLaunchKernelGGL(order_slots_kernel, dim3(heads), dim3(256), (size_t)n_occ * sizeof(int32_t), st,
                           c.pos, c.k, n_occ, order);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    // one-dimensional grid: heads x blocks per head (at most 2^24 x 4352 / 8 < 2^34 is refused below)
#define H2O_CC(RB)                                                                               \
    do {                                                                                         \
        const int bph = (ncat + 256 / (RB / 16) - 1) / (256 / (RB / 16));                        \
        if ((long long)heads * bph > 0x7fffffffLL) return hipErrorInvalidValue;                  \
        hipLaunchKernelGGL((concat_kernel<RB>), dim3((unsigned)(heads * bph)), dim3(256), 0, st, \
                           c.K, c.V, c.acc, c.pos, order, static_cast<const char *>(Kn),         \
                           static_cast<const char *>(Vn), c.k, n_occ, m, c.t, bph,               \
                           static_cast<char *>(Kcat), static_cast<char *>(Vcat), base, pos_cat); \
    } while (0)
    switch (rowb) {
    case 128: H2O_CC(128); break;
    case 256: H2O_CC(256); break;
    case 512: H2O_CC(512); break;
    default: return hipErrorInvalidValue;
    }
#undef H2O_CC
    return hipGetLastError();
}
