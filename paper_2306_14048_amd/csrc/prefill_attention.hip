// Causal attention over the prompt on gfx950 (MFMA), with the row statistics
// that the column-sum pass needs as a by-product.  The nq queries are the last
// nq of nk key positions (nq = nk: the whole prompt; nq < nk: a chunk of the
// prompt attending to cached tokens in front of it): query i sees keys
// j <= nk - nq + i.
//
// The prompt phase of H2O is ordinary full attention over the prompt (App. A,
// generation commentary: the prompt is processed with the full cache and only
// then compressed); the accumulated scores are the column sums of the same
// softmax matrix (Algorithm 2's accumulate line over the prompt rows).  A layer
// therefore needs  O = softmax(scale * Q K^T) V  anyway, and the log-sum-exp of
// every row falls out of it: with this kernel the scoring costs one extra
// matrix pass (the column sums) instead of two.
//
// Shape of the computation.  A workgroup of 8 waves owns 256 queries (32 per
// wave, kept in registers as MFMA B-operand fragments) and streams 64-key
// tiles.  Per tile and wave:
//     S^T (keys x queries)  = K_tile . Q^T          16 MFMAs 32x32x16
//     online softmax over the keys seen so far (per query = per lane)
//     O^T (dims x queries) += V^T_tile . P^T        16 MFMAs 32x32x16 (d = 128)
// In the 32x32 result layout a lane holds ONE query's products with 16 keys
// (S^T) or 16 output dims (O^T): row maximum, normaliser and the rescaling of
// the output accumulator are per-lane scalars; the only cross-lane traffic is
// one exchange of the tile maximum between the two lane halves that share a
// query.  V is needed with the key index innermost (A operand of the second
// product); it is transposed once per call into the workspace ([head][d][n],
// zero padded to whole tiles), after which its tiles are copied and read
// exactly like key tiles.  The key rows of a tile are visited in an order that
// makes the 8 probabilities a lane holds for one MFMA step belong to 8
// consecutive keys, so P^T goes from the accumulator registers into the second
// product without any shuffle and the V^T fragment is one 128-bit LDS read.
//
// Schedule: as in the scoring passes, two groups of four waves run one barrier
// apart; one group's matrix phase (P.V of the previous tile, then Q.K of this
// one: 32 MFMAs) overlaps the other group's vector phase (softmax of its tile).
#include "h2o_internal.h"
#include "lds_copy.h"
#include <type_traits>

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

template <int DT>
__device__ inline f32x16 mma16(const uint4 &a, const uint4 &b, f32x16 acc)
{
    if constexpr (DT == H2O_BF16) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(
            *reinterpret_cast<const bf16x8 *>(&a), *reinterpret_cast<const bf16x8 *>(&b), acc, 0, 0, 0);
    } else {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(
            *reinterpret_cast<const f16x8 *>(&a), *reinterpret_cast<const f16x8 *>(&b), acc, 0, 0, 0);
    }
}

// two floats -> one register of two 16-bit values (round to nearest even)
template <int DT> __device__ inline unsigned pack2(float a, float b)
{
    const f32x2 v = {a, b};
    if constexpr (DT == H2O_BF16) {
        const bf16x2 h = __builtin_convertvector(v, bf16x2);
        return *reinterpret_cast<const unsigned *>(&h);
    } else {
        const f16x2 h = __builtin_convertvector(v, f16x2);
        return *reinterpret_cast<const unsigned *>(&h);
    }
}

// value of the lane that shares this lane's query (lane ^ 32), combined with op
__device__ inline float other_half(float x)
{
    const unsigned own = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(own, own, false, false);
    // one of the two results is this lane's own value, the other the partner's
    return __uint_as_float(r[0] == own ? r[1] : r[0]);
}

constexpr int ANW = 8;       // waves per workgroup
constexpr int ANS = 3;       // stages (key tile + value tile each); copies run two tiles ahead
constexpr int ABN = 64;      // keys per tile

// ---- V -> V^T ([head][n][d] -> [head][d][npad]), zero padded ----------------------
template <int D>
__global__ __launch_bounds__(256) void transpose_v_kernel(const uint16_t *__restrict__ V,
                                                          uint16_t *__restrict__ Vt, int n, int npad)
{
    // rows go into LDS in 32-bit pieces; the pitch of D + 2 elements (an odd number of
    // words) spreads the column reads below over the banks
    constexpr int PITCH = D + 2;
    __shared__ __align__(4) uint16_t tile[ABN * PITCH];
    const int head = blockIdx.x, j0 = blockIdx.y * ABN, tid = threadIdx.x;
    const uint16_t *Vh = V + (size_t)head * n * D;
    uint16_t *Vth = Vt + (size_t)head * D * npad;
    constexpr int CPR = D / 8;                       // 16-byte chunks per row
    for (int q = tid; q < ABN * CPR; q += 256) {
        const int r = q / CPR, c = q % CPR;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (j0 + r < n) v = *reinterpret_cast<const uint4 *>(Vh + (size_t)(j0 + r) * D + c * 8);
        unsigned *dst = reinterpret_cast<unsigned *>(tile + r * PITCH + c * 8);
        dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
    }
    __syncthreads();
    for (int q = tid; q < D * (ABN / 8); q += 256) {
        const int d = q / (ABN / 8), c = q % (ABN / 8);
        uint16_t e[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) e[i] = tile[(c * 8 + i) * PITCH + d];
        *reinterpret_cast<uint4 *>(Vth + (size_t)d * npad + j0 + c * 8) = *reinterpret_cast<const uint4 *>(e);
    }
}

// ---- attention -------------------------------------------------------------------
template <int DT, int D>
__global__ __launch_bounds__(ANW * 64, 2) void prefill_attn_kernel(
    const char *__restrict__ Qg, const char *__restrict__ Kg, const char *__restrict__ Vtg, int nq,
    int nk, int npad, int heads, float c2, float *__restrict__ lse2, float *__restrict__ lse_nat,
    char *__restrict__ Og)
{
    const int off = nk - nq;               // key position of query 0
    constexpr int ROWB = D * 2;            // bytes per Q/K row
    constexpr int NF = ROWB / 32;          // 16-byte fragments per row per lane half
    constexpr int MB = ABN / 32;           // 32-key blocks per tile
    constexpr int NDB = D / 32;            // 32-dim blocks of the output
    constexpr int KS = ABN / 16;           // MFMA steps of the second product per tile
    constexpr int TILEK = ABN * ROWB;      // key tile bytes
    constexpr int VROWB = ABN * 2;         // bytes per V^T tile row (128)
    constexpr int TILEV = D * VROWB;       // value tile bytes
    constexpr int STAGE = TILEK + TILEV;
    // XOR swizzle of 16-byte chunks inside a row (see the scoring passes)
    constexpr int CPRK = ROWB / 16, RSHK = ROWB >= 256 ? 0 : 1, KMASKK = (CPRK < 16 ? CPRK : 16) - 1;
    constexpr int CPRV = VROWB / 16, RSHV = 1, KMASKV = CPRV - 1;
    constexpr int NT = ANW * 64;
    constexpr int SROWS = ANW * 32;
    constexpr int CPTK = ABN * CPRK / NT, CPTV = D * CPRV / NT;
    constexpr int CPF = CPTK + CPTV;       // copy instructions per wave per stage
    static_assert(ABN * CPRK % NT == 0 && D * CPRV % NT == 0 && CPTK >= 1 && CPTV >= 1, "copy split");

    extern __shared__ __align__(16) unsigned char smem[];   // [ANS][STAGE]

    const int tid = threadIdx.x, lane = tid & 63;
    // (the wave index as a scalar: branches on it are then uniform for the compiler
    // too, which otherwise keeps a second copy of the accumulators around them)
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;
    const int grp = wave >> 2;
    const int nblk = (nq + SROWS - 1) / SROWS;
    // a head lives on one XCD (one L2); heaviest (last) row blocks first
    constexpr int HG = 8;
    const int xcd = blockIdx.x & 7, turn = blockIdx.x >> 3;
    const int group = turn / (HG * nblk), idx = turn % (HG * nblk);
    const int head = (group * HG + idx % HG) * 8 + xcd;
    if (head >= heads) return;
    const int blk = nblk - 1 - idx / HG;
    const int s0 = blk * SROWS;
    const char *Qh = Qg + (size_t)head * nq * ROWB;
    const char *Kh = Kg + (size_t)head * nk * ROWB;
    const char *Vth = Vtg + (size_t)head * D * npad * 2;

    const int srow = s0 + wave * 32 + l32;           // this lane's query
    uint4 st[NF];
#pragma unroll
    for (int f = 0; f < NF; ++f)
        st[f] = *reinterpret_cast<const uint4 *>(Qh + (size_t)min(srow, nq - 1) * ROWB + (2 * f + half) * 16);
    if (srow >= nq) {
#pragma unroll
        for (int f = 0; f < NF; ++f) st[f] = make_uint4(0, 0, 0, 0);
    }

    // key tiles of this block (>= 1): up to the one that holds the last query's own key
    const int T = min((nk + ABN - 1) / ABN, (off + s0 + SROWS + ABN - 1) / ABN);

    // copy plan: instruction c of wave w fills LDS chunks [(c*ANW + w)*64, +64)
    unsigned koff[CPTK], kchunk[CPTK], voff[CPTV];
#pragma unroll
    for (int c = 0; c < CPTK; ++c) {
        const unsigned q = (unsigned)(c * ANW + wave) * 64u + lane;
        const unsigned r = q / CPRK, pos = q % CPRK;
        koff[c] = r * ROWB;
        kchunk[c] = (pos ^ ((r >> RSHK) & KMASKK)) * 16u;
    }
#pragma unroll
    for (int c = 0; c < CPTV; ++c) {
        const unsigned q = (unsigned)(c * ANW + wave) * 64u + lane;
        const unsigned r = q / CPRV, pos = q % CPRV;
        voff[c] = r * (unsigned)npad * 2u + (pos ^ ((r >> RSHV) & KMASKV)) * 16u;
    }
    const i32x4 rsrc_k = make_rsrc(Kh, (unsigned)nk * ROWB);
    const i32x4 rsrc_v = make_rsrc(Vth, (unsigned)D * (unsigned)npad * 2u);
    const unsigned lds_w = __builtin_amdgcn_readfirstlane(
        (unsigned)reinterpret_cast<size_t>(smem) + wave * 1024);
    const unsigned last_row_off = (unsigned)(nk - 1) * ROWB;
    // stage u holds what matrix phase u reads: key tile u and value tile u-1
    // (indices clamped to existing tiles: the first stage's value tile and the
    // last stage's key tile are never read)
    auto fetch = [&](int u, int stg) {
        const int kt = min(u, T - 1), vt = min(max(u - 1, 0), T - 1);
        const unsigned t0 = (unsigned)kt * (ABN * ROWB);
        const unsigned base = lds_w + stg * STAGE;
        if (t0 + ABN * ROWB <= (unsigned)nk * ROWB) {
#pragma unroll
            for (int c = 0; c < CPTK; ++c) dma16(rsrc_k, koff[c] + kchunk[c], t0, base + c * ANW * 1024);
        } else {                                       // ragged last tile: rows past nk repeat row nk-1
#pragma unroll
            for (int c = 0; c < CPTK; ++c)
                dma16(rsrc_k, min(t0 + koff[c], last_row_off) + kchunk[c], 0u, base + c * ANW * 1024);
        }
#pragma unroll
        for (int c = 0; c < CPTV; ++c)
            dma16(rsrc_v, voff[c], (unsigned)vt * VROWB, base + TILEK + c * ANW * 1024);
    };

    // LDS read offsets.  Key rows are visited so that MFMA row 16a + 8b + 4c + e
    // of a 32-row block is key 16a + 8c + 4b + e (bits 2 and 3 exchanged): the
    // accumulator registers 8s..8s+7 of lane half h then hold keys
    // 16s + 8h + (0..7) of the block, which is exactly what the second
    // product's B operand needs.
    const int krow = (l32 & ~12) | ((l32 & 4) << 1) | ((l32 & 8) >> 1);
    unsigned ka[NF][MB], va[NDB][KS];
#pragma unroll
    for (int f = 0; f < NF; ++f)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const int row = mb * 32 + krow;
            ka[f][mb] = row * ROWB + (((2 * f + half) ^ ((row >> RSHK) & KMASKK)) * 16);
        }
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int row = db * 32 + l32;
            va[db][ks] = TILEK + row * VROWB + (((2 * ks + half) ^ ((row >> RSHV) & KMASKV)) * 16);
        }

    float m_run = -INFINITY, l_run = 0.f;   // running maximum of the raw products / normaliser part
    f32x16 oacc[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[db][v] = 0.f;
    uint4 pfrag[KS];                        // probabilities of the previous tile, packed 16-bit
    bool live_prev = false;

    fetch(0, 0);
    fetch(1, 1);
    dma_wait_upto<CPF>();
#pragma unroll
    for (int f = 0; f < NF; ++f)
        asm volatile("" ::"v"(st[f].x), "v"(st[f].y), "v"(st[f].z), "v"(st[f].w));
    wg_barrier();
    if (grp == 1) wg_barrier();            // second group runs one phase behind

    int stg = 0;
    // Iteration u: matrix phase = P.V of tile u-1 and Q.K of tile u, vector phase
    // = softmax of tile u.  MASKED: tile u touches the diagonal of this block's
    // rows; LAST: u == T (only the trailing P.V).
    auto step = [&](int u, auto masked_tag, auto last_tag) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        constexpr bool LAST = decltype(last_tag)::value;
        fetch(u + 2, stg == 0 ? ANS - 1 : stg - 1);          // into the stage of iteration u-1
        const unsigned char *sb = smem + stg * STAGE;
        const int r0 = u * ABN;
        const int w0 = s0 + wave * 32;
        // keys r0.. are visible to this wave only if r0 <= its last query
        const bool live = !LAST && (!MASKED || r0 <= off + w0 + 31);
        f32x16 sacc[MB];
        __builtin_amdgcn_s_setprio(2);
        // Only one wave per SIMD is in its matrix phase, so nothing else hides the
        // LDS latency of its operand reads: they run PF fragments ahead of the
        // MFMAs that use them (a ring of PF registers quadruples).
        constexpr int PF = 4;
        if (live_prev) {
            constexpr int N = KS * NDB;
            uint4 ring[PF];
#pragma unroll
            for (int i = 0; i < PF; ++i)
                ring[i] = *reinterpret_cast<const uint4 *>(sb + va[i % NDB][i / NDB]);
#pragma unroll
            for (int i = 0; i < N; ++i) {
                const int ks = i / NDB, db = i % NDB;
                __builtin_amdgcn_sched_barrier(0);      // keep the reads PF ahead (the scheduler would pull them back)
                oacc[db] = mma16<DT>(ring[i % PF], pfrag[ks], oacc[db]);
                if (i + PF < N)
                    ring[i % PF] = *reinterpret_cast<const uint4 *>(sb + va[(i + PF) % NDB][(i + PF) / NDB]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (live) {
            constexpr int N = NF * MB;
            uint4 ring[PF];
#pragma unroll
            for (int i = 0; i < PF; ++i)
                ring[i] = *reinterpret_cast<const uint4 *>(sb + ka[i / MB][i % MB]);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int v = 0; v < 16; ++v) sacc[mb][v] = 0.f;
#pragma unroll
            for (int i = 0; i < N; ++i) {
                const int f = i / MB, mb = i % MB;
                __builtin_amdgcn_sched_barrier(0);
                sacc[mb] = mma16<DT>(ring[i % PF], st[f], sacc[mb]);
                if (i + PF < N)
                    ring[i % PF] = *reinterpret_cast<const uint4 *>(sb + ka[(i + PF) / MB][(i + PF) % MB]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        __builtin_amdgcn_s_setprio(0);
        dma_wait_upto<CPF>();
        wg_barrier();

        if (live) {
            if constexpr (MASKED) {
                // a wave whose 32 queries all see the whole tile needs no mask (wave-uniform)
                if (r0 + ABN - 1 > off + w0) {
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int j = r0 + mb * 32 + 16 * (v >> 3) + 8 * half + (v & 7);
                            if (j > off + srow) sacc[mb][v] = -INFINITY;
                        }
                }
            }
            float mx = m_run;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int v = 0; v < 16; v += 2) mx = fmaxf(fmaxf(mx, sacc[mb][v]), sacc[mb][v + 1]);
            mx = fmaxf(mx, other_half(mx));              // both halves of a query use one reference
            // mx is finite from the first tile on: key 0 is visible to every query
            if (__builtin_amdgcn_ballot_w64(mx > m_run) != 0) {      // rescale only when a maximum moved
                float alpha = __builtin_amdgcn_exp2f((m_run - mx) * c2);         // 0 on the first tile
                l_run *= alpha;
                // in place (written as an instruction so that the branch leaves the
                // accumulator in the registers it already occupies).  The compiler does
                // not see what an asm statement reads, so the wait states a consumer of
                // a transcendental result needs are spelled out here.
                asm volatile("s_nop 4" : "+v"(alpha));
#pragma unroll
                for (int db = 0; db < NDB; ++db)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        asm volatile("v_mul_f32 %0, %0, %1" : "+v"(oacc[db][v]) : "v"(alpha));
                m_run = mx;
            }
            const float nms = -m_run * c2;
            float sum0 = 0.f, sum1 = 0.f;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    float p[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        p[e] = __builtin_amdgcn_exp2f(fmaf(sacc[mb][8 * s + e], c2, nms));
                    sum0 += (p[0] + p[2]) + (p[4] + p[6]);
                    sum1 += (p[1] + p[3]) + (p[5] + p[7]);
                    pfrag[2 * mb + s] = make_uint4(pack2<DT>(p[0], p[1]), pack2<DT>(p[2], p[3]),
                                                   pack2<DT>(p[4], p[5]), pack2<DT>(p[6], p[7]));
                }
            l_run += sum0 + sum1;
        }
        live_prev = live;
        stg = stg == ANS - 1 ? 0 : stg + 1;
        dma_wait_upto<CPF>();
        wg_barrier();
    };
    {
        const int t_diag0 = min(T, (off + s0 + 1) / ABN);   // tiles every query of the block sees in full
        for (int u = 0; u < t_diag0; ++u) step(u, std::false_type{}, std::false_type{});
        for (int u = t_diag0; u < T; ++u) step(u, std::true_type{}, std::false_type{});
        step(T, std::false_type{}, std::true_type{});
    }
    if (grp == 0) wg_barrier();
    dma_wait_upto<0>();                    // trailing requests land before the LDS is released

    // ---- normalise and store ------------------------------------------------------
    const float l_tot = l_run + other_half(l_run);
    const float inv = 1.0f / l_tot;
    if (srow < nq) {
        using E = Elem<DT>;
        typename E::T *orow = reinterpret_cast<typename E::T *>(Og) + ((size_t)head * nq + srow) * D;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                typename E::T o4[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) o4[e] = E::from_f(oacc[db][4 * g + e] * inv);
                *reinterpret_cast<uint2 *>(orow + 32 * db + 8 * g + 4 * half) = *reinterpret_cast<const uint2 *>(o4);
            }
        if (half == 0) {
            const float l2 = m_run * c2 + __builtin_amdgcn_logf(l_tot);      // log2 of the row's normaliser
            lse2[(size_t)head * nq + srow] = l2;
            if (lse_nat) lse_nat[(size_t)head * nq + srow] = l2 * 0.69314718055994531f;
        }
    }
}

template <int DT, int D>
hipError_t launch_attn(const h2o_config &cfg, double scale, const void *Q, const void *K,
                       const void *V, int nq, int nk, void *vt, float *lse2, float *lse_nat, void *out,
                       hipStream_t st)
{
    const int heads = cfg.batch * cfg.heads;
    const int npad = (nk + ABN - 1) / ABN * ABN;
    hipLaunchKernelGGL((transpose_v_kernel<D>), dim3(heads, npad / ABN), dim3(256), 0, st,
                       static_cast<const uint16_t *>(V), static_cast<uint16_t *>(vt), nk, npad);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    constexpr size_t smem = (size_t)ANS * (ABN * D * 2 + D * ABN * 2);
    auto kern = prefill_attn_kernel<DT, D>;
    static bool raised = false;
    if (smem > 48 * 1024 && !raised) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        raised = true;
    }
    const int nblk = (nq + ANW * 32 - 1) / (ANW * 32);
    const float c2 = (float)(scale * 1.4426950408889634);
    hipLaunchKernelGGL(kern, dim3((unsigned)((heads + 63) / 64) * 64 * nblk), dim3(ANW * 64), smem, st,
                       static_cast<const char *>(Q), static_cast<const char *>(K),
                       static_cast<const char *>(vt), nq, nk, npad, heads, c2, lse2, lse_nat,
                       static_cast<char *>(out));
    return hipGetLastError();
}

}  // namespace

size_t h2o_attn_vt_bytes(const h2o_config &cfg, int n)
{
    const size_t npad = ((size_t)n + ABN - 1) / ABN * ABN;
    return (size_t)cfg.batch * cfg.heads * cfg.head_dim * npad * 2;
}

hipError_t h2o_launch_prefill_attention(const h2o_config &cfg, double scale, const void *Q,
                                        const void *K, const void *V, int nq, int nk, void *vt,
                                        float *lse2, float *lse_nat, void *out, hipStream_t st)
{
    const int d = cfg.head_dim;
    if (nq < 1 || nq > nk) return hipErrorInvalidValue;
    if (cfg.dtype == H2O_F16)
        return d == 64 ? launch_attn<H2O_F16, 64>(cfg, scale, Q, K, V, nq, nk, vt, lse2, lse_nat, out, st)
                       : launch_attn<H2O_F16, 128>(cfg, scale, Q, K, V, nq, nk, vt, lse2, lse_nat, out, st);
    return d == 64 ? launch_attn<H2O_BF16, 64>(cfg, scale, Q, K, V, nq, nk, vt, lse2, lse_nat, out, st)
                   : launch_attn<H2O_BF16, 128>(cfg, scale, Q, K, V, nq, nk, vt, lse2, lse_nat, out, st);
}
