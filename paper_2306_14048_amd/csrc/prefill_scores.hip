// Prompt scoring for H2O on gfx950 (MFMA): the column sums of the prompt's
// causal softmax matrix, which seed the accumulated attention scores
// (exact generative process of App. D "Eviction policy"; Algorithm 2's
// accumulate line applied to every prompt row).
//
//   pass 1 (row statistics) : LSE_i = log sum_{j<=i} exp(scale * <Q_i, K_j>)
//   pass 2 (column sums)    : c_j   = sum_{i>=j} exp(scale * <Q_i, K_j> - LSE_i)
//
// Both passes are the same dense contraction QK^T and run on the matrix cores;
// they differ in which operand stays in registers.  A workgroup of NWV waves owns
// 32*NWV "stationary" rows (queries in pass 1, keys in pass 2; 32 per wave, kept
// in registers as MFMA B-operand fragments) and streams tiles of the other
// operand through LDS (double buffered) as A-operand fragments.  Eight waves
// share one streamed tile: the copy into LDS and its address arithmetic are paid
// once per 256 stationary rows, which matters because the matrix pipe, the
// vector ALU (one exponential per product) and the vector memory path are all
// close to saturated by this loop.  With the 32x32 MFMA
// result layout a lane then holds one stationary row's products with 16 streamed
// rows per tile, so the reduction each pass needs (over keys for the row
// statistics, over queries for the column sums) runs inside a lane across the
// whole stream and needs no cross-lane traffic and no atomics; the two lane
// halves are merged once at the end.
//
// Everything is computed in base 2: x = (scale*log2 e) * <q,k>, the stored row
// statistic is log2 of the row's normaliser.
#include "h2o_internal.h"
#include "lds_copy.h"
#include <type_traits>

namespace {

#define CPR_OF(rowb) ((rowb) / 16)

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;


template <int DT>
__device__ inline f32x16 mma(const uint4 &a, const uint4 &b, f32x16 acc)
{
    if constexpr (DT == H2O_BF16) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(
            *reinterpret_cast<const bf16x8 *>(&a), *reinterpret_cast<const bf16x8 *>(&b), acc, 0, 0, 0);
    } else if constexpr (DT == H2O_F16) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(
            *reinterpret_cast<const f16x8 *>(&a), *reinterpret_cast<const f16x8 *>(&b), acc, 0, 0, 0);
    } else {
        const float *af = reinterpret_cast<const float *>(&a);
        const float *bf = reinterpret_cast<const float *>(&b);
#pragma unroll
        for (int e = 0; e < 4; ++e)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(af[e], bf[e], acc, 0, 0, 0);
        return acc;
    }
}

constexpr int NWV = 8;         // waves per workgroup
constexpr int NTB = 3;         // streamed-tile buffers (copies run two tiles ahead)
constexpr int NLB = 4;         // row-statistic buffers (pass 2; read one phase later than the tile)

// DT: element type; D: head_dim; MB: 32-row blocks per streamed tile;
// COLSUM: false = pass 1 (row statistics), true = pass 2 (column sums).
//
// Schedule.  Per streamed tile a wave has a matrix phase (16 MFMAs fed from LDS)
// and a vector phase (scale, exponential and sum of its 32x64 products), about
// equally long.  A SIMD runs both pipes at once only if its waves are in
// different phases, and waves that start together and meet at a barrier per
// tile stay in the same phase.  The eight waves therefore form two groups of
// four (wave w and w+4 sit on the same SIMD) that are kept one phase apart by
// the barriers themselves: the second group enters the loop one barrier late,
// so whenever one group is in its matrix phase the other is in its vector
// phase ("ping-pong").  s_setprio lets the matrix phase win the issue slot.
template <int DT, int D, int MB, bool COLSUM>
__global__ __launch_bounds__(NWV * 64, 4) void prefill_pass_kernel(
    const char *__restrict__ Qg, const char *__restrict__ Kg, int nq, int nk, int heads, float c2,
    float *__restrict__ lse2, float *__restrict__ colsum)
{
    constexpr int ES = DT == H2O_F32 ? 4 : 2;
    constexpr int ROWB = D * ES;          // bytes per row
    constexpr int NF = ROWB / 32;         // 16-byte fragments per row per lane half
    constexpr int BN = 32 * MB;           // streamed rows per tile
    constexpr int LROW = ROWB;            // LDS row pitch (chunks are XOR-swizzled instead of padded)
    constexpr int TILEB = BN * LROW;
    // Swizzle: 16-byte chunk c of tile row r is stored at chunk position
    // c ^ key(r), key = low bits of the row (of the row pair for 128-byte rows,
    // two of which span the banks once), so the 16 or 32 lanes that read the same
    // chunk of consecutive rows hit different banks.
    constexpr int RSH = ROWB >= 256 ? 0 : 1;
    constexpr int KMASK = (CPR_OF(ROWB) < 16 ? CPR_OF(ROWB) : 16) - 1;
    constexpr int CPR = ROWB / 16;        // 16-byte chunks per row
    constexpr int CHUNKS = BN * CPR;      // 16-byte chunks per tile
    constexpr int NT = NWV * 64;          // threads per workgroup
    constexpr int SROWS = NWV * 32;       // stationary rows per workgroup
    constexpr int CPT = CHUNKS / NT;      // tile-copy instructions per wave per tile
    constexpr int CPF = CPT + (COLSUM ? 1 : 0);   // copy instructions per wave per fetch
    constexpr int LPW = BN / NWV;         // row statistics each wave copies per tile
    static_assert(CHUNKS % NT == 0 && CPT >= 1, "every thread moves the same number of chunks");
    static_assert(SROWS % BN == 0 && BN % NWV == 0, "tiles divide the workgroup's rows");

    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char *tile_l = smem;                                        // [NTB][TILEB]
    float *lse_l = reinterpret_cast<float *>(smem + NTB * TILEB);        // [NLB][BN] (pass 2)

    const int tid = threadIdx.x, lane = tid & 63;
    // (the wave index as a scalar: branches on it are then uniform for the compiler too)
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;
    const int grp = wave >> 2;            // ping-pong group
    // The nq queries are the LAST nq positions of the nk keys (nq == nk for a whole
    // prompt; nq < nk when a chunk of new tokens attends to nk - nq cached tokens in
    // front of it): query row i sits at key position off + i and sees keys <= off + i.
    const int off = nk - nq;
    const int ns = COLSUM ? nk : nq;      // stationary rows
    const int nt = COLSUM ? nq : nk;      // streamed rows
    const int nblk = (ns + SROWS - 1) / SROWS;
    // Workgroups are handed to the 8 XCDs round-robin by linear id, and each XCD
    // has its own L2.  All blocks of a head share the streamed operand, so a head
    // lives on ONE XCD (ids that agree modulo 8) and its blocks run close together
    // in time: the operand is then fetched from HBM about once instead of once
    // per block.  On an XCD, heads are taken in groups of HG (about as many
    // workgroups as the XCD holds at once); inside a group the order is by block
    // weight, heaviest first over all its heads, so that the kernel does not end
    // on a few long blocks.
    constexpr int HG = 8;
    const int xcd = blockIdx.x & 7, turn = blockIdx.x >> 3;
    const int group = turn / (HG * nblk), idx = turn % (HG * nblk);
    const int head = (group * HG + idx % HG) * 8 + xcd;
    if (head >= heads) return;                       // padding of the last head group
    const int ord = idx / HG;
    // heaviest blocks first: pass 1's last row block sees every key tile,
    // pass 2's first key block sees every query tile
    const int blk = COLSUM ? ord : nblk - 1 - ord;
    const int s0 = blk * SROWS;
    const char *Sg = (COLSUM ? Kg : Qg) + (size_t)head * ns * ROWB;     // stationary operand
    const char *Tg = (COLSUM ? Qg : Kg) + (size_t)head * nt * ROWB;     // streamed operand

    const int srow = s0 + wave * 32 + l32;           // this lane's stationary row
    // Rows past the end are clamped to the last row (in bounds) and zeroed after arrival.
    uint4 st[NF];
#pragma unroll
    for (int f = 0; f < NF; ++f)
        st[f] = *reinterpret_cast<const uint4 *>(Sg + (size_t)min(srow, ns - 1) * ROWB + (2 * f + half) * 16);
    if (srow >= ns) {
#pragma unroll
        for (int f = 0; f < NF; ++f) st[f] = make_uint4(0, 0, 0, 0);
    }

    const int ntile_all = (nt + BN - 1) / BN;
    // pass 1 streams the keys its last query can see; pass 2 streams the queries
    // from the first one that sees this block's first key
    const int t_begin = COLSUM ? max(0, s0 - off) / BN : 0;
    const int t_end = COLSUM ? ntile_all : min(ntile_all, (off + s0 + SROWS + BN - 1) / BN);

    // Staging of a streamed tile: copy instruction c of wave w fills LDS chunks
    // [(c*NWV + w)*64, +64) of the buffer; lane l's chunk q = that base + l sits in
    // tile row q / CPR at position q % CPR and comes from global chunk
    // (q % CPR) ^ key(row).  A head's operand is < 4 GiB: a 32-bit per-lane offset
    // inside the tile plus the tile's wave-uniform offset.  Rows past the end (only in a
    // ragged last tile) are clamped to the last row; what they hold is never used
    // (both passes mask them).  Pass 2 also copies the tile's BN row statistics,
    // LPW lanes of every wave taking LPW of them, so that every wave issues the
    // same number of copy instructions per tile and one wait count fits all.
    unsigned goff[CPT], gchunk[CPT];
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
        const unsigned q = (unsigned)(c * NWV + wave) * 64u + lane;
        const unsigned r = q / CPR, pos = q % CPR;
        goff[c] = r * ROWB;
        gchunk[c] = ((pos ^ ((r >> RSH) & KMASK)) * 16u);
    }
    const i32x4 rsrc = make_rsrc(Tg, (unsigned)nt * ROWB);
    const i32x4 rsrc_lse = make_rsrc(lse2 + (size_t)head * nq, (unsigned)nq * 4u);
    // the low 32 bits of a generic pointer into LDS are the LDS byte offset
    const unsigned lds_w = __builtin_amdgcn_readfirstlane(
        (unsigned)reinterpret_cast<size_t>(tile_l) + wave * 1024);
    const unsigned lds_lse = (unsigned)reinterpret_cast<size_t>(lse_l);
    const unsigned last_row_off = (unsigned)(nt - 1) * ROWB;
    const bool lse_lane = lane / LPW == wave;        // (lane < BN follows from wave < NWV)
    // i = index of the tile in this block's sequence (selects the buffers)
    auto fetch = [&](int tile, int tb, int lb) {
        const unsigned t0 = (unsigned)tile * (BN * ROWB);
        if (t0 + BN * ROWB <= (unsigned)nt * ROWB) {           // whole tile inside the operand
#pragma unroll
            for (int c = 0; c < CPT; ++c)
                dma16(rsrc, goff[c] + gchunk[c], t0, lds_w + tb * TILEB + c * NWV * 1024);
        } else {
#pragma unroll
            for (int c = 0; c < CPT; ++c)
                dma16(rsrc, min(t0 + goff[c], last_row_off) + gchunk[c], 0u,
                      lds_w + tb * TILEB + c * NWV * 1024);
        }
        if constexpr (COLSUM) {
            // lane l writes LDS word l of the buffer; statistics past nq read as 0
            // (end of the descriptor) or as the next head's and are masked later
            if (lse_lane) dma4(rsrc_lse, (unsigned)lane * 4u, (unsigned)tile * (BN * 4u), lds_lse + lb * (BN * 4));
        }
    };

    float m_run = -INFINITY, l_run = 0.f;   // pass 1: running max / sum (base 2)
    float c_run = 0.f;                      // pass 2: running column sum

    // Every block has at least one tile.  The first two are requested
    // here; waiting for the first also completes the stationary loads above
    // (vector loads finish in order).  Requests past the block's last tile repeat
    // that tile (harmless, keeps the request count per iteration constant).
    fetch(t_begin, 0, 0);
    fetch(min(t_begin + 1, t_end - 1), 1, 1);
    dma_wait_upto<CPF>();
    // tell the compiler that the stationary fragments have arrived (it cannot see
    // the wait above), or it would re-wait for them, and with them for the tile
    // copies in flight, in front of the MFMAs of every iteration
#pragma unroll
    for (int f = 0; f < NF; ++f)
        asm volatile("" ::"v"(st[f].x), "v"(st[f].y), "v"(st[f].z), "v"(st[f].w));
    wg_barrier();
    if (grp == 1) wg_barrier();            // second group runs one phase behind

    int tb = 0, lb = 0;                    // buffers of the current tile
    // One streamed tile.  MASKED = the tile touches the causal diagonal of this
    // workgroup's rows or runs past the prompt's end; those tiles run in loops of
    // their own so that the others (most) carry no masking arithmetic at all.
    // In a diagonal tile a wave whose 32 rows see none of the tile's rows skips
    // the arithmetic (it still copies its share of a later tile and meets the
    // barriers).
    //
    // Buffer life times: the tile two ahead is requested at the start of the
    // matrix phase into the buffer of the previous tile, which both groups have
    // finished reading (the later group's matrix phase of that tile ended at the
    // barrier this group has just passed).  Row statistics are read in the vector
    // phase, one barrier later, hence one buffer more.  Before either barrier a
    // wave waits until only its newest request is outstanding, so that by the
    // barrier in front of any matrix phase every wave's share of that tile has
    // landed.
    auto tile_step = [&](int tile, auto masked_tag) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        const int tb2 = tb == 0 ? NTB - 1 : tb - 1;               // (tb + 2) % 3
        fetch(min(tile + 2, t_end - 1), tb2, (lb + 2) & (NLB - 1));
        const int r0 = tile * BN;
        const int w0 = s0 + wave * 32;            // first stationary row of this wave
        // pass 1: keys r0.. are visible to the queries at positions >= r0; pass 2:
        // the queries up to position off+r0+BN-1 see the keys up to there
        const bool live = !MASKED || (COLSUM ? off + r0 + BN - 1 >= w0 : r0 <= off + w0 + 31);
        // Of the tiles that touch the block's diagonal, a wave's own 32 rows straddle
        // only one; those in front of it are fully visible to the wave and need no
        // mask arithmetic (wave-uniform test).
        const bool clear = COLSUM ? (off + r0 >= w0 + 31 && r0 + BN <= nq) : (r0 + BN - 1 <= off + w0);
        f32x16 acc[MB];
        if (live) {
            __builtin_amdgcn_s_setprio(2);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[mb][v] = 0.f;
            const unsigned char *tbp = tile_l + tb * TILEB;
            auto fragment = [&](int f, int mb) {
                const int row = mb * 32 + l32;
                return *reinterpret_cast<const uint4 *>(
                    tbp + row * LROW + (((2 * f + half) ^ ((row >> RSH) & KMASK)) * 16));
            };
            if constexpr (ROWB >= 256) {
                // the fragments of k-step f + 1 are requested before the MFMAs of k-step f
                // are issued (the scheduling fences keep it that way; left alone the compiler
                // requests a k-step's fragments and waits for them on the spot): an LDS read
                // then has two MFMAs' time to come back
                uint4 a_cur[MB], a_nxt[MB];
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) a_cur[mb] = fragment(0, mb);
#pragma unroll
                for (int f = 0; f < NF; ++f) {
                    if (f + 1 < NF) {
#pragma unroll
                        for (int mb = 0; mb < MB; ++mb) a_nxt[mb] = fragment(f + 1, mb);
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) acc[mb] = mma<DT>(a_cur[mb], st[f], acc[mb]);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) a_cur[mb] = a_nxt[mb];
                }
            } else {
                // (128-byte rows: four k-steps per tile; the read-ahead's eight registers
                // would cost pass 2 its third workgroup per CU, which is worth more)
#pragma unroll
                for (int f = 0; f < NF; ++f)
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) acc[mb] = mma<DT>(fragment(f, mb), st[f], acc[mb]);
            }
            __builtin_amdgcn_s_setprio(0);
        }
        dma_wait_upto<CPF>();
        wg_barrier();

        if (live) {
            if constexpr (!COLSUM) {
                // streamed rows are keys j, this lane's row is the query at position
                // off + srow: need j <= off + srow.
                // m_run tracks the maximum of the raw products (c2 > 0 keeps the order);
                // the scale is folded into the exponent's fma
                if constexpr (MASKED) {
                    if (!clear) {
#pragma unroll
                        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                            for (int v = 0; v < 16; ++v) {
                                const int j = r0 + mb * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
                                if (j > off + srow) acc[mb][v] = -INFINITY;
                            }
                    }
                }
                float mx = m_run;
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int v = 0; v < 16; v += 2) mx = fmaxf(fmaxf(mx, acc[mb][v]), acc[mb][v + 1]);
                const float ms = mx == -INFINITY ? 0.f : mx;
                const float nms = -ms * c2;
                float sum0 = 0.f, sum1 = 0.f;
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int v = 0; v < 16; v += 2) {
                        sum0 += __builtin_amdgcn_exp2f(fmaf(acc[mb][v], c2, nms));
                        sum1 += __builtin_amdgcn_exp2f(fmaf(acc[mb][v + 1], c2, nms));
                    }
                l_run = l_run * __builtin_amdgcn_exp2f((m_run - ms) * c2) + (sum0 + sum1);
                m_run = mx;
            } else {
                // streamed rows are queries i (at position off + i), this lane's row is
                // key j = srow: need j <= off + i, i < nq
                const float *ll = lse_l + lb * BN;
                float sum0 = 0.f, sum1 = 0.f;
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int gq = 0; gq < 4; ++gq) {
                        const float4 l4 = *reinterpret_cast<const float4 *>(ll + mb * 32 + 8 * gq + 4 * half);
                        const float lv[4] = {l4.x, l4.y, l4.z, l4.w};
                        float x[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            x[e] = fmaf(acc[mb][4 * gq + e], c2, -lv[e]);
                        if constexpr (MASKED) {
                            if (!clear) {
#pragma unroll
                                for (int e = 0; e < 4; ++e) {
                                    const int i = r0 + mb * 32 + 8 * gq + 4 * half + e;
                                    if (off + i < srow || i >= nq) x[e] = -INFINITY;
                                }
                            }
                        }
                        sum0 += __builtin_amdgcn_exp2f(x[0]) + __builtin_amdgcn_exp2f(x[2]);
                        sum1 += __builtin_amdgcn_exp2f(x[1]) + __builtin_amdgcn_exp2f(x[3]);
                    }
                c_run += sum0 + sum1;
            }
        }
        tb = tb == NTB - 1 ? 0 : tb + 1;
        lb = (lb + 1) & (NLB - 1);
        dma_wait_upto<CPF>();
        // The step's closing barrier takes the running sums as operands: pass 1's vector
        // phase touches no memory, so only this data dependence keeps its arithmetic in
        // front of the barrier.  (Left free, a build has put the whole vector phase behind
        // it; the two wave groups then take turns instead of overlapping.)
        if constexpr (COLSUM)
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" : "+v"(c_run) : : "memory");
        else
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" : "+v"(m_run), "+v"(l_run) : : "memory");
    };
    // Tiles that need the mask: in pass 1 from the first key tile that reaches past
    // the position of this block's first query; in pass 2 up to the last query tile
    // that does not yet see this block's last key.
    if constexpr (!COLSUM) {
        const int t_diag0 = min(t_end, (off + s0 + 1) / BN);
        for (int tile = t_begin; tile < t_diag0; ++tile) tile_step(tile, std::false_type{});
        for (int tile = t_diag0; tile < t_end; ++tile) tile_step(tile, std::true_type{});
    } else {
        const int x = s0 + SROWS - 1 - off;      // first query (local) that sees the whole block
        const int t_diag1 = min(t_end, max(t_begin, x > 0 ? (x + BN - 1) / BN : 0));
        // a ragged last tile holds rows past nq: it takes the masking path as well
        const int t_rag = (nq % BN) ? max(t_diag1, t_end - 1) : t_end;
        for (int tile = t_begin; tile < t_diag1; ++tile) tile_step(tile, std::true_type{});
        for (int tile = t_diag1; tile < t_rag; ++tile) tile_step(tile, std::false_type{});
        for (int tile = t_rag; tile < t_end; ++tile) tile_step(tile, std::true_type{});
    }
    if (grp == 0) wg_barrier();            // the barrier the second group spent at the start
    dma_wait_upto<0>();                    // trailing repeat requests land before the LDS is released

    if constexpr (!COLSUM) {
        const float m2 = __shfl_xor(m_run, 32, 64), l2 = __shfl_xor(l_run, 32, 64);
        const float M = fmaxf(m_run, m2);            // finite: key 0 is visible to every query
        const float L = l_run * __builtin_amdgcn_exp2f((m_run - M) * c2) +
                        l2 * __builtin_amdgcn_exp2f((m2 - M) * c2);
        if (half == 0 && srow < nq) lse2[(size_t)head * nq + srow] = M * c2 + __builtin_amdgcn_logf(L);
    } else {
        const float c = c_run + __shfl_xor(c_run, 32, 64);
        if (half == 0 && srow < nk) colsum[(size_t)head * nk + srow] = c;
    }
}

template <int DT, int D, bool COLSUM>
hipError_t launch_pass(const h2o_config &cfg, double scale, const void *Q, const void *K, int nq,
                       int nk, float *lse2, float *colsum, hipStream_t st)
{
    constexpr int SROWS = NWV * 32;
    constexpr int ES = DT == H2O_F32 ? 4 : 2;
    constexpr int MB = (D * ES >= 512) ? 1 : 2;      // keep the two tile buffers under 48 KiB
    constexpr int BN = 32 * MB;
    constexpr size_t smem = NTB * (size_t)BN * (D * ES) + NLB * BN * sizeof(float);
    const int heads = cfg.batch * cfg.heads;
    const int nblk = ((COLSUM ? nk : nq) + SROWS - 1) / SROWS;
    const float c2 = (float)(scale * 1.4426950408889634);
    auto kern = prefill_pass_kernel<DT, D, MB, COLSUM>;
    if (smem > 48 * 1024) {
        static bool raised = false;
        if (!raised) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
            if (e != hipSuccess) return e;
            raised = true;
        }
    }
    hipLaunchKernelGGL(kern,
                       dim3((unsigned)((heads + 63) / 64) * 64 * nblk),
                       dim3(NWV * 64), smem, st, static_cast<const char *>(Q),
                       static_cast<const char *>(K), nq, nk, heads, c2, lse2, colsum);
    return hipGetLastError();
}

template <bool COLSUM>
hipError_t dispatch(const h2o_config &cfg, double scale, const void *Q, const void *K, int nq,
                    int nk, float *lse2, float *colsum, hipStream_t st)
{
    const int d = cfg.head_dim;
    switch (cfg.dtype) {
    case H2O_F32:
        return d == 64 ? launch_pass<H2O_F32, 64, COLSUM>(cfg, scale, Q, K, nq, nk, lse2, colsum, st)
                       : launch_pass<H2O_F32, 128, COLSUM>(cfg, scale, Q, K, nq, nk, lse2, colsum, st);
    case H2O_F16:
        return d == 64 ? launch_pass<H2O_F16, 64, COLSUM>(cfg, scale, Q, K, nq, nk, lse2, colsum, st)
                       : launch_pass<H2O_F16, 128, COLSUM>(cfg, scale, Q, K, nq, nk, lse2, colsum, st);
    default:
        return d == 64 ? launch_pass<H2O_BF16, 64, COLSUM>(cfg, scale, Q, K, nq, nk, lse2, colsum, st)
                       : launch_pass<H2O_BF16, 128, COLSUM>(cfg, scale, Q, K, nq, nk, lse2, colsum, st);
    }
}

}  // namespace

hipError_t h2o_launch_prefill_lse(const h2o_config &cfg, double scale, const void *Q,
                                  const void *K, int nq, int nk, float *lse, hipStream_t st)
{
    return dispatch<false>(cfg, scale, Q, K, nq, nk, lse, nullptr, st);
}

hipError_t h2o_launch_prefill_colsum(const h2o_config &cfg, double scale, const void *Q,
                                     const void *K, int nq, int nk, const float *lse,
                                     float *colsum, hipStream_t st)
{
    return dispatch<true>(cfg, scale, Q, K, nq, nk, const_cast<float *>(lse), colsum, st);
}
