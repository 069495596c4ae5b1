// Fused H2O generation step over a cache that stores 4-bit codes (group-wise
// min-max quantisation along the head dimension, Sec. 5.4 and the appendix on
// combining H2O with quantisation): one workgroup per (batch, head).
//
// The step is the one of the unquantised kernel (Definition 2.2 softmax over the
// cached tokens and the token itself, Algorithm 2 accumulate, evict the smallest
// score outside the recent window, overwrite in place) on the stored values
// x = min + code * scale; the new token attends to itself with its key and value
// as given and is quantised when it is written into its slot.
//
// Memory plan.  A stored row is D/2 bytes of codes followed by D/64 (scale, min)
// pairs.  LPR = D/32 neighbouring lanes read a row's codes with one 128-bit load
// each (32 codes per lane) and the pair of the group they fall in with one
// 64-bit load, so a wave covers RPW = 64/LPR rows per round.  All U key rounds
// of a wave are requested up front; a round's registers are refilled with the
// value row of the same slot as soon as the key has been used, so the value
// stream is in flight during the softmax.  Nothing is dequantised into memory.
//
// Arithmetic.  Logits: with the row's (scale s_g, min m_g) per group g,
//     <q, x> = sum_g  s_g * sum_{e in g} q_e c_e  +  m_g * sum_{e in g} q_e .
// The inner sums are formed in fp64 without converting the codes: a code placed
// in mantissa bits [p, p+4) of the high word of a double whose exponent makes
// that field's unit 1 IS the number 2^(20-p) + c, one bit-field insert per code;
// the surplus sum_e q_e 2^(20-p_e) is a per-lane constant taken off afterwards
// (fp64 keeps 2^20 |q| + q c to ~1e-9 absolute, far below what the scores need).
// Output: the same idea in half precision, (c << 6) | 0x4C00 is the half 16 + c,
// two codes per AND-OR, multiplied by the fp32 weight p * s_g in a mixed-precision
// fma with fp32 accumulation; 16 * sum p s_g and sum p m_g are settled once per lane.
#include "wave_ops.h"
#include <type_traits>

namespace {

template <int CTRL> __device__ inline float dpp_f(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
constexpr int DPP_ROR2 = 0x122, DPP_ROR4 = 0x124, DPP_ROR8 = 0x128;   // rotate inside 16 lanes

// sum over the LANES (2 or 4) neighbouring lanes of a row; every one of them gets it
template <int LANES> __device__ inline double row_lanes_sum(double a)
{
    a += dpp<DPP_XOR1>(a);
    if (LANES >= 4) a += dpp<DPP_XOR2>(a);
    return a;
}

// Streaming loads addressed as uniform base + 32-bit lane offset (the form that
// needs one address register per lane instead of a 64-bit pair).
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ inline f32x2 load_pair_stream(const char *base, unsigned byte_off)
{
    return __builtin_nontemporal_load(reinterpret_cast<const f32x2 *>(base + byte_off));
}
__device__ inline uint4 load_codes_stream(const char *base, unsigned byte_off)
{
    return load_stream(base + byte_off);
}

// Bit position of code j (0..7) of a word inside the high word of the double it is
// turned into: codes 0..4 stay where they are (bits 0, 4, .., 16), codes 5..7 are
// taken from the word shifted right by 12 (bits 8, 12, 16).
__host__ __device__ constexpr int code_bit(int j) { return j < 5 ? 4 * j : 4 * (j - 3); }

// Registers: a lane keeps its 32 elements of q as doubles (64 registers) next to
// the rounds in flight (7 registers each), which is why everything that is only
// needed after the key pass (slot bookkeeping, the new token once more) is
// requested after it, and why no loaded value may ever be spilled: a spill of a
// register a load is still writing waits for the whole stream.  Four-wave
// workgroups: 256 slots fit 128 registers (four workgroups per CU), 512 slots 168
// (three per CU); deeper rings run at two waves per SIMD.  Eight waves per head
// with half the rounds each were measured slower (more waves redo the softmax and
// bookkeeping than the shorter rounds save).
// PAT: built for a sparse-attention pattern as the protected set (the plain recent
// window's build carries none of that code).
template <int DT, int D, int NW, int U, bool PAT>
__global__ __launch_bounds__(NW * 64, U * (64 / (D / 32)) == 64 ? 4 : (NW == 4 && U * (64 / (D / 32)) == 128) ? 3 : 2)
void decode_q4_kernel(
    char *__restrict__ Kc, char *__restrict__ Vc, float *__restrict__ acc_g,
    int32_t *__restrict__ pos_g, const char *__restrict__ q_g,
    const char *__restrict__ kn_g, const char *__restrict__ vn_g,
    char *__restrict__ out_g, int k, int n_occ, int t, int recent, double scale, int rank, int protect,
    int stride)
{
    using E = Elem<DT>;
    using T = typename E::T;
    constexpr int CODEB = D / 2;                // bytes of codes per row
    constexpr unsigned ROWB = H2O_Q4_ROW_BYTES(D);
    constexpr int LPR = D / 32;                 // lanes per row, 32 codes each
    constexpr int RPW = 64 / LPR;               // rows per wave per round
    constexpr int RPI = NW * RPW;               // rows per workgroup-wide round
    constexpr int OWN = U * RPW;                // slots a wave owns
    constexpr int SPL = OWN / 64;               // ... per lane
    constexpr int QL = D / 8;                   // lanes holding the new key, 8 elements each
    constexpr int QPITCH = 34;                  // doubles per 32-element slice of q in LDS (bank spread)
    constexpr int OPITCH = D + 4;               // floats per row of partial outputs in LDS (bank spread)
    static_assert(NW * 64 >= D, "one thread per element of q");
    static_assert(OWN % 64 == 0 && SPL >= 1, "whole slots per lane");
    static_assert(D == 64 || D == 128, "head dimension");

    const int head = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int sub = lane / LPR, li = lane % LPR;

    extern __shared__ __align__(16) unsigned char smem[];
    double *s_l = reinterpret_cast<double *>(smem);                    // [NW][OWN] logits
    double *red_sum = s_l + NW * OWN;                                  // [NW]
    double *red_max = red_sum + NW;                                    // [NW] (overflow path)
    double *red_key = red_max + NW;                                    // [NW]
    double *qd_l = red_key + NW;                                       // [LPR][QPITCH] q as doubles
    float *p_l = reinterpret_cast<float *>(qd_l + LPR * QPITCH);       // [NW][OWN]
    float *fix_l = p_l + NW * OWN;                                     // [NW][4]
    unsigned *new_l = reinterpret_cast<unsigned *>(fix_l + NW * 4);    // [3][32] the new token as stored
    float *o_l = reinterpret_cast<float *>(new_l + 96);                // [NW * RPW][OPITCH]
    double *s_w = s_l + wave * OWN;
    float *p_w = p_l + wave * OWN;

    const size_t hoff = (size_t)head * k;
    char *Kb = Kc + hoff * ROWB;
    char *Vb = Vc + hoff * ROWB;
    const T *qh = reinterpret_cast<const T *>(q_g) + (size_t)head * D;
    const T *knh = reinterpret_cast<const T *>(kn_g) + (size_t)head * D;
    const T *vnh = reinterpret_cast<const T *>(vn_g) + (size_t)head * D;

    const int row0 = wave * RPW + sub;          // this lane's row inside a round
    const int last = max(n_occ, 1) - 1;         // clamp target
    int my_slot[SPL];
    bool owner[SPL];
#pragma unroll
    for (int s = 0; s < SPL; ++s) {
        const int o = lane + 64 * s;            // entry of the wave's tile: round o / RPW, row o % RPW
        my_slot[s] = (o / RPW) * RPI + wave * RPW + (o % RPW);
        owner[s] = my_slot[s] < n_occ;
    }

    // ---- requests: q, the new token, then the whole key stream ------------------
    const T q_elem = qh[tid % D];               // threads [0, D) widen q once for the workgroup
    // 8 elements of q and of the new key per lane (lanes [0, QL) cover the row): the token's own logit
    const int e8 = (lane % QL) * 8;
    float q8[8], k8[8];
    load8<DT>(qh + e8, q8);
    load8<DT>(knh + e8, k8);

    unsigned off[U];                            // byte offset of this lane's 16 bytes of codes
    const unsigned to_pair = (unsigned)CODEB + (unsigned)(li / 2) * 8u - (unsigned)li * 16u;   // ... on to its group's pair
    uint4 buf[U];
    f32x2 par[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        off[u] = __umul24((unsigned)min(u * RPI + row0, last), ROWB) + (unsigned)li * 16u;
        buf[u] = load_codes_stream(Kb, off[u]);
        par[u] = load_pair_stream(Kb, off[u] + to_pair);
    }
    __builtin_amdgcn_sched_barrier(0);

    // ---- the token's own logit (while the stream arrives) ------------------------
    double s_self;
    {
        double a = 0.0;
#pragma unroll
        for (int i = 0; i < 8; ++i) a = fma((double)q8[i], (double)k8[i], a);
        s_self = lane_value(group_sum<QL>(a), 0) * scale;     // lanes [0, QL) hold q.k_new
    }

    // ---- this lane's 32 elements of q, widened exactly (once per workgroup, via LDS) ---
    if (tid < D) qd_l[(tid / 32) * QPITCH + (tid % 32)] = (double)E::to_f(q_elem);
    lds_barrier();
    double qd[32];
    double qsum = 0.0, surplus = 0.0;           // sum q_e and sum q_e 2^(20 - bit(e))
    {
#pragma unroll
        for (int i = 0; i < 32; i += 2) {
            const double2 two = *reinterpret_cast<const double2 *>(qd_l + li * QPITCH + i);
            qd[i] = two.x;
            qd[i + 1] = two.y;
        }
        double by_bit[5] = {0.0, 0.0, 0.0, 0.0, 0.0};        // codes that sit at bit 0, 4, 8, 12, 16
#pragma unroll
        for (int e = 0; e < 32; ++e) by_bit[code_bit(e % 8) / 4] += qd[e];
#pragma unroll
        for (int b = 0; b < 5; ++b) {
            qsum += by_bit[b];
            surplus = fma(by_bit[b], (double)(1 << (20 - 4 * b)), surplus);
        }
    }

    // The constants that are OR-ed around a code live in vector registers: the fused
    // AND-OR instruction takes one scalar operand only (the mask), and a constant the
    // compiler can see would be split off into an instruction of its own.
    unsigned exp_bits[5];                       // exponent of 2^(20 - bit) for bit = 0, 4, .., 16
#pragma unroll
    for (int b = 0; b < 5; ++b) {
        exp_bits[b] = (1023u + 20u - 4u * (unsigned)b) << 20;
        asm volatile("" : "+v"(exp_bits[b]));
    }

    // ---- logits: one pass over the cached keys ------------------------------------
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (u * RPI + wave * RPW < n_occ) {     // wave-uniform: rounds past the occupied slots cost no arithmetic
            pin(buf[u]);
            const unsigned w[4] = {buf[u].x, buf[u].y, buf[u].z, buf[u].w};
            double a0 = 0.0, a1 = 0.0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const unsigned hi12 = w[i] >> 12;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int b = code_bit(j);
                    const unsigned src = j < 5 ? w[i] : hi12;
                    const unsigned hi = (src & (0xFu << b)) | exp_bits[b / 4];
                    const double c = __hiloint2double((int)hi, 0);      // 2^(20-b) + code
                    if (j & 1) a1 = fma(c, qd[i * 8 + j], a1);
                    else a0 = fma(c, qd[i * 8 + j], a0);
                }
            }
            const double part = fma((double)par[u].x, (a0 + a1) - surplus, (double)par[u].y * qsum);
            const double tot = row_lanes_sum<LPR>(part);
            if (li == 0) s_w[u * RPW + sub] = tot * scale;
        }
        // the value row takes the registers; the pair's offset is worked out here, from a
        // copy the compiler cannot see through, so that it is not kept for every round
        unsigned o = off[u];
        asm volatile("" : "+v"(o));
        buf[u] = load_codes_stream(Vb, o);
        par[u] = load_pair_stream(Vb, o + to_pair);
        __builtin_amdgcn_sched_barrier(0);
    }
    // What is needed after the value pass, requested behind the value stream (loads
    // complete in order): the owned slots' bookkeeping, the new token once more (lanes
    // [0, QL): 8 elements of its key, lanes [QL, 2 QL): of its value) and the column of
    // its value this thread adds to the output.  All unconditional: a load behind a
    // branch would be waited for on the spot.
    int pos_j[SPL];
    float acc_j[SPL];
#pragma unroll
    for (int s = 0; s < SPL; ++s) {
        pos_j[s] = pos_g[hoff + min(my_slot[s], last)];
        acc_j[s] = acc_g[hoff + min(my_slot[s], last)];
    }
    float n8[8];
    load8<DT>((lane / QL) == 1 ? vnh + e8 : knh + e8, n8);
    const T v_self_raw = vnh[tid % D];
    __builtin_amdgcn_wave_barrier();

    // ---- exact softmax over the occupied slots + the token itself -------------------
    double s_j[SPL], e_j[SPL];
    double e_sum = 0.0;
#pragma unroll
    for (int s = 0; s < SPL; ++s) {
        s_j[s] = owner[s] ? s_w[lane + 64 * s] : 0.0;
        e_j[s] = owner[s] ? exp(s_j[s] - s_self) : 0.0;
        e_sum += e_j[s];
    }
    double e_self = 1.0;
    {
        const double dw = wave_sum(e_sum);
        if (lane == 0) red_sum[wave] = dw;
    }
    lds_barrier();
    double den = e_self;
#pragma unroll
    for (int w = 0; w < NW; ++w) den += red_sum[w];
    if (!(den <= 1.79769313486231570815e+308)) {
        // some logit is > ~709 above the token's own: redo with the true maximum
        double m = -INFINITY;
#pragma unroll
        for (int s = 0; s < SPL; ++s) m = fmax(m, owner[s] ? s_j[s] : -INFINITY);
        const double mw = wave_max(m);
        if (lane == 0) red_max[wave] = mw;
        lds_barrier();
        double mx = s_self;
#pragma unroll
        for (int w = 0; w < NW; ++w) mx = fmax(mx, red_max[w]);
        e_sum = 0.0;
#pragma unroll
        for (int s = 0; s < SPL; ++s) {
            e_j[s] = owner[s] ? exp(s_j[s] - mx) : 0.0;
            e_sum += e_j[s];
        }
        e_self = exp(s_self - mx);
        const double dw = wave_sum(e_sum);
        if (lane == 0) red_sum[wave] = dw;
        lds_barrier();
        den = e_self;
#pragma unroll
        for (int w = 0; w < NW; ++w) den += red_sum[w];
    }
    const float p_self = (float)(e_self / den);

    // ---- probabilities to the lanes that read the value rows ------------------------
    float p_j[SPL];
#pragma unroll
    for (int s = 0; s < SPL; ++s) {
        p_j[s] = (float)(e_j[s] / den);
        p_w[lane + 64 * s] = p_j[s];                         // 0 for unoccupied rows
    }
    __builtin_amdgcn_wave_barrier();

    // ---- output: one pass over the cached values --------------------------------------
    // Accumulated in fp32, except for binary32 element types: there the output has to
    // hold 1e-5 relative, and the sums of p s_g (16 + c) are an order of magnitude larger
    // than the output they leave once 16 sum p s_g and sum p m_g are taken off (a
    // dequantised value is itself the small difference of m_g and c s_g), so fp32
    // rounding of the large sums would show.  fp64 then, settled per lane before the
    // columns meet in LDS.
    using OT = typename std::conditional<DT == H2O_F32, double, float>::type;
    OT o[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) o[i] = (OT)0;
    unsigned half16 = 0x4C004C00u;              // two halves of value 16 (in a vector register, as above)
    asm volatile("" : "+v"(half16));
    OT wsum = (OT)0, msum = (OT)0;              // sum p s_g and sum p m_g over this lane's rows
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (u * RPI + wave * RPW < n_occ) {
            pin(buf[u]);
            // rows past the occupied slots repeat the last occupied row with p = 0
            const float p = p_w[u * RPW + sub];
            OT wgt;
            if constexpr (DT == H2O_F32) {
                wgt = (double)p * (double)par[u].x;
                msum = fma((double)p, (double)par[u].y, msum);
            } else {
                wgt = p * par[u].x;
                msum = fmaf(p, par[u].y, msum);
            }
            wsum += wgt;
            const unsigned w[4] = {buf[u].x, buf[u].y, buf[u].z, buf[u].w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                // codes (j, j + 4) of the word as the two halves 16 + c of one register
                const unsigned x[4] = {w[i] << 6, w[i] << 2, w[i] >> 2, w[i] >> 6};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const unsigned h2 = (x[j] & 0x03C003C0u) | half16;
                    const _Float16 lo = __builtin_bit_cast(_Float16, (unsigned short)(h2 & 0xffffu));
                    const _Float16 hi = __builtin_bit_cast(_Float16, (unsigned short)(h2 >> 16));
                    if constexpr (DT == H2O_F32) {
                        o[i * 8 + j] = fma(wgt, (double)(float)lo, o[i * 8 + j]);
                        o[i * 8 + j + 4] = fma(wgt, (double)(float)hi, o[i * 8 + j + 4]);
                    } else {
                        o[i * 8 + j] = fmaf(wgt, (float)lo, o[i * 8 + j]);
                        o[i * 8 + j + 4] = fmaf(wgt, (float)hi, o[i * 8 + j + 4]);
                    }
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    {
        // every lane hands its 32 partial columns to LDS (o_l[row of the round][column]);
        // the two constants, which belong to all 32 columns alike, are added up over
        // the wave's rows first: fix_l[wave][li] (fp64 accumulation: taken off per lane)
        float *dst = o_l + (wave * RPW + sub) * OPITCH + li * 32;
        float fix;
        if constexpr (DT == H2O_F32) {
            const double fixd = msum - 16.0 * wsum;
#pragma unroll
            for (int i = 0; i < 32; i += 4)
                *reinterpret_cast<float4 *>(dst + i) =
                    make_float4((float)(o[i] + fixd), (float)(o[i + 1] + fixd), (float)(o[i + 2] + fixd),
                                (float)(o[i + 3] + fixd));
            fix = 0.f;
        } else {
#pragma unroll
            for (int i = 0; i < 32; i += 4)
                *reinterpret_cast<float4 *>(dst + i) = make_float4(o[i], o[i + 1], o[i + 2], o[i + 3]);
            fix = msum - 16.f * wsum;
        }
        fix += dpp_f<DPP_ROR8>(fix);
        fix += dpp_f<DPP_ROR4>(fix);
        if (LPR == 2) fix += dpp_f<DPP_ROR2>(fix);
        fix += __shfl_xor(fix, 16, 64);
        fix += __shfl_xor(fix, 32, 64);
        if (lane < LPR) fix_l[wave * 4 + lane] = fix;
    }

    // ---- the new token as it will be stored (one wave works it out for whichever
    // wave turns out to own the slot) ---------------------------------------------------
    if (wave == 0) {
        float new_scale, new_min;
        const unsigned new_word = q4_quantise8(n8, new_scale, new_min);
        if (lane < 32) {
            new_l[lane] = new_word;
            new_l[32 + lane] = __float_as_uint(new_scale);
            new_l[64 + lane] = __float_as_uint(new_min);
        }
    }

    // ---- score update (Algorithm 2, accumulate line: binary32 add of the binary32
    // probability) and the eviction candidate: smallest (rank value, position) outside
    // the window
    // (with a sparse-attention pattern as the protected set the candidates are the slots
    // it does not cover; the minimum over all slots is reduced alongside for the case
    // that it covers them all, in the LDS words of the overflow path, idle by now)
    unsigned long long key = NO_CANDIDATE, key_all = NO_CANDIDATE;
    int key_slot = -1, key_all_slot = -1;
#pragma unroll
    for (int s = 0; s < SPL; ++s) {
        acc_j[s] += p_j[s];
        if (owner[s]) {
            const unsigned long long c =
                ((unsigned long long)__float_as_uint(rank_value(acc_j[s], pos_j[s], t, rank)) << 32) |
                (unsigned)pos_j[s];
            if (PAT ? !is_protected(pos_j[s], t, recent, protect, stride) : pos_j[s] <= t - recent) {
                if (c < key) { key = c; key_slot = my_slot[s]; }
            }
            if (PAT && c < key_all) { key_all = c; key_all_slot = my_slot[s]; }
        }
    }
    {
        const double kw = wave_min_f64(__longlong_as_double((long long)key));
        if (lane == 0) red_key[wave] = kw;
    }
    if constexpr (PAT) {
        const double ka = wave_min_f64(__longlong_as_double((long long)key_all));
        if (lane == 0) red_max[wave] = ka;
    }
    lds_barrier();

    // ---- write-back ---------------------------------------------------------------------
    if (tid < D) {
        float r0 = p_self * E::to_f(v_self_raw), r1 = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) r1 += fix_l[w * 4 + tid / 32];
#pragma unroll 8
        for (int row = 0; row < NW * RPW; row += 2) {
            r0 += o_l[row * OPITCH + tid];
            r1 += o_l[(row + 1) * OPITCH + tid];
        }
        reinterpret_cast<T *>(out_g)[(size_t)head * D + tid] = E::from_f(r0 + r1);
    }
    int tslot = -1;          // wave-uniform: the slot this wave has to fill, if any
    int lost_slot = -1;      // per lane: its slot that has just been evicted
    if (n_occ < k) {
        if (wave == 0) tslot = n_occ;
    } else {
        double wd = red_key[0];
#pragma unroll
        for (int w = 1; w < NW; ++w) wd = fmin(wd, red_key[w]);
        if (PAT && wd != wd) {                               // the pattern covers every slot
            wd = red_max[0];
#pragma unroll
            for (int w = 1; w < NW; ++w) wd = fmin(wd, red_max[w]);
            key = key_all;
            key_slot = key_all_slot;
        }
        const unsigned long long win = (unsigned long long)__double_as_longlong(wd);
        const unsigned long long self_key =
            ((unsigned long long)__float_as_uint(p_self) << 32) | (unsigned)t;
        const bool evict = wd == wd && (PAT || recent != 0 || win < self_key);
        const bool mine = evict && key == win && key != NO_CANDIDATE;   // keys are unique (positions are)
        if (mine) lost_slot = key_slot;
        const unsigned long long b = __ballot(mine);
        if (b != 0) tslot = __builtin_amdgcn_readlane(key_slot, __ffsll((long long)b) - 1);
    }
#pragma unroll
    for (int s = 0; s < SPL; ++s)
        if (owner[s] && my_slot[s] != lost_slot) acc_g[hoff + my_slot[s]] = acc_j[s];
    if (tslot >= 0) {
        if (lane == 0) { pos_g[hoff + tslot] = t; acc_g[hoff + tslot] = p_self; }
        // lanes [0, QL) hold the new key's codes, lanes [QL, 2 QL) the new value's
        if (lane < 2 * QL) {
            char *row = (lane < QL ? Kb : Vb) + (size_t)tslot * ROWB;
            const int l = lane % QL;
            *reinterpret_cast<unsigned *>(row + l * 4) = new_l[lane];
            if ((l & 7) == 0)
                *reinterpret_cast<f32x2 *>(row + CODEB + (l / 8) * 8) =
                    f32x2{__uint_as_float(new_l[32 + lane]), __uint_as_float(new_l[64 + lane])};
        }
    }
}

#define H2O_DECODE_ARGS                                                                         \
    c.K, c.V, c.acc, c.pos, static_cast<const char *>(q), static_cast<const char *>(kn),        \
        static_cast<const char *>(vn), static_cast<char *>(out), c.k, (c.t < c.k ? c.t : c.k),  \
        c.t, c.cfg.recent, c.scale, c.cfg.rank, c.cfg.protect, c.cfg.stride

template <int DT, int D, int NW, int U>
hipError_t launch_q4(const h2o_cache &c, const void *q, const void *kn, const void *vn, void *out,
                     hipStream_t st)
{
    constexpr int LPR = D / 32, RPW = 64 / LPR, OWN = U * RPW;
    constexpr size_t smem = (size_t)NW * OWN * 8 + (size_t)NW * 24 + (size_t)LPR * 34 * 8 +
                            (size_t)NW * OWN * 4 + (size_t)NW * 16 + 384 +
                            (size_t)NW * RPW * (D + 4) * 4 + 16;
    auto launch = [&](auto kern, bool &raised) -> hipError_t {
        if (smem > 48 * 1024 && !raised) {
            const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
            if (e != hipSuccess) return e;
            raised = true;
        }
        hipLaunchKernelGGL(kern, dim3(c.cfg.batch * c.cfg.heads), dim3(NW * 64), smem, st, H2O_DECODE_ARGS);
        return hipGetLastError();
    };
    static bool raised_window = false, raised_pattern = false;
    if (c.cfg.protect == H2O_PROTECT_RECENT) return launch(decode_q4_kernel<DT, D, NW, U, false>, raised_window);
    return launch(decode_q4_kernel<DT, D, NW, U, true>, raised_pattern);
}

// Rounds per wave follow the number of occupied slots (capacity NW * U * RPW).
template <int DT, int D>
hipError_t pick_q4(const h2o_cache &c, const void *q, const void *kn, const void *vn, void *out,
                   hipStream_t st)
{
    constexpr int RPW = 64 / (D / 32);
    constexpr int U0 = 64 / RPW;                // fewest rounds that give every lane a slot
    const int occ = c.t < c.k ? c.t : c.k;
    if (occ <= 4 * U0 * RPW) return launch_q4<DT, D, 4, U0>(c, q, kn, vn, out, st);           // 256 slots
    if (occ <= 4 * 2 * U0 * RPW) return launch_q4<DT, D, 4, 2 * U0>(c, q, kn, vn, out, st);   // 512
    if (occ <= 4 * 4 * U0 * RPW) return launch_q4<DT, D, 4, 4 * U0>(c, q, kn, vn, out, st);   // 1024
    if (occ <= 8 * 4 * U0 * RPW) return launch_q4<DT, D, 8, 4 * U0>(c, q, kn, vn, out, st);   // 2048
    return hipErrorInvalidValue;               // beyond H2O_Q4_MAX_BUDGET: refused at configuration time
}

}  // namespace

hipError_t h2o_launch_decode_q4(const h2o_cache &c, const void *q, const void *k_new,
                                const void *v_new, void *out, hipStream_t st)
{
    const int d = c.cfg.head_dim;
    switch (c.cfg.dtype) {
    case H2O_F32:
        return d == 64 ? pick_q4<H2O_F32, 64>(c, q, k_new, v_new, out, st)
                       : pick_q4<H2O_F32, 128>(c, q, k_new, v_new, out, st);
    case H2O_F16:
        return d == 64 ? pick_q4<H2O_F16, 64>(c, q, k_new, v_new, out, st)
                       : pick_q4<H2O_F16, 128>(c, q, k_new, v_new, out, st);
    default:
        return d == 64 ? pick_q4<H2O_BF16, 64>(c, q, k_new, v_new, out, st)
                       : pick_q4<H2O_BF16, 128>(c, q, k_new, v_new, out, st);
    }
}
