// Fused H2O generation step for gfx950: one workgroup per (batch, head).
//
// Per head the kernel reads the k cached key rows once (logits), does an exact
// softmax over the occupied slots and the new token itself (Definition 2.2: the
// normaliser only counts tokens that are in the cache; the token attends to
// itself as in the exact process), reads the k cached value rows once (output),
// adds the probabilities to the per-slot accumulated scores (Algorithm 2,
// accumulate line), picks the slot to give up (Definition 4.3 with the sum of
// accumulated scores as F_score: the smallest score outside the recent window)
// and overwrites it in place with the new token (Sec. 4.2 implementation
// details: no swap, fill directly).
//
// Memory plan.  A cache row (head_dim elements) is read by LPR = row_bytes/16
// neighbouring lanes with one 128-bit load each, so a wave covers 64/LPR whole
// rows = 1 KiB of contiguous memory per load instruction and the workgroup
// covers RPI rows per "round".  The key rounds followed by the value rounds
// form one stream that is pulled through a ring of U register buffers per
// wave: a buffer is refilled with the entry U places ahead as soon as it has
// been consumed, so value rows are already in flight while the workgroup sits
// in the softmax barriers and HBM never idles.  Logits, probabilities and the
// per-slot bookkeeping live in LDS.
//
// Arithmetic.  q.k products are accumulated in fp64 (inputs widened exactly),
// reduced over the row's lanes with DPP moves, and the softmax is evaluated in
// fp64; each probability is rounded once to binary32 and added to the binary32
// score.  That makes the stored scores, and with them the eviction decisions,
// reproducible against an fp64 reference; the kernel is HBM-bound and the extra
// ALU work hides behind the stream.  P.V is accumulated in fp32.
#include "h2o_internal.h"

namespace {

// Workgroup barrier that waits for this wave's LDS traffic only, so global
// loads issued earlier (prefetched rows) stay in flight across it.
__device__ inline void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// 128-bit load of a cache row piece with the non-temporal hint: the cache is
// streamed once per step, and hinting that lifts the achieved read bandwidth by
// 12-14 % on this part (measured with a plain streaming-read kernel).
__device__ inline uint4 load_stream(const char *p)
{
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
    return make_uint4(t.x, t.y, t.z, t.w);
}

// ---- DPP helpers (row = 16 lanes) ---------------------------------------------
constexpr int DPP_XOR1 = 0xB1;         // quad_perm [1,0,3,2]
constexpr int DPP_XOR2 = 0x4E;         // quad_perm [2,3,0,1]
constexpr int DPP_HALF_MIRROR = 0x141; // lane i <-> 7-i inside each 8 lanes
constexpr int DPP_MIRROR = 0x140;      // lane i <-> 15-i inside each 16 lanes

template <int CTRL> __device__ inline int dpp(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true);
}
template <int CTRL> __device__ inline double dpp(double v)
{
    return __hiloint2double(dpp<CTRL>(__double2hiint(v)), dpp<CTRL>(__double2loint(v)));
}
template <int CTRL> __device__ inline unsigned long long dpp(unsigned long long v)
{
    const unsigned hi = (unsigned)dpp<CTRL>((int)(v >> 32)), lo = (unsigned)dpp<CTRL>((int)v);
    return ((unsigned long long)hi << 32) | lo;
}

// After the xor-1 and xor-2 steps all four lanes of a quad agree, so the two
// mirror steps act as xor-4 and xor-8: every lane ends with its group's total.
template <int LANES> __device__ inline double group_sum(double a)
{
    a += dpp<DPP_XOR1>(a);
    a += dpp<DPP_XOR2>(a);
    if (LANES >= 8) a += dpp<DPP_HALF_MIRROR>(a);
    if (LANES >= 16) a += dpp<DPP_MIRROR>(a);
    if (LANES >= 32) a += __shfl_xor(a, 16, 64);
    if (LANES >= 64) a += __shfl_xor(a, 32, 64);
    return a;
}
__device__ inline double row_max(double a)
{
    a = fmax(a, dpp<DPP_XOR1>(a));
    a = fmax(a, dpp<DPP_XOR2>(a));
    a = fmax(a, dpp<DPP_HALF_MIRROR>(a));
    return fmax(a, dpp<DPP_MIRROR>(a));
}
__device__ inline unsigned long long umin64(unsigned long long a, unsigned long long b)
{
    return a < b ? a : b;
}
__device__ inline unsigned long long row_min(unsigned long long a)
{
    a = umin64(a, dpp<DPP_XOR1>(a));
    a = umin64(a, dpp<DPP_XOR2>(a));
    a = umin64(a, dpp<DPP_HALF_MIRROR>(a));
    return umin64(a, dpp<DPP_MIRROR>(a));
}
// value of lane L of the wave, as a wave-uniform scalar
__device__ inline double lane_value(double v, int L)
{
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), L),
                            __builtin_amdgcn_readlane(__double2loint(v), L));
}
__device__ inline unsigned long long lane_value(unsigned long long v, int L)
{
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(v >> 32), L);
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)v, L);
    return ((unsigned long long)hi << 32) | lo;
}
__device__ inline double wave_max(double v)
{
    v = row_max(v);
    return fmax(fmax(lane_value(v, 0), lane_value(v, 16)), fmax(lane_value(v, 32), lane_value(v, 48)));
}
__device__ inline double wave_min_f64(double v)   // NaN entries are ignored
{
    v = fmin(v, dpp<DPP_XOR1>(v));
    v = fmin(v, dpp<DPP_XOR2>(v));
    v = fmin(v, dpp<DPP_HALF_MIRROR>(v));
    v = fmin(v, dpp<DPP_MIRROR>(v));
    return fmin(fmin(lane_value(v, 0), lane_value(v, 16)), fmin(lane_value(v, 32), lane_value(v, 48)));
}
__device__ inline double wave_sum(double v)
{
    v = group_sum<16>(v);
    return (lane_value(v, 0) + lane_value(v, 16)) + (lane_value(v, 32) + lane_value(v, 48));
}
__device__ inline unsigned long long wave_min(unsigned long long v)
{
    v = row_min(v);
    return umin64(umin64(lane_value(v, 0), lane_value(v, 16)),
                  umin64(lane_value(v, 32), lane_value(v, 48)));
}
constexpr unsigned long long NO_CANDIDATE = ~0ull;

// ---- pieces shared by the two kernels -------------------------------------------

// Adds this lane's fp32 partial output (EPL columns of row group `sub`) into the
// workgroup's output row, multiplies nothing: o_l[wave][column] gets the wave's sum.
template <int EPL, int LPR, int D>
__device__ inline void wave_output_to_lds(float (&o)[EPL], float *o_l, int wave, int sub, int li)
{
#pragma unroll
    for (int m = LPR; m < 64; m <<= 1) {
#pragma unroll
        for (int i = 0; i < EPL; ++i) o[i] += __shfl_xor(o[i], m, 64);
    }
    if (sub == 0) {
#pragma unroll
        for (int i = 0; i < EPL; ++i) o_l[wave * D + li * EPL + i] = o[i];
    }
}

// Final writes of a step: the output row, and the new token into slot `target`
// (K row, V row, first score, position); target < 0 = the token is not kept.
template <int DT, int D, int NW>
__device__ inline void write_back(const float *o_l, float p_self, int target, int t, size_t hoff,
                                  int head, char *Kb, char *Vb, float *acc_g, int32_t *pos_g,
                                  const typename Elem<DT>::T *knh, const typename Elem<DT>::T *vnh,
                                  char *out_g)
{
    using E = Elem<DT>;
    using T = typename E::T;
    constexpr int EPL = E::EPL, LPR = D / EPL;
    constexpr unsigned ROWB = D * sizeof(T);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid < D) {
        float r = p_self * E::to_f(vnh[tid]);
#pragma unroll
        for (int w = 0; w < NW; ++w) r += o_l[w * D + tid];
        reinterpret_cast<T *>(out_g)[(size_t)head * D + tid] = E::from_f(r);
    }
    if (target >= 0) {
        if (tid == 0) { pos_g[hoff + target] = t; acc_g[hoff + target] = p_self; }
        if (wave == NW - 1) {            // a wave that is not busy with the output row
            if (lane < LPR) {
                const uint4 v = *reinterpret_cast<const uint4 *>(knh + lane * EPL);
                *reinterpret_cast<uint4 *>(Kb + (size_t)target * ROWB + lane * 16) = v;
            } else if (lane < 2 * LPR) {
                const int l2 = lane - LPR;
                const uint4 v = *reinterpret_cast<const uint4 *>(vnh + l2 * EPL);
                *reinterpret_cast<uint4 *>(Vb + (size_t)target * ROWB + l2 * 16) = v;
            }
        }
    }
}

// ---- register-resident kernel: every row of the head fits the ring -----------------
//
// Requires n_occ <= U * RPI and U * RPW <= 64.  Straight-line code: the U key
// loads of a wave go out first, each buffer is refilled with the matching value
// row as soon as it has been used, and no load is conditional, so the compiler
// can wait for exactly the load it needs (vector loads complete in issue order;
// a load behind a branch would make every later wait conservative).  Rounds past
// the occupied slots re-read the last occupied row and are ignored.
//
// A wave owns the slots whose rows it reads (U * RPW of them, one per lane): the
// lanes' fp64 partial dot products go to a wave-private LDS tile and lane l adds
// up the row of its slot, so a slot's logit, probability, score and position
// live in registers of one lane and nothing but the softmax normaliser and the
// final results cross waves: two workgroup barriers per step.
//
// Softmax shift: exp(s_j - s_self), the token's own logit, which is known before
// the key stream arrives (no maximum pass, no barrier for it).  In fp64 this is
// exact to rounding unless some logit exceeds s_self by ~709; then the
// normaliser overflows, which is detected, and the step is redone with the true
// maximum (a rare, workgroup-uniform branch).
template <int DT, int D, int NW, int U>
__global__ __launch_bounds__(NW * 64, 4) void decode_resident_kernel(
    char *__restrict__ Kc, char *__restrict__ Vc, float *__restrict__ acc_g,
    int32_t *__restrict__ pos_g, const char *__restrict__ q_g,
    const char *__restrict__ kn_g, const char *__restrict__ vn_g,
    char *__restrict__ out_g, int k, int n_occ, int t, int recent, double scale)
{
    using E = Elem<DT>;
    using T = typename E::T;
    constexpr int EPL = E::EPL;          // elements per lane per 16-byte load
    constexpr int LPR = D / EPL;         // lanes per row
    constexpr int RPW = 64 / LPR;        // rows per wave per load
    constexpr int RPI = NW * RPW;        // rows per workgroup-wide round
    constexpr int OWN = U * RPW;         // slots a wave owns (one per lane)
    constexpr int PITCH = LPR + 1;       // doubles per row of partials (bank spread)
    constexpr unsigned ROWB = D * sizeof(T);
    static_assert(LPR >= 8 && LPR <= 32, "a row is read by 8, 16 or 32 lanes");
    static_assert(OWN <= 64, "one slot per lane");

    const int head = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane / LPR, li = lane % LPR;

    extern __shared__ __align__(16) unsigned char smem[];
    double *part_l = reinterpret_cast<double *>(smem);                 // [NW][OWN][PITCH]
    double *red_sum = part_l + NW * OWN * PITCH;                       // [NW]
    double *red_max = red_sum + NW;                                    // [NW] (overflow path)
    double *red_key = red_max + NW;                                    // [NW]
    float *p_l = reinterpret_cast<float *>(red_key + NW);              // [NW][OWN]
    float *o_l = p_l + NW * OWN;                                       // [NW][D]
    double *part_w = part_l + wave * OWN * PITCH;
    float *p_w = p_l + wave * OWN;

    const size_t hoff = (size_t)head * k;
    char *Kb = Kc + hoff * ROWB;                                       // uniform bases
    char *Vb = Vc + hoff * ROWB;
    const T *qh = reinterpret_cast<const T *>(q_g) + (size_t)head * D;
    const T *knh = reinterpret_cast<const T *>(kn_g) + (size_t)head * D;
    const T *vnh = reinterpret_cast<const T *>(vn_g) + (size_t)head * D;

    const int row0 = wave * RPW + sub;   // this lane's row inside a round
    const int last = max(n_occ, 1) - 1;  // clamp target: slot 0 exists even when empty
    // the slot this lane owns: the row that lane group (lane % RPW) reads in round lane / RPW
    const int my_slot = (lane / RPW) * RPI + wave * RPW + (lane % RPW);
    const bool owner = lane < OWN && my_slot < n_occ;

    // q, the new key and the new value first: whatever the first arithmetic needs
    // must be requested before the long key stream
    const uint4 qraw = *reinterpret_cast<const uint4 *>(qh + li * EPL);
    const uint4 kraw = *reinterpret_cast<const uint4 *>(knh + li * EPL);
    const uint4 vraw = *reinterpret_cast<const uint4 *>(vnh + li * EPL);
    unsigned off[U];
    uint4 buf[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        off[u] = (unsigned)min(u * RPI + row0, last) * ROWB + (unsigned)li * 16u;
        buf[u] = load_stream(Kb + off[u]);
    }
    // the owned slot's bookkeeping (unconditional, clamped: a conditional load
    // would be merged with its default right here and stall on the whole stream)
    const int pos_j = pos_g[hoff + min(my_slot, last)];
    float acc_j = acc_g[hoff + min(my_slot, last)];
    __builtin_amdgcn_sched_barrier(0);   // every request above leaves before any arithmetic

    // this lane's slice of q (widened exactly) and the token's own logit
    double qd[EPL];
    double s_self;
    {
        const T *qe = reinterpret_cast<const T *>(&qraw);
        const T *ke = reinterpret_cast<const T *>(&kraw);
        double a = 0.0;
#pragma unroll
        for (int i = 0; i < EPL; ++i) {
            qd[i] = (double)E::to_f(qe[i]);
            a = fma((double)E::to_f(ke[i]), qd[i], a);
        }
        s_self = group_sum<LPR>(a) * scale;
    }

    // ---- logits: one pass over the cached keys --------------------------------
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const T *x = reinterpret_cast<const T *>(&buf[u]);
        double a0 = 0.0, a1 = 0.0;
#pragma unroll
        for (int i = 0; i < EPL; i += 2) {
            a0 = fma((double)E::to_f(x[i]), qd[i], a0);
            a1 = fma((double)E::to_f(x[i + 1]), qd[i + 1], a1);
        }
        buf[u] = load_stream(Vb + off[u]);   // value row takes the buffer
        part_w[(u * RPW + sub) * PITCH + li] = a0 + a1;
        __builtin_amdgcn_sched_barrier(0);   // one row at a time: bounds live registers
    }
    __builtin_amdgcn_wave_barrier();     // the tile is private to the wave: LDS runs in order

    // ---- exact softmax over the occupied slots + the token itself -------------
    double s_j = 0.0;
    if (lane < OWN) {
        const double *pr = part_w + lane * PITCH;
        double a = pr[0], b = pr[1];
#pragma unroll
        for (int c = 2; c < LPR; c += 2) { a += pr[c]; b += pr[c + 1]; }
        s_j = (a + b) * scale;
    }
    double e_j = owner ? exp(s_j - s_self) : 0.0;
    double e_self = 1.0;
    {
        const double dw = wave_sum(e_j);
        if (lane == 0) red_sum[wave] = dw;
    }
    lds_barrier();
    double den = e_self;
#pragma unroll
    for (int w = 0; w < NW; ++w) den += red_sum[w];
    if (!(den <= 1.79769313486231570815e+308)) {
        // some logit is > ~709 above the token's own: redo with the true maximum
        const double mw = wave_max(owner ? s_j : -INFINITY);
        if (lane == 0) red_max[wave] = mw;
        lds_barrier();
        double mx = s_self;
#pragma unroll
        for (int w = 0; w < NW; ++w) mx = fmax(mx, red_max[w]);
        e_j = owner ? exp(s_j - mx) : 0.0;
        e_self = exp(s_self - mx);
        const double dw = wave_sum(e_j);
        if (lane == 0) red_sum[wave] = dw;
        lds_barrier();
        den = e_self;
#pragma unroll
        for (int w = 0; w < NW; ++w) den += red_sum[w];
    }
    const float p_self = (float)(e_self / den);
    const float p_j = (float)(e_j / den);

    // ---- score update; probabilities to the lanes that read the value rows ----
    acc_j += p_j;                                            // binary32 accumulate
    if (lane < OWN) p_w[lane] = p_j;                         // 0 for unoccupied rows
    __builtin_amdgcn_wave_barrier();

    // ---- output: one pass over the cached values ------------------------------
    float o[EPL];
    {
        // the token's own contribution rides with wave 0's first lane group
        const float ps = (wave == 0 && sub == 0) ? p_self : 0.f;
        const T *x = reinterpret_cast<const T *>(&vraw);
#pragma unroll
        for (int i = 0; i < EPL; ++i) o[i] = ps * E::to_f(x[i]);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const float p = p_w[u * RPW + sub];
        const T *x = reinterpret_cast<const T *>(&buf[u]);
#pragma unroll
        for (int i = 0; i < EPL; ++i) o[i] = fmaf(p, E::to_f(x[i]), o[i]);
        __builtin_amdgcn_sched_barrier(0);
    }
    wave_output_to_lds<EPL, LPR, D>(o, o_l, wave, sub, li);

    // ---- eviction candidate: smallest (score, position) outside the window -----
    // The 64-bit key (score bits, position) of a finite non-negative score is
    // also a positive double with the same order, and "no candidate" is a NaN,
    // which fmin drops: the key reduction is a plain fp64 minimum.
    unsigned long long key = NO_CANDIDATE;
    if (owner && pos_j <= t - recent)                        // window after this step = {t-R+1..t}
        key = ((unsigned long long)__float_as_uint(acc_j) << 32) | (unsigned)pos_j;
    {
        const double kw = wave_min_f64(__longlong_as_double((long long)key));
        if (lane == 0) red_key[wave] = kw;
    }
    lds_barrier();

    // ---- write-back -----------------------------------------------------------
    if (tid < D) {
        float r = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) r += o_l[w * D + tid];
        reinterpret_cast<T *>(out_g)[(size_t)head * D + tid] = E::from_f(r);
    }
    // Which slot receives the new token: the first free one if any; else the
    // evicted one.  With recent == 0 the token itself competes with its first
    // score and may lose, in which case nothing is written.
    int tslot = -1;          // wave-uniform: the slot this wave has to fill, if any
    bool evicted_mine = false;
    if (n_occ < k) {
        if (wave == 0) tslot = n_occ;
    } else {
        double wd = red_key[0];
#pragma unroll
        for (int w = 1; w < NW; ++w) wd = fmin(wd, red_key[w]);
        const unsigned long long win = (unsigned long long)__double_as_longlong(wd);
        const unsigned long long self_key =
            ((unsigned long long)__float_as_uint(p_self) << 32) | (unsigned)t;
        const bool evict = wd == wd && (recent != 0 || win < self_key);
        evicted_mine = evict && owner && key == win;         // keys are unique (positions are)
        const unsigned long long b = __ballot(evicted_mine);
        if (b != 0) tslot = __builtin_amdgcn_readlane(my_slot, __ffsll((long long)b) - 1);
    }
    if (owner && !evicted_mine) acc_g[hoff + my_slot] = acc_j;
    if (tslot >= 0) {
        if (lane == 0) { pos_g[hoff + tslot] = t; acc_g[hoff + tslot] = p_self; }
        // lane group 0 holds the new key row, lane group 1 the new value row
        if (lane < LPR)
            *reinterpret_cast<uint4 *>(Kb + (size_t)tslot * ROWB + li * 16) = kraw;
        else if (lane < 2 * LPR)
            *reinterpret_cast<uint4 *>(Vb + (size_t)tslot * ROWB + li * 16) = vraw;
    }
}

// ---- streaming kernel: any budget up to H2O_MAX_BUDGET --------------------------------
//
// The key rounds followed by the value rounds form one stream pulled through a
// ring of U register buffers per wave: a buffer is refilled with the entry U
// places ahead as soon as it has been consumed.  Logits, probabilities and the
// per-slot bookkeeping live in LDS; thread j % NT handles slot j.
template <int DT, int D, int NW, int U>
__global__ __launch_bounds__(NW * 64, 4) void decode_stream_kernel(
    char *__restrict__ Kc, char *__restrict__ Vc, float *__restrict__ acc_g,
    int32_t *__restrict__ pos_g, const char *__restrict__ q_g,
    const char *__restrict__ kn_g, const char *__restrict__ vn_g,
    char *__restrict__ out_g, int k, int n_occ, int t, int recent, double scale)
{
    using E = Elem<DT>;
    using T = typename E::T;
    constexpr int EPL = E::EPL;
    constexpr int LPR = D / EPL;
    constexpr int RPW = 64 / LPR;
    constexpr int NT = NW * 64;
    constexpr int RPI = NW * RPW;
    constexpr unsigned ROWB = D * sizeof(T);
    static_assert(LPR >= 8 && LPR <= 32, "a row is read by 8, 16 or 32 lanes");

    const int head = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane / LPR, li = lane % LPR;
    const int kp = (k + 2) & ~1;         // keeps the arrays 8-byte aligned

    extern __shared__ __align__(16) unsigned char smem[];
    double *s_l = reinterpret_cast<double *>(smem);            // [kp] logits, then exp
    float *p_l = reinterpret_cast<float *>(s_l + kp);          // [kp] probabilities
    float *acc_l = p_l + kp;                                   // [kp] updated scores
    int *pos_l = reinterpret_cast<int *>(acc_l + kp);          // [kp]
    float *o_l = reinterpret_cast<float *>(pos_l + kp);        // [NW][D]
    double *red_max = reinterpret_cast<double *>(o_l + NW * D);
    double *red_sum = red_max + NW;
    unsigned long long *red_key = reinterpret_cast<unsigned long long *>(red_sum + NW);
    int *target_l = reinterpret_cast<int *>(red_key + NW);     // [1]

    const size_t hoff = (size_t)head * k;
    char *Kb = Kc + hoff * ROWB;
    char *Vb = Vc + hoff * ROWB;
    const T *qh = reinterpret_cast<const T *>(q_g) + (size_t)head * D;
    const T *knh = reinterpret_cast<const T *>(kn_g) + (size_t)head * D;
    const T *vnh = reinterpret_cast<const T *>(vn_g) + (size_t)head * D;

    const int rounds = (n_occ + RPI - 1) / RPI;
    const int row0 = wave * RPW + sub;
    const int vbase = (rounds + U - 1) / U * U;   // stream index of value round 0
    // stream entry e: key round e for e < rounds, value round e - vbase for
    // vbase <= e < vbase + rounds, nothing in between; entry e lives in buf[e % U]
    auto load_row = [&](const char *base, int round) -> uint4 {
        const unsigned rc = (unsigned)min(round * RPI + row0, max(n_occ, 1) - 1);   // in bounds
        return load_stream(base + (rc * ROWB + (unsigned)li * 16u));
    };

    const uint4 qraw = *reinterpret_cast<const uint4 *>(qh + li * EPL);
    const uint4 kraw = *reinterpret_cast<const uint4 *>(knh + li * EPL);
    uint4 buf[U];
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (u < rounds) buf[u] = load_row(Kb, u);

    double qd[EPL];
    double s_self;
    {
        const T *qe = reinterpret_cast<const T *>(&qraw);
        const T *ke = reinterpret_cast<const T *>(&kraw);
        double a = 0.0;
#pragma unroll
        for (int i = 0; i < EPL; ++i) {
            qd[i] = (double)E::to_f(qe[i]);
            a = fma((double)E::to_f(ke[i]), qd[i], a);
        }
        s_self = group_sum<LPR>(a) * scale;
    }

    // ---- logits ---------------------------------------------------------------
    double m_run = s_self;               // running maximum (the softmax shift)
    for (int r = 0; r < rounds; r += U) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int e = r + u;
            if (e < rounds) {
                const T *x = reinterpret_cast<const T *>(&buf[u]);
                double a = 0.0;
#pragma unroll
                for (int i = 0; i < EPL; ++i) a = fma((double)E::to_f(x[i]), qd[i], a);
                const int nx = e + U;
                if (nx < rounds) buf[u] = load_row(Kb, nx);
                else if (nx >= vbase && nx - vbase < rounds) buf[u] = load_row(Vb, nx - vbase);
                a = group_sum<LPR>(a) * scale;
                const int row = e * RPI + row0;
                if (li == 0 && row < n_occ) s_l[row] = a;
                m_run = fmax(m_run, a);          // clamped duplicates repeat a real row
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    {
        // value rounds the ring has not requested yet (the ring positions that
        // held no entry between the last key round and value round 0)
        const int primed = rounds + U - vbase;
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (u >= primed && u < rounds) buf[u] = load_row(Vb, u);
    }
    {
        const double mw = wave_max(m_run);
        if (lane == 0) red_max[wave] = mw;
    }
    for (int j = tid; j < n_occ; j += NT) {
        pos_l[j] = pos_g[hoff + j];
        acc_l[j] = acc_g[hoff + j];
    }
    lds_barrier();

    // ---- exact softmax (slot j is always handled by thread j % NT, so pos_l /
    // acc_l entries are only ever touched by the thread that wrote them) --------
    double mx = red_max[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) mx = fmax(mx, red_max[w]);
    double d_loc = 0.0;
    for (int j = tid; j < n_occ; j += NT) {
        const double e = exp(s_l[j] - mx);
        s_l[j] = e;
        d_loc += e;
    }
    const double e_self = exp(s_self - mx);
    {
        const double dw = wave_sum(d_loc);
        if (lane == 0) red_sum[wave] = dw;
    }
    lds_barrier();
    double den = e_self;
#pragma unroll
    for (int w = 0; w < NW; ++w) den += red_sum[w];
    const float p_self = (float)(e_self / den);

    // ---- score update and eviction candidates ---------------------------------
    unsigned long long key = NO_CANDIDATE;
    const int last_cand = t - recent;    // window after this step = {t-R+1 .. t}
    for (int j = tid; j < n_occ; j += NT) {
        const float p = (float)(s_l[j] / den);
        p_l[j] = p;
        const float a = acc_l[j] + p;                     // binary32 accumulate
        acc_l[j] = a;
        const int pj = pos_l[j];
        if (pj <= last_cand)
            key = umin64(key, ((unsigned long long)__float_as_uint(a) << 32) | (unsigned)pj);
    }
    {
        const unsigned long long kw = wave_min(key);
        if (lane == 0) red_key[wave] = kw;
        if (tid == 0) *target_l = n_occ < k ? n_occ : -1;
    }
    lds_barrier();
    if (n_occ >= k) {
        key = red_key[0];
#pragma unroll
        for (int w = 1; w < NW; ++w) key = umin64(key, red_key[w]);
        const unsigned long long self_key =
            ((unsigned long long)__float_as_uint(p_self) << 32) | (unsigned)t;
        if (key != NO_CANDIDATE && (recent != 0 || key < self_key)) {
            const int wpos = (int)(unsigned)(key & 0xffffffffu);
            for (int j = tid; j < n_occ; j += NT)
                if (pos_l[j] == wpos) *target_l = j;      // positions are unique
        }
    }

    // ---- output ---------------------------------------------------------------
    float o[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) o[i] = 0.f;
    for (int r = 0; r < rounds; r += U) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int vr = r + u;
            if (vr < rounds) {
                const int row = vr * RPI + row0;
                const float p = row < n_occ ? p_l[row] : 0.f;   // clamped duplicates add nothing
                const uint4 raw = buf[u];
                const int nx = vr + U;
                if (nx < rounds) buf[u] = load_row(Vb, nx);
                const T *x = reinterpret_cast<const T *>(&raw);
#pragma unroll
                for (int i = 0; i < EPL; ++i) o[i] = fmaf(p, E::to_f(x[i]), o[i]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    wave_output_to_lds<EPL, LPR, D>(o, o_l, wave, sub, li);
    lds_barrier();

    // ---- write-back -----------------------------------------------------------
    const int target = *target_l;
    for (int j = tid; j < n_occ; j += NT)
        if (j != target) acc_g[hoff + j] = acc_l[j];
    write_back<DT, D, NW>(o_l, p_self, target, t, hoff, head, Kb, Vb, acc_g, pos_g, knh, vnh, out_g);
}

inline hipError_t raise_lds_limit(const void *kern, size_t smem, bool &raised)
{
    if (smem > 48 * 1024 && !raised) {
        hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           150 * 1024);
        if (e != hipSuccess) return e;
        raised = true;
    }
    return hipSuccess;
}

#define H2O_DECODE_ARGS                                                                         \
    c.K, c.V, c.acc, c.pos, static_cast<const char *>(q), static_cast<const char *>(kn),        \
        static_cast<const char *>(vn), static_cast<char *>(out), c.k, (c.t < c.k ? c.t : c.k),  \
        c.t, c.cfg.recent, c.scale

template <int DT, int D, int NW, int U>
hipError_t launch_resident(const h2o_cache &c, const void *q, const void *kn, const void *vn,
                           void *out, hipStream_t st)
{
    constexpr int LPR = D / Elem<DT>::EPL;
    constexpr int OWN = U * (64 / LPR);
    constexpr size_t smem = (size_t)NW * OWN * (LPR + 1) * 8 + (size_t)NW * 24 +
                            (size_t)NW * OWN * 4 + (size_t)NW * D * 4 + 16;
    auto kern = decode_resident_kernel<DT, D, NW, U>;
    static bool raised = false;
    hipError_t e = raise_lds_limit(reinterpret_cast<const void *>(kern), smem, raised);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(c.cfg.batch * c.cfg.heads), dim3(NW * 64), smem, st,
                       H2O_DECODE_ARGS);
    return hipGetLastError();
}

template <int DT, int D, int NW, int U>
hipError_t launch_stream(const h2o_cache &c, const void *q, const void *kn, const void *vn,
                         void *out, hipStream_t st)
{
    const int kp = (c.k + 2) & ~1;
    const size_t smem = (size_t)kp * 20 + (size_t)NW * D * 4 + (size_t)NW * 24 + 16;
    auto kern = decode_stream_kernel<DT, D, NW, U>;
    static bool raised = false;
    hipError_t e = raise_lds_limit(reinterpret_cast<const void *>(kern), smem, raised);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(c.cfg.batch * c.cfg.heads), dim3(NW * 64), smem, st,
                       H2O_DECODE_ARGS);
    return hipGetLastError();
}

template <int DT, int D>
hipError_t pick(const h2o_cache &c, const void *q, const void *kn, const void *vn, void *out,
                hipStream_t st)
{
    // Waves per head and ring depth follow the number of occupied slots: while
    // every row fits the ring (at most UMAX rounds, and at most one slot per
    // thread) the head is register-resident, with 4 waves per head for small
    // budgets so that more heads share a CU, else 8; beyond that the 8-wave
    // kernel streams the rows through a 13-deep ring.
    constexpr int LPR = D / Elem<DT>::EPL;
    constexpr int RPW = 64 / LPR;
    constexpr int UMAX = RPW * 13 <= 64 ? 13 : 8;
    const int occ = c.t < c.k ? c.t : c.k;
    if (occ <= 4 * RPW * UMAX) {
        const int rounds = (occ + 4 * RPW - 1) / (4 * RPW);
        if (rounds <= 4) return launch_resident<DT, D, 4, 4>(c, q, kn, vn, out, st);
        if (rounds <= 8) return launch_resident<DT, D, 4, 8>(c, q, kn, vn, out, st);
        if constexpr (UMAX > 8) return launch_resident<DT, D, 4, 13>(c, q, kn, vn, out, st);
    }
    const int rounds = (occ + 8 * RPW - 1) / (8 * RPW);
    if (rounds <= 8) return launch_resident<DT, D, 8, 8>(c, q, kn, vn, out, st);
    if constexpr (UMAX > 8) {
        if (rounds <= 13) return launch_resident<DT, D, 8, 13>(c, q, kn, vn, out, st);
    }
    return launch_stream<DT, D, 8, 13>(c, q, kn, vn, out, st);
}

}  // namespace

hipError_t h2o_launch_decode(const h2o_cache &c, const void *q, const void *k_new,
                             const void *v_new, void *out, hipStream_t st)
{
    const int d = c.cfg.head_dim;
    switch (c.cfg.dtype) {
    case H2O_F32:
        return d == 64 ? pick<H2O_F32, 64>(c, q, k_new, v_new, out, st)
                       : pick<H2O_F32, 128>(c, q, k_new, v_new, out, st);
    case H2O_F16:
        return d == 64 ? pick<H2O_F16, 64>(c, q, k_new, v_new, out, st)
                       : pick<H2O_F16, 128>(c, q, k_new, v_new, out, st);
    default:
        return d == 64 ? pick<H2O_BF16, 64>(c, q, k_new, v_new, out, st)
                       : pick<H2O_BF16, 128>(c, q, k_new, v_new, out, st);
    }
}
