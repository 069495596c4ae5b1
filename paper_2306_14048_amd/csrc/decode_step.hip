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
#include "wave_ops.h"
#include <type_traits>

namespace {

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
// PAT: a sparse-attention pattern is the protected set (cfg.protect != 0); the plain
// recent-window build carries none of that code.
template <int DT, int D, int NW, int U, bool PAT>
__global__ __launch_bounds__(NW * 64, 4) void decode_resident_kernel(
    char *__restrict__ Kc, char *__restrict__ Vc, float *__restrict__ acc_g,
    int32_t *__restrict__ pos_g, const char *__restrict__ q_g,
    const char *__restrict__ kn_g, const char *__restrict__ vn_g,
    char *__restrict__ out_g, int k, int n_occ, int t, int recent, double scale, int rank, int protect,
    int stride)
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
    // With a sparse-attention pattern as the protected set (protect != 0) the
    // candidates are the slots the pattern does not cover; should it cover them
    // all, protection is void and every slot competes: the minimum over all slots
    // is reduced alongside (in the LDS words of the overflow path, idle by now).
    unsigned long long key = NO_CANDIDATE, own_key = NO_CANDIDATE;
    if constexpr (PAT) {
        if (owner) {
            own_key = ((unsigned long long)__float_as_uint(rank_value(acc_j, pos_j, t, rank)) << 32) |
                      (unsigned)pos_j;
            if (!is_protected(pos_j, t, recent, protect, stride)) key = own_key;
        }
        const double ka = wave_min_f64(__longlong_as_double((long long)own_key));
        if (lane == 0) red_max[wave] = ka;
    } else {
        if (owner && pos_j <= t - recent)                    // window after this step = {t-R+1..t}
            key = ((unsigned long long)__float_as_uint(rank_value(acc_j, pos_j, t, rank)) << 32) |
                  (unsigned)pos_j;
    }
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
        if constexpr (PAT) {
            if (wd != wd) {                                  // the pattern covers every slot
                wd = red_max[0];
#pragma unroll
                for (int w = 1; w < NW; ++w) wd = fmin(wd, red_max[w]);
                key = own_key;
            }
        }
        const unsigned long long win = (unsigned long long)__double_as_longlong(wd);
        const unsigned long long self_key =
            ((unsigned long long)__float_as_uint(p_self) << 32) | (unsigned)t;
        // (a pattern always covers the new token; with the plain window of width 0 it competes)
        const bool evict = wd == wd && (PAT || recent != 0 || win < self_key);
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

// ---- chunked kernel: any budget up to H2O_MAX_BUDGET ----------------------------------
//
// The same straight-line body as the register-resident kernel, run over the
// head in chunks of U rounds (CH = U * RPI slots).  The chunks' key rounds
// followed by their value rounds form one stream through the ring of U
// register buffers: the buffer of round u of a chunk is refilled with round u
// of the next chunk (after the last key chunk: of the first value chunk) as
// soon as it has been consumed, so the ring stays full across chunk borders
// and across the softmax barrier.  No load is conditional (addresses are
// clamped to the last occupied row); the last value chunk, which has nothing
// left to request, is a second copy of the body without refills.
//
// A wave owns the slots whose rows it reads, per chunk one per lane; the fp64
// logits of all chunks are kept in a wave-private LDS array (8 bytes per slot),
// from which the exponentials are evaluated twice: once for the normaliser
// (key phase) and once for the probabilities (value phase; the normaliser is
// only known after the last key chunk).  Scores and positions are read one
// chunk ahead of their use.  Softmax shift and overflow fallback as above.
template <int DT, int D, int NW, int U, bool PAT>
__global__ __launch_bounds__(NW * 64, 4) void decode_chunked_kernel(
    char *__restrict__ Kc, char *__restrict__ Vc, float *__restrict__ acc_g,
    int32_t *__restrict__ pos_g, const char *__restrict__ q_g,
    const char *__restrict__ kn_g, const char *__restrict__ vn_g,
    char *__restrict__ out_g, int k, int n_occ, int t, int recent, double scale, int rank, int protect,
    int stride, int chunks)
{
    using E = Elem<DT>;
    using T = typename E::T;
    constexpr int EPL = E::EPL;
    constexpr int LPR = D / EPL;
    constexpr int RPW = 64 / LPR;
    constexpr int RPI = NW * RPW;
    constexpr int OWN = U * RPW;
    constexpr int CH = U * RPI;          // slots per chunk
    constexpr int PITCH = LPR + 1;
    constexpr unsigned ROWB = D * sizeof(T);
    static_assert(LPR >= 8 && LPR <= 32, "a row is read by 8, 16 or 32 lanes");
    static_assert(OWN <= 64, "one slot per lane and chunk");

    const int head = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane / LPR, li = lane % LPR;

    extern __shared__ __align__(16) unsigned char smem[];
    double *part_l = reinterpret_cast<double *>(smem);                 // [NW][OWN][PITCH]
    double *s_l = part_l + NW * OWN * PITCH;                           // [NW][chunks][OWN] logits
    double *red_sum = s_l + (size_t)NW * chunks * OWN;                 // [NW]
    double *red_max = red_sum + NW;                                    // [NW]
    double *red_key = red_max + NW;                                    // [NW]
    float *p_l = reinterpret_cast<float *>(red_key + NW);              // [NW][OWN]
    float *o_l = p_l + NW * OWN;                                       // [NW][D]
    double *part_w = part_l + wave * OWN * PITCH;
    double *s_w = s_l + (size_t)wave * chunks * OWN;
    float *p_w = p_l + wave * OWN;

    const size_t hoff = (size_t)head * k;
    char *Kb = Kc + hoff * ROWB;
    char *Vb = Vc + hoff * ROWB;
    const T *qh = reinterpret_cast<const T *>(q_g) + (size_t)head * D;
    const T *knh = reinterpret_cast<const T *>(kn_g) + (size_t)head * D;
    const T *vnh = reinterpret_cast<const T *>(vn_g) + (size_t)head * D;

    const int row0 = wave * RPW + sub;   // this lane's row inside a round
    const int last = n_occ - 1;          // n_occ > CH >= 1 here
    // slot this lane owns inside a chunk: the row its lane group reads in round lane / RPW
    const int my_sc = (lane / RPW) * RPI + wave * RPW + (lane % RPW);

    const uint4 qraw = *reinterpret_cast<const uint4 *>(qh + li * EPL);
    const uint4 kraw = *reinterpret_cast<const uint4 *>(knh + li * EPL);
    const uint4 vraw = *reinterpret_cast<const uint4 *>(vnh + li * EPL);
    // byte offset of this lane's piece of round u of chunk c (clamped, in bounds)
    auto row_off = [&](int c, int u) -> unsigned {
        return (unsigned)min(c * CH + u * RPI + row0, last) * ROWB + (unsigned)li * 16u;
    };
    uint4 buf[U];
#pragma unroll
    for (int u = 0; u < U; ++u) buf[u] = load_stream(Kb + row_off(0, u));
    // bookkeeping of the slot owned in chunk 0 (requested behind the first key rounds)
    int pos_nx = pos_g[hoff + min(my_sc, last)];
    float acc_nx = acc_g[hoff + min(my_sc, last)];
    __builtin_amdgcn_sched_barrier(0);

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

    // ---- key phase -----------------------------------------------------------------
    double m_loc = -INFINITY;
    for (int c = 0; c < chunks; ++c) {
        // what refills the ring: the next key chunk, or the first value chunk
        const bool more_keys = c + 1 < chunks;
        const char *nbase = more_keys ? Kb : Vb;
        const int nc = more_keys ? c + 1 : 0;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            pin(buf[u]);
            float x[EPL];
            piece_to_float<DT>(buf[u], x);
            double a0 = 0.0, a1 = 0.0;
#pragma unroll
            for (int i = 0; i < EPL; i += 2) {
                a0 = fma((double)x[i], qd[i], a0);
                a1 = fma((double)x[i + 1], qd[i + 1], a1);
            }
            buf[u] = load_stream(nbase + row_off(nc, u));
            part_w[(u * RPW + sub) * PITCH + li] = a0 + a1;
            __builtin_amdgcn_sched_barrier(0);
        }
        __builtin_amdgcn_wave_barrier();
        if (lane < OWN) {
            const double *pr = part_w + lane * PITCH;
            double a = pr[0], b2 = pr[1];
#pragma unroll
            for (int i = 2; i < LPR; i += 2) { a += pr[i]; b2 += pr[i + 1]; }
            const double s_j = (a + b2) * scale;
            s_w[c * OWN + lane] = s_j;
            if (c * CH + my_sc < n_occ) m_loc = fmax(m_loc, s_j);
        }
        __builtin_amdgcn_wave_barrier();     // the partial-sum tile is reused by the next chunk
    }

    // ---- normaliser (shift = the token's own logit; true maximum on overflow) --------
    // (the exponentials are summed here, not in the key loop: q is no longer live)
    double shift = s_self, e_self = 1.0;
    double d_loc = 0.0;
    if (lane < OWN)
        for (int c = 0; c < chunks; ++c)
            if (c * CH + my_sc < n_occ) d_loc += exp(s_w[c * OWN + lane] - shift);
    {
        const double dw = wave_sum(d_loc);
        if (lane == 0) red_sum[wave] = dw;
    }
    lds_barrier();
    double den = e_self;
#pragma unroll
    for (int w = 0; w < NW; ++w) den += red_sum[w];
    if (!(den <= 1.79769313486231570815e+308)) {
        const double mw = wave_max(m_loc);
        if (lane == 0) red_max[wave] = mw;
        lds_barrier();
        shift = s_self;
#pragma unroll
        for (int w = 0; w < NW; ++w) shift = fmax(shift, red_max[w]);
        d_loc = 0.0;
        if (lane < OWN)
            for (int c = 0; c < chunks; ++c)
                if (c * CH + my_sc < n_occ) d_loc += exp(s_w[c * OWN + lane] - shift);
        e_self = exp(s_self - shift);
        const double dw = wave_sum(d_loc);
        if (lane == 0) red_sum[wave] = dw;
        lds_barrier();
        den = e_self;
#pragma unroll
        for (int w = 0; w < NW; ++w) den += red_sum[w];
    }
    const float p_self = (float)(e_self / den);

    // ---- value phase -----------------------------------------------------------------
    float o[EPL];
    {
        const float ps = (wave == 0 && sub == 0) ? p_self : 0.f;
        const T *x = reinterpret_cast<const T *>(&vraw);
#pragma unroll
        for (int i = 0; i < EPL; ++i) o[i] = ps * E::to_f(x[i]);
    }
    unsigned long long best = NO_CANDIDATE;  // smallest (score, position) among this lane's candidate slots
    int best_slot = 0;
    unsigned long long best_all = NO_CANDIDATE;   // ... among all its slots (pattern modes: see the resident kernel)
    int best_all_slot = 0;
    auto value_chunk = [&](int c, auto refill_tag) {
        constexpr bool REFILL = decltype(refill_tag)::value;
        const int slot = c * CH + my_sc;
        const bool owner = lane < OWN && slot < n_occ;
        const int pos_j = pos_nx;
        float acc_j = acc_nx;
        if (REFILL) {                        // the next chunk's bookkeeping, one chunk ahead
            pos_nx = pos_g[hoff + min(slot + CH, last)];
            acc_nx = acc_g[hoff + min(slot + CH, last)];
        }
        const double e_j = owner ? exp(s_w[c * OWN + min(lane, OWN - 1)] - shift) : 0.0;
        const float p_j = (float)(e_j / den);
        acc_j += p_j;                                            // binary32 accumulate
        if (lane < OWN) p_w[lane] = p_j;
        if (owner) {
            acc_g[hoff + slot] = acc_j;
            if constexpr (PAT) {
                const unsigned long long key =
                    ((unsigned long long)__float_as_uint(rank_value(acc_j, pos_j, t, rank)) << 32) |
                    (unsigned)pos_j;
                if (!is_protected(pos_j, t, recent, protect, stride) && key < best) { best = key; best_slot = slot; }
                if (key < best_all) { best_all = key; best_all_slot = slot; }
            } else if (pos_j <= t - recent) {                    // window after this step = {t-R+1..t}
                const unsigned long long key =
                    ((unsigned long long)__float_as_uint(rank_value(acc_j, pos_j, t, rank)) << 32) |
                    (unsigned)pos_j;
                if (key < best) { best = key; best_slot = slot; }
            }
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float p = p_w[u * RPW + sub];
            pin(buf[u]);
            float x[EPL];
            piece_to_float<DT>(buf[u], x);
#pragma unroll
            for (int i = 0; i < EPL; ++i) o[i] = fmaf(p, x[i], o[i]);
            __builtin_amdgcn_sched_barrier(0);   // the row is consumed before its buffer is requested again
            if (REFILL) buf[u] = load_stream(Vb + row_off(c + 1, u));
            __builtin_amdgcn_sched_barrier(0);
        }
        __builtin_amdgcn_wave_barrier();     // the probability row is reused by the next chunk
    };
    for (int c = 0; c + 1 < chunks; ++c) value_chunk(c, std::true_type{});
    value_chunk(chunks - 1, std::false_type{});
    wave_output_to_lds<EPL, LPR, D>(o, o_l, wave, sub, li);
    {
        const double kw = wave_min_f64(__longlong_as_double((long long)best));
        if (lane == 0) red_key[wave] = kw;
    }
    if constexpr (PAT) {
        const double ka = wave_min_f64(__longlong_as_double((long long)best_all));
        if (lane == 0) red_max[wave] = ka;
    }
    lds_barrier();

    // ---- write-back -----------------------------------------------------------------
    if (tid < D) {
        float r = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) r += o_l[w * D + tid];
        reinterpret_cast<T *>(out_g)[(size_t)head * D + tid] = E::from_f(r);
    }
    int tslot = -1;          // wave-uniform: the slot this wave has to fill, if any
    if (n_occ < k) {
        if (wave == 0) tslot = n_occ;
    } else {
        double wd = red_key[0];
#pragma unroll
        for (int w = 1; w < NW; ++w) wd = fmin(wd, red_key[w]);
        if constexpr (PAT) {
            if (wd != wd) {                                  // the pattern covers every slot
                wd = red_max[0];
#pragma unroll
                for (int w = 1; w < NW; ++w) wd = fmin(wd, red_max[w]);
                best = best_all;
                best_slot = best_all_slot;
            }
        }
        const unsigned long long win = (unsigned long long)__double_as_longlong(wd);
        const unsigned long long self_key =
            ((unsigned long long)__float_as_uint(p_self) << 32) | (unsigned)t;
        const bool evict = wd == wd && (PAT || recent != 0 || win < self_key);
        // keys are unique (positions are); the lane that holds the winner also wrote
        // that slot's score above, so its stores below are ordered behind that one
        const unsigned long long b = __ballot(evict && best == win);
        if (b != 0) tslot = __builtin_amdgcn_readlane(best_slot, __ffsll((long long)b) - 1);
    }
    if (tslot >= 0) {
        if (n_occ < k) {
            if (lane == 0) { pos_g[hoff + tslot] = t; acc_g[hoff + tslot] = p_self; }
        } else if (best_slot == tslot && best != NO_CANDIDATE) {
            pos_g[hoff + tslot] = t;
            acc_g[hoff + tslot] = p_self;
        }
        if (lane < LPR)
            *reinterpret_cast<uint4 *>(Kb + (size_t)tslot * ROWB + li * 16) = kraw;
        else if (lane < 2 * LPR)
            *reinterpret_cast<uint4 *>(Vb + (size_t)tslot * ROWB + li * 16) = vraw;
    }
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
        c.t, c.cfg.recent, c.scale, c.cfg.rank, c.cfg.protect, c.cfg.stride

template <int DT, int D, int NW, int U>
hipError_t launch_resident(const h2o_cache &c, const void *q, const void *kn, const void *vn,
                           void *out, hipStream_t st)
{
    constexpr int LPR = D / Elem<DT>::EPL;
    constexpr int OWN = U * (64 / LPR);
    constexpr size_t smem = (size_t)NW * OWN * (LPR + 1) * 8 + (size_t)NW * 24 +
                            (size_t)NW * OWN * 4 + (size_t)NW * D * 4 + 16;
    if (c.cfg.protect != H2O_PROTECT_RECENT) {
        auto kern = decode_resident_kernel<DT, D, NW, U, true>;
        static bool raised = false;
        hipError_t e = raise_lds_limit(reinterpret_cast<const void *>(kern), smem, raised);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, dim3(c.cfg.batch * c.cfg.heads), dim3(NW * 64), smem, st, H2O_DECODE_ARGS);
        return hipGetLastError();
    }
    auto kern = decode_resident_kernel<DT, D, NW, U, false>;
    static bool raised = false;
    hipError_t e = raise_lds_limit(reinterpret_cast<const void *>(kern), smem, raised);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(c.cfg.batch * c.cfg.heads), dim3(NW * 64), smem, st,
                       H2O_DECODE_ARGS);
    return hipGetLastError();
}

template <int DT, int D, int NW, int U>
hipError_t launch_chunked(const h2o_cache &c, const void *q, const void *kn, const void *vn,
                          void *out, hipStream_t st)
{
    constexpr int LPR = D / Elem<DT>::EPL;
    constexpr int RPW = 64 / LPR;
    constexpr int OWN = U * RPW;
    constexpr int CH = U * NW * RPW;
    const int occ = c.t < c.k ? c.t : c.k;
    const int chunks = (occ + CH - 1) / CH;
    const size_t smem = (size_t)NW * OWN * (LPR + 1) * 8 + (size_t)NW * chunks * OWN * 8 +
                        (size_t)NW * 24 + (size_t)NW * OWN * 4 + (size_t)NW * D * 4 + 16;
    if (c.cfg.protect != H2O_PROTECT_RECENT) {
        auto kern = decode_chunked_kernel<DT, D, NW, U, true>;
        static bool raised = false;
        hipError_t e = raise_lds_limit(reinterpret_cast<const void *>(kern), smem, raised);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, dim3(c.cfg.batch * c.cfg.heads), dim3(NW * 64), smem, st, H2O_DECODE_ARGS,
                           chunks);
        return hipGetLastError();
    }
    auto kern = decode_chunked_kernel<DT, D, NW, U, false>;
    static bool raised = false;
    hipError_t e = raise_lds_limit(reinterpret_cast<const void *>(kern), smem, raised);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(c.cfg.batch * c.cfg.heads), dim3(NW * 64), smem, st,
                       H2O_DECODE_ARGS, chunks);
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
    // kernel works through the head in chunks of that size.
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
        // two more rounds still fit the registers of two workgroups per CU
        if (rounds <= 14) return launch_resident<DT, D, 8, 14>(c, q, kn, vn, out, st);
        if (rounds <= 15) return launch_resident<DT, D, 8, 15>(c, q, kn, vn, out, st);
    }
    // Chunked: the ring depth that wastes the fewest rounds on the last chunk
    // (rounds past the occupied slots re-read the last row)
    constexpr int U1 = UMAX - 2, U2 = UMAX - 4, U3 = UMAX - 6;
    auto waste = [&](int u) { return (rounds + u - 1) / u * u - rounds; };
    int u = UMAX;
    if (waste(U1) < waste(u)) u = U1;
    if (waste(U2) < waste(u)) u = U2;
    if (U3 >= 2 && waste(U3) < waste(u)) u = U3;
    if (u == U1) return launch_chunked<DT, D, 8, U1>(c, q, kn, vn, out, st);
    if (u == U2) return launch_chunked<DT, D, 8, U2>(c, q, kn, vn, out, st);
    if constexpr (U3 >= 2) {
        if (u == U3) return launch_chunked<DT, D, 8, U3>(c, q, kn, vn, out, st);
    }
    return launch_chunked<DT, D, 8, UMAX>(c, q, kn, vn, out, st);
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
