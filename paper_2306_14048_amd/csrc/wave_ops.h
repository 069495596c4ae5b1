// Wave-level building blocks of the generation-step kernels: streaming loads,
// DPP reductions over 4..64 lanes, wave-uniform broadcasts, the eviction rank.
// Everything lives in an unnamed namespace: each translation unit gets its own copy.
#pragma once
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

// Marks the point from which a loaded row may be unpacked: inside a loop the
// compiler otherwise moves the unpacking of 16-bit pairs to the end of the
// previous iteration, right behind the loads, and with it the wait for them.
__device__ inline void pin(uint4 &v)
{
    asm volatile("" : "+v"(v.x), "+v"(v.y), "+v"(v.z), "+v"(v.w));
}

// The elements of a loaded 16-byte piece as floats, taken from its four 32-bit
// words with integer operations (a 16-bit element view of the registers makes the
// compiler carry every half in a register of its own across loop iterations).
template <int DT>
__device__ inline void piece_to_float(const uint4 &v, float (&f)[Elem<DT>::EPL])
{
    const unsigned w[4] = {v.x, v.y, v.z, v.w};
    if constexpr (DT == H2O_F32) {
#pragma unroll
        for (int i = 0; i < 4; ++i) f[i] = __uint_as_float(w[i]);
    } else if constexpr (DT == H2O_F16) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = (float)__builtin_bit_cast(_Float16, (unsigned short)(w[i] & 0xffffu));
            f[2 * i + 1] = (float)__builtin_bit_cast(_Float16, (unsigned short)(w[i] >> 16));
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
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
constexpr unsigned long long NO_CANDIDATE = ~0ull;

// What ranks a slot for eviction after the query at position t: its accumulated
// score, or (averaged ranking) that score over the number of queries that have
// scored the token, t - pos + 1, as a correctly rounded binary32 quotient.  The
// new token itself has been scored once, so its value is its first score either way.
__device__ inline float rank_value(float acc, int pos, int t, int rank)
{
    return rank == H2O_RANK_AVERAGED ? __fdiv_rn(acc, (float)(t - pos + 1)) : acc;
}

// What an eviction may not touch when the query sits at position t.  protect 0:
// the last `recent` positions (the method's recent window).  Otherwise the
// positions a sparse-attention pattern lets that query attend to (Sec. 5.2,
// the strided and fixed patterns combined with heavy hitters): strided = a band
// of `recent` positions and every stride-th position counted back from t;
// fixed = the block of `stride` positions holding t and the last `recent`
// positions of every block.
__device__ inline bool is_protected(int p, int t, int recent, int protect, int stride)
{
    if (protect == H2O_PROTECT_STRIDED) return t - p < recent || (t - p) % stride == 0;
    if (protect == H2O_PROTECT_FIXED) return p / stride == t / stride || p % stride >= stride - recent;
    return p > t - recent;
}

// ---- 4-bit group-wise storage ------------------------------------------------------
//
// A lane holds 8 consecutive elements of a row (exact binary32 images); the 8
// lanes of an aligned group of 8 together hold one quantisation group of 64.
// Returns the lane's 8 codes packed into one word (element i in bits 4i..4i+3)
// and the group's (scale, min).  Every operation is a single correctly rounded
// binary32 operation, in the order the storage format is defined in.
__device__ inline unsigned q4_quantise8(const float (&x)[8], float &scale, float &mn)
{
    float lo = x[0], hi = x[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) { lo = fminf(lo, x[i]); hi = fmaxf(hi, x[i]); }
    lo = fminf(lo, __int_as_float(dpp<DPP_XOR1>(__float_as_int(lo))));
    hi = fmaxf(hi, __int_as_float(dpp<DPP_XOR1>(__float_as_int(hi))));
    lo = fminf(lo, __int_as_float(dpp<DPP_XOR2>(__float_as_int(lo))));
    hi = fmaxf(hi, __int_as_float(dpp<DPP_XOR2>(__float_as_int(hi))));
    lo = fminf(lo, __int_as_float(dpp<DPP_HALF_MIRROR>(__float_as_int(lo))));
    hi = fmaxf(hi, __int_as_float(dpp<DPP_HALF_MIRROR>(__float_as_int(hi))));
    mn = lo;
    scale = __fdiv_rn(__fsub_rn(hi, lo), 15.0f);
    unsigned word = 0;
    if (scale > 0.0f) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float c = rintf(__fdiv_rn(__fsub_rn(x[i], lo), scale));   // half to even
            c = fminf(fmaxf(c, 0.0f), 15.0f);
            word |= (unsigned)c << (4 * i);
        }
    }
    return word;
}

// 8 consecutive elements starting at p (16-byte aligned for 16-bit types, 32 for binary32)
template <int DT>
__device__ inline void load8(const typename Elem<DT>::T *p, float (&f)[8])
{
    if constexpr (DT == H2O_F32) {
        const float4 a = *reinterpret_cast<const float4 *>(p);
        const float4 b = *reinterpret_cast<const float4 *>(p + 4);
        f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w;
        f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
    } else {
        const uint4 v = *reinterpret_cast<const uint4 *>(p);
        piece_to_float<DT>(v, f);
    }
}

}  // namespace
