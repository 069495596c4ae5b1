// Direct global -> LDS copies and the waits that go with them, shared by the
// prompt-phase kernels (scoring passes and attention).
//
// The copies are written as inline assembly so that the compiler does not order
// later LDS reads of the OTHER tile buffers behind them; their completion is
// awaited explicitly (dma_wait_upto).  The instruction takes the LDS base
// address from the scalar register m0: the statements name m0 as an input
// operand, so the compiler itself puts the address there and knows that the
// register is used (nothing is written to m0 behind its back).  The s_nop
// covers the wait state between a scalar write of m0 and its use by the copy,
// which the compiler cannot insert for an instruction inside an asm statement.
#pragma once
#include <hip/hip_runtime.h>

namespace {

typedef int i32x4 __attribute__((ext_vector_type(4)));

// Raw buffer descriptor (no stride, no swizzle, 32-bit data format) over `bytes`
// bytes at `base`; reads past the end return zero.
__device__ inline i32x4 make_rsrc(const void *base, unsigned bytes)
{
    const size_t b = reinterpret_cast<size_t>(base);
    i32x4 r;
    r.x = __builtin_amdgcn_readfirstlane((int)(unsigned)b);
    r.y = __builtin_amdgcn_readfirstlane((int)(unsigned)(b >> 32));
    r.z = __builtin_amdgcn_readfirstlane((int)bytes);
    r.w = 0x00020000;
    return r;
}

// Asynchronous 16-byte-per-lane copy: the wave's 64 lanes fill 1 KiB of LDS
// starting at the wave-uniform byte offset `lds_base`, lane l at +16*l, each from
// byte `voff + soff` of the buffer that `rsrc` describes (voff per lane, soff
// wave-uniform: a per-tile advance costs no vector instruction).
__device__ inline void dma16(i32x4 rsrc, unsigned voff, unsigned soff, unsigned lds_base)
{
    asm volatile("s_nop 0\n\tbuffer_load_dwordx4 %0, %1, %2 offen lds"
                 :
                 : "v"(voff), "s"(rsrc), "s"(soff), "{m0}"(lds_base)
                 : "memory");
}

// Same for one dword per lane (lane l writes LDS word l from `lds_base`); lanes
// that are switched off copy nothing.
__device__ inline void dma4(i32x4 rsrc, unsigned voff, unsigned soff, unsigned lds_base)
{
    asm volatile("s_nop 0\n\tbuffer_load_dword %0, %1, %2 offen lds"
                 :
                 : "v"(voff), "s"(rsrc), "s"(soff), "{m0}"(lds_base)
                 : "memory");
}

// Waits until at most N of this wave's vector-memory requests are outstanding.
template <int N> __device__ inline void dma_wait_upto()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Workgroup barrier that first drains this wave's LDS reads (so that a buffer is
// really free once every wave has passed) but leaves global requests in flight.
__device__ inline void wg_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

}  // namespace
