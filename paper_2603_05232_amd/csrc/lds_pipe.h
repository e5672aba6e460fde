// Building blocks of the LDS-staged GEMM kernels: direct global -> LDS loads, wait-counter and barrier
// wrappers that leave loads in flight, and the XOR-swizzled row-major operand tile.
#pragma once
#include "ss_common.h"

namespace ss {

constexpr int ROWB = 128; // bytes of one LDS row of a row-major operand tile (one cache line)

typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void gbl_void;

// 16 (or 4) bytes per lane, global -> LDS; the LDS address is wave-uniform base + lane * size.  The global
// address is given as a wave-uniform pointer plus a 32-bit lane offset; the empty asm pins the uniform part
// in scalar registers so that the load uses its scalar-base addressing form and the lane part stays one
// 32-bit register (otherwise the compiler keeps a 64-bit per-lane address alive for every load stream).
__device__ inline void lds_dma16(const uint8_t* uniform_base, uint32_t lane_off, void* lds_wave_base)
{
    asm volatile("" : "+s"(uniform_base));
    __builtin_amdgcn_global_load_lds((gbl_void*)(uniform_base + lane_off), (lds_void*)lds_wave_base, 16, 0, 0);
}
__device__ inline void lds_dma4(const uint8_t* uniform_base, uint32_t lane_off, void* lds_wave_base)
{
    asm volatile("" : "+s"(uniform_base));
    __builtin_amdgcn_global_load_lds((gbl_void*)(uniform_base + lane_off), (lds_void*)lds_wave_base, 4, 0, 0);
}

// Lane id read from the hardware.  Code that runs once per tile (loader set-up, epilogue) takes the lane id from
// here instead of keeping threadIdx-derived values alive through the k loop, where every register is taken:
// what the compiler cannot keep it spills, and a spill reload waits for all direct loads in flight.
__device__ inline int fresh_lane()
{
    int l;
    asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(l));
    return l;
}

// Wait until at most N of this wave's direct loads are still in flight and all of its LDS reads
// have returned (gfx9 s_waitcnt encoding: vmcnt = bits [3:0] and [15:14], lgkmcnt = bits [11:8]).
template <int N> __device__ inline void wait_vmcnt()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0x0 << 8));
    asm volatile("" ::: "memory");
}

// all LDS reads of this wave have returned (loads in flight are left alone)
__device__ inline void wait_lgkm0()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0xF | (0x3 << 14) | (0x7 << 4) | (0x0 << 8));
    asm volatile("" ::: "memory");
}

// Workgroup barrier without the memory fence of __syncthreads(): direct-to-LDS loads in flight
// for later units must stay in flight.  The empty asm statements keep the compiler from moving
// LDS accesses or load issues across it.
__device__ inline void wg_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// ---- LDS tile of a row-major operand: rows of 128 bytes, XOR-swizzled at 16-byte granularity ----
__device__ inline int swz(int row) { return (row >> 1) & 7; }

__device__ inline const v4i* tile_chunk(const uint8_t* lds_tile, int row, int lc)
{
    return reinterpret_cast<const v4i*>(lds_tile + row * ROWB + ((lc ^ swz(row)) << 4));
}

}  // namespace ss
