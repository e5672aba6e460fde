// Building blocks of the LDS-staged GEMM kernels: direct global -> LDS loads, wait-counter and barrier
// wrappers that leave loads in flight, and the XOR-swizzled row-major operand tile.
#pragma once
#include "ss_common.h"

namespace ss {

constexpr int ROWB = 128; // bytes of one LDS row of a row-major operand tile (one cache line)

typedef __attribute__((address_space(3))) void lds_void;

// 16 (or 4) bytes per lane, global -> LDS; the LDS address is wave-uniform base + lane * size (the base
// goes through M0).  The global address is a wave-uniform pointer in scalar registers plus a 32-bit lane
// offset (the scalar-base form of the load: one address register per lane, no 64-bit address arithmetic).
// The loads are written as assembly on purpose: the compiler's wait-count insertion treats a direct-to-LDS
// load as an access to both address spaces and from then on turns every wait for an LDS read into a wait
// for all of them; as opaque statements they leave its count of LDS reads exact (s_waitcnt lgkmcnt(n)
// with n > 0 between the matrix instructions), and the kernels wait for the loads themselves with
// explicit vmcnt counts anyway.
__device__ inline uint32_t lds_address(const void* lds_ptr)
{
    return __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(const lds_void*)lds_ptr);
}
__device__ inline void lds_dma16_at(const uint8_t* uniform_base, uint32_t lane_off, uint32_t lds_wave_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_wave_addr), "v"(lane_off), "s"(uniform_base) : "memory", "m0");
}
__device__ inline void lds_dma4_at(const uint8_t* uniform_base, uint32_t lane_off, uint32_t lds_wave_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" ::"s"(lds_wave_addr), "v"(lane_off), "s"(uniform_base) : "memory", "m0");
}
__device__ inline void lds_dma16(const uint8_t* uniform_base, uint32_t lane_off, const void* lds_wave_base)
{
    lds_dma16_at(uniform_base, lane_off, lds_address(lds_wave_base));
}
__device__ inline void lds_dma4(const uint8_t* uniform_base, uint32_t lane_off, const void* lds_wave_base)
{
    lds_dma4_at(uniform_base, lane_off, lds_address(lds_wave_base));
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
