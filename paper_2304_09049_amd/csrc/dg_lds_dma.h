// Loads from global memory straight into LDS (global_load_lds_dwordx4), for kernels that stage operands there.
//
// Why they stage: the address unit of a compute unit takes a load instruction at about one cache line per cycle, so 64
// lanes reading 16 bytes each from 64 different rows cost 94 cycles, from 32 rows 34 - 44, from 16 rows (four
// neighbouring lanes per row) 15 - 20 and contiguous 15 (measured, loads only, L2-resident data); a matrix
// instruction's operand layout, a row per lane, is the worst case.  A staged load lets neighbouring lanes read
// neighbouring bytes; every lane then picks its row's bytes out of LDS.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

// 16 bytes per lane: lane l's land at LDS byte `lds` + 16 l (`lds`: a wavefront-uniform LDS byte address, handed over
// in M0; one wait state between writing M0 and the load).  Written as assembly because the compiler, which cannot tell
// staging buffers apart, would wait for every such load before the next LDS read of any kind; here the wavefront counts
// its own loads (dg_wait_for_loads), and the "memory" clobbers keep the compiler's LDS reads on their side of the loads
// and the waits.  Loads complete in order, so waiting until at most n are outstanding means all but the last n are in.
__device__ __forceinline__ void dg_load16_to_lds(const uint8_t *base, int32_t offset, uint32_t lds)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(offset), "s"(base), "s"(__builtin_amdgcn_readfirstlane(lds)) : "memory", "m0");
}
__device__ __forceinline__ void dg_load16_to_lds(const uint8_t *address, uint32_t lds)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :: "v"(address), "s"(__builtin_amdgcn_readfirstlane(lds)) : "memory", "m0");
}
template <int OUTSTANDING = 0>
__device__ __forceinline__ void dg_wait_for_loads()
{
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(OUTSTANDING) : "memory");
}
// The same with a count known at run time only (the same in every lane), rounded down to a multiple of 4 (waiting for
// more than asked is always correct).  The counter counts every vector memory instruction of the wavefront, stores
// included, and they complete in the order they were issued: a kernel that stores between its staged loads allows for
// the stores it knows it has issued since.
__device__ __forceinline__ void dg_wait_for_loads_at_most(int n)
{
    if (n >= 40) dg_wait_for_loads<40>();
    else if (n >= 36) dg_wait_for_loads<36>();
    else if (n >= 32) dg_wait_for_loads<32>();
    else if (n >= 28) dg_wait_for_loads<28>();
    else if (n >= 24) dg_wait_for_loads<24>();
    else if (n >= 20) dg_wait_for_loads<20>();
    else if (n >= 16) dg_wait_for_loads<16>();
    else if (n >= 12) dg_wait_for_loads<12>();
    else if (n >= 8) dg_wait_for_loads<8>();
    else if (n >= 4) dg_wait_for_loads<4>();
    else dg_wait_for_loads<0>();
}
// (the numeric value of a pointer into LDS is its LDS byte address)
__device__ __forceinline__ uint32_t dg_lds_address(const void *p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void *)p;
}
