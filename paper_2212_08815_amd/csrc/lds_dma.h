// Device helpers shared by the convolution kernels: direct-to-LDS buffer loads and the
// vector-memory wait that goes with them (gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fscnn {

// s_waitcnt with only the vector-memory counter set (gfx9 encoding: vmcnt is split over
// bits 3:0 and 15:14; expcnt and lgkmcnt fields are left at "no wait")
template <int N> __device__ inline void wait_vmcnt()
{
    __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 15) | ((N >> 4) << 14));
}

typedef int int4v __attribute__((ext_vector_type(4)));
typedef float f4v __attribute__((ext_vector_type(4)));

// One buffer load that writes LDS directly (MUBUF with LDS=1): lane l deposits the dword it
// loads at LDS byte address lds_addr + 4*l (or its four dwords at lds_addr + 16*l); a lane whose
// offset is out of the descriptor's range deposits 0.0.  Written as inline assembly on purpose:
// the compiler does not count it as an LDS store, so it puts no vmcnt wait in front of later LDS
// reads of the OTHER buffer.  The caller waits (vmcnt(0), then a barrier) before anyone reads what
// was loaded.  M0 carries the LDS address; it is a register the compiler reserves for itself, so
// its value is saved and put back around the load.
__device__ inline void lds_dma_dwordx4(int4v rsrc, uint32_t lds_addr, int voff)
{
    uint32_t saved;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\t"
                 "buffer_load_dwordx4 %2, %3, 0 offen lds\n\ts_mov_b32 m0, %0"
                 : "=&s"(saved)
                 : "s"(lds_addr), "v"(voff), "s"(rsrc)
                 : "memory");
}
__device__ inline void lds_dma_dword(int4v rsrc, uint32_t lds_addr, int voff)
{
    uint32_t saved;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\t"
                 "buffer_load_dword %2, %3, 0 offen lds\n\ts_mov_b32 m0, %0"
                 : "=&s"(saved)
                 : "s"(lds_addr), "v"(voff), "s"(rsrc)
                 : "memory");
}

}  // namespace fscnn
