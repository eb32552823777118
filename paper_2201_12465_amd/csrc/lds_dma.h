// Direct-to-LDS loads (global_load_lds_dwordx4) and the wait that orders them.
#pragma once
#include <hip/hip_runtime.h>

namespace fl {

// vmcnt(n) only (gfx9 encoding: vmcnt = imm[3:0] | imm[15:14]<<4; expcnt, lgkmcnt left at "no wait")
#define FL_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | (7 << 4) | (15 << 8))

// One wave-level direct-to-LDS load: lane l's 16 bytes at `src` land at LDS byte address lds_base + 16*l
// (lds_base is wave-uniform and travels in M0).  Written as inline assembly on purpose: through the
// compiler's builtin the instruction counts as a flat access that may touch LDS, and from then on every
// wait the compiler inserts for an LDS read is a wait for ALL outstanding LDS reads (lgkmcnt(0)) -- the
// fragment reads requested ahead for the next step included, which serialises a pipelined loop.  The
// kernels order these loads themselves (s_waitcnt vmcnt + s_barrier before any read of what they wrote),
// so the compiler has nothing to track.  One wait state is required between the write of M0 and the load.
__device__ __forceinline__ void lds_dma16(const void *src, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :
               : "v"(src), "s"(lds_base)
               : "memory", "m0");
}
__device__ __forceinline__ unsigned lds_address(const void *p) {
  return (unsigned)(size_t)(__attribute__((address_space(3))) const unsigned char *)p;
}

}  // namespace fl
