// Copies from memory straight into LDS, without a stop in registers.
#pragma once
#include <hip/hip_runtime.h>

namespace pipesd {

// One 1 KB piece: lane i's 16 bytes at src_lane land at dst_wave + 16 i (dst_wave is the same for
// the whole wave).  The copy counts as one outstanding vector-memory load of the wave until it has
// landed; whoever reads the LDS waits for it by hand (s_waitcnt vmcnt), counting the loads issued
// since.
//
// Written as an instruction, not through the compiler's builtin: the compiler books the builtin as
// an access that may touch memory and LDS at once and from there on turns every wait of the wave,
// for ordinary loads and for LDS reads alike, into a wait for zero outstanding operations, which
// undoes reading ahead.  Issued this way the compiler does not know of the copy.  Its own waits stay
// correct: loads complete in the order issued, and it waits until at most as many are outstanding
// as IT has issued since the one it needs, which is never more than really have been.
// (A write of M0 needs one wait state before a load to LDS reads it.)
__device__ __forceinline__ void lds_dma16(const void* src_lane, void* dst_wave) {
  const unsigned lds_addr = (unsigned)(unsigned long long)(__attribute__((address_space(3))) char*)dst_wave;
  asm volatile("s_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src_lane), "{m0}"(lds_addr) : "memory");
}

}  // namespace pipesd
