// Global memory -> LDS without passing through registers (gfx950 "buffer_load ... lds"), shared
// by the kernels that stage their operand tiles this way.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dpbk {

typedef __attribute__((ext_vector_type(4))) int i32x4;

// A lane whose byte offset has bit 31 set lies past any descriptor size used here: it fetches zeros.
constexpr unsigned OOB = 0x80000000u;

// Raw buffer descriptor (stride 0) over `bytes` bytes at `base`.
__device__ __forceinline__ i32x4 make_rsrc(const void* base, unsigned bytes) {
  const uint64_t p = reinterpret_cast<uint64_t>(base);
  i32x4 r;
  r[0] = (int)(uint32_t)p;
  r[1] = (int)(uint32_t)(p >> 32) & 0xFFFF;
  r[2] = (int)bytes;
  r[3] = 0x00020000;
  return r;
}

// 16 bytes per lane from buffer `rsrc` at byte voff + soff to LDS at lds_base + 16 * lane
// (lds_base wave-uniform).  The range check sees voff alone: a lane whose voff is at or past the
// descriptor's size (bit 31 set, or a row past the end of the slab) fetches zeros whatever soff is.
__device__ __forceinline__ void load_to_lds(i32x4 rsrc, unsigned voff, unsigned soff, unsigned lds_base) {
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "s_nop 0\n\t"
      "buffer_load_dwordx4 %1, %2, %3 offen lds"
      :
      : "s"(lds_base), "v"(voff), "s"(rsrc), "s"(soff)
      : "memory", "m0");
}

// Nothing moves across this point in the compiler's instruction scheduling.
#define DP_PIN() __builtin_amdgcn_sched_barrier(0)

}  // namespace dpbk
