// gfx950 primitives shared by every kernel that stages through LDS without registers: the direct
// global->LDS load, its wait, the raw buffer descriptor whose out-of-range offsets read zeros, and
// the XCD-aware renumbering of workgroups.
#pragma once
#include <hip/hip_runtime.h>

namespace relay {

typedef int intx4 __attribute__((ext_vector_type(4)));

constexpr unsigned kOob = 0x80000000u;  // a buffer offset beyond any num_records this library accepts: reads zeros

// The statement overwrites M0 and says so in its clobber list.  The compiler treats M0 as a reserved
// register (it sets M0 itself right before each of its own instructions that read it and keeps no
// value live there), warns about reserved registers in a clobber list, and honours the entry all the same.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void lds_dma16(intx4 rsrc, unsigned lds_base, unsigned voff) {
  // m0 = wave-uniform LDS byte address; lane i lands at m0 + 16*i
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(lds_base), "v"(voff),
               "s"(rsrc)
               : "memory", "m0");
}
#pragma clang diagnostic pop

// Wait until at most N of this wave's global->LDS loads are pending and all of its LDS reads
// have returned (so that the stage they read may be refilled after the barrier).
template <int N>
__device__ __forceinline__ void wait_loads() {
  asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(N) : "memory");
}

__device__ __forceinline__ intx4 make_rsrc(const void* p, unsigned bytes) {
  const unsigned long long pa = reinterpret_cast<unsigned long long>(p);
  intx4 r;
  r[0] = (int)(unsigned)pa;
  r[1] = (int)(unsigned)((pa >> 32) & 0xffffu);  // stride 0: raw buffer
  r[2] = (int)bytes;                            // num_records
  r[3] = 0x00020000;                            // 32-bit data format, no swizzle
  return r;
}

// Workgroup id -> logical tile id such that consecutive logical ids run on the same XCD
// (workgroups are dealt round-robin over the 8 XCDs, each with its own L2): tiles that
// share input rows or filter tiles then share an L2.
__device__ __forceinline__ int xcd_remap(int bid, int nb) {
  const int xcd = bid & 7, idx = bid >> 3;
  const int per = nb >> 3, rem = nb & 7;
  return xcd < rem ? xcd * (per + 1) + idx : rem * (per + 1) + (xcd - rem) * per + idx;
}

}  // namespace relay
