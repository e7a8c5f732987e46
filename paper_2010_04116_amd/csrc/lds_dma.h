// Direct HBM/L2 -> LDS loads for gfx950 (buffer_load ... lds), issued so that they overlap
// with the LDS reads of the tile being multiplied.
//
// The loads are written as inline assembly on purpose.  Issued through the compiler's builtin,
// every later LDS read is assumed to alias the pending transfer and is preceded by a wait for
// ALL outstanding loads, including the ones just issued for the next tile: nothing overlaps.
// With the instruction opaque to the compiler, the kernel orders the transfers itself:
//   * wait_vmcnt<n>() before the barrier that publishes a stage (loads retire in issue order,
//     so "at most n outstanding" means every older load has landed),
//   * a workgroup barrier between the last LDS read of a stage and the loads that refill it.
// Each load writes 64 lanes x SIZE bytes at consecutive LDS addresses starting at `lds_addr`
// (wave-uniform, taken from M0); a lane whose byte offset lies outside the descriptor's range
// writes zeros.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace il {

typedef int BufRsrc __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void lds_void;

constexpr uint32_t kOob = 0x80000000u;  // byte offset beyond every buffer: the load returns 0

// Raw buffer descriptor over [base, base+bytes), bytes < 2^31: stride 0, range checked against the
// per-lane byte offset (the scalar offset is not part of the check and is kept at zero).
__device__ inline BufRsrc make_rsrc(const void *base, size_t bytes) {
  const uint64_t a = (uint64_t)base;
  BufRsrc r;  // wave-uniform by construction; readfirstlane pins it to scalar registers
  r.x = __builtin_amdgcn_readfirstlane((int)(uint32_t)a);
  r.y = __builtin_amdgcn_readfirstlane((int)((uint32_t)(a >> 32) & 0xFFFFu));
  r.z = __builtin_amdgcn_readfirstlane((int)(uint32_t)bytes);
  r.w = 0x00020000;
  return r;
}

__device__ inline uint32_t lds_address(const void *p) {
  return (uint32_t)__builtin_amdgcn_readfirstlane((int)(uintptr_t)(lds_void *)p);
}

// (the host pass parses device functions too but cannot check gfx950 assembly)
__device__ inline void dma16(BufRsrc rs, uint32_t lds_addr, uint32_t byte_off) {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
               :: "s"(lds_addr), "v"(byte_off), "s"(rs) : "memory", "m0");
#else
  (void)rs; (void)lds_addr; (void)byte_off;
#endif
}
__device__ inline void dma4(BufRsrc rs, uint32_t lds_addr, uint32_t byte_off) {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds"
               :: "s"(lds_addr), "v"(byte_off), "s"(rs) : "memory", "m0");
#else
  (void)rs; (void)lds_addr; (void)byte_off;
#endif
}

// s_waitcnt with only the vector-memory counter constrained (6-bit field split 4 + 2 on gfx9).
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }
template <int N>
__device__ inline void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt(vmcnt_imm(N));
}

}  // namespace il
