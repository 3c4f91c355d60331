// Global -> LDS loads and the barrier that goes with them (gfx950).
#pragma once
#include <cstdint>

#include <hip/hip_runtime.h>

namespace distdl {

typedef uint32_t lds_u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) char* lds_char_ptr;

// Raw buffer descriptor (base, stride 0, bytes covered, data format word): offsets at or beyond `bytes` are out
// of range (loads return zero).
__device__ inline lds_u32x4 lds_direct_rsrc(const void* p, uint32_t bytes) {
  const uint64_t a = (uint64_t)(uintptr_t)p;
  return lds_u32x4{(uint32_t)a, (uint32_t)(a >> 32), bytes, 0x00020000u};
}

// One global -> LDS load of 16 bytes per lane: lane L's piece lands at LDS address lds_addr + 16 L (measured), an
// out-of-range lane writes zeros (measured).  Written as inline assembly on purpose: the compiler then does not know
// that a load is filling LDS, so it neither waits for every outstanding load (vmcnt(0)) in front of each LDS read
// that it cannot tell apart from the landing area, nor counts these loads; kernels that use it wait with explicit
// s_waitcnt vmcnt(...) counts, which are exact as long as these are the only vector memory loads in flight.
// M0 is written inside the statement and cannot be named as clobbered (the compiler reserves it and refuses it in a
// clobber list); that is sound because the compiler never keeps a value in M0 across other instructions: it loads M0
// immediately before each instruction of its own that reads it.
// The LDS address, the descriptor and soff must be wave-uniform; they are passed through readfirstlane so that they
// sit in scalar registers also where the compiler computed a uniform value with vector instructions.
__device__ inline void load_to_lds(lds_u32x4 desc, uint32_t lds_addr, uint32_t voff, uint32_t soff) {
  lds_addr = __builtin_amdgcn_readfirstlane(lds_addr);
  soff = __builtin_amdgcn_readfirstlane(soff);
  desc = lds_u32x4{(uint32_t)__builtin_amdgcn_readfirstlane(desc[0]), (uint32_t)__builtin_amdgcn_readfirstlane(desc[1]),
                   (uint32_t)__builtin_amdgcn_readfirstlane(desc[2]), (uint32_t)__builtin_amdgcn_readfirstlane(desc[3])};
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :
               : "s"(lds_addr), "v"(voff), "s"(desc), "s"(soff)
               : "memory");
}
__device__ inline uint32_t lds_address(const void* p) { return (uint32_t)(size_t)(lds_char_ptr)p; }

// Workgroup barrier without the fences of __syncthreads(): those make the compiler wait for every outstanding
// global -> LDS load it knows of.  Waits for this wave's LDS operations, then for the other waves; the memory
// clobber keeps the compiler from moving LDS accesses across it.  The caller waits for the loads it needs
// (s_waitcnt vmcnt) before it.
__device__ inline void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// s_waitcnt immediates (vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8; a field of all ones does not wait)
constexpr int kWaitVmcnt0 = 0x0F70, kWaitVmcnt4 = 0x0F74, kWaitVmcnt8 = 0x0F78, kWaitVmcnt16 = 0x4F70;
constexpr int kWaitLgkmcnt0 = 0xC07F;

}  // namespace distdl
