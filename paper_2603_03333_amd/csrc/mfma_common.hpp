// Pieces shared by the two bf16 MFMA contraction kernels: vector types, the LDS-DMA copy
// instruction, explicit waits and barriers (the compiler does not model LDS-DMA).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

#define DM_GLOBAL_PTR(p) ((const void __attribute__((address_space(1)))*)(p))
#define DM_LDS_PTR(p) ((void __attribute__((address_space(3)))*)(p))

// s_waitcnt with only vmcnt set (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[15:14])
#define DM_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))
// s_barrier that the compiler may not move LDS accesses across
#define DM_BARRIER()               \
  do {                             \
    asm volatile("" ::: "memory"); \
    __builtin_amdgcn_s_barrier();  \
    asm volatile("" ::: "memory"); \
  } while (0)

// One LDS-DMA copy instruction: every lane moves 16 bytes from (uniform base + its 32-bit offset)
// to LDS address (uniform dst + 16 * lane).  Written out so that the address needs no vector ALU
// instruction: the copy wavefronts share their SIMD with wavefronts that keep the vector ALU busy
// with MFMAs (measured on the 256 x 256 kernel: one v_mov per copy cost 6 % of MFMA peak).
__device__ __forceinline__ void dma_copy16(const char* base, uint32_t lane_off, unsigned char* lds_dst) {
  const uint32_t dst = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds_dst;
  asm volatile(
      "s_mov_b32 m0, %2\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %0, %1"
      :
      : "v"(lane_off), "s"(base), "s"(dst)
      : "memory", "m0");
}

// The same copy marked non-temporal, for data that is used once per call: its lines should be the
// first to leave L2.
__device__ __forceinline__ void dma_copy16_stream(const char* base, uint32_t lane_off, unsigned char* lds_dst) {
  const uint32_t dst = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds_dst;
  asm volatile(
      "s_mov_b32 m0, %2\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %0, %1 nt"
      :
      : "v"(lane_off), "s"(base), "s"(dst)
      : "memory", "m0");
}

}  // namespace dm
