// Global -> LDS DMA building blocks shared by the DMA-ring kernels (bf16 GEMM, 3x3 conv).
// Device code only; not part of the ABI.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

typedef __attribute__((address_space(3))) void* lds_void_ptr;

// s_waitcnt immediate that waits for vmcnt <= n only (gfx9 encoding: vmcnt in bits 3:0 and
// 15:14, expcnt 6:4 and lgkmcnt 11:8 left at "do not wait")
constexpr uint32_t vm_wait(uint32_t n) { return (n & 15u) | ((n >> 4) << 14) | 0x0F70u; }

// 16 bytes per lane from global memory straight into LDS at lds_addr + 16 * lane (lds_addr is
// wave-uniform, no register staging).  Written as asm so that the compiler does not serialise
// every later LDS read behind it (it would put vmcnt(0) before each one); completion is awaited
// with explicit vmcnt waits, and the kernel must drain them before it ends.  The asm writes M0
// (the LDS base of the transfer); M0 is reserved by the compiler, which uses it for nothing else
// in these kernels (the build silences its note that such a clobber is not modelled).
__device__ __forceinline__ void dma16(const void* g, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(g), "s"(lds_addr) : "memory", "m0");
}

// Chunk swizzle of an unpadded 64-byte LDS row (4 chunks of 16 bytes): physical chunk = logical
// chunk ^ row_swz(row).  16 consecutive rows read at one logical chunk hit 16 different 16-byte
// slots of a 256-byte bank sweep, 8 consecutive rows 8 different slots of a 128-byte sweep.
// The DMA realises it by letting each lane fetch the global chunk that belongs at its LDS slot.
__device__ __forceinline__ uint32_t row_swz(uint32_t row) { return ((row >> 2) & 3u) ^ (((row >> 1) & 1u) << 1); }

// wave-uniform LDS byte address of a dynamic shared array
__device__ __forceinline__ uint32_t lds_address_of(const void* smem) {
  return __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_void_ptr)smem);
}
