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

// The same transfer through a buffer resource: lane address = resource base + voff + soff, where
// soff is wave-uniform (a scalar register), so that walking along k needs no vector arithmetic.
// It matters to a kernel that runs one wave per SIMD: every vector-ALU instruction issued between
// two MFMAs holds the matrix pipe up for ~14 clocks (the 64-bit add that forms a global address
// counts) and a load with a 64-bit vector address for 10-17 more, while scalar instructions, LDS
// reads and loads with a scalar base and a 32-bit vector offset, like this one, are free
// (measured: a loop of 64 fp32 MFMAs with one such instruction after every fourth).
// The resource is raw (stride 0) and bounds-checked by the hardware: a lane whose offset lies at
// or beyond `bytes` receives zeros and touches no memory.  Callers keep a resource to the piece
// one workgroup (or one tile) reads, so its size always fits 32 bits.
typedef uint32_t buf_rsrc __attribute__((ext_vector_type(4)));

__device__ __forceinline__ buf_rsrc make_buf_rsrc(const void* base, uint32_t bytes) {
  const uint64_t b = (uint64_t)(uintptr_t)base;
  buf_rsrc r;
  r.x = __builtin_amdgcn_readfirstlane((uint32_t)b);
  r.y = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));                  // stride 0 in the upper half
  r.z = __builtin_amdgcn_readfirstlane(bytes);
  r.w = 0x00020000u;                                                         // 32-bit data format, raw addressing
  return r;
}

__device__ __forceinline__ void buf_dma16(uint32_t voff, buf_rsrc rsrc, uint32_t soff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\tbuffer_load_dwordx4 %0, %1, %3 offen lds"
               : : "v"(voff), "s"(rsrc), "s"(lds_addr), "s"(soff) : "memory", "m0");
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
