// Diagnostic kernels.
//  * cu_trace: record on which physical compute unit each workgroup ran; used to show that a
//    placement's CU-masked stream confines work to its granules and that disjoint granule sets
//    are disjoint sets of physical CUs.
//  * stream_copy: a plain 16-byte-per-lane device copy of known size; the measured ceiling the
//    HBM-bound kernels are compared with, and the calibration point for traffic counters.
//  * mfma_loop: matrix instructions on registers only, 16 independent accumulator blocks per
//    wave, one wave per SIMD on every CU; the rate the matrix cores sustain on this part (clocks
//    included) when nothing else is in the way, the measured ceiling of the MFMA-bound kernels.
#include "../../include/mgb.h"
#include "launch_util.h"

#include <hip/hip_runtime.h>

namespace {

__global__ __launch_bounds__(64) void cu_trace_kernel(uint32_t* __restrict__ out, uint32_t spin_clocks) {
  uint32_t hw_id, xcc_id;
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw_id));
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc_id));
  // stay resident for a bounded while so that later workgroups land on other CUs
  const unsigned long long t0 = clock64();
  while (clock64() - t0 < (unsigned long long)spin_clocks) {
  }
  if (threadIdx.x == 0) {
    const uint32_t cu = (hw_id >> 8) & 0xfu, se = (hw_id >> 13) & 0x7u, xcc = xcc_id & 0xfu;
    out[blockIdx.x] = (xcc << 8) | (se << 4) | cu;
  }
}

__global__ __launch_bounds__(256) void stream_copy_kernel(uint4* __restrict__ dst,
                                                         const uint4* __restrict__ src, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256u;
  for (size_t i = (size_t)blockIdx.x * 256u + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// Operand values of the MFMA loop: a fixed integer hash of (block, lane, element) mapped to
// [-1, 1) in steps of 2^-23, so that successive instructions see unrelated full-width mantissas
// as they do in a GEMM on real data (constant operands draw less power and clock higher).
__device__ __forceinline__ float loop_operand(uint32_t b, uint32_t lane, uint32_t e) {
  uint32_t h = lane * 2654435761u + b * 40503u + e * 9973u + 12345u;
  h ^= h >> 15;
  h *= 0x2c1b3c6du;
  h ^= h >> 12;
  return (float)(h >> 8) * (1.0f / 8388608.0f) - 1.0f;
}

template <bool BF16>
__global__ __launch_bounds__(256, 1) void mfma_loop_kernel(float* __restrict__ out, uint32_t iters) {
  f32x16 acc[16];
#pragma unroll
  for (int b = 0; b < 16; ++b)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[b][r] = 0.f;
  const uint32_t lane = threadIdx.x & 63u;
  float x[16];
  bf16x8 hx[16];
#pragma unroll
  for (int b = 0; b < 16; ++b) {
    x[b] = loop_operand(b, lane, 0);
#pragma unroll
    for (int e = 0; e < 8; ++e) hx[b][e] = (__bf16)loop_operand(b, lane, e);
  }
  for (uint32_t i = 0; i < iters; ++i) {
#pragma unroll
    for (int b = 0; b < 16; ++b) {
      if (BF16) acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hx[b], hx[b], acc[b], 0, 0, 0);
      else acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(x[b], x[b], acc[b], 0, 0, 0);
    }
  }
  float sum = 0.f;
#pragma unroll
  for (int b = 0; b < 16; ++b)
#pragma unroll
    for (int r = 0; r < 16; ++r) sum += acc[b][r];
  out[(size_t)blockIdx.x * 256u + threadIdx.x] = sum;      // keeps the loop alive
}

}  // namespace

// Marks, in a profiler's kernel trace, which partition a hardware queue belongs to: an empty
// kernel whose grid encodes the partition (first granule * 64 + number of granules workgroups of
// one wave).  Launched by mgb_task_launch in front of a task's kernels when MGB_TAG_PARTITIONS is
// set in the environment.
__global__ __launch_bounds__(64) void partition_tag_kernel() {}

int mgb_internal_tag_partition(hipStream_t stream, uint32_t first_granule, uint32_t n_granules) {
  hipLaunchKernelGGL(partition_tag_kernel, dim3(first_granule * 64u + n_granules), dim3(64), 0, stream);
  return mgb_check_launch("partition_tag_kernel");
}

// Rate at which a CU moves operand rows from memory into LDS with the DMA instruction the ring
// kernels use (16 bytes per lane, 1 KiB per instruction).  Every wave walks its own sequence of
// places through a footprint; an instruction's 64 lanes cover 1024 / row_bytes rows of row_bytes
// bytes, `pitch` bytes apart (row_bytes = 1024: one contiguous KiB).
__global__ __launch_bounds__(256, 2) void fetch_rate_kernel(const uint8_t* src, uint32_t* sink, uint32_t iters, uint32_t row_bytes,
                                                            uint32_t pitch, uint32_t places, uint32_t place_bytes) {
  extern __shared__ __attribute__((aligned(1024))) uint8_t fetch_lds[];
  const uint32_t lds_base = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)fetch_lds);
  const uint32_t tid = threadIdx.x, lane = tid & 63u;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t per_row = row_bytes / 16u;                       // lanes per row
  const size_t lane_off = row_bytes == 1024u ? 16u * lane : (size_t)(lane / per_row) * pitch + 16u * (lane % per_row);
  uint32_t cur = ((blockIdx.x * 4u + wave) * 2654435761u) % places;
  for (uint32_t it = 0; it < iters; ++it) {
#pragma unroll
    for (uint32_t h = 0; h < 8u; ++h) {
      const uint8_t* g = src + (size_t)cur * place_bytes + lane_off;
      const uint32_t at = lds_base + (wave * 8u + h) * 1024u;
      asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(g), "s"(at) : "memory", "m0");
      cur += 7u;
      if (cur >= places) cur -= places;
    }
    __builtin_amdgcn_s_waitcnt(0x0F78);                            // vmcnt(8): one round in flight behind this one
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);                              // vmcnt(0)
  __syncthreads();
  const uint32_t v = reinterpret_cast<const uint32_t*>(fetch_lds)[tid];
  if (v == 0x12345678u) sink[0] = v;                               // (keeps the copies alive)
}

// Rate at which a CU's waves read 16-byte MFMA fragments from LDS: 32 rows of 128 bytes, the
// chunk of a row XOR-swizzled as in the conv kernels (`swizzled` != 0) or not (every lane of a
// half-wave on the same banks).
__global__ __launch_bounds__(256, 2) void lds_read_rate_kernel(uint32_t* sink, uint32_t iters, uint32_t swizzled) {
  __shared__ __attribute__((aligned(16))) uint32_t rows[4u * 2048u];
  const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
  for (uint32_t i = tid; i < 4u * 2048u; i += 256u) rows[i] = i;
  __syncthreads();
  const uint32_t row = lane & 31u, hi = lane >> 5;
  const uint32_t swz = swizzled ? (((row >> 1) & 3u) | (((row ^ (row >> 3)) & 1u) << 2)) : 0u;
  const uint32_t base = wave * 8192u + row * 128u + ((hi ^ swz) << 4);
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (uint32_t it = 0; it < iters; ++it) {
#pragma unroll
    for (uint32_t u = 0; u < 8u; ++u)
      acc ^= *reinterpret_cast<const u32x4*>(reinterpret_cast<const uint8_t*>(rows) + (base ^ ((u & 3u) << 5)));
    asm volatile("" : "+v"(acc) : : "memory");
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678u) sink[0] = acc.x;
}

extern "C" int mgb_mfma_loop_enqueue(void* stream, uint32_t bf16, uint32_t n_blocks, uint32_t iters,
                                     float* out, double* flops) {
  if (!out || n_blocks == 0u || n_blocks > 65536u || iters == 0u || iters > (1u << 24)) return MGB_E_INVAL;
  // per wave and iteration: 16 blocks of 32 x 32 x (16 | 2) multiply-adds
  if (flops) *flops = (double)n_blocks * 4.0 * (double)iters * 16.0 * 2.0 * 32.0 * 32.0 * (bf16 ? 16.0 : 2.0);
  if (bf16) hipLaunchKernelGGL(mfma_loop_kernel<true>, dim3(n_blocks), dim3(256), 0, (hipStream_t)stream, out, iters);
  else hipLaunchKernelGGL(mfma_loop_kernel<false>, dim3(n_blocks), dim3(256), 0, (hipStream_t)stream, out, iters);
  return mgb_check_launch("mfma_loop_kernel");
}

extern "C" int mgb_cu_trace_enqueue(void* stream, uint32_t* out, uint32_t n_blocks) {
  if (!out || n_blocks == 0u || n_blocks > (1u << 20)) return MGB_E_INVAL;
  hipLaunchKernelGGL(cu_trace_kernel, dim3(n_blocks), dim3(64), 0, (hipStream_t)stream, out, 20000u);
  return mgb_check_launch("cu_trace_kernel");
}

extern "C" int mgb_copy_enqueue(void* stream, void* dst, const void* src, uint64_t bytes) {
  if (!dst || !src || bytes == 0u || (bytes & 15u)) return MGB_E_INVAL;
  if (((uintptr_t)dst | (uintptr_t)src) & 15u) return MGB_E_INVAL;
  const size_t n16 = bytes / 16u;
  size_t blocks = (n16 + 255u) / 256u;
  if (blocks > 16384u) blocks = 16384u;          // grid-stride beyond that
  hipLaunchKernelGGL(stream_copy_kernel, dim3((uint32_t)blocks), dim3(256), 0, (hipStream_t)stream,
                     (uint4*)dst, (const uint4*)src, n16);
  return mgb_check_launch("stream_copy_kernel");
}

extern "C" int mgb_fetch_rate_enqueue(void* stream, const void* src, uint64_t footprint_bytes, uint32_t row_bytes,
                                      uint32_t pitch, uint32_t n_blocks, uint32_t iters, uint32_t* sink, double* bytes) {
  if (!src || !sink || n_blocks == 0u || n_blocks > 65536u || iters == 0u || iters > (1u << 20)) return MGB_E_INVAL;
  if (row_bytes != 64u && row_bytes != 128u && row_bytes != 1024u) return MGB_E_INVAL;
  if ((uintptr_t)src & 15u) return MGB_E_INVAL;
  if (row_bytes != 1024u && (pitch < row_bytes || (pitch & 15u))) return MGB_E_INVAL;
  // what one instruction spans, and the granularity of a wave's places
  const uint64_t span = row_bytes == 1024u ? 1024u : (uint64_t)(1024u / row_bytes) * pitch;
  const uint32_t place_bytes = row_bytes == 1024u || pitch == row_bytes ? 1024u : row_bytes;
  if (footprint_bytes < span + place_bytes || (footprint_bytes - span) / place_bytes > 0xffffffffull) return MGB_E_INVAL;
  const uint32_t places = (uint32_t)((footprint_bytes - span) / place_bytes);
  static hipError_t attr = hipFuncSetAttribute((const void*)fetch_rate_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 32768);
  if (attr != hipSuccess) {
    mgb_internal_set_error("fetch_rate_kernel: dynamic LDS size", attr);
    return MGB_E_BACKEND;
  }
  if (bytes) *bytes = (double)n_blocks * 4.0 * (double)iters * 8.0 * 1024.0;
  hipLaunchKernelGGL(fetch_rate_kernel, dim3(n_blocks), dim3(256), 32768, (hipStream_t)stream, (const uint8_t*)src, sink, iters,
                     row_bytes, pitch, places, place_bytes);
  return mgb_check_launch("fetch_rate_kernel");
}

extern "C" int mgb_lds_read_rate_enqueue(void* stream, uint32_t swizzled, uint32_t n_blocks, uint32_t iters, uint32_t* sink,
                                         double* bytes) {
  if (!sink || n_blocks == 0u || n_blocks > 65536u || iters == 0u || iters > (1u << 24)) return MGB_E_INVAL;
  if (bytes) *bytes = (double)n_blocks * 256.0 * (double)iters * 8.0 * 16.0;
  hipLaunchKernelGGL(lds_read_rate_kernel, dim3(n_blocks), dim3(256), 0, (hipStream_t)stream, sink, iters, swizzled);
  return mgb_check_launch("lds_read_rate_kernel");
}
