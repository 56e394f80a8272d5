// Diagnostic kernels.
//  * cu_trace: record on which physical compute unit each workgroup ran; used to show that a
//    placement's CU-masked stream confines work to its granules and that disjoint granule sets
//    are disjoint sets of physical CUs.
//  * stream_copy: a plain 16-byte-per-lane device copy of known size; the measured ceiling the
//    HBM-bound kernels are compared with, and the calibration point for traffic counters.
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

}  // namespace

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
