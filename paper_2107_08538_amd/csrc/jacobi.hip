// fp32 5-point Jacobi relaxation, one kernel launch per sweep.
//
// HBM-bound: the ideal traffic is one read and one write of every cell per
// sweep (8 bytes per cell update).  Each thread owns four adjacent columns
// (one 16-byte access per row) and marches down JB_ROWS rows keeping the
// north / centre / south rows in registers, so every cell is read from memory
// once per workgroup plus a two-row halo.  West / east neighbours come from
// the neighbouring lane through a wave shuffle; only the two edge lanes of a
// wave issue an extra scalar load (an L1/L2 hit on a line the neighbouring
// wave is streaming anyway).
//
// The arithmetic is exactly v = 0.25f * ((N + S) + (W + E)): two roundings of
// pair sums, one rounding of their sum, an exact scaling.  No FMA can form.
#include "../../include/mgb.h"
#include "launch_util.h"

#include <hip/hip_runtime.h>

namespace {

constexpr uint32_t JB_THREADS = 256;   // 4 waves
constexpr uint32_t JB_ROWS = 16;       // interior rows per workgroup
constexpr uint32_t JB_COLS_V4 = JB_THREADS * 4;

// Workgroups are dealt round-robin to the 8 XCDs in launch order; give each
// XCD one contiguous band of tiles so that the halo rows shared by vertically
// adjacent tiles meet in the same L2.
__device__ __forceinline__ bool tile_of_block(uint32_t tiles_x, uint32_t tiles_y, uint32_t* tx,
                                              uint32_t* ty) {
  const uint32_t total = tiles_x * tiles_y;
  const uint32_t lin = blockIdx.x;
  const uint32_t per_xcd = (total + 7u) / 8u;
  const uint32_t tile = (lin & 7u) * per_xcd + (lin >> 3);
  if ((lin >> 3) >= per_xcd || tile >= total) return false;
  *tx = tile % tiles_x;
  *ty = tile / tiles_x;
  return true;
}

// n % 4 == 0: rows are 16-byte aligned, every thread's four columns are either
// all inside the grid or all outside.
__global__ __launch_bounds__(JB_THREADS) void jacobi_sweep_v4(const float* __restrict__ u,
                                                             float* __restrict__ v, uint32_t n,
                                                             uint32_t tiles_x, uint32_t tiles_y) {
  uint32_t tx, ty;
  if (!tile_of_block(tiles_x, tiles_y, &tx, &ty)) return;
  const uint32_t c0 = tx * JB_COLS_V4 + threadIdx.x * 4u;
  const uint32_t r0 = 1u + ty * JB_ROWS;
  if (c0 >= n) return;
  const uint32_t r1 = min(r0 + JB_ROWS, n - 1u);  // exclusive
  const uint32_t lane = threadIdx.x & 63u;
  const bool has_w = c0 > 0u, has_e = c0 + 4u < n;
  const bool first_col = c0 == 0u, last_col = c0 + 4u == n;

  float4 north = *reinterpret_cast<const float4*>(u + (size_t)(r0 - 1u) * n + c0);
  float4 centre = *reinterpret_cast<const float4*>(u + (size_t)r0 * n + c0);
  // Fixed trip count so the loop unrolls fully and the row loads are issued
  // ahead of use; on the ragged last tile row indices are clamped to stay in
  // bounds and the stores are predicated.
#pragma unroll
  for (uint32_t i = 0; i < JB_ROWS; ++i) {
    const uint32_t r = r0 + i;
    const float* pc = u + (size_t)min(r, n - 1u) * n + c0;
    const float4 south = *reinterpret_cast<const float4*>(u + (size_t)min(r + 1u, n - 1u) * n + c0);
    float west = __shfl_up(centre.w, 1);
    float east = __shfl_down(centre.x, 1);
    if (lane == 0u) west = has_w ? pc[-1] : 0.f;
    if (lane == 63u) east = has_e ? pc[4] : 0.f;
    float4 o;
    o.x = 0.25f * ((north.x + south.x) + (west + centre.y));
    o.y = 0.25f * ((north.y + south.y) + (centre.x + centre.z));
    o.z = 0.25f * ((north.z + south.z) + (centre.y + centre.w));
    o.w = 0.25f * ((north.w + south.w) + (centre.z + east));
    if (first_col) o.x = centre.x;   // boundary columns keep their value
    if (last_col) o.w = centre.w;
    if (r < r1) *reinterpret_cast<float4*>(v + (size_t)r * n + c0) = o;
    north = centre;
    centre = south;
  }
}

// any n: one column per thread.
__global__ __launch_bounds__(JB_THREADS) void jacobi_sweep_v1(const float* __restrict__ u,
                                                             float* __restrict__ v, uint32_t n,
                                                             uint32_t tiles_x, uint32_t tiles_y) {
  uint32_t tx, ty;
  if (!tile_of_block(tiles_x, tiles_y, &tx, &ty)) return;
  const uint32_t c = tx * JB_THREADS + threadIdx.x;
  const uint32_t r0 = 1u + ty * JB_ROWS;
  if (c == 0u || c + 1u >= n) return;
  const uint32_t r1 = min(r0 + JB_ROWS, n - 1u);
  const float* p = u + (size_t)(r0 - 1u) * n + c;
  float north = p[0];
  p += n;
  float centre = p[0];
  for (uint32_t r = r0; r < r1; ++r) {
    const float south = p[n];
    v[(size_t)r * n + c] = 0.25f * ((north + south) + (p[-1] + p[1]));
    north = centre;
    centre = south;
    p += n;
  }
}

struct Geometry {
  uint32_t tiles_x, tiles_y, blocks;
  bool vec4;
};

Geometry geometry(uint32_t n) {
  Geometry g;
  g.vec4 = (n % 4u) == 0u;
  g.tiles_x = g.vec4 ? (n + JB_COLS_V4 - 1u) / JB_COLS_V4 : (n + JB_THREADS - 1u) / JB_THREADS;
  g.tiles_y = (n - 2u + JB_ROWS - 1u) / JB_ROWS;
  const uint32_t total = g.tiles_x * g.tiles_y;
  g.blocks = ((total + 7u) / 8u) * 8u;   // whole rounds over the 8 XCDs
  return g;
}

}  // namespace

extern "C" {

int mgb_jacobi_probe(uint32_t n, uint32_t iters, uint64_t* mem_bytes, mgb_dim3* grid,
                     mgb_dim3* block) {
  (void)iters;
  if (!mem_bytes || !grid || !block) return MGB_E_INVAL;
  if (n < 3u || n > 65536u) return MGB_E_UNSUPPORTED;
  const Geometry g = geometry(n);
  *mem_bytes = 2ull * n * n * sizeof(float);
  *grid = mgb_dim3{g.blocks, 1u, 1u};
  *block = mgb_dim3{JB_THREADS, 1u, 1u};
  return MGB_OK;
}

int mgb_jacobi_enqueue(void* stream, float* u0, float* u1, uint32_t n, uint32_t iters) {
  if (!u0 || !u1 || u0 == u1) return MGB_E_INVAL;
  if (n < 3u || n > 65536u) return MGB_E_UNSUPPORTED;
  if (((uintptr_t)u0 | (uintptr_t)u1) & 15u) return MGB_E_INVAL;
  const Geometry g = geometry(n);
  hipStream_t st = (hipStream_t)stream;
  const float* src = u0;
  float* dst = u1;
  for (uint32_t t = 0; t < iters; ++t) {
    if (g.vec4)
      hipLaunchKernelGGL(jacobi_sweep_v4, dim3(g.blocks), dim3(JB_THREADS), 0, st, src, dst, n,
                         g.tiles_x, g.tiles_y);
    else
      hipLaunchKernelGGL(jacobi_sweep_v1, dim3(g.blocks), dim3(JB_THREADS), 0, st, src, dst, n,
                         g.tiles_x, g.tiles_y);
    float* tmp = const_cast<float*>(src);
    src = dst;
    dst = tmp;
  }
  return mgb_check_launch("jacobi_sweep");
}

}  // extern "C"
