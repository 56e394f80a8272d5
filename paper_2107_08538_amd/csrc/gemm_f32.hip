// fp32 GEMM C = A * B (all row-major) on the fp32 matrix cores.
//
// MFMA-bound for all but tiny shapes (2*m*n*k flop over 4*(mk + kn + mn)
// bytes).  One workgroup of 4 waves owns a 128 x 128 tile of C; each wave a
// 64 x 64 quadrant as 2 x 2 blocks of v_mfma_f32_32x32x2_f32.  A and B tiles
// of depth 16 are staged through LDS (double buffered, one barrier per step);
// A is transposed on the way in so that both operands are read from LDS as
// 32 consecutive floats per half-wave (no bank conflicts).
//
// MFMA 32x32x2 operand layout (lane l of 64): a = A[l % 32][l / 32],
// b = B[l / 32][l % 32], acc[r] = C[8*(r/4) + 4*(l/32) + r%4][l % 32].
#include "../../include/mgb.h"
#include "launch_util.h"

#include <hip/hip_runtime.h>

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr uint32_t GF_BM = 128, GF_BN = 128, GF_BK = 16, GF_THREADS = 256;

// FAST: m % 128 == 0, n % 128 == 0, k % 16 == 0 -> unguarded 16-byte loads.
// otherwise every global access is guarded and scalar.
template <bool FAST>
__global__ __launch_bounds__(GF_THREADS) void gemm_f32_kernel(const float* __restrict__ A,
                                                             const float* __restrict__ B,
                                                             float* __restrict__ C, uint32_t M,
                                                             uint32_t N, uint32_t K,
                                                             uint32_t tiles_n, uint32_t tiles_total) {
  __shared__ float As[2][GF_BK][GF_BM];   // [k][m]
  __shared__ float Bs[2][GF_BK][GF_BN];   // [k][n]

  // XCD-aware tile order: consecutive workgroup ids go to different XCDs, so
  // give each XCD a contiguous run of tiles (neighbours share A rows / B cols
  // in that XCD's L2).
  const uint32_t per_xcd = (tiles_total + 7u) / 8u;
  const uint32_t tile = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
  if ((blockIdx.x >> 3) >= per_xcd || tile >= tiles_total) return;
  const uint32_t bm = (tile / tiles_n) * GF_BM;
  const uint32_t bn = (tile % tiles_n) * GF_BN;

  const uint32_t tid = threadIdx.x;
  const uint32_t lane = tid & 63u, wave = tid >> 6;
  const uint32_t wm = (wave >> 1) * 64u, wn = (wave & 1u) * 64u;
  const uint32_t l32 = lane & 31u, lhi = lane >> 5;

  // global -> register staging: A: row = tid % 128, k-quads {tid/128, tid/128 + 2}
  //                             B: rows {tid/32, tid/32 + 8}, column quad tid % 32
  const uint32_t a_row = tid & 127u, a_kq = tid >> 7;
  const uint32_t b_row = tid >> 5, b_cq = tid & 31u;
  float4 ra[2], rb[2];

  auto load_tiles = [&](uint32_t k0) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint32_t kq = a_kq + 2u * h;
      const uint32_t gr = bm + a_row, gk = k0 + 4u * kq;
      if (FAST) {
        ra[h] = *reinterpret_cast<const float4*>(A + (size_t)gr * K + gk);
      } else {
        float t[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) t[i] = (gr < M && gk + i < K) ? A[(size_t)gr * K + gk + i] : 0.f;
        ra[h] = make_float4(t[0], t[1], t[2], t[3]);
      }
      const uint32_t gkb = k0 + b_row + 8u * h, gc = bn + 4u * b_cq;
      if (FAST) {
        rb[h] = *reinterpret_cast<const float4*>(B + (size_t)gkb * N + gc);
      } else {
        float t[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) t[i] = (gkb < K && gc + i < N) ? B[(size_t)gkb * N + gc + i] : 0.f;
        rb[h] = make_float4(t[0], t[1], t[2], t[3]);
      }
    }
  };
  auto store_tiles = [&](uint32_t buf) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint32_t kq = a_kq + 2u * h;
      As[buf][4u * kq + 0u][a_row] = ra[h].x;
      As[buf][4u * kq + 1u][a_row] = ra[h].y;
      As[buf][4u * kq + 2u][a_row] = ra[h].z;
      As[buf][4u * kq + 3u][a_row] = ra[h].w;
      *reinterpret_cast<float4*>(&Bs[buf][b_row + 8u * h][4u * b_cq]) = rb[h];
    }
  };

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const uint32_t nk = (K + GF_BK - 1u) / GF_BK;
  load_tiles(0);
  store_tiles(0);
  __syncthreads();
  for (uint32_t kt = 0; kt < nk; ++kt) {
    const uint32_t buf = kt & 1u;
    if (kt + 1u < nk) load_tiles((kt + 1u) * GF_BK);
#pragma unroll
    for (uint32_t kk = 0; kk < GF_BK; kk += 2u) {
      const float a0 = As[buf][kk + lhi][wm + l32];
      const float a1 = As[buf][kk + lhi][wm + 32u + l32];
      const float b0 = Bs[buf][kk + lhi][wn + l32];
      const float b1 = Bs[buf][kk + lhi][wn + 32u + l32];
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
    }
    if (kt + 1u < nk) store_tiles(buf ^ 1u);
    __syncthreads();
  }

#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const uint32_t row = bm + wm + 32u * i + 8u * (r >> 2) + 4u * lhi + (r & 3);
        const uint32_t col = bn + wn + 32u * j + l32;
        if (FAST || (row < M && col < N)) C[(size_t)row * N + col] = acc[i][j][r];
      }
}

struct Geometry {
  uint32_t tiles_m, tiles_n, total, blocks;
  bool fast;
};

Geometry geometry(uint32_t m, uint32_t n, uint32_t k) {
  Geometry g;
  g.tiles_m = (m + GF_BM - 1u) / GF_BM;
  g.tiles_n = (n + GF_BN - 1u) / GF_BN;
  g.total = g.tiles_m * g.tiles_n;
  g.blocks = ((g.total + 7u) / 8u) * 8u;
  g.fast = m % GF_BM == 0u && n % GF_BN == 0u && k % GF_BK == 0u;
  return g;
}

bool shape_ok(uint32_t m, uint32_t n, uint32_t k) {
  return m >= 1u && n >= 1u && k >= 1u && m <= 65536u && n <= 65536u && k <= 65536u;
}

}  // namespace

extern "C" {

int mgb_gemm_f32_probe(uint32_t m, uint32_t n, uint32_t k, uint64_t* mem_bytes, mgb_dim3* grid,
                       mgb_dim3* block) {
  if (!mem_bytes || !grid || !block) return MGB_E_INVAL;
  if (!shape_ok(m, n, k)) return MGB_E_UNSUPPORTED;
  const Geometry g = geometry(m, n, k);
  *mem_bytes = ((uint64_t)m * k + (uint64_t)k * n + (uint64_t)m * n) * sizeof(float);
  *grid = mgb_dim3{g.blocks, 1u, 1u};
  *block = mgb_dim3{GF_THREADS, 1u, 1u};
  return MGB_OK;
}

int mgb_gemm_f32_enqueue(void* stream, const float* A, const float* B, float* C, uint32_t m,
                         uint32_t n, uint32_t k) {
  if (!A || !B || !C) return MGB_E_INVAL;
  if (!shape_ok(m, n, k)) return MGB_E_UNSUPPORTED;
  const Geometry g = geometry(m, n, k);
  const bool aligned = (((uintptr_t)A | (uintptr_t)B | (uintptr_t)C) & 15u) == 0u;
  hipStream_t st = (hipStream_t)stream;
  if (g.fast && aligned)
    hipLaunchKernelGGL(gemm_f32_kernel<true>, dim3(g.blocks), dim3(GF_THREADS), 0, st, A, B, C, m,
                       n, k, g.tiles_n, g.total);
  else
    hipLaunchKernelGGL(gemm_f32_kernel<false>, dim3(g.blocks), dim3(GF_THREADS), 0, st, A, B, C, m,
                       n, k, g.tiles_n, g.total);
  return mgb_check_launch("gemm_f32_kernel");
}

}  // extern "C"
