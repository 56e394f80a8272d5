// bf16 GEMM C(fp32) = A(bf16) * B(bf16), all row-major, fp32 accumulation on
// the bf16 matrix cores (v_mfma_f32_32x32x16_bf16).
//
// MFMA-bound above n ~ 1.3k, HBM-bound below.  One workgroup of 4 waves owns a
// 128 x 128 tile of C, each wave a 64 x 64 quadrant (2 x 2 MFMA blocks).  The
// MFMA wants, per lane, 8 consecutive k of one A row and 8 consecutive k of
// one B column.  A is row-major, so its tile is copied to LDS as is; B is
// k-major in memory, so its tile is transposed on the way into LDS (two k rows
// are zipped into 32-bit {k, k+1} pairs per column) and both operands are then
// fetched with one 16-byte LDS read per MFMA operand.
//
// MFMA 32x32x16 layout (lane l): a = A[l % 32][8*(l/32) .. +7],
// b = B[8*(l/32) .. +7][l % 32], acc[r] = C[8*(r/4) + 4*(l/32) + r%4][l % 32].
#include "../../include/mgb.h"
#include "launch_util.h"

#include <hip/hip_runtime.h>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr uint32_t GB_BM = 128, GB_BN = 128, GB_BK = 32, GB_THREADS = 256;
constexpr uint32_t GB_LD = GB_BK + 8;   // LDS row pitch in elements (80 bytes, keeps 16-byte alignment)

union Frag {
  uint4 q;
  uint32_t d[4];
  uint16_t h[8];
  bf16x8 v;
};

template <bool FAST>
__global__ __launch_bounds__(GB_THREADS) void gemm_bf16_kernel(const uint16_t* __restrict__ A,
                                                              const uint16_t* __restrict__ B,
                                                              float* __restrict__ C, uint32_t M,
                                                              uint32_t N, uint32_t K,
                                                              uint32_t tiles_n, uint32_t tiles_total) {
  __shared__ __attribute__((aligned(16))) uint16_t As[2][GB_BM][GB_LD];   // [m][k]
  __shared__ __attribute__((aligned(16))) uint16_t Bs[2][GB_BN][GB_LD];   // [n][k]

  const uint32_t per_xcd = (tiles_total + 7u) / 8u;
  const uint32_t tile = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
  if ((blockIdx.x >> 3) >= per_xcd || tile >= tiles_total) return;
  const uint32_t bm = (tile / tiles_n) * GB_BM;
  const uint32_t bn = (tile % tiles_n) * GB_BN;

  const uint32_t tid = threadIdx.x;
  const uint32_t lane = tid & 63u, wave = tid >> 6;
  const uint32_t wm = (wave >> 1) * 64u, wn = (wave & 1u) * 64u;
  const uint32_t l32 = lane & 31u, lhi = lane >> 5;

  // staging roles.  A: rows {tid/4, tid/4 + 64}, 8-element chunk tid % 4.
  //                 B: k pair tid / 16 (rows 2p, 2p+1), 8 columns starting at 8 * (tid % 16).
  const uint32_t a_row = tid >> 2, a_ch = tid & 3u;
  const uint32_t b_kp = tid >> 4, b_ng = tid & 15u;
  Frag ra[2], rb[2];

  auto load_tiles = [&](uint32_t k0) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint32_t gr = bm + a_row + 64u * h, gk = k0 + 8u * a_ch;
      if (FAST) {
        ra[h].q = *reinterpret_cast<const uint4*>(A + (size_t)gr * K + gk);
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) ra[h].h[i] = (gr < M && gk + i < K) ? A[(size_t)gr * K + gk + i] : (uint16_t)0;
      }
      const uint32_t gkb = k0 + 2u * b_kp + h, gc = bn + 8u * b_ng;
      if (FAST) {
        rb[h].q = *reinterpret_cast<const uint4*>(B + (size_t)gkb * N + gc);
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) rb[h].h[i] = (gkb < K && gc + i < N) ? B[(size_t)gkb * N + gc + i] : (uint16_t)0;
      }
    }
  };
  auto store_tiles = [&](uint32_t buf) {
#pragma unroll
    for (int h = 0; h < 2; ++h)
      *reinterpret_cast<uint4*>(&As[buf][a_row + 64u * h][8u * a_ch]) = ra[h].q;
    // zip rows k (rb[0]) and k+1 (rb[1]): column i gets the pair {B[k][i], B[k+1][i]}
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const uint32_t pair = (uint32_t)rb[0].h[i] | ((uint32_t)rb[1].h[i] << 16);
      *reinterpret_cast<uint32_t*>(&Bs[buf][8u * b_ng + i][2u * b_kp]) = pair;
    }
  };

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const uint32_t nk = (K + GB_BK - 1u) / GB_BK;
  load_tiles(0);
  store_tiles(0);
  __syncthreads();
  for (uint32_t kt = 0; kt < nk; ++kt) {
    const uint32_t buf = kt & 1u;
    if (kt + 1u < nk) load_tiles((kt + 1u) * GB_BK);
#pragma unroll
    for (uint32_t ks = 0; ks < GB_BK; ks += 16u) {
      Frag a0, a1, b0, b1;
      a0.q = *reinterpret_cast<const uint4*>(&As[buf][wm + l32][ks + 8u * lhi]);
      a1.q = *reinterpret_cast<const uint4*>(&As[buf][wm + 32u + l32][ks + 8u * lhi]);
      b0.q = *reinterpret_cast<const uint4*>(&Bs[buf][wn + l32][ks + 8u * lhi]);
      b1.q = *reinterpret_cast<const uint4*>(&Bs[buf][wn + 32u + l32][ks + 8u * lhi]);
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0.v, b0.v, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0.v, b1.v, acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1.v, b0.v, acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1.v, b1.v, acc[1][1], 0, 0, 0);
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
  g.tiles_m = (m + GB_BM - 1u) / GB_BM;
  g.tiles_n = (n + GB_BN - 1u) / GB_BN;
  g.total = g.tiles_m * g.tiles_n;
  g.blocks = ((g.total + 7u) / 8u) * 8u;
  g.fast = m % GB_BM == 0u && n % GB_BN == 0u && k % GB_BK == 0u;
  return g;
}

bool shape_ok(uint32_t m, uint32_t n, uint32_t k) {
  return m >= 1u && n >= 1u && k >= 1u && m <= 65536u && n <= 65536u && k <= 65536u;
}

}  // namespace

extern "C" {

int mgb_gemm_bf16_probe(uint32_t m, uint32_t n, uint32_t k, uint64_t* mem_bytes, mgb_dim3* grid,
                        mgb_dim3* block) {
  if (!mem_bytes || !grid || !block) return MGB_E_INVAL;
  if (!shape_ok(m, n, k)) return MGB_E_UNSUPPORTED;
  const Geometry g = geometry(m, n, k);
  *mem_bytes = ((uint64_t)m * k + (uint64_t)k * n) * 2 + (uint64_t)m * n * 4;
  *grid = mgb_dim3{g.blocks, 1u, 1u};
  *block = mgb_dim3{GB_THREADS, 1u, 1u};
  return MGB_OK;
}

int mgb_gemm_bf16_enqueue(void* stream, const uint16_t* A, const uint16_t* B, float* C, uint32_t m,
                          uint32_t n, uint32_t k) {
  if (!A || !B || !C) return MGB_E_INVAL;
  if (!shape_ok(m, n, k)) return MGB_E_UNSUPPORTED;
  const Geometry g = geometry(m, n, k);
  const bool aligned = (((uintptr_t)A | (uintptr_t)B | (uintptr_t)C) & 15u) == 0u;
  hipStream_t st = (hipStream_t)stream;
  if (g.fast && aligned)
    hipLaunchKernelGGL(gemm_bf16_kernel<true>, dim3(g.blocks), dim3(GB_THREADS), 0, st, A, B, C, m,
                       n, k, g.tiles_n, g.total);
  else
    hipLaunchKernelGGL(gemm_bf16_kernel<false>, dim3(g.blocks), dim3(GB_THREADS), 0, st, A, B, C, m,
                       n, k, g.tiles_n, g.total);
  return mgb_check_launch("gemm_bf16_kernel");
}

}  // extern "C"
