// fp32 GEMM C = A * B (all row-major) on the fp32 matrix cores.
//
// MFMA-bound for all but tiny shapes (2*m*n*k flop over 4*(mk + kn + mn)
// bytes).  One workgroup of 8 waves owns a 128 x 128 tile of C; each wave a
// 32 x 64 piece as 1 x 2 blocks of v_mfma_f32_32x32x2_f32.  A and B tiles of
// depth 16 are staged through LDS (double buffered, one barrier per step, next
// tile prefetched into registers during the MFMAs); A is transposed on the
// way in so that both operands are read from LDS as 32 consecutive floats per
// half-wave (no bank conflicts).  Operand fragments for the next k pair are
// fetched from LDS while the MFMAs of the current pair run.
//
// Eight waves per 128 x 128 tile keep the accumulators at 32 registers per
// lane, so eight waves fit a SIMD and a CU holds four workgroups: wave slots,
// not registers or LDS (32 KiB per workgroup), limit residency.
//
// MFMA 32x32x2 operand layout (lane l of 64): a = A[l % 32][l / 32],
// b = B[l / 32][l % 32], acc[r] = C[8*(r/4) + 4*(l/32) + r%4][l % 32].
#include "../../include/mgb.h"
#include "launch_util.h"

#include <hip/hip_runtime.h>

#ifndef GF_WAVES_M
#define GF_WAVES_M 4     // waves along m: 4 -> wave tile 32 x 64, 2 -> 64 x 64
#endif
#ifndef GF_BAND
#define GF_BAND 8        // tile rows per band of the tile sequence
#endif

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr uint32_t GF_BM = 128, GF_BN = 128, GF_BK = 16;
constexpr uint32_t GF_WM = GF_WAVES_M, GF_WN = 2;                  // wave grid
constexpr uint32_t GF_TM = GF_BM / (32u * GF_WM), GF_TN = GF_BN / (32u * GF_WN);   // MFMA blocks per wave
constexpr uint32_t GF_THREADS = 64u * GF_WM * GF_WN;
constexpr uint32_t GF_LOADS = 512u / GF_THREADS;                   // float4 per thread per operand tile

// FAST: m % 128 == 0, n % 128 == 0, k % 16 == 0, 16-byte aligned -> unguarded 16-byte
// accesses everywhere.  Otherwise the decision is taken per workgroup: a tile that lies fully
// inside C (and k % 16 == 0, n % 4 == 0, aligned pointers: `vec_ok`) still takes the 16-byte
// path, only the ragged edge tiles fall back to guarded scalar accesses.
template <bool FAST>
__global__ __launch_bounds__(GF_THREADS) void gemm_f32_kernel(const float* __restrict__ A,
                                                             const float* __restrict__ B,
                                                             float* __restrict__ C, uint32_t M,
                                                             uint32_t N, uint32_t K,
                                                             uint32_t tiles_n, uint32_t tiles_total,
                                                             uint32_t vec_ok) {
  __shared__ float As[2][GF_BK][GF_BM];   // [k][m]
  __shared__ float Bs[2][GF_BK][GF_BN];   // [k][n]

  // XCD-aware tile order.  Consecutive workgroup ids go to different XCDs, so XCD x takes the
  // contiguous run [x * per_xcd, (x+1) * per_xcd) of a tile sequence that walks C in bands of GF_BAND
  // tile rows, down the band first: the tiles resident in one XCD at a time then form a
  // squarish block and share both their A row slabs and their B column slabs in that XCD's L2.
  const uint32_t per_xcd = (tiles_total + 7u) / 8u;
  const uint32_t seq = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
  if ((blockIdx.x >> 3) >= per_xcd || seq >= tiles_total) return;
  const uint32_t tiles_m = tiles_total / tiles_n;
  constexpr uint32_t BAND = GF_BAND;
  const uint32_t band = seq / (BAND * tiles_n);
  const uint32_t band_rows = min(BAND, tiles_m - BAND * band);
  const uint32_t in_band = seq - band * BAND * tiles_n;
  const uint32_t bm = (BAND * band + in_band % band_rows) * GF_BM;
  const uint32_t bn = (in_band / band_rows) * GF_BN;

  const bool vec = FAST || (vec_ok != 0u && bm + GF_BM <= M && bn + GF_BN <= N);   // workgroup-uniform

  const uint32_t tid = threadIdx.x;
  const uint32_t lane = tid & 63u, wave = tid >> 6;
  const uint32_t wm = (wave / GF_WN) * (32u * GF_TM), wn = (wave % GF_WN) * (32u * GF_TN);
  const uint32_t l32 = lane & 31u, lhi = lane >> 5;

  // global -> register staging.  Operand tiles are 512 float4 each.
  //   A: float4 index f -> row f % 128, k-quad f / 128;  B: row f / 32, column quad f % 32.
  float4 ra[GF_LOADS], rb[GF_LOADS];

  auto load_tiles = [&](uint32_t k0) {
#pragma unroll
    for (uint32_t h = 0; h < GF_LOADS; ++h) {
      const uint32_t f = tid + GF_THREADS * h;
      const uint32_t gr = bm + (f & 127u), gk = k0 + 4u * (f >> 7);
      // edge tiles: a quad that lies fully inside the matrix is still one 16-byte load
      if (vec || (vec_ok != 0u && gr < M && gk + 4u <= K)) {
        ra[h] = *reinterpret_cast<const float4*>(A + (size_t)gr * K + gk);
      } else {
        float t[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) t[i] = (gr < M && gk + i < K) ? A[(size_t)gr * K + gk + i] : 0.f;
        ra[h] = make_float4(t[0], t[1], t[2], t[3]);
      }
      const uint32_t gkb = k0 + (f >> 5), gc = bn + 4u * (f & 31u);
      if (vec || (vec_ok != 0u && gkb < K && gc + 4u <= N)) {
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
    for (uint32_t h = 0; h < GF_LOADS; ++h) {
      const uint32_t f = tid + GF_THREADS * h;
      const uint32_t row = f & 127u, kq = f >> 7;
      As[buf][4u * kq + 0u][row] = ra[h].x;
      As[buf][4u * kq + 1u][row] = ra[h].y;
      As[buf][4u * kq + 2u][row] = ra[h].z;
      As[buf][4u * kq + 3u][row] = ra[h].w;
      *reinterpret_cast<float4*>(&Bs[buf][f >> 5][4u * (f & 31u)]) = rb[h];
    }
  };

  f32x16 acc[GF_TM][GF_TN];
#pragma unroll
  for (uint32_t i = 0; i < GF_TM; ++i)
#pragma unroll
    for (uint32_t j = 0; j < GF_TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const uint32_t nk = (K + GF_BK - 1u) / GF_BK;
  load_tiles(0);
  store_tiles(0);
  __syncthreads();
  for (uint32_t kt = 0; kt < nk; ++kt) {
    const uint32_t buf = kt & 1u;
    if (kt + 1u < nk) load_tiles((kt + 1u) * GF_BK);
    float fa[2][GF_TM], fb[2][GF_TN];
    auto fetch = [&](uint32_t kk, uint32_t slot) {
#pragma unroll
      for (uint32_t i = 0; i < GF_TM; ++i) fa[slot][i] = As[buf][kk + lhi][wm + 32u * i + l32];
#pragma unroll
      for (uint32_t j = 0; j < GF_TN; ++j) fb[slot][j] = Bs[buf][kk + lhi][wn + 32u * j + l32];
    };
    fetch(0, 0);
#pragma unroll
    for (uint32_t kk = 0; kk < GF_BK; kk += 2u) {
      const uint32_t cur = (kk >> 1) & 1u;
      if (kk + 2u < GF_BK) fetch(kk + 2u, cur ^ 1u);
#pragma unroll
      for (uint32_t i = 0; i < GF_TM; ++i)
#pragma unroll
        for (uint32_t j = 0; j < GF_TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[cur][i], fb[cur][j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1u < nk) store_tiles(buf ^ 1u);
    __syncthreads();
  }

#pragma unroll
  for (uint32_t i = 0; i < GF_TM; ++i)
#pragma unroll
    for (uint32_t j = 0; j < GF_TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const uint32_t row = bm + wm + 32u * i + 8u * (r >> 2) + 4u * lhi + (r & 3);
        const uint32_t col = bn + wn + 32u * j + l32;
        if (vec || (row < M && col < N)) C[(size_t)row * N + col] = acc[i][j][r];
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
  const uint32_t vec_ok = (aligned && k % GF_BK == 0u && n % 4u == 0u) ? 1u : 0u;
  if (g.fast && aligned)
    hipLaunchKernelGGL(gemm_f32_kernel<true>, dim3(g.blocks), dim3(GF_THREADS), 0, st, A, B, C, m,
                       n, k, g.tiles_n, g.total, 1u);
  else
    hipLaunchKernelGGL(gemm_f32_kernel<false>, dim3(g.blocks), dim3(GF_THREADS), 0, st, A, B, C, m,
                       n, k, g.tiles_n, g.total, vec_ok);
  return mgb_check_launch("gemm_f32_kernel");
}

}  // extern "C"
