// bf16 GEMM C(fp32) = A(bf16) * B(bf16), all row-major, fp32 accumulation on
// the bf16 matrix cores (v_mfma_f32_32x32x16_bf16).
//
// MFMA-bound above n ~ 1.3k, HBM-bound below.  One workgroup of 4 waves owns a
// 128 x 256 tile of C, each wave a 64 x 128 piece (2 x 4 MFMA blocks): at the
// bf16 MFMA rate a smaller wave tile would be bound by LDS read bandwidth
// (a 64 x 128 piece reads 6 KiB of operands per 8 MFMAs).
//
// The MFMA wants, per lane, 8 consecutive k of one A row and 8 consecutive k
// of one B column.  A is row-major, so its tile is copied to LDS as is and read
// back 16 bytes per lane.  B is k-major in memory; its tile is also copied to
// LDS as is (no shuffling in registers) and the k-contiguous operand is formed
// by the LDS transpose read of gfx950, ds_read_b64_tr_b16: within each group of
// 16 lanes, lane i receives element (i % 4) of the four 8-byte rows addressed by
// lanes i/4, i/4 + 4, i/4 + 8, i/4 + 12.  With lane s of a group pointing at
// B[k0 + s/4][n0 + 4*(s%4) ..], lane i gets B[k0 .. k0+3][n0 + i].
//
// LDS pitches: A rows 80 bytes (conflict-free 16-byte reads), B rows
// 2*256 + 64 bytes so that the four k rows one transpose read touches fall in
// different bank quarters.
//
// MFMA 32x32x16 layout (lane l): a = A[l % 32][8*(l/32) .. +7],
// b = B[8*(l/32) .. +7][l % 32], acc[r] = C[8*(r/4) + 4*(l/32) + r%4][l % 32].
#include "../../include/mgb.h"
#include "launch_util.h"

#include <hip/hip_runtime.h>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr uint32_t GB_BM = 128, GB_BN = 256, GB_BK = 32, GB_THREADS = 256;
constexpr uint32_t GB_LDA = GB_BK + 8;      // A pitch in elements (80 bytes)
constexpr uint32_t GB_LDB = GB_BN + 32;     // B pitch in elements (576 bytes)

typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // one 16-byte chunk (native vector: bit casts stay in registers)

// guarded element-wise gather of 8 consecutive bf16 into one 16-byte chunk (ragged shapes)
__device__ __forceinline__ u32x4 gather8(const uint16_t* __restrict__ p, bool row_ok, uint32_t first,
                                         uint32_t limit) {
  uint32_t w[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t lo = (row_ok && first + 2u * i < limit) ? p[2 * i] : 0u;
    const uint32_t hi = (row_ok && first + 2u * i + 1u < limit) ? p[2 * i + 1] : 0u;
    w[i] = lo | (hi << 16);
  }
  return u32x4{w[0], w[1], w[2], w[3]};
}

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 q) { return __builtin_bit_cast(bf16x8, q); }
__device__ __forceinline__ bf16x8 join_bf16x8(s16x4 lo, s16x4 hi) {
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;

template <bool FAST>
__global__ __launch_bounds__(GB_THREADS, 2) void gemm_bf16_kernel(const uint16_t* __restrict__ A,
                                                              const uint16_t* __restrict__ B,
                                                              float* __restrict__ C, uint32_t M,
                                                              uint32_t N, uint32_t K,
                                                              uint32_t tiles_n, uint32_t tiles_total,
                                                              uint32_t vec_ok) {
  __shared__ __attribute__((aligned(16))) uint16_t As[2][GB_BM][GB_LDA];   // [m][k]
  __shared__ __attribute__((aligned(16))) uint16_t Bs[2][GB_BK][GB_LDB];   // [k][n]

  // XCD-aware tile order (see the fp32 GEMM): bands of 8 tile rows, down the band first.
  const uint32_t per_xcd = (tiles_total + 7u) / 8u;
  const uint32_t seq = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
  if ((blockIdx.x >> 3) >= per_xcd || seq >= tiles_total) return;
  const uint32_t tiles_m = tiles_total / tiles_n;
  const uint32_t band = seq / (8u * tiles_n);
  const uint32_t band_rows = min(8u, tiles_m - 8u * band);
  const uint32_t in_band = seq - band * 8u * tiles_n;
  const uint32_t bm = (8u * band + in_band % band_rows) * GB_BM;
  const uint32_t bn = (in_band / band_rows) * GB_BN;

  // FAST: every tile is full and aligned.  Otherwise tiles that lie fully inside C still take
  // the 16-byte path when the shape allows it (vec_ok: k % 32 == 0, n % 8 == 0, aligned
  // pointers); only ragged edge tiles gather element-wise.  Workgroup-uniform.
  const bool vec = FAST || (vec_ok != 0u && bm + GB_BM <= M && bn + GB_BN <= N);

  const uint32_t tid = threadIdx.x;
  const uint32_t lane = tid & 63u, wave = tid >> 6;
  const uint32_t wm = (wave >> 1) * 64u, wn = (wave & 1u) * 128u;
  const uint32_t l32 = lane & 31u, lhi = lane >> 5;
  // transpose-read roles: 16-lane group q, lane s within it
  const uint32_t tq = lane >> 4, ts = lane & 15u;
  const uint32_t tr_row = 8u * (tq >> 1) + (ts >> 2);            // + ks + 4*r
  const uint32_t tr_col = 16u * (tq & 1u) + 4u * (ts & 3u);      // + wn + 32*j

  // staging: A tile = 512 chunks of 8 elements (row f/4, chunk f%4), 2 per thread;
  //          B tile = 1024 chunks (k row f/32, chunk f%32), 4 per thread.
  u32x4 ra[2], rb[4];
  auto load_tiles = [&](uint32_t k0) {
#pragma unroll
    for (uint32_t h = 0; h < 2; ++h) {
      const uint32_t f = tid + GB_THREADS * h;
      const uint32_t gr = bm + (f >> 2), gk = k0 + 8u * (f & 3u);
      // edge tiles: a chunk that lies fully inside the matrix is still one 16-byte load
      if (vec || (vec_ok != 0u && gr < M && gk + 8u <= K)) ra[h] = *reinterpret_cast<const u32x4*>(A + (size_t)gr * K + gk);
      else ra[h] = gather8(A + (size_t)gr * K + gk, gr < M, gk, K);
    }
#pragma unroll
    for (uint32_t h = 0; h < 4; ++h) {
      const uint32_t f = tid + GB_THREADS * h;
      const uint32_t gk = k0 + (f >> 5), gc = bn + 8u * (f & 31u);
      if (vec || (vec_ok != 0u && gk < K && gc + 8u <= N)) rb[h] = *reinterpret_cast<const u32x4*>(B + (size_t)gk * N + gc);
      else rb[h] = gather8(B + (size_t)gk * N + gc, gk < K, gc, N);
    }
  };
  auto store_tiles = [&](uint32_t buf) {
#pragma unroll
    for (uint32_t h = 0; h < 2; ++h) {
      const uint32_t f = tid + GB_THREADS * h;
      *reinterpret_cast<u32x4*>(&As[buf][f >> 2][8u * (f & 3u)]) = ra[h];
    }
#pragma unroll
    for (uint32_t h = 0; h < 4; ++h) {
      const uint32_t f = tid + GB_THREADS * h;
      *reinterpret_cast<u32x4*>(&Bs[buf][f >> 5][8u * (f & 31u)]) = rb[h];
    }
  };

  f32x16 acc[2][4];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
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
      bf16x8 fa[2], fb[4];
#pragma unroll
      for (uint32_t i = 0; i < 2; ++i)
        fa[i] = as_bf16x8(*reinterpret_cast<const u32x4*>(&As[buf][wm + 32u * i + l32][ks + 8u * lhi]));
#pragma unroll
      for (uint32_t j = 0; j < 4; ++j) {
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (lds_s16x4_ptr)&Bs[buf][ks + tr_row][wn + 32u * j + tr_col]);
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (lds_s16x4_ptr)&Bs[buf][ks + 4u + tr_row][wn + 32u * j + tr_col]);
        fb[j] = join_bf16x8(lo, hi);
      }
#pragma unroll
      for (uint32_t i = 0; i < 2; ++i)
#pragma unroll
        for (uint32_t j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1u < nk) store_tiles(buf ^ 1u);
    __syncthreads();
  }

#pragma unroll
  for (uint32_t i = 0; i < 2; ++i)
#pragma unroll
    for (uint32_t j = 0; j < 4; ++j)
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
  const uint32_t vec_ok = (aligned && k % GB_BK == 0u && n % 8u == 0u) ? 1u : 0u;
  if (g.fast && aligned)
    hipLaunchKernelGGL(gemm_bf16_kernel<true>, dim3(g.blocks), dim3(GB_THREADS), 0, st, A, B, C, m,
                       n, k, g.tiles_n, g.total, 1u);
  else
    hipLaunchKernelGGL(gemm_bf16_kernel<false>, dim3(g.blocks), dim3(GB_THREADS), 0, st, A, B, C, m,
                       n, k, g.tiles_n, g.total, vec_ok);
  return mgb_check_launch("gemm_bf16_kernel");
}

}  // extern "C"
