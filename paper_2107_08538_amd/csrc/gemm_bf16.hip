// bf16 GEMM C(fp32) = A(bf16) * B(bf16), all row-major, fp32 accumulation on
// the bf16 matrix cores (v_mfma_f32_32x32x16_bf16).
//
// Three kernels.
//
// gemm_bf16_dma_a64_kernel (k % 64 == 0, n % 8 == 0, 16-byte aligned operands): the kernel
// described next, with A fetched in pieces of depth 64 (whole cache lines per row) into a ring of
// its own; see the comment at the kernel.
//
// gemm_bf16_dma_kernel (k % 32 == 0, n % 8 == 0, 16-byte aligned operands): one
// workgroup of 4 waves owns a 256 x 256 tile of C, each wave a 128 x 128 piece
// (4 x 4 MFMA blocks, 256 accumulator registers, one wave per SIMD).  At that
// size a wave reads 128 bytes of operands from LDS per lane for every 16 MFMAs
// and the workgroup pulls 32 KiB from L2 per 32 MFMAs per wave, which keeps
// both LDS and the L2 -> CU path below the MFMA time.  Operand tiles of depth
// 32 travel global -> LDS directly (global_load_lds_dwordx4, no register
// staging) into a ring of four 32 KiB stages, so three tiles are in flight
// while one is consumed and the latency of L2 misses is covered.  The LDS
// layout is unpadded (a DMA instruction fills 1 KiB contiguously, 16 bytes per
// lane) and XOR-swizzled through the choice of the global source chunk of each
// lane.  With one wave per SIMD nothing hides a stalled instruction, so the
// main loop is laid out by hand: after every MFMA exactly one memory
// instruction is issued (a fragment read for the next 16 k, or one DMA
// instruction of a later tile), pinned with scheduling barriers.
//
// gemm_bf16_kernel (any shape): 128 x 256 tiles, 4 waves of 64 x 128, register
// staged; guarded element-wise gathers on ragged edge tiles.
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
// LDS pitches of the register-staged kernel: A rows 80 bytes (conflict-free
// 16-byte reads), B rows 2*256 + 64 bytes so that the four k rows one transpose
// read touches fall in different bank quarters.
//
// MFMA 32x32x16 layout (lane l): a = A[l % 32][8*(l/32) .. +7],
// b = B[8*(l/32) .. +7][l % 32], acc[r] = C[8*(r/4) + 4*(l/32) + r%4][l % 32].
#include "../../include/mgb.h"
#include "launch_util.h"
#include "lds_dma.h"

#include <hip/hip_runtime.h>

#include <mutex>

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

// ---- global -> LDS DMA ring kernel: 2 x 2 waves of (32 WT) x (32 WT), WT = 4 or 2 -------------
constexpr uint32_t GD_BK = 32, GD_THREADS = 256, GD_NST = 4, GD_BAND = 4;
constexpr uint32_t gd_lds_bytes(uint32_t wt) { return GD_NST * (64u * wt * GD_BK * 2u) * 2u; }   // 128 / 64 KiB

// chunk swizzle of a B k-row (16-byte chunks): the four k rows of one transpose read land in
// different 64-byte quarters
__device__ __forceinline__ uint32_t b_swz(uint32_t k) { return (k & 3u) << 2; }

template <uint32_t WT>
__global__ __launch_bounds__(GD_THREADS, WT == 4u ? 1 : 2) void gemm_bf16_dma_kernel(const uint16_t* __restrict__ A,
                                                                                   const uint16_t* __restrict__ B,
                                                                                   float* __restrict__ C, uint32_t M,
                                                                                   uint32_t N, uint32_t K,
                                                                                   uint32_t tiles_n,
                                                                                   uint32_t tiles_total) {
  constexpr uint32_t BM = 64u * WT, BN = 64u * WT;             // workgroup tile
  constexpr uint32_t A_BYTES = BM * GD_BK * 2u, B_BYTES = GD_BK * BN * 2u, STAGE = A_BYTES + B_BYTES;
  constexpr uint32_t ND = BM / 64u;                            // DMA instructions per wave per operand per tile
  constexpr uint32_t B_ROW = BN * 2u;                          // bytes of a B k-row in LDS
  constexpr uint32_t B_CPR = BN / 8u;                          // 16-byte chunks of a B k-row
  constexpr uint32_t NF = 3u * WT;                             // fragment reads per half tile
  constexpr uint32_t NM = WT * WT;                             // MFMAs per half tile
  extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];

  // XCD-aware tile order (see the fp32 GEMM): bands of GD_BAND tile rows, down the band first.
  const uint32_t per_xcd = (tiles_total + 7u) / 8u;
  const uint32_t seq = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
  if ((blockIdx.x >> 3) >= per_xcd || seq >= tiles_total) return;
  const uint32_t tiles_m = tiles_total / tiles_n;
  const uint32_t band = seq / (GD_BAND * tiles_n);
  const uint32_t band_rows = min(GD_BAND, tiles_m - GD_BAND * band);
  const uint32_t in_band = seq - band * GD_BAND * tiles_n;
  const uint32_t bm = (GD_BAND * band + in_band % band_rows) * BM;
  const uint32_t bn = (in_band / band_rows) * BN;

  const uint32_t lds_base = lds_address_of(smem);
  const uint32_t tid = threadIdx.x, lane = tid & 63u;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t wm = (wave >> 1) * (32u * WT), wn = (wave & 1u) * (32u * WT);
  const uint32_t l32 = lane & 31u, lhi = lane >> 5;
  const uint32_t tq = lane >> 4, ts = lane & 15u;
  const uint32_t tr_row = 8u * (tq >> 1) + (ts >> 2);
  const uint32_t tr_col = 16u * (tq & 1u) + 4u * (ts & 3u);

  // DMA roles: wave w, instruction h fills the 1 KiB block b = ND*w + h of the A part and of the B
  // part of a stage.
  //   A block b: rows 16b .. 16b+15 (64 bytes each); lane -> row 16b + lane/4, LDS chunk lane%4.
  //   B block b: 1024 / B_ROW consecutive k rows;    lane -> k row and LDS chunk of its 16 bytes.
  // The lane fetches the global chunk whose swizzled position is its LDS chunk.  Rows beyond M
  // and column chunks beyond N are clamped to the last valid one: what they deliver only feeds
  // entries of C that are never stored.
  const uint16_t* ga[ND];
  const uint16_t* gb[ND];
#pragma unroll
  for (uint32_t h = 0; h < ND; ++h) {
    const uint32_t b = ND * wave + h;
    const uint32_t ar = 16u * b + (lane >> 2);
    ga[h] = A + (size_t)min(bm + ar, M - 1u) * K + 8u * ((lane & 3u) ^ row_swz(ar));
    const uint32_t bk = (1024u / B_ROW) * b + lane / B_CPR;
    gb[h] = B + (size_t)bk * N + min(bn + 8u * ((lane % B_CPR) ^ b_swz(bk)), N - 8u);
  }

  f32x16 acc[WT][WT];
#pragma unroll
  for (uint32_t i = 0; i < WT; ++i)
#pragma unroll
    for (uint32_t j = 0; j < WT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // fragment addresses inside a stage (bytes), for the two 16-wide k halves of a tile
  uint32_t a_off[2][WT], b_lo[2][WT], b_hi[2][WT];
  auto b_off = [&](uint32_t krow, uint32_t col) -> uint32_t {
    return A_BYTES + krow * B_ROW + (((col >> 3) ^ b_swz(krow)) << 4) + (col & 7u) * 2u;
  };
#pragma unroll
  for (uint32_t s = 0; s < 2; ++s) {
#pragma unroll
    for (uint32_t i = 0; i < WT; ++i) {
      const uint32_t row = wm + 32u * i + l32;
      a_off[s][i] = row * 64u + (((2u * s + lhi) ^ row_swz(row)) << 4);
    }
#pragma unroll
    for (uint32_t j = 0; j < WT; ++j) {
      b_lo[s][j] = b_off(16u * s + tr_row, wn + 32u * j + tr_col);
      b_hi[s][j] = b_off(16u * s + 4u + tr_row, wn + 32u * j + tr_col);
    }
  }

  u32x4 fa[2][WT];
  s16x4 blo[2][WT], bhi[2][WT];
  const uint32_t nk = K / GD_BK;
  // one fragment read: q = 0 -> a0; 1 .. 2 WT -> b0 lo, b0 hi, b1 lo, ..; then a1, a2, ..
  // (the order in which the next WT * WT MFMAs, row by row, need them)
  auto frag_load = [&](const uint8_t* st, uint32_t s, uint32_t slot, uint32_t q) {
    if (q == 0u || q > 2u * WT) {
      const uint32_t i = q == 0u ? 0u : q - 2u * WT;
      fa[slot][i] = *reinterpret_cast<const u32x4*>(st + a_off[s][i]);
    } else {
      const uint32_t j = (q - 1u) >> 1;
      if ((q - 1u) & 1u) bhi[slot][j] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(st + b_hi[s][j]));
      else blo[slot][j] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(st + b_lo[s][j]));
    }
  };
  // one DMA instruction of tile kt: part 0 = A, part 1 = B, h = 0 .. ND-1.  The tile index is
  // clamped so that every iteration issues the same number of loads (the vmcnt arithmetic below
  // relies on it); the redundant loads of the last iterations land in stages nobody reads any more.
  auto dma_one = [&](uint32_t kt, uint32_t part, uint32_t h) {
    const uint32_t t = min(kt, nk - 1u);
    const uint32_t st = lds_base + (kt % GD_NST) * STAGE + (ND * wave + h) * 1024u;
    if (part == 0u) dma16(ga[h] + (size_t)t * GD_BK, st);
    else dma16(gb[h] + (size_t)t * GD_BK * N, st + A_BYTES);
  };
  // NM MFMAs on fragment slot `slot`; spread evenly between them NF + ND memory instructions: the
  // fragment reads of (tile ft, half fs) into the other slot, then the DMA instructions of
  // (tile dt, part dpart).  WT = 4: one after every MFMA; WT = 2: two.
  auto block = [&](uint32_t slot, uint32_t ft, uint32_t fs, uint32_t dt, uint32_t dpart) {
    const uint8_t* fst = smem + (ft % GD_NST) * STAGE;
#pragma unroll
    for (uint32_t m = 0; m < NM; ++m) {
      const uint32_t i = m / WT, j = m % WT;
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(fa[slot][i]), join_bf16x8(blo[slot][j], bhi[slot][j]),
                                                          acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (uint32_t x = m * (NF + ND) / NM; x < (m + 1u) * (NF + ND) / NM; ++x) {
        if (x < NF) frag_load(fst, fs, slot ^ 1u, x);
        else dma_one(dt, dpart, x - NF);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // Order of DMA issue: A(0) B(0) .. A(NST-2) B(NST-2) A(NST-1) | B(NST-1) A(NST) | B(NST) A(NST+1) | ..
  // (ND instructions each; one `|` per loop iteration).  Tile t is complete once B(t) has landed.
#pragma unroll
  for (uint32_t t = 0; t < GD_NST - 1u; ++t)
#pragma unroll
    for (uint32_t p = 0; p < 2u; ++p)
#pragma unroll
      for (uint32_t h = 0; h < ND; ++h) dma_one(t, p, h);
#pragma unroll
  for (uint32_t h = 0; h < ND; ++h) dma_one(GD_NST - 1u, 0u, h);
  __builtin_amdgcn_s_waitcnt(vm_wait(2u * ND * (GD_NST - 2u) + ND));   // this wave's part of tile 0 has landed
  __syncthreads();                                                     // ... and everybody else's
#pragma unroll
  for (uint32_t q = 0; q < NF; ++q) frag_load(smem, 0u, 0u, q);
  for (uint32_t kt = 0; kt < nk; ++kt) {
    block(0u, kt, 1u, kt + GD_NST - 1u, 1u);            // second half of tile kt's fragments; B(kt + NST - 1)
    // 2 ND (NST - 2) instructions were issued after B(kt + 1): tile kt+1 has landed when no more
    // than that many are outstanding; the barrier extends that to every wave's part and tells
    // that all reads of tile kt are done (its fragments are in registers), which frees its stage
    __builtin_amdgcn_s_waitcnt(vm_wait(2u * ND * (GD_NST - 2u)));
    __syncthreads();
    block(1u, kt + 1u, 0u, kt + GD_NST, 0u);            // first half of tile kt+1's fragments; A(kt + NST) into the freed stage
  }
  __builtin_amdgcn_s_waitcnt(vm_wait(0));               // no DMA may be in flight when the LDS is given back

#pragma unroll
  for (uint32_t i = 0; i < WT; ++i)
#pragma unroll
    for (uint32_t j = 0; j < WT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const uint32_t row = bm + wm + 32u * i + 8u * (r >> 2) + 4u * lhi + (r & 3);
        const uint32_t col = bn + wn + 32u * j + l32;
        if (row < M && col < N) C[(size_t)row * N + col] = acc[i][j][r];
      }
}

// ---- DMA ring kernel, A fetched 64 deep (k % 64 == 0) -------------------------------------------
// Tiles, waves, the B ring, the order of fragment reads and the MFMA / memory interleave are those
// of gemm_bf16_dma_kernel.  What differs is how A travels.  A row of a depth-32 tile is 64 bytes,
// half a cache line, and a request for half a line costs the L2 -> CU path as much as one for a
// whole line (measured: 64-byte rows arrive at half the rate of 128-byte rows), so A took two
// thirds of the kernel's fetch time.  Here A is fetched in pieces of depth 64: rows of 128 bytes,
// 8 chunks, swizzled by row_swz8 through the lane's choice of source chunk, into a ring of its own
// with GA_NA = 3 stages; one A stage serves two consecutive tiles of B, which keeps its ring of
// four depth-32 stages (rows of 2 BN bytes are whole lines already).  LDS: 3 x 32 KiB + 4 x 16 KiB
// = 160 KiB for 256 x 256 tiles, all a CU has; half of that per workgroup for 128 x 128 tiles.
//
// Order of DMA issue per wave (ND = WT instructions per item; A(u) = columns 64 u .. 64 u + 63 of
// the A tile in two halves of ND instructions, B(t) = rows 32 t .. 32 t + 31 of the B tile):
//   A(0) B(0) B(1) A(1) B(2) A(2)h0 | B(3) A(2)h1 | B(4) A(3)h0 | B(5) A(3)h1 | ...
// one `|` per loop iteration.  Iteration t needs tile t + 1 = B(t + 1) and A((t + 1) / 2) at its
// barrier; 4 ND instructions follow B(t + 1) in this order and A((t + 1) / 2) precedes it, so
// "at most 4 ND outstanding" says both have landed.  A(u + 3) goes into the stage of A(u), which
// the barrier of iteration 2 u + 1 frees (every wave has then issued its last reads of it).
constexpr uint32_t GA_NA = 3;
constexpr uint32_t ga_lds_bytes(uint32_t wt) { return GA_NA * (64u * wt * 128u) + GD_NST * (GD_BK * 64u * wt * 2u); }

// chunk swizzle of an unpadded 128-byte LDS row (8 chunks): 16 consecutive rows read at one logical
// chunk fall into 16 different 16-byte slots of a 256-byte bank sweep
__device__ __forceinline__ uint32_t row_swz8(uint32_t row) {
  return ((row >> 1) & 3u) | (((row ^ (row >> 3)) & 1u) << 2);
}

// The main loop holds no vector arithmetic and no load with a 64-bit vector address: with one wave
// per SIMD each vector-ALU instruction between two MFMAs holds the matrix pipe up for ~14 clocks
// (an MFMA here lasts 32) and such a load for ~17 more, while scalar instructions, LDS reads and
// loads with a scalar base and a 32-bit vector offset cost nothing.  So the loop is unrolled over
// twelve tiles (three A stages of two tiles, four B stages), which makes every stage offset an
// immediate of the LDS read, and the DMA goes through buffer resources: A's walk along k is a
// scalar offset, B's resource is rebased for every tile by the scalar unit.
typedef const u32x4 __attribute__((address_space(3))) * lds_u32x4_ptr;

template <uint32_t WT>
__global__ __launch_bounds__(GD_THREADS, WT == 4u ? 1 : 2) void gemm_bf16_dma_a64_kernel(const uint16_t* __restrict__ A,
                                                                                       const uint16_t* __restrict__ B,
                                                                                       float* __restrict__ C, uint32_t M,
                                                                                       uint32_t N, uint32_t K,
                                                                                       uint32_t tiles_n,
                                                                                       uint32_t tiles_total) {
  constexpr uint32_t BM = 64u * WT, BN = 64u * WT;
  constexpr uint32_t A_BYTES = BM * 128u;                      // one A stage: BM rows of depth 64
  constexpr uint32_t B_BYTES = GD_BK * BN * 2u;                // one B stage: 32 k rows
  constexpr uint32_t B_BASE = GA_NA * A_BYTES;
  constexpr uint32_t ND = WT;                                  // DMA instructions per wave: B tile, half an A stage
  constexpr uint32_t B_ROW = BN * 2u, B_CPR = BN / 8u;
  constexpr uint32_t NF = 3u * WT, NM = WT * WT;
  static_assert(2u * A_BYTES <= 65536u && GD_NST * B_BYTES <= 65536u, "stage offsets must fit the offset field of an LDS read");
  extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];

  const uint32_t per_xcd = (tiles_total + 7u) / 8u;
  const uint32_t seq = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
  if ((blockIdx.x >> 3) >= per_xcd || seq >= tiles_total) return;
  const uint32_t tiles_m = tiles_total / tiles_n;
  const uint32_t band = seq / (GD_BAND * tiles_n);
  const uint32_t band_rows = min(GD_BAND, tiles_m - GD_BAND * band);
  const uint32_t in_band = seq - band * GD_BAND * tiles_n;
  const uint32_t bm = (GD_BAND * band + in_band % band_rows) * BM;
  const uint32_t bn = (in_band / band_rows) * BN;

  const uint32_t lds_base = lds_address_of(smem);
  const uint32_t tid = threadIdx.x, lane = tid & 63u;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t wm = (wave >> 1) * (32u * WT), wn = (wave & 1u) * (32u * WT);
  const uint32_t l32 = lane & 31u, lhi = lane >> 5;
  const uint32_t tq = lane >> 4, ts = lane & 15u;
  const uint32_t tr_row = 8u * (tq >> 1) + (ts >> 2);
  const uint32_t tr_col = 16u * (tq & 1u) + 4u * (ts & 3u);

  // DMA roles.  A: wave w, instruction g (0 .. 2 ND - 1) fills the 1 KiB block b = 2 ND w + g of an
  // A stage = rows 8 b .. 8 b + 7 (128 bytes each); lane -> row 8 b + lane / 8, LDS chunk lane % 8.
  // B: as in gemm_bf16_dma_kernel.  Rows beyond M and column chunks beyond N are clamped.
  // A's resource covers this workgroup's rows (at most 2^25 bytes; the scalar offset walks along
  // k), B's is rebased for every tile to its 32 k rows (at most 2^22 bytes).
  const buf_rsrc rsrc_a = make_buf_rsrc(A + (size_t)bm * K, min(BM, M - bm) * K * 2u);
  uint32_t va[2u * ND], vb[ND];
#pragma unroll
  for (uint32_t g = 0; g < 2u * ND; ++g) {
    const uint32_t ar = 8u * (2u * ND * wave + g) + (lane >> 3);
    va[g] = (min(bm + ar, M - 1u) - bm) * K * 2u + 16u * ((lane & 7u) ^ row_swz8(ar));
  }
#pragma unroll
  for (uint32_t h = 0; h < ND; ++h) {
    const uint32_t b = ND * wave + h;
    const uint32_t bk = (1024u / B_ROW) * b + lane / B_CPR;
    vb[h] = (bk * N + min(bn + 8u * ((lane % B_CPR) ^ b_swz(bk)), N - 8u)) * 2u;
  }

  f32x16 acc[WT][WT];
#pragma unroll
  for (uint32_t i = 0; i < WT; ++i)
#pragma unroll
    for (uint32_t j = 0; j < WT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // LDS addresses of the fragments (integers; a stage is added as a constant that becomes the
  // read's immediate offset).  A: quarter s4 (16 k) of a stage; two bases, for stages 0 - 1 and
  // for stage 2, because the offset field reaches 64 KiB; block row i is 4096 i further on
  // (rows 32 apart share their swizzle).  B: half s of a stage, block column j.
  uint32_t a_adr[2][4], b_lo[2][WT], b_hi[2][WT];
  auto b_off = [&](uint32_t krow, uint32_t col) -> uint32_t {
    return lds_base + B_BASE + krow * B_ROW + (((col >> 3) ^ b_swz(krow)) << 4) + (col & 7u) * 2u;
  };
#pragma unroll
  for (uint32_t s4 = 0; s4 < 4u; ++s4) {
    const uint32_t row = wm + l32;
    a_adr[0][s4] = lds_base + row * 128u + (((2u * s4 + lhi) ^ row_swz8(row)) << 4);
    a_adr[1][s4] = a_adr[0][s4] + 2u * A_BYTES;
    asm volatile("" : "+v"(a_adr[1][s4]));      // kept in a register of its own: recomputed from a_adr[0] it is a vector add in the loop
  }
#pragma unroll
  for (uint32_t s = 0; s < 2; ++s)
#pragma unroll
    for (uint32_t j = 0; j < WT; ++j) {
      b_lo[s][j] = b_off(16u * s + tr_row, wn + 32u * j + tr_col);
      b_hi[s][j] = b_off(16u * s + 4u + tr_row, wn + 32u * j + tr_col);
    }

  u32x4 fa[2][WT];
  s16x4 blo[2][WT], bhi[2][WT];
  const uint32_t nk = K / GD_BK, nk2 = K / 64u;
  // one fragment read, in the order of gemm_bf16_dma_kernel: a0, b0 lo, b0 hi, b1 lo, .., a1, a2, ..
  // sa: A stage (0 .. 2), s4: its quarter; sb: B stage (0 .. 3), s: its half -- constants where called
  auto frag_load = [&](uint32_t sa, uint32_t s4, uint32_t sb, uint32_t s, uint32_t slot, uint32_t q) {
    if (q == 0u || q > 2u * WT) {
      const uint32_t i = q == 0u ? 0u : q - 2u * WT;
      fa[slot][i] = *(lds_u32x4_ptr)(uintptr_t)(a_adr[sa >> 1][s4] + ((sa & 1u) * A_BYTES + 4096u * i));
    } else {
      const uint32_t j = (q - 1u) >> 1;
      if ((q - 1u) & 1u) bhi[slot][j] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(uintptr_t)(b_hi[s][j] + sb * B_BYTES));
      else blo[slot][j] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(uintptr_t)(b_lo[s][j] + sb * B_BYTES));
    }
  };
  // tile / piece indices beyond the end are clamped: every iteration issues the same number of
  // loads (the vmcnt arithmetic relies on it), the redundant ones land in stages nobody reads again
  const uint32_t dst_a = lds_base + 2u * ND * wave * 1024u, dst_b = lds_base + B_BASE + ND * wave * 1024u;
  auto b_rsrc = [&](uint32_t t) -> buf_rsrc {
    return make_buf_rsrc(B + (size_t)min(t, nk - 1u) * GD_BK * N, GD_BK * N * 2u);
  };
  auto dma_b = [&](const buf_rsrc& rb, uint32_t sb, uint32_t h) { buf_dma16(vb[h], rb, 0u, dst_b + sb * B_BYTES + h * 1024u); };
  auto dma_a = [&](uint32_t u, uint32_t sa, uint32_t g) {
    buf_dma16(va[g], rsrc_a, min(u, nk2 - 1u) * 128u, dst_a + sa * A_BYTES + g * 1024u);
  };
  // NM MFMAs on fragment slot `slot`; between them the NF fragment reads of the next half tile into
  // the other slot, then ND DMA instructions: of B tile dt into B stage dsb (dpart 1), or of half
  // dhalf of A piece dt into A stage dsa (dpart 0)
  auto block = [&](uint32_t slot, uint32_t sa, uint32_t s4, uint32_t sb, uint32_t s, uint32_t dpart, uint32_t dt,
                   uint32_t dstage, uint32_t dhalf) {
    const buf_rsrc rb = b_rsrc(dt);
#pragma unroll
    for (uint32_t m = 0; m < NM; ++m) {
      const uint32_t i = m / WT, j = m % WT;
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(fa[slot][i]), join_bf16x8(blo[slot][j], bhi[slot][j]),
                                                          acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (uint32_t x = m * (NF + ND) / NM; x < (m + 1u) * (NF + ND) / NM; ++x) {
        if (x < NF) frag_load(sa, s4, sb, s, slot ^ 1u, x);
        else if (dpart == 1u) dma_b(rb, dstage, x - NF);
        else dma_a(dt, dstage, dhalf * ND + (x - NF));
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // prologue: A(0) B(0) B(1) A(1) B(2) A(2)h0
#pragma unroll
  for (uint32_t g = 0; g < 2u * ND; ++g) dma_a(0u, 0u, g);
  {
    const buf_rsrc r0 = b_rsrc(0u), r1 = b_rsrc(1u), r2 = b_rsrc(2u);
#pragma unroll
    for (uint32_t h = 0; h < ND; ++h) dma_b(r0, 0u, h);
#pragma unroll
    for (uint32_t h = 0; h < ND; ++h) dma_b(r1, 1u, h);
#pragma unroll
    for (uint32_t g = 0; g < 2u * ND; ++g) dma_a(1u, 1u, g);
#pragma unroll
    for (uint32_t h = 0; h < ND; ++h) dma_b(r2, 2u, h);
  }
#pragma unroll
  for (uint32_t g = 0; g < ND; ++g) dma_a(2u, 2u, g);
  __builtin_amdgcn_s_waitcnt(vm_wait(5u * ND));            // this wave's part of A(0) and B(0) has landed
  __syncthreads();
#pragma unroll
  for (uint32_t q = 0; q < NF; ++q) frag_load(0u, 0u, 0u, 0u, 0u, q);
  // piece u of A (tiles 2 u and 2 u + 1 of B) lives in A stage u % 3, tile t in B stage t % 4: six
  // pieces per pass make every stage index below a constant
  for (uint32_t u0 = 0; u0 < nk2; u0 += 6u) {
#pragma unroll
    for (uint32_t p = 0; p < 6u; ++p) {
      const uint32_t u = u0 + p, kt = 2u * u;
      if (u < nk2) {
        const uint32_t sa = p % 3u, sb = (2u * p) % 4u;
        block(0u, sa, 1u, sb, 1u, 1u, kt + 3u, (sb + 3u) % 4u, 0u);                 // B(kt + 3)
        __builtin_amdgcn_s_waitcnt(vm_wait(4u * ND));          // tile kt + 1 has landed (this wave's part)
        __syncthreads();                                       // ... everybody's; all reads of B(kt) are issued
        block(1u, sa, 2u, (sb + 1u) % 4u, 0u, 0u, u + 2u, (sa + 2u) % 3u, 1u);      // second half of A(u + 2)
        block(0u, sa, 3u, (sb + 1u) % 4u, 1u, 1u, kt + 4u, sb, 0u);                 // B(kt + 4)
        __builtin_amdgcn_s_waitcnt(vm_wait(4u * ND));
        __syncthreads();                                       // all reads of B(kt + 1) and of A(u) are issued
        block(1u, (sa + 1u) % 3u, 0u, (sb + 2u) % 4u, 0u, 0u, u + 3u, sa, 0u);      // first half of A(u + 3) into the stage just freed
      }
    }
  }
  __builtin_amdgcn_s_waitcnt(vm_wait(0));                  // no DMA may be in flight when the LDS is given back

#pragma unroll
  for (uint32_t i = 0; i < WT; ++i)
#pragma unroll
    for (uint32_t j = 0; j < WT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const uint32_t row = bm + wm + 32u * i + 8u * (r >> 2) + 4u * lhi + (r & 3);
        const uint32_t col = bn + wn + 32u * j + l32;
        if (row < M && col < N) C[(size_t)row * N + col] = acc[i][j][r];
      }
}

struct Geometry {
  uint32_t tiles_m, tiles_n, total, blocks;
  bool dma;        // shape fits the DMA kernel (operand alignment is checked at enqueue)
  uint32_t wt;     // DMA kernel: wave tile 32 wt x 32 wt, workgroup tile 64 wt x 64 wt
  bool fast;       // register-staged kernel: every tile full
};

// 256 x 256 tiles unless they would leave half of the 256 CUs without one; then 128 x 128
// (measured crossover: 2816^2 runs at 804 TFLOP/s on small tiles, 3072^2 at 880 on big ones).
constexpr uint32_t GD_MIN_BIG_TILES = 128;

Geometry geometry(uint32_t m, uint32_t n, uint32_t k) {
  Geometry g;
  g.dma = k % GD_BK == 0u && n % 8u == 0u;
  g.wt = 4u;
  if (g.dma && ((m + 255u) / 256u) * ((n + 255u) / 256u) < GD_MIN_BIG_TILES) g.wt = 2u;
  const uint32_t bm = g.dma ? 64u * g.wt : GB_BM, bn = g.dma ? 64u * g.wt : GB_BN;
  g.tiles_m = (m + bm - 1u) / bm;
  g.tiles_n = (n + bn - 1u) / bn;
  g.total = g.tiles_m * g.tiles_n;
  g.blocks = ((g.total + 7u) / 8u) * 8u;
  g.fast = m % GB_BM == 0u && n % GB_BN == 0u && k % GB_BK == 0u;
  return g;
}

Geometry staged_geometry(uint32_t m, uint32_t n, uint32_t k) {
  Geometry g;
  g.dma = false;
  g.wt = 0u;
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

uint32_t mgb_gemm_bf16_residency(uint32_t m, uint32_t n, uint32_t k) {
  if (!shape_ok(m, n, k)) return 0u;
  const Geometry g = geometry(m, n, k);
  // 256 x 256 tiles: 512 registers per lane and rings of 128 KiB (160 KiB when A travels 64 deep),
  // one workgroup per CU; 128 x 128: 64 KiB (80 KiB); the register-staged kernel: 207 registers
  // per lane, two waves per SIMD
  return g.dma ? (g.wt == 4u ? 1u : 2u) : 2u;
}

int mgb_gemm_bf16_enqueue(void* stream, const uint16_t* A, const uint16_t* B, float* C, uint32_t m,
                          uint32_t n, uint32_t k) {
  if (!A || !B || !C) return MGB_E_INVAL;
  if (!shape_ok(m, n, k)) return MGB_E_UNSUPPORTED;
  const bool aligned = (((uintptr_t)A | (uintptr_t)B | (uintptr_t)C) & 15u) == 0u;
  hipStream_t st = (hipStream_t)stream;
  Geometry g = geometry(m, n, k);
  if (g.dma && aligned) {
    static std::once_flag once;
    static hipError_t attr = hipSuccess;
    std::call_once(once, [] {
      attr = hipFuncSetAttribute((const void*)gemm_bf16_dma_kernel<4>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                 (int)gd_lds_bytes(4));
      if (attr == hipSuccess)
        attr = hipFuncSetAttribute((const void*)gemm_bf16_dma_kernel<2>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (int)gd_lds_bytes(2));
    });
    if (attr != hipSuccess) {
      mgb_internal_set_error("gemm_bf16_dma_kernel: dynamic LDS size", attr);
      return MGB_E_BACKEND;
    }
    if (k % 64u == 0u) {
      // A fetched 64 deep: whole cache lines per row
      static std::once_flag once64;
      static hipError_t attr64 = hipSuccess;
      std::call_once(once64, [] {
        attr64 = hipFuncSetAttribute((const void*)gemm_bf16_dma_a64_kernel<4>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)ga_lds_bytes(4));
        if (attr64 == hipSuccess)
          attr64 = hipFuncSetAttribute((const void*)gemm_bf16_dma_a64_kernel<2>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)ga_lds_bytes(2));
      });
      if (attr64 != hipSuccess) {
        mgb_internal_set_error("gemm_bf16_dma_a64_kernel: dynamic LDS size", attr64);
        return MGB_E_BACKEND;
      }
      if (g.wt == 4u)
        hipLaunchKernelGGL(gemm_bf16_dma_a64_kernel<4>, dim3(g.blocks), dim3(GD_THREADS), ga_lds_bytes(4), st, A, B, C,
                           m, n, k, g.tiles_n, g.total);
      else
        hipLaunchKernelGGL(gemm_bf16_dma_a64_kernel<2>, dim3(g.blocks), dim3(GD_THREADS), ga_lds_bytes(2), st, A, B, C,
                           m, n, k, g.tiles_n, g.total);
      return mgb_check_launch("gemm_bf16_dma_a64_kernel");
    }
    if (g.wt == 4u)
      hipLaunchKernelGGL(gemm_bf16_dma_kernel<4>, dim3(g.blocks), dim3(GD_THREADS), gd_lds_bytes(4), st, A, B, C, m,
                         n, k, g.tiles_n, g.total);
    else
      hipLaunchKernelGGL(gemm_bf16_dma_kernel<2>, dim3(g.blocks), dim3(GD_THREADS), gd_lds_bytes(2), st, A, B, C, m,
                         n, k, g.tiles_n, g.total);
    return mgb_check_launch("gemm_bf16_dma_kernel");
  }
  // any other shape, or operands that are not 16-byte aligned (the probe assumed they were)
  g = staged_geometry(m, n, k);
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
