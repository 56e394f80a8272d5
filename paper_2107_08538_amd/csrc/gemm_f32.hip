// fp32 GEMM C = A * B (all row-major) on the fp32 matrix cores.
//
// Two kernels: gemm_f32_dma_kernel (k % 16 == 0, n % 4 == 0, 16-byte aligned operands; described
// where it is defined) and the register-staged gemm_f32_kernel for every other shape:
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
#include "lds_dma.h"

#include <hip/hip_runtime.h>

#include <mutex>

#ifndef GF_WAVES_M
#define GF_WAVES_M 4     // waves along m: 4 -> wave tile 32 x 64, 2 -> 64 x 64
#endif
#ifndef GF_BAND
#define GF_BAND 8        // tile rows per band of the tile sequence
#endif

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));      // native vector: a load through it is one 16-byte LDS read
typedef const f32x4 __attribute__((address_space(3))) * lds_f4_ptr;
typedef const float __attribute__((address_space(3))) * lds_f1_ptr;

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

// ---- global -> LDS DMA ring kernel (k % 16 == 0, n % 4 == 0, 16-byte aligned operands) ---------
//
// The fp32 MFMA needs only 128 bytes of operands from L2 per instruction at 128 x 128 tiles, so
// the kernel is bound by MFMA issue alone; what the register-staged kernel loses is issue slots
// (global loads, the transposing LDS stores, a barrier per 16 k).  Here the tiles go global -> LDS
// by DMA into a ring of four stages and the loop is laid out by hand: the LDS reads and DMA
// instructions are spread between the MFMAs and pinned.
//
// WGM x WGN waves, each TM x TN MFMA blocks of 32 x 32:
//   2 x 2 waves of 128 x 128: 256 x 256 tile, 256 threads, 256 accumulator registers, one workgroup
//                             per CU (12 LDS reads and 4 DMA instructions per 64 MFMAs)
//   2 x 4 waves of 64 x 32:   128 x 128 tile, 512 threads, when there are too few 256 x 256 tiles
//   2 x 2 waves of 32 x 32:   64 x 64 tile, 256 threads, when there are too few 128 x 128 tiles
// Depth 16 per tile: an A row is 64 bytes, the same byte geometry (and swizzle) as the bf16 kernels.
//
// k order inside a tile: the MFMA's two k slots (lane / 32) take k = 8 * (lane / 32) + s in step
// s = 0..7, so a lane's A operands of four steps are 16 contiguous bytes (one ds_read_b128), and
// its B operand of step s is the float at k row 8 * (lane / 32) + s.  (Any assignment of the 16 k
// of a tile to steps and slots gives the same sum up to rounding order.)
constexpr uint32_t FD_BK = 16, FD_NST = 4, FD_BAND = 8;
constexpr uint32_t fd_lds_bytes(uint32_t bm, uint32_t bn) { return FD_NST * (bm + bn) * FD_BK * 4u; }

// With one wave per SIMD nothing hides what a wave issues between two MFMAs, and not everything is
// free there: a vector-ALU instruction (an address add) holds the matrix pipe up for about 14
// clocks, a load with a 64-bit vector address for 10-17 more, while scalar instructions, LDS
// reads and loads with a scalar base and a 32-bit vector offset cost nothing (measured with a
// loop of 64 MFMAs and one such instruction after every fourth: the mix this loop used to have,
// an add before each LDS read and before each DMA, ran at 90 % of the MFMA-only rate, the
// present mix at 100 %).  So the main loop holds no vector arithmetic at
// all: the ring is walked by unrolling the loop over its four stages, which turns every stage
// offset into the immediate offset of the LDS read (the A ring and the B ring are 64 KiB or less
// each, the reach of that field), and the DMA goes through buffer resources whose walk along k is
// a scalar offset (A) or a new base (B), computed by the scalar unit.
template <uint32_t WGM, uint32_t WGN, uint32_t TM, uint32_t TN>
__global__ __launch_bounds__(64 * WGM * WGN, TM * TN >= 16 ? 1 : 2) void gemm_f32_dma_kernel(const float* __restrict__ A,
                                                                       const float* __restrict__ B,
                                                                       float* __restrict__ C, uint32_t M,
                                                                       uint32_t N, uint32_t K, uint32_t tiles_n,
                                                                       uint32_t tiles_total) {
  constexpr uint32_t NW = WGM * WGN;
  constexpr uint32_t BM = 32u * TM * WGM, BN = 32u * TN * WGN;
  constexpr uint32_t A_BYTES = BM * 64u, B_BYTES = FD_BK * BN * 4u;
  constexpr uint32_t B_BASE = FD_NST * A_BYTES;      // LDS: the four A stages, then the four B stages
  static_assert(FD_NST * A_BYTES <= 65536u && FD_NST * B_BYTES <= 65536u, "a stage offset must fit the offset field of an LDS read");
  constexpr uint32_t NDA = BM / 16u / NW, NDB = BN / 16u / NW;   // DMA instructions per wave per tile
  static_assert(NDA >= 1u && NDB >= 1u, "every wave takes part in both operand copies");
  constexpr uint32_t B_ROW = BN * 4u;                // bytes of a B k-row in LDS
  constexpr uint32_t B_CPR = BN / 4u;                // 16-byte chunks of a B k-row
  constexpr uint32_t NF = TM + 2u * TN;              // fragment reads per half tile (4 steps; B two steps at a time)
  constexpr uint32_t NM = 4u * TM * TN;              // MFMAs per half tile
  extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];

  const uint32_t per_xcd = (tiles_total + 7u) / 8u;
  const uint32_t seq = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
  if ((blockIdx.x >> 3) >= per_xcd || seq >= tiles_total) return;
  const uint32_t tiles_m = tiles_total / tiles_n;
  const uint32_t band = seq / (FD_BAND * tiles_n);
  const uint32_t band_rows = min(FD_BAND, tiles_m - FD_BAND * band);
  const uint32_t in_band = seq - band * FD_BAND * tiles_n;
  const uint32_t bm = (FD_BAND * band + in_band % band_rows) * BM;
  const uint32_t bn = (in_band / band_rows) * BN;

  const uint32_t lds_base = lds_address_of(smem);
  const uint32_t tid = threadIdx.x, lane = tid & 63u;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t wm = (wave / WGN) * (32u * TM), wn = (wave % WGN) * (32u * TN);
  const uint32_t l32 = lane & 31u, lhi = lane >> 5;

  // chunk swizzle of a B k-row: rows 8..15 are shifted by 128 bytes against rows 0..7, so that the
  // two halves of a wave (k rows s and 8 + s) read different banks
  auto b_swz = [](uint32_t k) -> uint32_t { return ((k >> 3) & 1u) << 3; };

  // DMA roles: wave w, instruction h fills the 1 KiB block b = ND*w + h of an operand stage.
  //   A block b: rows 16b .. 16b+15 (64 bytes = 16 k each); lane -> row 16b + lane/4, chunk lane%4
  //   B block b: 1024 / B_ROW consecutive k rows;             lane -> its k row and chunk
  // Rows beyond M and column chunks beyond N are clamped: they only feed entries never stored.
  // A's resource covers this workgroup's rows (at most 2^26 bytes; the scalar offset walks along
  // k), B's is rebased for every tile to its 16 k rows (at most 2^22 bytes).
  const buf_rsrc rsrc_a = make_buf_rsrc(A + (size_t)bm * K, min(BM, M - bm) * K * 4u);
  uint32_t va[NDA], vb[NDB];
#pragma unroll
  for (uint32_t h = 0; h < NDA; ++h) {
    const uint32_t ar = 16u * (NDA * wave + h) + (lane >> 2);
    va[h] = (min(bm + ar, M - 1u) - bm) * K * 4u + 16u * ((lane & 3u) ^ row_swz(ar));
  }
#pragma unroll
  for (uint32_t h = 0; h < NDB; ++h) {
    const uint32_t bk = (1024u / B_ROW) * (NDB * wave + h) + lane / B_CPR;
    vb[h] = (bk * N + min(bn + 4u * ((lane % B_CPR) ^ b_swz(bk)), N - 4u)) * 4u;
  }

  f32x16 acc[TM][TN];
#pragma unroll
  for (uint32_t i = 0; i < TM; ++i)
#pragma unroll
    for (uint32_t j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // LDS addresses of the fragments in stage 0 of each ring: half hf covers steps 4 hf .. 4 hf + 3.
  // They are kept as integers and a stage is added as a constant, which the LDS read takes as its
  // immediate offset (formed from the array's address the constant stays a vector add).
  uint32_t a_off[2][TM], b_off[2][2][TN];   // B: steps 0 and 2 of a half; steps 1 and 3 are one row further
#pragma unroll
  for (uint32_t hf = 0; hf < 2; ++hf) {
#pragma unroll
    for (uint32_t i = 0; i < TM; ++i) {
      const uint32_t row = wm + 32u * i + l32;
      a_off[hf][i] = lds_base + row * 64u + (((2u * lhi + hf) ^ row_swz(row)) << 4);      // k = 8 lhi + 4 hf .. + 3
    }
#pragma unroll
    for (uint32_t s = 0; s < 2; ++s)
#pragma unroll
      for (uint32_t j = 0; j < TN; ++j) {
        const uint32_t krow = 8u * lhi + 4u * hf + 2u * s, col = wn + 32u * j + l32;
        b_off[hf][s][j] = lds_base + B_BASE + krow * B_ROW + (((col >> 2) ^ b_swz(krow)) << 4) + (col & 3u) * 4u;
      }
  }

  f32x4 fa[2][TM];             // [slot][block row]: A operands of four steps
  float fb[2][4][TN];          // [slot][step][block column]
  const uint32_t nk = K / FD_BK;
  // one fragment read of a half tile of the tile in ring stage `st` (a constant where it is called),
  // in the order the MFMAs need them: the A operands (one read serves four steps), then the B
  // operands, two steps (two k rows, one two-address LDS read) at a time
  auto frag_load = [&](uint32_t st, uint32_t hf, uint32_t slot, uint32_t q) {
    if (q < TM) fa[slot][q] = *(lds_f4_ptr)(uintptr_t)(a_off[hf][q] + st * A_BYTES);
    else {
      // the next step's k row is the next LDS row (same swizzle: a half never crosses k = 8), a
      // constant distance away, so the pair becomes one two-address read
      const uint32_t x = q - TM, s2 = 2u * (x / TN), j = x % TN;
      const uint32_t p = b_off[hf][s2 / 2u][j] + st * B_BYTES;
      fb[slot][s2][j] = *(lds_f1_ptr)(uintptr_t)p;
      fb[slot][s2 + 1u][j] = *(lds_f1_ptr)(uintptr_t)(p + B_ROW);
    }
  };
  // tile indices beyond the end are clamped: the schedule never changes (see the wait counts), the
  // redundant loads land in stages nobody reads any more
  const uint32_t dst_a = lds_base + NDA * wave * 1024u, dst_b = lds_base + B_BASE + NDB * wave * 1024u;
  auto b_rsrc = [&](uint32_t kt) -> buf_rsrc {
    const uint32_t t = min(kt, nk - 1u);
    return make_buf_rsrc(B + (size_t)t * FD_BK * N, FD_BK * N * 4u);
  };
  auto dma_a = [&](uint32_t kt, uint32_t st, uint32_t h) {
    buf_dma16(va[h], rsrc_a, min(kt, nk - 1u) * (FD_BK * 4u), dst_a + st * A_BYTES + h * 1024u);
  };
  auto dma_b = [&](const buf_rsrc& rb, uint32_t st, uint32_t h) { buf_dma16(vb[h], rb, 0u, dst_b + st * B_BYTES + h * 1024u); };
  // NM MFMAs (4 steps) on fragment slot `slot`; spread between them: the NF fragment reads of
  // (stage fst, half fh) into the other slot, then the DMA instructions of tile dt into stage dst
  // (dpart 0: its A part, 1: its B part)
  auto block = [&](uint32_t slot, uint32_t fst, uint32_t fh, uint32_t dt, uint32_t dst, uint32_t dpart) {
    const uint32_t nd = dpart == 0u ? NDA : NDB;
    const buf_rsrc rb = b_rsrc(dt);
#pragma unroll
    for (uint32_t m = 0; m < NM; ++m) {
      const uint32_t s = m / (TM * TN), i = (m / TN) % TM, j = m % TN;
      const float a = s == 0u ? fa[slot][i].x : s == 1u ? fa[slot][i].y : s == 2u ? fa[slot][i].z : fa[slot][i].w;
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, fb[slot][s][j], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (uint32_t x = m * (NF + nd) / NM; x < (m + 1u) * (NF + nd) / NM; ++x) {
        if (x < NF) frag_load(fst, fh, slot ^ 1u, x);
        else if (dpart == 0u) dma_a(dt, dst, x - NF);
        else dma_b(rb, dst, x - NF);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // DMA issue order: A(0) B(0) .. A(NST-2) B(NST-2) A(NST-1) | B(NST-1) A(NST) | B(NST) A(NST+1) | ..
#pragma unroll
  for (uint32_t t = 0; t < FD_NST - 1u; ++t) {
#pragma unroll
    for (uint32_t h = 0; h < NDA; ++h) dma_a(t, t, h);
    const buf_rsrc rb = b_rsrc(t);
#pragma unroll
    for (uint32_t h = 0; h < NDB; ++h) dma_b(rb, t, h);
  }
#pragma unroll
  for (uint32_t h = 0; h < NDA; ++h) dma_a(FD_NST - 1u, FD_NST - 1u, h);
  __builtin_amdgcn_s_waitcnt(vm_wait((NDA + NDB) * (FD_NST - 2u) + NDA));   // this wave's part of tile 0 has landed
  __syncthreads();
#pragma unroll
  for (uint32_t q = 0; q < NF; ++q) frag_load(0u, 0u, 0u, q);
  for (uint32_t kt0 = 0; kt0 < nk; kt0 += FD_NST) {
#pragma unroll
    for (uint32_t u = 0; u < FD_NST; ++u) {           // tile kt lives in stage u: every stage index below is a constant
      const uint32_t kt = kt0 + u;
      if (kt < nk) {
        block(0u, u, 1u, kt + FD_NST - 1u, (u + FD_NST - 1u) % FD_NST, 1u);   // reads the second half of tile kt; B(kt + NST - 1)
        // tile kt+1 has landed when no more than the (NDA + NDB)(NST-2) instructions issued after it
        // are outstanding; the barrier makes that true for every wave and frees tile kt's stage
        __builtin_amdgcn_s_waitcnt(vm_wait((NDA + NDB) * (FD_NST - 2u)));
        __syncthreads();
        block(1u, (u + 1u) % FD_NST, 0u, kt + FD_NST, u, 0u);                 // reads the first half of tile kt+1; A(kt + NST)
      }
    }
  }
  __builtin_amdgcn_s_waitcnt(vm_wait(0));             // no DMA may be in flight when the LDS is given back

#pragma unroll
  for (uint32_t i = 0; i < TM; ++i)
#pragma unroll
    for (uint32_t j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const uint32_t row = bm + wm + 32u * i + 8u * (r >> 2) + 4u * lhi + (r & 3);
        const uint32_t col = bn + wn + 32u * j + l32;
        if (row < M && col < N) C[(size_t)row * N + col] = acc[i][j][r];
      }
}

struct Geometry {
  uint32_t tiles_m, tiles_n, total, blocks, threads;
  bool dma;        // shape fits the DMA kernel (operand alignment is checked at enqueue)
  uint32_t tile;   // 256, 128 or 64 (DMA kernel); 128 (register-staged kernel)
  bool fast;       // register-staged kernel: every tile full
};

// Which tile: the one that is done first by this estimate.  A CU works its tiles off one after the
// other (two or five resident workgroups share its matrix pipes), so a launch takes as many tile
// times as the busiest CU has tiles, ceil(tiles / 256), and a tile time is its area over the
// rate a CU reaches with that tile.  Rates measured on square shapes from 512 to 8192, in TFLOP/s
// over the device when every CU is equally loaded: 153 with 256 x 256 tiles, 150 with 128 x 128,
// 143 with 64 x 64 up to k = 5632 and 128 beyond (the small tile re-reads its operands more often
// and the slabs of a band of tile rows no longer fit L2).  The estimate picks the fastest or
// second-fastest tile (within 3 % of the fastest up to 5000, within 10 % beyond) on every shape of that sweep:
// 2176^3 runs at 109 TFLOP/s (64 x 64) instead of 86 (128 x 128), 2944^3 at 132 instead of 105,
// 4160^3 at 140 instead of 125 (128 x 128) or 79 (256 x 256), 4096^3 and 8192^3 keep the big tile.
// cost = ceil(tiles / 256) * tile^2 * (100000 / rate), in integers; ties go to the larger tile.
uint32_t pick_tile(uint32_t m, uint32_t n, uint32_t k) {
  const uint32_t tile[3] = {256u, 128u, 64u};
  const uint64_t inv_rate[3] = {100000u / 153u, 100000u / 150u, 100000u / (k <= 5632u ? 143u : 128u)};
  uint32_t best = 256u;
  uint64_t best_cost = ~0ull;
  for (int i = 0; i < 3; ++i) {
    const uint64_t tiles = (uint64_t)((m + tile[i] - 1u) / tile[i]) * ((n + tile[i] - 1u) / tile[i]);
    const uint64_t cost = ((tiles + 255u) / 256u) * tile[i] * tile[i] * inv_rate[i];
    if (cost < best_cost) {
      best_cost = cost;
      best = tile[i];
    }
  }
  return best;
}

Geometry geometry(uint32_t m, uint32_t n, uint32_t k, bool allow_dma = true) {
  Geometry g;
  g.dma = allow_dma && k % FD_BK == 0u && n % 4u == 0u;
  g.tile = 128u;
  if (g.dma) g.tile = pick_tile(m, n, k);
  g.tiles_m = (m + g.tile - 1u) / g.tile;
  g.tiles_n = (n + g.tile - 1u) / g.tile;
  g.total = g.tiles_m * g.tiles_n;
  g.blocks = ((g.total + 7u) / 8u) * 8u;
  g.threads = g.dma && g.tile != 128u ? 256u : GF_THREADS;
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
  *block = mgb_dim3{g.threads, 1u, 1u};
  return MGB_OK;
}

uint32_t mgb_gemm_f32_residency(uint32_t m, uint32_t n, uint32_t k) {
  if (!shape_ok(m, n, k)) return 0u;
  const Geometry g = geometry(m, n, k);
  // LDS: the ring takes 128 KiB (256 x 256 tiles, which also need all 512 registers of a lane),
  // 64 KiB (128 x 128) or 32 KiB (64 x 64) of a CU's 160 KiB; the register-staged kernel is limited
  // by its 8 waves per workgroup
  return g.dma ? (g.tile == 256u ? 1u : g.tile == 128u ? 2u : 5u) : 4u;
}

int mgb_gemm_f32_enqueue(void* stream, const float* A, const float* B, float* C, uint32_t m,
                         uint32_t n, uint32_t k) {
  if (!A || !B || !C) return MGB_E_INVAL;
  if (!shape_ok(m, n, k)) return MGB_E_UNSUPPORTED;
  const bool aligned = (((uintptr_t)A | (uintptr_t)B | (uintptr_t)C) & 15u) == 0u;
  const Geometry g = geometry(m, n, k, aligned);     // the probe assumed aligned operands
  hipStream_t st = (hipStream_t)stream;
  if (g.dma) {
    static std::once_flag once;
    static hipError_t attr = hipSuccess;
    std::call_once(once, [] {
      attr = hipFuncSetAttribute((const void*)gemm_f32_dma_kernel<2, 2, 4, 4>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                 (int)fd_lds_bytes(256, 256));
      if (attr == hipSuccess)
        attr = hipFuncSetAttribute((const void*)gemm_f32_dma_kernel<2, 4, 2, 1>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (int)fd_lds_bytes(128, 128));
      if (attr == hipSuccess)
        attr = hipFuncSetAttribute((const void*)gemm_f32_dma_kernel<2, 2, 1, 1>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (int)fd_lds_bytes(64, 64));
    });
    if (attr != hipSuccess) {
      mgb_internal_set_error("gemm_f32_dma_kernel: dynamic LDS size", attr);
      return MGB_E_BACKEND;
    }
    if (g.tile == 256u)
      hipLaunchKernelGGL((gemm_f32_dma_kernel<2, 2, 4, 4>), dim3(g.blocks), dim3(g.threads), fd_lds_bytes(256, 256), st,
                         A, B, C, m, n, k, g.tiles_n, g.total);
    else if (g.tile == 128u)
      hipLaunchKernelGGL((gemm_f32_dma_kernel<2, 4, 2, 1>), dim3(g.blocks), dim3(g.threads), fd_lds_bytes(128, 128), st,
                         A, B, C, m, n, k, g.tiles_n, g.total);
    else
      hipLaunchKernelGGL((gemm_f32_dma_kernel<2, 2, 1, 1>), dim3(g.blocks), dim3(g.threads), fd_lds_bytes(64, 64), st,
                         A, B, C, m, n, k, g.tiles_n, g.total);
    return mgb_check_launch("gemm_f32_dma_kernel");
  }
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
