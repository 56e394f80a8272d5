// 3x3 convolution + ReLU (padding 1, stride 1 or 2) on the bf16 matrix cores, and a chain of
// such layers run as one task.
//
// GEMM view: rows = output pixels (n, oh, ow), columns = output channels, depth = (r, s, c) =
// 9 * c_in.  Activations are N,H,W,C and weights K,3,3,C, so for a fixed filter tap the channel
// run is contiguous for both operands and neither needs a transpose.
//
// Kernels (each described where it is defined; geometry() says which layer gets which):
//   conv3x3_patch_kernel       stride 1, c_in % 64 == 0: the input patch of a 2-D output tile in
//                              LDS, read nine times at shifted positions; weights through a ring
//   conv3x3_s2c32_kernel       stride 2 from 32 channels: filter and patch in LDS; inside a chain it
//                              also computes the 3-channel first layer in front of it
//   conv3x3_dma_kernel         implicit GEMM, c_in % 32 == 0: every DMA lane gathers its own
//   conv3x3_dma64_kernel         pixel; the same with stages of depth 64 (c_in % 64 == 0) and both
//                              operands through buffer resources (no vector arithmetic in its loop)
//   conv3x3_dma_ksplit_kernel  layers with few tiles: the depth split over the waves of a
//                              workgroup and, inside a chain, over workgroups
//                              (conv_split_reduce_kernel adds the parts); buffer resources too
//   conv3x3_c3_kernel          the 3-channel first layer on its own
//   conv3x3_kernel             register-staged, any other shape
// At the sizes of the net none of them is bound by the matrix pipes or by bytes: a CU holds two of
// their workgroups (LDS), and what a workgroup's waves spend on addresses, set-up and result stores
// is not hidden by anyone else.  Hence store_tile_via_lds, FastDiv, the source tables and the
// buffer resources with scalar offsets below.
#include "../../include/mgb.h"
#include "launch_util.h"
#include "lds_dma.h"

#include <hip/hip_runtime.h>

#include <mutex>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // one 16-byte chunk of 8 bf16

constexpr uint32_t CV_BM = 128, CV_THREADS = 256;

// Unsigned division by a number fixed at launch: q = n / d for every 32-bit n, as a multiply-high
// and two shifts (the round-up method for invariant divisors).  The kernels decode tile and pixel
// indices with it; the compiler's general division costs some forty instructions each, and a
// workgroup's set-up runs a dozen or two of them per lane before its first load can be issued.
struct FastDiv {
  uint32_t d, m, s1, s2;
};

FastDiv fast_div(uint32_t d) {
  uint32_t l = 0u;
  while (l < 32u && (1ull << l) < d) ++l;                       // ceil(log2(d)), d >= 1
  FastDiv f;
  f.d = d;
  f.m = (uint32_t)(((1ull << 32) * ((1ull << l) - d)) / d + 1ull);
  f.s1 = l < 1u ? l : 1u;
  f.s2 = l > 0u ? l - 1u : 0u;
  return f;
}

__device__ __forceinline__ uint32_t operator/(uint32_t n, const FastDiv& f) {
  const uint32_t t = __umulhi(f.m, n);
  return (t + ((n - t) >> f.s1)) >> f.s2;
}

struct ConvArgs {
  const uint16_t* x;
  const uint16_t* w;
  void* y;
  uint32_t batch, H, W, C, K, stride, Ho, Wo;
  uint32_t pixels, depth;      // batch*Ho*Wo, 9*C
  uint32_t tiles_n, tiles_total, out_f32;
  uint32_t splits;             // depth-split kernel only: workgroups that share one output tile
  float* work;                 // splits > 1: fp32 partial sums [split][pixel][channel]
  uint32_t th, tw, tiles_y, tiles_x;   // patch kernels only: output tile of th x tw pixels, tiles per image
  FastDiv by_tiles_n, by_plane, by_wo; // divisors tiles_n, Ho * Wo, Wo
  FastDiv by_tiles_x, by_tiles_y, by_pw, by_tw;   // patch kernels only: tiles_x, tiles_y, patch width, tw
  const uint16_t* w_first;             // fused first two layers only: the 3-channel layer's filter
  FastDiv by_iw;                       // the same: patch width + 2
};

// 16 bytes of zeros in device memory: the source of every padded / out-of-range operand chunk
__device__ __attribute__((aligned(16))) uint32_t g_zero16[4];

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t w = __float_as_uint(f);
  return (uint16_t)((w + 0x7fffu + ((w >> 16) & 1u)) >> 16);
}

// two floats to two bf16 (round to nearest even) in one word, low half first: the hardware's
// packed conversion, one instruction instead of eight integer ones
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 q) { return __builtin_bit_cast(bf16x8, q); }

// p if ok (0 or 1) else z, as a select on the address bits (two conditional moves; written on
// pointers the compiler may turn it into a branch around the load that follows)
__device__ __forceinline__ const uint16_t* pick(const uint16_t* p, const uint16_t* z, uint32_t ok) {
  const uintptr_t a = (uintptr_t)p, b = (uintptr_t)z;
  const uint32_t lo = ok ? (uint32_t)a : (uint32_t)b, hi = ok ? (uint32_t)(a >> 32) : (uint32_t)(b >> 32);
  return (const uint16_t*)(((uintptr_t)hi << 32) | lo);
}

// Register-staged kernel for shapes none of the others takes.  A workgroup of 4 waves (2 x 2)
// owns 128 pixels x BN channels; the A tile is gathered from the input image (zeros outside it)
// into LDS, 8 channels per 16-byte load when c_in % 8 == 0 (VEC, depth 64 per step), element-wise
// otherwise (depth 32 per step).  The tiles of the next two steps are kept in flight in registers
// while the MFMAs of the current step run from LDS.
template <uint32_t BN, bool VEC>
__global__ __launch_bounds__(CV_THREADS, 2) void conv3x3_kernel(ConvArgs a) {
  constexpr uint32_t CV_BK = VEC ? 64u : 32u;
  constexpr uint32_t CV_LD = CV_BK + 8u;            // LDS pitch in elements
  constexpr uint32_t CPR = CV_BK / 8u;              // 8-element chunks per tile row
  constexpr uint32_t RSTEP = CV_THREADS / CPR;      // rows covered by one pass of the workgroup
  __shared__ __attribute__((aligned(16))) uint16_t As[2][CV_BM][CV_LD];   // [pixel][k]
  __shared__ __attribute__((aligned(16))) uint16_t Bs[2][BN][CV_LD];      // [channel][k]
  constexpr uint32_t NT = BN / 64u;                 // MFMA blocks per wave along the channels
  constexpr uint32_t ACH = CV_BM / RSTEP;           // A chunks per thread per step
  constexpr uint32_t BCH = BN / RSTEP;              // weight chunks per thread per step

  const uint32_t per_xcd = (a.tiles_total + 7u) / 8u;
  const uint32_t tile = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
  if ((blockIdx.x >> 3) >= per_xcd || tile >= a.tiles_total) return;
  const uint32_t bm = (tile / a.tiles_n) * CV_BM;
  const uint32_t bn = (tile % a.tiles_n) * BN;

  const uint32_t tid = threadIdx.x;
  const uint32_t lane = tid & 63u, wave = tid >> 6;
  const uint32_t wm = (wave >> 1) * 64u, wn = (wave & 1u) * (BN / 2u);
  const uint32_t l32 = lane & 31u, lhi = lane >> 5;
  // staging roles: 8-element chunk ch of rows row0, row0 + RSTEP, ...
  const uint32_t ch = tid % CPR, row0 = tid / CPR;

  // the pixels this thread gathers for
  int32_t ih0[ACH], iw0[ACH];
  uint32_t img[ACH];
  bool pv[ACH];
#pragma unroll
  for (uint32_t h = 0; h < ACH; ++h) {
    const uint32_t p = bm + row0 + RSTEP * h;
    pv[h] = p < a.pixels;
    const uint32_t pp = pv[h] ? p : 0u;
    const uint32_t b = pp / a.by_plane;
    const uint32_t rem = pp - b * a.Ho * a.Wo;
    const uint32_t oh = rem / a.by_wo, ow = rem - oh * a.Wo;
    ih0[h] = (int32_t)(oh * a.stride) - 1;
    iw0[h] = (int32_t)(ow * a.stride) - 1;
    img[h] = b * a.H * a.W;                          // pixel index of the image origin
  }

  // Taps outside the image, pixels / channels past the end and depth padding read from a
  // 16-byte block of zeros instead of the tensors: every load is unconditional and its
  // result goes to LDS untouched, so no branch or select sits between a load and its use and
  // the loads of two steps can stay in flight across the MFMAs.
  const uint16_t* zeros = reinterpret_cast<const uint16_t*>(g_zero16);
  auto load_tiles = [&](uint32_t k0, u32x4 (&ra)[ACH], u32x4 (&rb)[BCH]) {
    const uint32_t k = k0 + 8u * ch;
    if (VEC) {
      // the 8 k-values share one filter tap (c_in % 8 == 0, so depth % 8 == 0)
      const bool kok = k < a.depth;
      const uint32_t tap = k / a.C, c = k - tap * a.C;
      const int32_t r = (int32_t)(tap / 3u), s = (int32_t)(tap - 3u * (tap / 3u));
#pragma unroll
      for (uint32_t h = 0; h < ACH; ++h) {
        const int32_t ih = ih0[h] + r, iw = iw0[h] + s;
        const uint32_t ok = (uint32_t)pv[h] & (uint32_t)kok & (uint32_t)((uint32_t)ih < a.H) & (uint32_t)((uint32_t)iw < a.W);
        const uint16_t* in_img = a.x + ((int64_t)img[h] + (int64_t)ih * a.W + iw) * a.C + c;
        ra[h] = *reinterpret_cast<const u32x4*>(pick(in_img, zeros, ok));
      }
#pragma unroll
      for (uint32_t j = 0; j < BCH; ++j) {
        const uint32_t n = bn + row0 + RSTEP * j;
        const uint16_t* in_w = a.w + (size_t)n * a.depth + k;
        rb[j] = *reinterpret_cast<const u32x4*>(pick(in_w, zeros, (uint32_t)(n < a.K) & (uint32_t)kok));
      }
    } else {
#pragma unroll
      for (uint32_t h = 0; h < ACH; ++h) {
        uint32_t wd[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (uint32_t i = 0; i < 8; ++i) {
          const uint32_t kk = k + i;
          const uint32_t tap = kk / a.C, c = kk - tap * a.C;
          const int32_t r = (int32_t)(tap / 3u), s = (int32_t)(tap - 3u * (tap / 3u));
          const int32_t ih = ih0[h] + r, iw = iw0[h] + s;
          const uint32_t ok = (uint32_t)pv[h] & (uint32_t)(kk < a.depth) & (uint32_t)((uint32_t)ih < a.H) & (uint32_t)((uint32_t)iw < a.W);
          const uint16_t* in_img = a.x + ((int64_t)img[h] + (int64_t)ih * a.W + iw) * a.C + c;
          wd[i >> 1] |= (uint32_t)*pick(in_img, zeros, ok) << (16u * (i & 1u));
        }
        ra[h] = u32x4{wd[0], wd[1], wd[2], wd[3]};
      }
#pragma unroll
      for (uint32_t j = 0; j < BCH; ++j) {
        const uint32_t n = bn + row0 + RSTEP * j;
        uint32_t wd[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (uint32_t i = 0; i < 8; ++i) {
          const uint16_t* in_w = a.w + (size_t)n * a.depth + k + i;
          wd[i >> 1] |= (uint32_t)*pick(in_w, zeros, (uint32_t)(n < a.K) & (uint32_t)(k + i < a.depth)) << (16u * (i & 1u));
        }
        rb[j] = u32x4{wd[0], wd[1], wd[2], wd[3]};
      }
    }
  };
  auto store_tiles = [&](uint32_t buf, const u32x4 (&ra)[ACH], const u32x4 (&rb)[BCH]) {
#pragma unroll
    for (uint32_t h = 0; h < ACH; ++h)
      *reinterpret_cast<u32x4*>(&As[buf][row0 + RSTEP * h][8u * ch]) = ra[h];
#pragma unroll
    for (uint32_t j = 0; j < BCH; ++j)
      *reinterpret_cast<u32x4*>(&Bs[buf][row0 + RSTEP * j][8u * ch]) = rb[j];
  };

  f32x16 acc[2][NT];
#pragma unroll
  for (uint32_t i = 0; i < 2; ++i)
#pragma unroll
    for (uint32_t j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  auto compute = [&](uint32_t buf) {
#pragma unroll
    for (uint32_t ks = 0; ks < CV_BK; ks += 16u) {
      bf16x8 fa[2], fb[NT];
#pragma unroll
      for (uint32_t i = 0; i < 2; ++i)
        fa[i] = as_bf16x8(*reinterpret_cast<const u32x4*>(&As[buf][wm + 32u * i + l32][ks + 8u * lhi]));
#pragma unroll
      for (uint32_t j = 0; j < NT; ++j)
        fb[j] = as_bf16x8(*reinterpret_cast<const u32x4*>(&Bs[buf][wn + 32u * j + l32][ks + 8u * lhi]));
#pragma unroll
      for (uint32_t i = 0; i < 2; ++i)
#pragma unroll
        for (uint32_t j = 0; j < NT; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
  };

  // Software pipeline, two steps deep: while step kt computes from LDS[kt & 1], the tiles of
  // step kt+1 sit in one register set (stored to LDS at the end of the step) and the loads of
  // step kt+2 are in flight into the other.  The loop body handles two steps so that the
  // register sets keep fixed names.
  const uint32_t nk = (a.depth + CV_BK - 1u) / CV_BK;
  const uint32_t last = (nk - 1u) * CV_BK;          // loads issued past the end re-read the last step
  u32x4 ra0[ACH], rb0[BCH], ra1[ACH], rb1[BCH];
  load_tiles(0, ra0, rb0);
  store_tiles(0, ra0, rb0);
  load_tiles(min(CV_BK, last), ra1, rb1);
  __syncthreads();
  for (uint32_t kt = 0; kt < nk; kt += 2u) {
    // step kt: LDS[0]; set 1 holds step kt+1; set 0 receives step kt+2
    load_tiles(min((kt + 2u) * CV_BK, last), ra0, rb0);
    compute(0);
    store_tiles(1, ra1, rb1);                        // unused if kt+1 == nk
    __syncthreads();
    if (kt + 1u >= nk) break;
    // step kt+1: LDS[1]; set 0 holds step kt+2; set 1 receives step kt+3
    load_tiles(min((kt + 3u) * CV_BK, last), ra1, rb1);
    compute(1);
    store_tiles(0, ra0, rb0);                        // unused if kt+2 == nk
    __syncthreads();
  }

  // ReLU, then bf16 (nearest even) or fp32
#pragma unroll
  for (uint32_t i = 0; i < 2; ++i)
#pragma unroll
    for (uint32_t j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const uint32_t p = bm + wm + 32u * i + 8u * (r >> 2) + 4u * lhi + (r & 3);
        const uint32_t col = bn + wn + 32u * j + l32;
        if (p < a.pixels && col < a.K) {
          const float v = fmaxf(acc[i][j][r], 0.f);
          if (a.out_f32)
            reinterpret_cast<float*>(a.y)[(size_t)p * a.K + col] = v;
          else
            reinterpret_cast<uint16_t*>(a.y)[(size_t)p * a.K + col] = f32_to_bf16_rne(v);
        }
      }
}

// ---- results of a wave's 64 pixels x 64 channels to memory through LDS --------------------------
//
// In the out^T accumulator layout (weights as the MFMA's first operand) a lane holds, per quad,
// four consecutive channels of one pixel: stored straight from the registers that is 8 bytes per
// lane into 32 different cache lines per instruction, and the write path takes about twice as
// long over it as the whole depth loop of a 64-channel layer.  Here the wave first lays its tile
// out in LDS as [pixel][channel] (16-byte chunks XOR-swizzled by the pixel) and then writes 16
// bytes per lane, the lanes of a pixel's row side by side: whole 128-byte lines (bf16; fp32: 256
// bytes per pixel).  `stage` is this wave's own 16 KiB of LDS (OUT_STAGE_BYTES; with TABLE 256
// bytes more), free of other use (NI = 1: a wave of 32 pixels x 64 channels, half of all that).  Where the wave's pixels go: with TABLE, pix[i] is the output
// pixel of lane block i (l32 = lane % 32), negative if there is none, and the lanes exchange them
// through a table behind the tile; without, pixel r of the tile is output pixel pix[0] + r as long
// as that is below pix[1].  ch0 is the first of the 64 channels (channels >= c_out are dropped;
// c_out % 8 == 0).
constexpr uint32_t OUT_STAGE_BYTES = 64u * 256u;

template <bool TABLE, uint32_t NI = 2u>
__device__ __forceinline__ void store_tile_via_lds(uint8_t* stage, const f32x16 (&acc)[NI][2], const int32_t (&pix)[2],
                                                   uint32_t ch0, uint32_t K, uint32_t out_f32, void* y) {
  const uint32_t lane = threadIdx.x & 63u, l32 = lane & 31u, lhi = lane >> 5;
  int32_t* index = reinterpret_cast<int32_t*>(stage + NI * 32u * 256u);
  if (TABLE && lhi == 0u) {
    index[l32] = pix[0];
    if (NI == 2u) index[32u + l32] = pix[1];
  }
  auto pixel_of = [&](uint32_t px) -> int32_t {
    if (TABLE) return index[px];
    const int32_t p = pix[0] + (int32_t)px;
    return p < pix[1] ? p : -1;
  };
  if (!out_f32) {
    // bf16: rows of 128 bytes, chunk = 8 channels; a lane owns half a chunk per quad
#pragma unroll
    for (uint32_t i = 0; i < NI; ++i) {
      const uint32_t px = 32u * i + l32;
#pragma unroll
      for (uint32_t j = 0; j < 2; ++j)
#pragma unroll
        for (uint32_t g = 0; g < 4; ++g) {
          uint2 q;
          q.x = pack_bf16x2(fmaxf(acc[i][j][4u * g], 0.f), fmaxf(acc[i][j][4u * g + 1u], 0.f));
          q.y = pack_bf16x2(fmaxf(acc[i][j][4u * g + 2u], 0.f), fmaxf(acc[i][j][4u * g + 3u], 0.f));
          *reinterpret_cast<uint2*>(stage + px * 128u + (((4u * j + g) ^ ((px ^ (px >> 3)) & 7u)) << 4) + 8u * lhi) = q;
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    uint16_t* out = reinterpret_cast<uint16_t*>(y);
#pragma unroll
    for (uint32_t it = 0; it < 4u * NI; ++it) {
      const uint32_t px = 8u * it + (lane >> 3), c = lane & 7u;
      const u32x4 v = *reinterpret_cast<const u32x4*>(stage + px * 128u + ((c ^ ((px ^ (px >> 3)) & 7u)) << 4));
      const int32_t p = pixel_of(px);
      const uint32_t ch = ch0 + 8u * c;
      if (p >= 0 && ch < K) *reinterpret_cast<u32x4*>(out + (size_t)p * K + ch) = v;
    }
  } else {
    // fp32: rows of 256 bytes, chunk = 4 channels = one quad of a lane
#pragma unroll
    for (uint32_t i = 0; i < NI; ++i) {
      const uint32_t px = 32u * i + l32;
#pragma unroll
      for (uint32_t j = 0; j < 2; ++j)
#pragma unroll
        for (uint32_t g = 0; g < 4; ++g) {
          const float4 q = make_float4(fmaxf(acc[i][j][4u * g], 0.f), fmaxf(acc[i][j][4u * g + 1u], 0.f),
                                       fmaxf(acc[i][j][4u * g + 2u], 0.f), fmaxf(acc[i][j][4u * g + 3u], 0.f));
          *reinterpret_cast<float4*>(stage + px * 256u + (((8u * j + 2u * g + lhi) ^ (px & 15u)) << 4)) = q;
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    float* out = reinterpret_cast<float*>(y);
#pragma unroll
    for (uint32_t it = 0; it < 8u * NI; ++it) {
      const uint32_t px = 4u * it + (lane >> 4), c = lane & 15u;
      const float4 v = *reinterpret_cast<const float4*>(stage + px * 256u + ((c ^ (px & 15u)) << 4));
      const int32_t p = pixel_of(px);
      const uint32_t ch = ch0 + 4u * c;
      if (p >= 0 && ch < K) *reinterpret_cast<float4*>(out + (size_t)p * K + ch) = v;
    }
  }
}

// ---- DMA-ring implicit GEMM (c_in % 32 == 0, c_out % 8 == 0, 16-byte aligned tensors) -----------
//
// Same pipeline as the DMA bf16 GEMM: operand tiles of depth 32 go global -> LDS directly
// (global_load_lds_dwordx4) into a ring of four stages, three tiles in flight while one is
// consumed; unpadded, XOR-swizzled LDS rows of 64 bytes; the main loop is laid out by hand, the
// fragment reads and DMA instructions spread between the MFMAs and pinned with scheduling
// barriers.  The gather of the activation operand is free with DMA: every lane names its own
// source address (its pixel shifted by the filter tap), and a tap outside the image, or a pixel
// past the end, names a 16-byte block of zeros instead.  With c_in % 32 == 0 a depth-32 tile
// lies inside one filter tap, so the tap is uniform per tile.
//
// The weights are the MFMA's first operand and the pixels its second (out^T = w * patch^T): a
// lane then owns 4 consecutive channels of one pixel per accumulator quad and stores them as
// 8 bytes (bf16) or 16 bytes (fp32).
//
// WM x WN waves (64 threads each), every wave 64 pixels x 64 channels (2 x 2 MFMA blocks):
//   2 x 2: 128 x 128 tile          4 x 1: 256 pixels x 64 channels (c_out <= 64)
//   1 x 1: 64 x 64 tile, one wave per workgroup (layers too small to give every CU a big tile)
constexpr uint32_t CD_BK = 32, CD_NST = 4;

template <uint32_t WM, uint32_t WN>
__global__ __launch_bounds__(64 * WM * WN, 2) void conv3x3_dma_kernel(ConvArgs a) {
  constexpr uint32_t NW = WM * WN;
  constexpr uint32_t BMP = 64u * WM, BNC = 64u * WN;             // pixels x channels per workgroup
  constexpr uint32_t A_BYTES = BMP * 64u, B_BYTES = BNC * 64u, STAGE = A_BYTES + B_BYTES;
  constexpr uint32_t NA = BMP / 16u / NW, NB = BNC / 16u / NW;   // DMA instructions per wave per tile
  static_assert(NA >= 1u && NB >= 1u, "every wave takes part in both operand copies");
  extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];

  const uint32_t per_xcd = (a.tiles_total + 7u) / 8u;
  const uint32_t tile = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
  if ((blockIdx.x >> 3) >= per_xcd || tile >= a.tiles_total) return;
  const uint32_t tile_m = tile / a.by_tiles_n;
  const uint32_t bm = tile_m * BMP;
  const uint32_t bn = (tile - tile_m * a.tiles_n) * BNC;

  const uint32_t lds_base = lds_address_of(smem);
  const uint32_t tid = threadIdx.x, lane = tid & 63u;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t wm = (wave / WN) * 64u, wn = (wave % WN) * 64u;
  const uint32_t l32 = lane & 31u, lhi = lane >> 5;
  const uint16_t* zeros = reinterpret_cast<const uint16_t*>(g_zero16);

  // DMA roles.  Instruction h of wave w fills the 1 KiB block b = N*w + h of an operand part:
  // rows 16b .. 16b+15, lane -> row 16b + lane/4, LDS chunk lane%4, source chunk swizzled.
  //   pixels:   source = x[img][ih0 + r][iw0 + s][c0 + 8*chunk ..] for tap (r, s), or zeros
  //   weights:  source = w[n][k0 + 8*chunk ..], rows past c_out clamped (they feed channels
  //             that are never stored)
  int64_t a_src[NA];        // element offset of the pixel's (ih0, iw0) corner, plus the chunk
  uint32_t a_taps[NA];      // bit 3r+s: tap (r, s) lies inside the image (0 for pixels past the end)
  const uint16_t* b_src[NB];
#pragma unroll
  for (uint32_t h = 0; h < NA; ++h) {
    const uint32_t row = 16u * (NA * wave + h) + (lane >> 2);
    const uint32_t p = bm + row;
    const bool pv = p < a.pixels;
    const uint32_t pp = pv ? p : 0u;
    const uint32_t b = pp / a.by_plane;
    const uint32_t rem = pp - b * a.Ho * a.Wo;
    const uint32_t oh = rem / a.by_wo, ow = rem - oh * a.Wo;
    const int32_t ih0 = (int32_t)(oh * a.stride) - 1, iw0 = (int32_t)(ow * a.stride) - 1;
    uint32_t taps = 0u;
#pragma unroll
    for (int32_t r = 0; r < 3; ++r)
#pragma unroll
      for (int32_t t = 0; t < 3; ++t)
        if (pv && (uint32_t)(ih0 + r) < a.H && (uint32_t)(iw0 + t) < a.W) taps |= 1u << (3 * r + t);
    a_taps[h] = taps;
    a_src[h] = (((int64_t)b * a.H + ih0) * a.W + iw0) * a.C + 8u * ((lane & 3u) ^ row_swz(row));
  }
#pragma unroll
  for (uint32_t h = 0; h < NB; ++h) {
    const uint32_t row = 16u * (NB * wave + h) + (lane >> 2);
    b_src[h] = a.w + (size_t)min(bn + row, a.K - 1u) * a.depth + 8u * ((lane & 3u) ^ row_swz(row));
  }

  const uint32_t nk = a.depth / CD_BK;
  // cursors of the two DMA streams (tile index clamped to the last tile: the schedule issues the
  // same number of loads in every iteration and the surplus lands in stages nobody reads)
  uint32_t ta = 0u, a_tap = 0u, a_c0 = 0u;    // pixels: tile, its filter tap, first channel
  uint32_t tb = 0u;                           // weights: tile
  auto dma_pixels = [&](uint32_t h) {
    const uint32_t r = (a_tap * 11u) >> 5, t = a_tap - 3u * r;
    const int64_t delta = ((int64_t)r * a.W + t) * a.C + a_c0;
    const uint32_t ok = (a_taps[h] >> a_tap) & 1u;
    dma16(pick(a.x + a_src[h] + delta, zeros, ok), lds_base + (ta % CD_NST) * STAGE + (NA * wave + h) * 1024u);
  };
  auto next_pixels = [&]() {
    if (ta + 1u < nk) {
      a_c0 += CD_BK;
      if (a_c0 == a.C) { a_c0 = 0u; ++a_tap; }
    }
    ++ta;                                    // the ring position advances even when the source is clamped
  };
  auto dma_weights = [&](uint32_t h) {
    dma16(b_src[h] + (size_t)min(tb, nk - 1u) * CD_BK, lds_base + (tb % CD_NST) * STAGE + A_BYTES + (NB * wave + h) * 1024u);
  };

  f32x16 acc[2][2];                          // [pixel block][channel block]
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // fragment addresses inside a stage, for the two 16-wide halves of a tile
  uint32_t p_off[2][2], w_off[2][2];
#pragma unroll
  for (uint32_t s = 0; s < 2; ++s)
#pragma unroll
    for (uint32_t i = 0; i < 2; ++i) {
      const uint32_t prow = wm + 32u * i + l32, wrow = wn + 32u * i + l32;
      p_off[s][i] = prow * 64u + (((2u * s + lhi) ^ row_swz(prow)) << 4);
      w_off[s][i] = A_BYTES + wrow * 64u + (((2u * s + lhi) ^ row_swz(wrow)) << 4);
    }
  u32x4 fp[2][2], fw[2][2];                  // [slot][block]
  auto frag_load = [&](const uint8_t* st, uint32_t s, uint32_t slot, uint32_t q) {   // q: w0, p0, p1, w1
    if (q == 0u) fw[slot][0] = *reinterpret_cast<const u32x4*>(st + w_off[s][0]);
    else if (q == 3u) fw[slot][1] = *reinterpret_cast<const u32x4*>(st + w_off[s][1]);
    else fp[slot][q - 1u] = *reinterpret_cast<const u32x4*>(st + p_off[s][q - 1u]);
  };
  // 4 MFMAs on fragment slot `slot` (order (j, i) = (0,0) (0,1) (1,0) (1,1)); spread between them
  // the 4 fragment reads of (tile ft, half fs) into the other slot and one part of a tile's DMA
  auto block = [&](uint32_t slot, uint32_t ft, uint32_t fs, bool weights_part) {
    const uint8_t* fst = smem + (ft % CD_NST) * STAGE;
    constexpr uint32_t ND = NA > NB ? NA : NB;
#pragma unroll
    for (uint32_t m = 0; m < 4u; ++m) {
      const uint32_t j = m >> 1, i = m & 1u;
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(fw[slot][j]), as_bf16x8(fp[slot][i]), acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      frag_load(fst, fs, slot ^ 1u, m);
#pragma unroll
      for (uint32_t h = m * ND / 4u; h < (m + 1u) * ND / 4u; ++h) {
        if (weights_part) { if (h < NB) dma_weights(h); }
        else { if (h < NA) dma_pixels(h); }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if (weights_part) ++tb; else next_pixels();
  };

  // DMA issue order: P(0) W(0) .. P(NST-2) W(NST-2) P(NST-1) | W(NST-1) P(NST) | W(NST) P(NST+1) | ..
  // (`|` = one loop iteration); tile t is complete once W(t) has landed.
#pragma unroll
  for (uint32_t t = 0; t < CD_NST - 1u; ++t) {
#pragma unroll
    for (uint32_t h = 0; h < NA; ++h) dma_pixels(h);
    next_pixels();
#pragma unroll
    for (uint32_t h = 0; h < NB; ++h) dma_weights(h);
    ++tb;
  }
#pragma unroll
  for (uint32_t h = 0; h < NA; ++h) dma_pixels(h);
  next_pixels();
  __builtin_amdgcn_s_waitcnt(vm_wait((CD_NST - 2u) * (NA + NB) + NA));   // this wave's part of tile 0 has landed
  __syncthreads();
#pragma unroll
  for (uint32_t q = 0; q < 4u; ++q) frag_load(smem, 0u, 0u, q);
  for (uint32_t kt = 0; kt < nk; ++kt) {
    block(0u, kt, 1u, true);                 // second half of tile kt's fragments; W(kt + NST - 1)
    // (NST-2) * (NA+NB) instructions were issued after W(kt+1): tile kt+1 has landed when no more
    // are outstanding; the barrier extends that to every wave's part, and tells that tile kt's
    // fragments are all in registers, which frees its stage
    __builtin_amdgcn_s_waitcnt(vm_wait((CD_NST - 2u) * (NA + NB)));
    __syncthreads();
    block(1u, kt + 1u, 0u, false);           // first half of tile kt+1's fragments; P(kt + NST) into the freed stage
  }
  __builtin_amdgcn_s_waitcnt(vm_wait(0));    // no DMA may be in flight when the LDS is given back

  // every wave is done with the ring: each takes a part of the LDS to stage its 64 pixels x 64 channels
  __syncthreads();
  const int32_t pix[2] = {(int32_t)(bm + wm), (int32_t)a.pixels};
  store_tile_via_lds<false>(smem + wave * OUT_STAGE_BYTES, acc, pix, bn + wn, a.K, a.out_f32, a.y);
}

// ---- DMA-ring implicit GEMM with the depth split over the waves of a workgroup ------------------
//
// For layers too small to give every CU a 128 x 128 tile (c_in % 64 == 0, c_out % 8 == 0).  A
// workgroup of four waves owns a 64 x 64 output tile; ring stages hold depth-64 operand tiles
// (rows of 128 bytes, 8 chunks, XOR-swizzled), and wave w multiplies only the w-th 16-deep slice
// of every stage, so the four matrix units of a CU work on one small tile at once.  The four
// partial accumulators are added through LDS (in the fixed order w = 0, 1, 2, 3) before ReLU.
//
// A layer with so few tiles that most CUs would still idle is split once more: `splits`
// workgroups share a tile, each takes a contiguous range of the depth and writes its fp32 partial
// sums to a workspace; conv_split_reduce_kernel adds them in split order and applies ReLU.
constexpr uint32_t KS_BK = 64, KS_NST = 4, KS_PART = 64u * 128u, KS_STAGE = 2u * KS_PART;
constexpr uint32_t KS_LDS = KS_NST * KS_STAGE;

__device__ __forceinline__ uint32_t row_swz8(uint32_t row) {
  return ((row >> 1) & 3u) | (((row ^ (row >> 3)) & 1u) << 2);
}

__global__ __launch_bounds__(256, 2) void conv3x3_dma_ksplit_kernel(ConvArgs a) {
  extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
  const uint32_t per_xcd = (a.tiles_total + 7u) / 8u;
  const uint32_t tile = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
  if ((blockIdx.x >> 3) >= per_xcd || tile >= a.tiles_total) return;    // tiles_total counts (tile, split) pairs
  const uint32_t split = tile % a.splits, otile = tile / a.splits;
  const uint32_t tile_m = otile / a.by_tiles_n;
  const uint32_t bm = tile_m * 64u;
  const uint32_t bn = (otile - tile_m * a.tiles_n) * 64u;
  const uint32_t kt0 = split * (a.depth / KS_BK) / a.splits;             // this workgroup's depth tiles [kt0, kt0 + nk)
  const uint32_t nk = (split + 1u) * (a.depth / KS_BK) / a.splits - kt0;

  const uint32_t lds_base = lds_address_of(smem);
  const uint32_t tid = threadIdx.x, lane = tid & 63u;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t l32 = lane & 31u, lhi = lane >> 5;

  // A workgroup advances one depth tile per pass over its loop with one wave per SIMD and only
  // four MFMAs per wave and tile, so what is issued between the MFMAs decides its speed: the loop
  // holds no vector arithmetic and no load with a 64-bit vector address (see the depth-64 ring
  // kernel).  Both operands travel through buffer resources.  Pixels: the resource spans what this
  // workgroup's 64 pixels can read, from the tap (0, 0) pixel of its first pixel to the tap (2, 2)
  // pixel of its last (input pixel indices grow with output pixel indices, also across images), so
  // its size fits 32 bits whatever the tensor's; a lane's offset changes only with the filter
  // tap, and a tap in the padding ring takes the offset `beyond`, for which the hardware delivers
  // zeros.  The walk along the depth is a scalar offset.
  auto corner = [&](uint32_t p) -> uint32_t {            // input pixel under tap (1, 1) of output pixel p
    const uint32_t b = p / a.by_plane;
    const uint32_t rem = p - b * a.Ho * a.Wo;
    const uint32_t oh = rem / a.by_wo, ow = rem - oh * a.Wo;
    return (b * a.H + oh * a.stride) * a.W + ow * a.stride;
  };
  const uint32_t lin0 = corner(bm), lin1 = corner(min(bm + 64u, a.pixels) - 1u);
  const uint32_t beyond = (lin1 - lin0 + 2u * a.W + 3u) * a.C * 2u;
  const buf_rsrc rsrc_x = make_buf_rsrc(a.x + ((int64_t)lin0 - (int64_t)a.W - 1) * a.C, beyond);
  const buf_rsrc rsrc_w = make_buf_rsrc(a.w + (size_t)bn * a.depth, min(64u, a.K - bn) * a.depth * 2u);

  // DMA roles: instruction h of wave w fills the 1 KiB block b = 2w + h of an operand part
  // (rows 8b .. 8b+7; lane -> row 8b + lane/8, LDS chunk lane%8, source chunk swizzled)
  uint32_t a_voff[2], a_taps[2], b_voff[2];
#pragma unroll
  for (uint32_t h = 0; h < 2; ++h) {
    const uint32_t row = 8u * (2u * wave + h) + (lane >> 3);
    const uint32_t p = bm + row;
    const bool pv = p < a.pixels;
    const uint32_t pp = pv ? p : bm;
    const uint32_t b = pp / a.by_plane;
    const uint32_t rem = pp - b * a.Ho * a.Wo;
    const uint32_t oh = rem / a.by_wo, ow = rem - oh * a.Wo;
    const int32_t ih0 = (int32_t)(oh * a.stride) - 1, iw0 = (int32_t)(ow * a.stride) - 1;
    uint32_t taps = 0u;
#pragma unroll
    for (int32_t r = 0; r < 3; ++r)
#pragma unroll
      for (int32_t t = 0; t < 3; ++t)
        if (pv && (uint32_t)(ih0 + r) < a.H && (uint32_t)(iw0 + t) < a.W) taps |= 1u << (3 * r + t);
    a_taps[h] = taps;
    const uint32_t chunk = (lane & 7u) ^ row_swz8(row);
    a_voff[h] = ((((b * a.H + oh * a.stride) * a.W + ow * a.stride) - lin0) * a.C + 8u * chunk) * 2u;
    b_voff[h] = ((min(bn + row, a.K - 1u) - bn) * a.depth + 8u * chunk) * 2u;
  }

  // DMA cursor: tile relative to kt0, its tap, first channel, and this lane's pixel offsets for
  // that tap.  At the last tile the cursor stops: the requests past it re-read that tile into
  // stages nobody reads any more.
  uint32_t td = 0u, a_tap = kt0 * KS_BK / a.C, a_c0 = kt0 * KS_BK - a_tap * a.C;
  uint32_t a_cur[2];
  auto new_tap = [&]() {
#pragma unroll
    for (uint32_t q = 0; q < 2u; ++q) a_cur[q] = ((a_taps[q] >> a_tap) & 1u) ? a_voff[q] : beyond;
  };
  new_tap();
  const uint32_t dst_a = lds_base + 2u * wave * 1024u, dst_b = dst_a + KS_PART;
  auto dma_tile_part = [&](uint32_t st, uint32_t q) {     // st: ring stage; q = 0, 1: pixel blocks; 2, 3: weight blocks
    if (q < 2u) {
      const uint32_t r = (a_tap * 11u) >> 5, t = a_tap - 3u * r;
      buf_dma16(a_cur[q], rsrc_x, ((r * a.W + t) * a.C + a_c0) * 2u, dst_a + st * KS_STAGE + q * 1024u);
    } else {
      buf_dma16(b_voff[q - 2u], rsrc_w, (kt0 + min(td, nk - 1u)) * (2u * KS_BK), dst_b + st * KS_STAGE + (q - 2u) * 1024u);
    }
  };
  auto next_tile = [&]() {
    ++td;
    if (td < nk) {
      a_c0 += KS_BK;
      if (a_c0 == a.C) {
        a_c0 = 0u;
        ++a_tap;
        new_tap();
      }
    }
  };

  f32x16 acc[2][2];                          // [pixel block][channel block]
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // LDS address of this wave's 16-deep slice (chunks 2*wave, 2*wave + 1) of pixel block 0 in stage
  // 0; pixel block 1 lies 4096 bytes further on (same swizzle), the weight blocks KS_PART further,
  // a stage KS_STAGE further: all immediates of the reads
  const uint32_t p_adr = lds_base + l32 * 128u + (((2u * wave + lhi) ^ row_swz8(l32)) << 4);
  typedef const u32x4 __attribute__((address_space(3))) * lds_u32x4_ptr;
  u32x4 fp[2][2], fw[2][2];                  // [slot][block]
  auto frag_load = [&](uint32_t st, uint32_t slot, uint32_t q) {   // st: stage, a constant where called; q: w0, p0, p1, w1
    if (q == 0u) fw[slot][0] = *(lds_u32x4_ptr)(uintptr_t)(p_adr + (st * KS_STAGE + KS_PART));
    else if (q == 3u) fw[slot][1] = *(lds_u32x4_ptr)(uintptr_t)(p_adr + (st * KS_STAGE + KS_PART + 4096u));
    else fp[slot][q - 1u] = *(lds_u32x4_ptr)(uintptr_t)(p_adr + (st * KS_STAGE + (q - 1u) * 4096u));
  };
  // tile kt, which lives in stage st: 4 MFMAs on slot `slot`; between them the fragment reads of
  // tile kt+1 into the other slot and this wave's part of tile kt + NST, which goes into the stage
  // tile kt leaves
  auto step = [&](uint32_t slot, uint32_t st) {
    // 2 tiles' worth of instructions were issued after tile kt+1's: it has landed when no more
    // are outstanding; the barrier extends that to every wave's part and tells that tile kt's
    // fragments are in registers everywhere
    __builtin_amdgcn_s_waitcnt(vm_wait((KS_NST - 2u) * 4u));
    __syncthreads();
#pragma unroll
    for (uint32_t m = 0; m < 4u; ++m) {
      const uint32_t j = m >> 1, i = m & 1u;
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(fw[slot][j]), as_bf16x8(fp[slot][i]), acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      frag_load((st + 1u) % KS_NST, slot ^ 1u, m);
      dma_tile_part(st, m);
      __builtin_amdgcn_sched_barrier(0);
    }
    next_tile();
  };

#pragma unroll
  for (uint32_t t = 0; t < KS_NST; ++t) {
#pragma unroll
    for (uint32_t q = 0; q < 4u; ++q) dma_tile_part(t, q);
    next_tile();
  }
  __builtin_amdgcn_s_waitcnt(vm_wait((KS_NST - 1u) * 4u));   // this wave's part of tile 0
  __syncthreads();
#pragma unroll
  for (uint32_t q = 0; q < 4u; ++q) frag_load(0u, 0u, q);
  // four tiles per pass: the ring stage and the fragment slot of each are constants
  for (uint32_t kt = 0u; kt < nk; kt += KS_NST) {
#pragma unroll
    for (uint32_t u = 0; u < KS_NST; ++u)
      if (kt + u < nk) step(u & 1u, u);
  }
  __builtin_amdgcn_s_waitcnt(vm_wait(0));    // no DMA in flight, then the ring becomes the reduction buffer
  __syncthreads();

  // partial of wave w: floats [w][pixel][quad ^ (pixel & 15)][4], quad = 4 consecutive channels
  float* part = reinterpret_cast<float*>(smem);
#pragma unroll
  for (uint32_t i = 0; i < 2; ++i) {
    const uint32_t px = 32u * i + l32;
#pragma unroll
    for (uint32_t j = 0; j < 2; ++j)
#pragma unroll
      for (uint32_t g = 0; g < 4; ++g) {
        const uint32_t quad = 8u * j + 2u * g + lhi;
        *reinterpret_cast<float4*>(part + wave * 4096u + px * 64u + ((quad ^ (px & 15u)) << 2)) =
            make_float4(acc[i][j][4u * g], acc[i][j][4u * g + 1u], acc[i][j][4u * g + 2u], acc[i][j][4u * g + 3u]);
      }
  }
  __syncthreads();
#pragma unroll
  for (uint32_t r = 0; r < 4; ++r) {
    const uint32_t px = (tid >> 4) + 16u * r, quad = tid & 15u;
    const float* src = part + px * 64u + ((quad ^ (px & 15u)) << 2);
    float4 v = *reinterpret_cast<const float4*>(src);
#pragma unroll
    for (uint32_t w = 1; w < 4; ++w) {
      const float4 u = *reinterpret_cast<const float4*>(src + w * 4096u);
      v.x += u.x; v.y += u.y; v.z += u.z; v.w += u.w;
    }
    const uint32_t p = bm + px, ch = bn + 4u * quad;
    if (p < a.pixels && ch < a.K) {                       // c_out % 4 == 0: a quad is inside or outside as a whole
      if (a.splits > 1u) {
        *reinterpret_cast<float4*>(a.work + ((size_t)split * a.pixels + p) * a.K + ch) = v;
        continue;
      }
      v.x = fmaxf(v.x, 0.f); v.y = fmaxf(v.y, 0.f); v.z = fmaxf(v.z, 0.f); v.w = fmaxf(v.w, 0.f);
      if (a.out_f32) {
        *reinterpret_cast<float4*>(reinterpret_cast<float*>(a.y) + (size_t)p * a.K + ch) = v;
      } else {
        uint2 q;
        q.x = pack_bf16x2(v.x, v.y);
        q.y = pack_bf16x2(v.z, v.w);
        *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(a.y) + (size_t)p * a.K + ch) = q;
      }
    }
  }
}

// y = ReLU(sum over splits of work[split]) for 4 consecutive outputs per thread
__global__ __launch_bounds__(256) void conv_split_reduce_kernel(const float* __restrict__ work, void* y, uint32_t splits,
                                                                uint32_t quads, uint32_t out_f32) {
  const uint32_t q = blockIdx.x * 256u + threadIdx.x;
  if (q >= quads) return;
  const float4* src = reinterpret_cast<const float4*>(work) + q;
  float4 v = src[0];
#pragma unroll 4
  for (uint32_t s = 1; s < splits; ++s) {
    const float4 u = src[(size_t)s * quads];
    v.x += u.x; v.y += u.y; v.z += u.z; v.w += u.w;
  }
  v.x = fmaxf(v.x, 0.f); v.y = fmaxf(v.y, 0.f); v.z = fmaxf(v.z, 0.f); v.w = fmaxf(v.w, 0.f);
  if (out_f32) {
    reinterpret_cast<float4*>(y)[q] = v;
  } else {
    uint2 o;
    o.x = pack_bf16x2(v.x, v.y);
    o.y = pack_bf16x2(v.z, v.w);
    reinterpret_cast<uint2*>(y)[q] = o;
  }
}

// ---- DMA-ring implicit GEMM with operand tiles of depth 64 (c_in % 64 == 0) ---------------------
//
// The tiles of conv3x3_dma_kernel with rows of 128 bytes instead of 64.  A row of an operand tile
// is then one whole cache line of the tensor (a pixel's 64 consecutive channels, a filter's 64
// consecutive depth values) instead of half of one: the 64-byte rows of the depth-32 tiles make
// the vector cache fetch every line twice, in two steps a few hundred nanoseconds apart, by which
// time a CU's two workgroups have pushed it out again, and a load that uses half of each line it
// touches runs at half the rate (measured: 28 against 56 bytes per clock and CU out of L2, 4.7
// against 10 TB/s out of the last-level cache, where the activations of a large batch live).
//
// The ring has two stages of depth 64 (the same bytes as four of depth 32).  A stage is consumed
// as four 16-deep slices; the whole DMA of tile t+2 is issued between the MFMAs of slice 3 of tile
// t, right after the barrier that frees tile t's stage, and has the three other slices of tile
// t+1 (and the CU's other workgroup) to land.  Rows are XOR-swizzled in 16-byte chunks
// (row_swz8) through each lane's choice of source chunk.
//
// The loop holds no vector arithmetic and no load with a 64-bit vector address (each of those
// between two MFMAs holds the matrix pipe up: ~14 clocks per vector-ALU instruction, 10-17 per
// such load, halved but not gone with two waves per SIMD).  Both operands travel through buffer
// resources: a lane's offset into the tensor is a 32-bit register that changes only when the
// filter tap does (then it is either the pixel's offset or, where the tap falls into the padding
// ring, an offset beyond the resource, for which the hardware delivers zeros), the walk along the
// depth is a scalar offset; the two stages are told apart by unrolling the loop over them, which
// makes a stage the immediate offset of an LDS read.  The host takes this kernel only for inputs
// below 2 GiB (the reach of the offsets).
template <uint32_t WM, uint32_t WN>
__global__ __launch_bounds__(64 * WM * WN, 2) void conv3x3_dma64_kernel(ConvArgs a) {
  constexpr uint32_t NW = WM * WN;
  constexpr uint32_t BMP = 64u * WM, BNC = 64u * WN;             // pixels x channels per workgroup
  constexpr uint32_t A_BYTES = BMP * 128u, B_BYTES = BNC * 128u, STAGE = A_BYTES + B_BYTES;
  constexpr uint32_t NA = BMP / 8u / NW, NB = BNC / 8u / NW;     // DMA instructions per wave per tile
  constexpr uint32_t ND = NA + NB;
  static_assert(NA >= 1u && NB >= 1u, "every wave takes part in both operand copies");
  static_assert(STAGE + 4096u < 65536u, "the second stage must be within reach of an LDS read's offset field");
  extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];

  const uint32_t per_xcd = (a.tiles_total + 7u) / 8u;
  const uint32_t tile = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
  if ((blockIdx.x >> 3) >= per_xcd || tile >= a.tiles_total) return;
  const uint32_t tile_m = tile / a.by_tiles_n;
  const uint32_t bm = tile_m * BMP;
  const uint32_t bn = (tile - tile_m * a.tiles_n) * BNC;

  const uint32_t lds_base = lds_address_of(smem);
  const uint32_t tid = threadIdx.x, lane = tid & 63u;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t wm = (wave / WN) * 64u, wn = (wave % WN) * 64u;
  const uint32_t l32 = lane & 31u, lhi = lane >> 5;

  // Resources.  Pixels: the whole input, its base moved back by one image row and one pixel (the
  // padding shift), so that the offset of a pixel's tap (0, 0) corner is never negative; nothing
  // in front of the tensor is ever read, because a tap outside the image takes the offset
  // `beyond` instead.  Weights: the rows of this workgroup's channels.
  const uint32_t shift = (a.W + 1u) * a.C * 2u;
  const uint32_t beyond = a.batch * a.H * a.W * a.C * 2u + shift;
  const buf_rsrc rsrc_x = make_buf_rsrc(reinterpret_cast<const uint8_t*>(a.x) - shift, beyond);
  const buf_rsrc rsrc_w = make_buf_rsrc(a.w + (size_t)bn * a.depth, min(BNC, a.K - bn) * a.depth * 2u);

  // DMA roles.  Instruction h of wave w fills the 1 KiB block b = N*w + h of an operand part:
  // rows 8b .. 8b+7, lane -> row 8b + lane/8, LDS chunk lane%8, source chunk swizzled.
  uint32_t a_voff[NA];      // byte offset of the pixel's tap (0, 0) corner in the pixel resource, plus the chunk
  uint32_t a_taps[NA];      // bit 3r+s: tap (r, s) lies inside the image (0 for pixels past the end)
  uint32_t b_voff[NB];
#pragma unroll
  for (uint32_t h = 0; h < NA; ++h) {
    const uint32_t row = 8u * (NA * wave + h) + (lane >> 3);
    const uint32_t p = bm + row;
    const bool pv = p < a.pixels;
    const uint32_t pp = pv ? p : 0u;
    const uint32_t b = pp / a.by_plane;
    const uint32_t rem = pp - b * a.Ho * a.Wo;
    const uint32_t oh = rem / a.by_wo, ow = rem - oh * a.Wo;
    const int32_t ih0 = (int32_t)(oh * a.stride) - 1, iw0 = (int32_t)(ow * a.stride) - 1;
    uint32_t taps = 0u;
#pragma unroll
    for (int32_t r = 0; r < 3; ++r)
#pragma unroll
      for (int32_t t = 0; t < 3; ++t)
        if (pv && (uint32_t)(ih0 + r) < a.H && (uint32_t)(iw0 + t) < a.W) taps |= 1u << (3 * r + t);
    a_taps[h] = taps;
    a_voff[h] = (((b * a.H + oh * a.stride) * a.W + ow * a.stride) * a.C + 8u * ((lane & 7u) ^ row_swz8(row))) * 2u;
  }
#pragma unroll
  for (uint32_t h = 0; h < NB; ++h) {
    const uint32_t row = 8u * (NB * wave + h) + (lane >> 3);
    b_voff[h] = ((min(bn + row, a.K - 1u) - bn) * a.depth + 8u * ((lane & 7u) ^ row_swz8(row))) * 2u;
  }

  const uint32_t nk = a.depth / 64u;
  uint32_t td = 0u, a_tap = 0u, a_c0 = 0u;   // DMA cursor: tile, its filter tap, first channel
  uint32_t a_cur[NA];                        // this lane's pixel offsets for the cursor's tap
  auto select_tap = [&]() {
#pragma unroll
    for (uint32_t h = 0; h < NA; ++h) a_cur[h] = ((a_taps[h] >> a_tap) & 1u) ? a_voff[h] : beyond;
  };
  select_tap();
  // instruction h of tile td's DMA (pixel blocks first, then weight blocks)
  auto dma_part = [&](uint32_t h) {
    const uint32_t stage = lds_base + (td & 1u) * STAGE;
    if (h < NA) {
      const uint32_t r = (a_tap * 11u) >> 5, t = a_tap - 3u * r;
      buf_dma16(a_cur[h], rsrc_x, ((r * a.W + t) * a.C + a_c0) * 2u, stage + (NA * wave + h) * 1024u);
    } else {
      buf_dma16(b_voff[h - NA], rsrc_w, min(td, nk - 1u) * 128u, stage + A_BYTES + (NB * wave + h - NA) * 1024u);
    }
  };
  // (the cursor stops at the last tile: the requests past it re-read that tile into a stage nobody
  // reads any more, so that every iteration issues the same instructions)
  auto next_tile = [&]() {
    if (td + 1u < nk) {
      a_c0 += 64u;
      if (a_c0 == a.C) {
        a_c0 = 0u;
        ++a_tap;
        select_tap();
      }
    }
    ++td;
  };

  f32x16 acc[2][2];                          // [pixel block][channel block]
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // LDS addresses of the fragments of block 0 in stage 0, one per 16-deep slice q (the slice flips
  // two bits of the swizzled chunk, so it is not an offset); block 1 lies 32 rows = 4096 bytes
  // further on with the same swizzle, stage 1 STAGE bytes further on: both immediates of the read
  uint32_t p_adr[4], w_adr[4];
  {
    const uint32_t prow = wm + l32, wrow = wn + l32;
#pragma unroll
    for (uint32_t q = 0; q < 4u; ++q) {
      p_adr[q] = lds_base + ((prow * 128u + ((lhi ^ row_swz8(prow)) << 4)) ^ (q << 5));
      w_adr[q] = lds_base + A_BYTES + ((wrow * 128u + ((lhi ^ row_swz8(wrow)) << 4)) ^ (q << 5));
    }
  }
  typedef const u32x4 __attribute__((address_space(3))) * lds_u32x4_ptr;
  u32x4 fp[2][2], fw[2][2];                  // [slot][block]
  auto frag_load = [&](uint32_t st, uint32_t q, uint32_t slot, uint32_t m) {   // m: w0, p0, p1, w1; st: stage, a constant
    if (m == 0u) fw[slot][0] = *(lds_u32x4_ptr)(uintptr_t)(w_adr[q] + st * STAGE);
    else if (m == 3u) fw[slot][1] = *(lds_u32x4_ptr)(uintptr_t)(w_adr[q] + (st * STAGE + 4096u));
    else fp[slot][m - 1u] = *(lds_u32x4_ptr)(uintptr_t)(p_adr[q] + (st * STAGE + (m - 1u) * 4096u));
  };
  // 4 MFMAs on fragment slot `slot` (order (j, i) = (0,0) (0,1) (1,0) (1,1)); spread between them
  // the 4 fragment reads of slice fq of stage fst into the other slot and, if `dma`, the
  // DMA of tile td
  auto block = [&](uint32_t slot, uint32_t fst, uint32_t fq, bool dma) {
#pragma unroll
    for (uint32_t m = 0; m < 4u; ++m) {
      const uint32_t j = m >> 1, i = m & 1u;
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(fw[slot][j]), as_bf16x8(fp[slot][i]), acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      frag_load(fst, fq, slot ^ 1u, m);
      if (dma) {
#pragma unroll
        for (uint32_t h = m * ND / 4u; h < (m + 1u) * ND / 4u; ++h) dma_part(h);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

#pragma unroll
  for (uint32_t t = 0; t < 2u; ++t) {        // depth = 9 * c_in: at least nine tiles
#pragma unroll
    for (uint32_t h = 0; h < ND; ++h) dma_part(h);
    next_tile();
  }
  __builtin_amdgcn_s_waitcnt(vm_wait(ND));   // this wave's part of tile 0 has landed
  __syncthreads();
#pragma unroll
  for (uint32_t m = 0; m < 4u; ++m) frag_load(0u, 0u, 0u, m);
  for (uint32_t kt0 = 0; kt0 < nk; kt0 += 2u) {
#pragma unroll
    for (uint32_t u = 0; u < 2u; ++u) {      // tile kt0 + u lives in stage u
      if (kt0 + u < nk) {
        block(0u, u, 1u, false);
        block(1u, u, 2u, false);
        block(0u, u, 3u, false);
        // Every fragment read of this tile has been issued; once they have returned and every DMA this
        // wave issued has landed (the last were the next tile's), the barrier tells that the next tile is
        // complete and that this tile's stage may be overwritten.
        __builtin_amdgcn_s_waitcnt(0x0070);      // vmcnt(0) and lgkmcnt(0)
        __syncthreads();
        block(1u, u ^ 1u, 0u, true);             // the tile after the next into the stage this tile leaves
        next_tile();
      }
    }
  }
  __builtin_amdgcn_s_waitcnt(vm_wait(0));    // no DMA may be in flight when the LDS is given back

  // every wave is done with the ring: each takes a part of the LDS to stage its 64 pixels x 64 channels
  __syncthreads();
  const int32_t pix[2] = {(int32_t)(bm + wm), (int32_t)a.pixels};
  store_tile_via_lds<false>(smem + wave * OUT_STAGE_BYTES, acc, pix, bn + wn, a.K, a.out_f32, a.y);
}

// ---- stride-1 layers with the input patch of a 2-D output tile held in LDS (c_in % 64 == 0) ------
//
// The implicit-GEMM kernels above fetch every activation once per filter tap: nine times, from L2
// or the last-level cache, and that traffic together with the address arithmetic of its DMA is
// what bounds them on the layers with many pixels.  Here a workgroup owns th x tw output pixels of
// one image (th * tw <= 256) and 64 output channels.  For each block of 64 input channels it
// copies the (th + 2) x (tw + 2) input pixels around its tile into LDS once (128 bytes per pixel,
// zeros for the padding ring outside the image), and the nine taps read their pixel operand from
// that patch at a shifted position: patch pixel (ty + r, tx + s) for output pixel (ty, tx) and tap
// (r, s).  Only the weights stream through a DMA ring (four stages of 64 channels x 64 depth
// values, one stage per tap).  The tile shape is chosen per layer on the host so that the tiles
// cover the image with little overhang.
//
// Four waves, each 64 pixels x 64 channels; pixel q = 64 * wave + 32 * i + l32 of the tile is
// (q / tw, q % tw).  Patch pixels and weight rows are 128-byte rows with their 16-byte chunks
// XOR-swizzled: weight rows by row_swz8 of the channel as in the depth-64 kernel; patch pixels by
// the low three bits of the pixel index, which keeps any eight consecutive pixels on different
// chunks whatever the tap's shift (row_swz8 assumes an even first row).
// Schedule per tap (one weight tile): four 16-deep slices of 4 MFMAs; the fragments of the next
// slice are read between the MFMAs of the current one; a barrier after slice 0 tells that the
// next weight tile has landed and that every wave is done with the previous tap, then the weight
// tile three taps ahead is requested into the stage the previous tap leaves.  The patch is single:
// when a channel block is finished the next one is requested and awaited (the CU's other
// workgroup computes meanwhile).  The results leave through store_tile_via_lds.
constexpr uint32_t PT_WST = 4u, PT_WTILE = 64u * 128u;
constexpr uint32_t PT_NPB = 11u;                          // patch DMA instructions per wave, 8 pixels each
constexpr uint32_t PT_MAX_SLOTS = 4u * PT_NPB * 8u;       // 352 patch pixels
constexpr uint32_t PT_PATCH = PT_MAX_SLOTS * 128u;        // 44 KiB
constexpr uint32_t PT_LDS = PT_PATCH + PT_WST * PT_WTILE; // 76 KiB: two workgroups per CU
constexpr uint32_t PT_MIN_TILES = 128u;                   // layers with fewer tiles take the depth-split kernel

__global__ __launch_bounds__(256, 2) void conv3x3_patch_kernel(ConvArgs a) {
  extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
  const uint32_t per_xcd = (a.tiles_total + 7u) / 8u;
  const uint32_t tile = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
  if ((blockIdx.x >> 3) >= per_xcd || tile >= a.tiles_total) return;
  uint32_t rest = tile / a.by_tiles_n;
  const uint32_t bn = (tile - rest * a.tiles_n) * 64u;
  uint32_t up = rest / a.by_tiles_x;
  const uint32_t tile_x = rest - up * a.tiles_x;
  const uint32_t img = up / a.by_tiles_y, tile_y = up - img * a.tiles_y;
  const uint32_t oh0 = tile_y * a.th, ow0 = tile_x * a.tw;
  const uint32_t pw = a.tw + 2u, slots = (a.th + 2u) * pw;
  const uint32_t nph = ((slots + 7u) / 8u + 3u) / 4u;    // patch DMA instructions per wave that carry pixels

  const uint32_t lds_base = lds_address_of(smem);
  const uint32_t tid = threadIdx.x, lane = tid & 63u;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t l32 = lane & 31u, lhi = lane >> 5;
  const uint16_t* zeros = reinterpret_cast<const uint16_t*>(g_zero16);
  const uint32_t ncb = a.C / 64u, nk = 9u * ncb;

  // Where the patch pixels come from: entry s of a table in LDS (in the weight stage that is filled
  // last) is the input pixel under patch pixel s, counted from the one under patch pixel (0, 0), or
  // all ones if s lies outside the image (the padding ring) or past the patch.  Each thread works
  // out at most two entries; the DMA roles below then cost a table read instead of a division and
  // four comparisons each.
  uint32_t* pixel_of_slot = reinterpret_cast<uint32_t*>(smem + PT_PATCH + (PT_WST - 1u) * PT_WTILE);
#pragma unroll
  for (uint32_t e = 0; e < (PT_MAX_SLOTS + 255u) / 256u; ++e) {
    const uint32_t slot = tid + 256u * e;
    const uint32_t py = slot / a.by_pw, px = slot - py * pw;
    const uint32_t ok = (uint32_t)(slot < slots) & (uint32_t)(oh0 + py - 1u < a.H) & (uint32_t)(ow0 + px - 1u < a.W);   // (- 1 wraps to a huge value above / left of the image)
    if (slot < PT_MAX_SLOTS) pixel_of_slot[slot] = ok ? py * a.W + px : 0xffffffffu;
  }
  __syncthreads();
  // Patch DMA roles: instruction h of wave w fills the 1 KiB block 4h + w = patch pixels
  // 8 * (4h + w) .. + 7; lane -> pixel + lane / 8, LDS chunk lane % 8, source chunk swizzled
  // (the pixel's low three bits are lane / 8 whatever h and w).  A pixel without a source reads
  // the block of zeros, and its source does not advance from one channel block to the next.
  // The first channel block is requested here, each instruction as soon as its address is known.
  // (origin: the input pixel under patch pixel (0, 0); it lies outside the tensor for tiles at the
  // top or left edge, and is only ever used with offsets that lead back inside)
  const uint16_t* origin = a.x + (((int64_t)img * a.H + oh0) * a.W + ow0 - (int64_t)a.W - 1) * a.C +
                           8u * ((lane & 7u) ^ ((lane >> 3) & 7u));
  const uint16_t* a_ptr[PT_NPB];
  uint32_t a_real = 0u;                      // bit h: instruction h of this lane reads the tensor
  uint32_t a_pixel[PT_NPB];                  // (all table reads first: a DMA request orders later LDS reads behind it)
#pragma unroll
  for (uint32_t h = 0; h < PT_NPB; ++h) a_pixel[h] = pixel_of_slot[8u * (4u * h + wave) + (lane >> 3)];
#pragma unroll
  for (uint32_t h = 0; h < PT_NPB; ++h) {
    if (h < nph) {
      const uint32_t pixel = a_pixel[h];
      const bool ok = pixel != 0xffffffffu;
      a_ptr[h] = ok ? origin + (uint64_t)pixel * a.C : zeros;
      a_real |= (ok ? 1u : 0u) << h;
      dma16(a_ptr[h], lds_base + (4u * h + wave) * 1024u);
      a_ptr[h] = reinterpret_cast<const uint16_t*>(reinterpret_cast<uintptr_t>(a_ptr[h]) + ((ok ? 1u : 0u) << 7));
    } else {
      a_ptr[h] = zeros;
    }
  }
  // (the table's stage takes weights only after the loop's first barrier, which every wave
  // reaches after it has used what it read here)
  // weights: instruction h of wave w fills rows 8 * (2w + h) .. + 7 of a stage.  They travel
  // through a buffer resource over this workgroup's 64 filters: the lane offset is fixed, the
  // tile's place in the depth a scalar offset, so that a request costs the loop no vector
  // arithmetic (see the depth-64 ring kernel)
  const buf_rsrc rsrc_w = make_buf_rsrc(a.w + (size_t)bn * a.depth, min(64u, a.K - bn) * a.depth * 2u);
  uint32_t b_voff[2];
#pragma unroll
  for (uint32_t h = 0; h < 2; ++h) {
    const uint32_t row = 8u * (2u * wave + h) + (lane >> 3);
    b_voff[h] = ((min(bn + row, a.K - 1u) - bn) * a.depth + 8u * ((lane & 7u) ^ row_swz8(row))) * 2u;
  }
  // weight tile t belongs to channel block t / 9 and tap t % 9: depth offset tap * C + 64 * block.
  // The cursor stops at the last tile; the requests past it land in stages nobody reads and
  // keep the count of outstanding requests the same in every iteration.
  uint32_t wt = 0u, w_tap = 0u, w_cb = 0u;
  auto dma_weights = [&]() {
    const uint32_t off = (w_tap * a.C + 64u * w_cb) * 2u;
    const uint32_t stage = lds_base + PT_PATCH + (wt & (PT_WST - 1u)) * PT_WTILE;
#pragma unroll
    for (uint32_t h = 0; h < 2; ++h) buf_dma16(b_voff[h], rsrc_w, off, stage + (2u * wave + h) * 1024u);
    if (wt + 1u < nk) {
      if (++w_tap == 9u) { w_tap = 0u; ++w_cb; }
    }
    ++wt;
  };
#pragma unroll
  for (uint32_t t = 0; t < PT_WST - 1u; ++t) dma_weights();   // depth = 9 * c_in: at least nine tiles

  f32x16 acc[2][2];                          // [pixel block][channel block]
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // this lane's two pixels: patch pixel index of tap (0, 0), and where the result goes
  uint32_t slot0[2];
  int64_t out_px[2];                         // output pixel index, -1 if the lane has none
#pragma unroll
  for (uint32_t i = 0; i < 2; ++i) {
    const uint32_t q = 64u * wave + 32u * i + l32;
    const uint32_t ty = q / a.by_tw, tx = q - ty * a.tw;
    const bool ok = q < a.th * a.tw && oh0 + ty < a.Ho && ow0 + tx < a.Wo;
    slot0[i] = q < a.th * a.tw ? ty * pw + tx : 0u;
    out_px[i] = ok ? ((int64_t)img * a.Ho + oh0 + ty) * a.Wo + ow0 + tx : -1;
  }
  // byte address (inside the patch) of slice 0 of the pixel fragment for a tap whose patch offset is `shift`
  auto patch_off = [&](uint32_t i, uint32_t shift) {
    const uint32_t slot = slot0[i] + shift;
    return slot * 128u + ((lhi ^ (slot & 7u)) << 4);
  };
  // LDS address of the weight fragment of block 0 in ring stage 0, one per 16-deep slice (the slice
  // flips two bits of the swizzled chunk); block 1 lies 32 rows = 4096 bytes further on.  A tap
  // adds its stage to the four of them in one go (w_at), so that no read waits for an add.
  uint32_t w_adr[4];
#pragma unroll
  for (uint32_t q = 0; q < 4u; ++q) w_adr[q] = lds_base + PT_PATCH + ((l32 * 128u + ((lhi ^ row_swz8(l32)) << 4)) ^ (q << 5));
  typedef const u32x4 __attribute__((address_space(3))) * lds_u32x4_ptr;

  u32x4 fp[2][2], fw[2][2];                  // [slot][block]
  // fragment m (w0, p0, p1, w1) of slice q: pixels at p_at[] inside the patch, weights at LDS address wq
  auto frag_load = [&](const uint32_t (&p_at)[2], uint32_t wq, uint32_t q, uint32_t slot, uint32_t m) {
    if (m == 0u) fw[slot][0] = *(lds_u32x4_ptr)(uintptr_t)wq;
    else if (m == 3u) fw[slot][1] = *(lds_u32x4_ptr)(uintptr_t)(wq + 4096u);
    else fp[slot][m - 1u] = *reinterpret_cast<const u32x4*>(smem + (p_at[m - 1u] ^ (q << 5)));
  };
  // 4 MFMAs on fragment slot `slot`; between them the 4 fragment reads of slice fq (pixels at
  // p_at, weights at wq) into the other slot and, if `dma`, the request for the next weight tile
  auto block = [&](uint32_t slot, const uint32_t (&p_at)[2], uint32_t wq, uint32_t fq, bool dma) {
#pragma unroll
    for (uint32_t m = 0; m < 4u; ++m) {
      const uint32_t j = m >> 1, i = m & 1u;
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(fw[slot][j]), as_bf16x8(fp[slot][i]), acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      frag_load(p_at, wq, fq, slot ^ 1u, m);
      if (dma && m == 1u) dma_weights();
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  uint32_t kt = 0u;
  for (uint32_t cb = 0; cb < ncb; ++cb) {
    if (cb != 0u) {
      // the patch of this channel block, once every wave has read the previous one to the end
      __builtin_amdgcn_s_waitcnt(0xC07Fu);   // lgkmcnt(0)
      __syncthreads();
#pragma unroll
      for (uint32_t h = 0; h < PT_NPB; ++h)
        if (h < nph) {
          dma16(a_ptr[h], lds_base + (4u * h + wave) * 1024u);
          a_ptr[h] = reinterpret_cast<const uint16_t*>(reinterpret_cast<uintptr_t>(a_ptr[h]) + (((a_real >> h) & 1u) << 7));
        }
    }
    __builtin_amdgcn_s_waitcnt(vm_wait(0));
    __syncthreads();
    uint32_t p_at[2] = {patch_off(0u, 0u), patch_off(1u, 0u)};
    {
      const uint32_t w0 = w_adr[0] + (kt & (PT_WST - 1u)) * PT_WTILE;
#pragma unroll
      for (uint32_t m = 0; m < 4u; ++m) frag_load(p_at, w0, 0u, 0u, m);
    }
#pragma unroll
    for (uint32_t tap = 0; tap < 9u; ++tap, ++kt) {       // (unrolled: a tap's patch offsets are then constants of the code)
      // this tap's stage for slices 1 .. 3, the next tap's for its slice 0
      const uint32_t cur = (kt & (PT_WST - 1u)) * PT_WTILE, nxt = ((kt + 1u) & (PT_WST - 1u)) * PT_WTILE;
      uint32_t w_at[4] = {w_adr[0] + nxt, w_adr[1] + cur, w_adr[2] + cur, w_adr[3] + cur};
      asm volatile("" : "+v"(w_at[0]), "+v"(w_at[1]), "+v"(w_at[2]), "+v"(w_at[3]));   // all four here, in one burst: left to
      __builtin_amdgcn_sched_barrier(0);                                                // itself the compiler sinks each add to its read
      block(0u, p_at, w_at[1], 1u, false);
      // At most the weight tile after the next is outstanding: the next one has landed, and the
      // barrier tells so for every wave's part.  It also tells that every wave has finished the
      // previous tap (its last MFMAs needed that tap's last fragments), whose stage the request
      // of the following block overwrites with the tile three taps ahead.
      __builtin_amdgcn_s_waitcnt(vm_wait(2));
      __syncthreads();
      block(1u, p_at, w_at[2], 2u, true);
      block(0u, p_at, w_at[3], 3u, false);
      const uint32_t nt = tap + 1u < 9u ? tap + 1u : 8u;     // (after the last tap the reads fetch bytes nobody uses)
      const uint32_t r = (nt * 11u) >> 5, t = nt - 3u * r;
      p_at[0] = patch_off(0u, r * pw + t);
      p_at[1] = patch_off(1u, r * pw + t);
      block(1u, p_at, w_at[0], 0u, false);
    }
  }
  __builtin_amdgcn_s_waitcnt(vm_wait(0));    // no DMA may be in flight when the LDS is given back

  // the patch and the ring are done with: every wave takes a part of the LDS to stage its results
  __syncthreads();
  const int32_t pix[2] = {(int32_t)out_px[0], (int32_t)out_px[1]};
  store_tile_via_lds<true>(smem + wave * (OUT_STAGE_BYTES + 256u), acc, pix, bn, a.K, a.out_f32, a.y);
}

// ---- stride-2 layer with 32 input channels (c_out % 8 == 0, c_out <= 64) -------------------------
//
// The second layer of the net: few channels, many pixels, nine depth tiles of 32 only.  As an
// implicit GEMM it spends its time in set-up, in 2.25 fetches of every activation and in
// half-used cache lines (a pixel's 32 channels are 64 bytes).  Here a workgroup owns th x tw output
// pixels of one image (th * tw <= 128) and all output channels, and holds in LDS
//   * the whole filter, c_out rows of 9 * 32 values (576 bytes), the low two bits of a row's
//     16-byte chunk index XORed with bits 2..3 of the row: the rows of 16 consecutive channels
//     then hit 16 different 16-byte slots of a 256-byte bank sweep;
//   * the (2 th + 1) x (2 tw + 1) input pixels its tile reads (64 bytes each, zeros outside the
//     image), every patch row stored as its even columns followed by its odd columns, so that the
//     pixels the 32 lanes of a fragment read for one tap are neighbours in LDS although they are
//     two apart in the image: output pixel (ty, tx), tap (r, s) reads row 2 ty + r, even column
//     tx (s = 0) or tx + 1 (s = 2), or odd column tx (s = 1).
// Nothing streams: one barrier after the copies, then 9 taps x 2 slices of 16 with no further
// synchronisation.  Four waves, each 32 pixels x 64 channels.  16-byte chunks of a pixel are
// XOR-swizzled by bits 2..3 of the pixel's LDS index.
//
// FUSED: the layer in front is the net's 3-channel first layer with 32 output channels, and the
// patch is computed here instead of being read: the workgroup loads the raw 3-channel pixels
// under its patch (two more rows and columns), runs the first layer on them exactly as
// conv3x3_c3_kernel does (three MFMA steps per 32 pixels, one per filter row, same operand
// layout, so the same bits come out), applies ReLU and the bf16 rounding and writes the values
// where the DMA would have put them (zeros where the patch leaves the image: that is the second
// layer's padding, not a first-layer output).  The first layer's output, 32 channels at full
// resolution and the largest tensor of the net, is then neither written nor read back.
constexpr uint32_t S2_NPB = 9u;                           // patch DMA instructions per wave, 16 pixels each
constexpr uint32_t S2_MAX_SLOTS = 4u * S2_NPB * 16u;      // 576 patch pixels
constexpr uint32_t S2_PATCH = S2_MAX_SLOTS * 64u;         // 36 KiB
constexpr uint32_t S2_WPITCH = 576u, S2_WBYTES = 64u * S2_WPITCH;
constexpr uint32_t S2_LDS = S2_PATCH + S2_WBYTES + S2_MAX_SLOTS * 4u;   // 76032 bytes: two workgroups per CU
constexpr uint32_t S2_MIN_TILES = 256u;
// tiles are kept to th + tw <= 30: patch height + width <= 62, so that the raw pixels under a
// patch (height + 2 by width + 2) are at most 576 + 2 * 62 + 4 = 704
constexpr uint32_t S2_MAX_SIDES = 30u;
constexpr uint32_t S2_FIRST_W = 32u * 27u * 2u;           // the first layer's filter, 1728 bytes
constexpr uint32_t S2_RAW_MAX = 704u;                     // raw pixels under a patch, 8 bytes each
constexpr uint32_t S2_LDS_FUSED = S2_PATCH + S2_WBYTES + S2_FIRST_W + (S2_RAW_MAX + 1u) * 8u;   // 81096 bytes: two per CU (one
                                                          // entry more: the padding tap of the last pixel reads it)

template <bool FUSED>
__global__ __launch_bounds__(256, 2) void conv3x3_s2c32_kernel(ConvArgs a) {
  extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
  const uint32_t per_xcd = (a.tiles_total + 7u) / 8u;
  const uint32_t tile = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
  if ((blockIdx.x >> 3) >= per_xcd || tile >= a.tiles_total) return;
  const uint32_t up = tile / a.by_tiles_x;
  const uint32_t tile_x = tile - up * a.tiles_x;
  const uint32_t img = up / a.by_tiles_y, tile_y = up - img * a.tiles_y;
  const uint32_t oh0 = tile_y * a.th, ow0 = tile_x * a.tw;
  const uint32_t pw = 2u * a.tw + 1u, slots = (2u * a.th + 1u) * pw;
  const uint32_t nph = ((slots + 15u) / 16u + 3u) / 4u;   // patch DMA instructions per wave that carry pixels

  const uint32_t lds_base = lds_address_of(smem);
  const uint32_t tid = threadIdx.x, lane = tid & 63u;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t l32 = lane & 31u, lhi = lane >> 5;
  const uint16_t* zeros = reinterpret_cast<const uint16_t*>(g_zero16);
  (void)zeros;
  uint8_t* wl = smem + S2_PATCH;

  // filter: 36 chunks of 16 bytes per channel, 2304 in all = 36 DMA instructions, 9 per wave.
  // Chunk c of channel row sits at LDS chunk 36 * row + (c with its low two bits ^ bits 2..3 of
  // the row); channels past c_out repeat the last one (they feed outputs that are never stored).
#pragma unroll
  for (uint32_t e = 0; e < 9u; ++e) {
    const uint32_t at = 64u * (4u * e + wave) + lane, row = at / 36u, pos = at - 36u * row;
    const uint32_t c = pos ^ ((row >> 2) & 3u);
    dma16(a.w + (size_t)min(row, a.K - 1u) * 288u + 8u * c, lds_base + S2_PATCH + (4u * e + wave) * 1024u);
  }

  if (FUSED) {
    // raw pixels under the patch: rows 2 oh0 - 2 .. 2 oh0 + 2 th, columns 2 ow0 - 2 .. 2 ow0 + 2 tw, each
    // padded to four channels (8 bytes), zeros outside the image; and the first layer's filter.
    // All loads are issued before the first of them is used.
    uint16_t* w0l = reinterpret_cast<uint16_t*>(smem + S2_PATCH + S2_WBYTES);
    uint2* raw = reinterpret_cast<uint2*>(smem + S2_PATCH + S2_WBYTES + S2_FIRST_W);
    const uint32_t rw = pw + 2u, raws = (2u * a.th + 3u) * rw;
    constexpr uint32_t RAW_ITERS = (S2_RAW_MAX + 255u) / 256u, W_ITERS = (32u * 27u + 255u) / 256u;
    uint32_t rc[RAW_ITERS][3], wv[W_ITERS];
    bool rok[RAW_ITERS];
#pragma unroll
    for (uint32_t it = 0; it < RAW_ITERS; ++it) {
      const uint32_t idx = tid + 256u * it;
      const uint32_t iy = idx / a.by_iw, ix = idx - iy * rw;
      const uint32_t gy = 2u * oh0 + iy - 2u, gx = 2u * ow0 + ix - 2u;      // (wraps to a huge value above / left of the image)
      rok[it] = idx < raws && gy < a.H && gx < a.W;
      const int64_t g = rok[it] ? ((int64_t)img * a.H + gy) * a.W + gx : 0;
#pragma unroll
      for (uint32_t c = 0; c < 3; ++c) rc[it][c] = a.x[g * 3 + c];
    }
#pragma unroll
    for (uint32_t it = 0; it < W_ITERS; ++it) {
      const uint32_t idx = tid + 256u * it;
      wv[it] = a.w_first[idx < 32u * 27u ? idx : 0u];
    }
#pragma unroll
    for (uint32_t it = 0; it < RAW_ITERS; ++it) {
      const uint32_t idx = tid + 256u * it;
      if (idx < S2_RAW_MAX) raw[idx] = rok[it] ? make_uint2(rc[it][0] | (rc[it][1] << 16), rc[it][2]) : make_uint2(0u, 0u);
    }
#pragma unroll
    for (uint32_t it = 0; it < W_ITERS; ++it) {
      const uint32_t idx = tid + 256u * it;
      if (idx < 32u * 27u) w0l[idx] = (uint16_t)wv[it];
    }
    __syncthreads();
    // first-layer weight fragments of filter row r: channel l32, operand e = (s, c) = (2*lhi + e/4, e%4)
    u32x4 f0[3];
#pragma unroll
    for (uint32_t r = 0; r < 3; ++r) {
      uint32_t wd[4] = {0u, 0u, 0u, 0u};
#pragma unroll
      for (uint32_t e = 0; e < 8; ++e) {
        const uint32_t t = 2u * lhi + (e >> 2), c = e & 3u;
        const uint32_t ok = (uint32_t)(t < 3u) & (uint32_t)(c < 3u);
        const uint32_t v = w0l[ok ? l32 * 27u + r * 9u + t * 3u + c : 0u];
        wd[e >> 1] |= (ok ? v : 0u) << (16u * (e & 1u));
      }
      f0[r] = u32x4{wd[0], wd[1], wd[2], wd[3]};
    }
    // the first layer on the patch, 32 patch pixels (row-major) per block, the waves taking turns;
    // two blocks at a time, so that one block's chain of three dependent MFMAs fills the gaps of the other's
    for (uint32_t first = 32u * wave; first < slots; first += 256u) {
      uint32_t py[2], px[2];
      bool in_patch[2];
      f32x16 z[2];
#pragma unroll
      for (uint32_t u = 0; u < 2; ++u) {
        const uint32_t qp = first + 128u * u + l32;
        in_patch[u] = qp < slots;
        const uint32_t qq = in_patch[u] ? qp : 0u;
        py[u] = qq / a.by_pw;
        px[u] = qq - py[u] * pw;
#pragma unroll
        for (int r = 0; r < 16; ++r) z[u][r] = 0.f;
      }
#pragma unroll
      for (uint32_t r = 0; r < 3; ++r)
#pragma unroll
        for (uint32_t u = 0; u < 2; ++u) {
          // taps s = 2*lhi and 2*lhi + 1 of row r: raw pixels (py + r, px + s), (py + r, px + s + 1)
          const uint2 d0 = raw[(py[u] + r) * rw + px[u] + 2u * lhi];
          const uint2 d1 = raw[(py[u] + r) * rw + px[u] + 2u * lhi + 1u];
          const uint32_t m1 = lhi ? 0u : 0xffffffffu;                        // s = 3 is padding
          z[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(f0[r]), as_bf16x8(u32x4{d0.x, d0.y, d1.x & m1, d1.y & m1}), z[u], 0, 0, 0);
        }
#pragma unroll
      for (uint32_t u = 0; u < 2; ++u) {
        // channels 8g + 4*lhi + (0..3) of patch pixel (py, px) -> its LDS place (even columns first)
        const bool real = 2u * oh0 + py[u] - 1u < a.H && 2u * ow0 + px[u] - 1u < a.W;
        const uint32_t slot = py[u] * pw + ((px[u] & 1u) ? a.tw + 1u + (px[u] >> 1) : (px[u] >> 1));
        if (in_patch[u]) {
#pragma unroll
          for (uint32_t g = 0; g < 4; ++g) {
            uint2 v;
            v.x = real ? pack_bf16x2(fmaxf(z[u][4u * g], 0.f), fmaxf(z[u][4u * g + 1u], 0.f)) : 0u;
            v.y = real ? pack_bf16x2(fmaxf(z[u][4u * g + 2u], 0.f), fmaxf(z[u][4u * g + 3u], 0.f)) : 0u;
            *reinterpret_cast<uint2*>(smem + slot * 64u + ((g ^ ((slot >> 2) & 3u)) << 4) + 8u * lhi) = v;
          }
        }
      }
    }
  } else {
    // entry s of the table: the input pixel stored at LDS index s, counted from the one under patch
    // pixel (0, 0), or all ones if it lies outside the image or s is past the patch
    uint32_t* pixel_of_slot = reinterpret_cast<uint32_t*>(smem + S2_PATCH + S2_WBYTES);
  #pragma unroll
    for (uint32_t e = 0; e < (S2_MAX_SLOTS + 255u) / 256u; ++e) {
      const uint32_t slot = tid + 256u * e;
      const uint32_t py = slot / a.by_pw, rem = slot - py * pw;
      const uint32_t px = rem <= a.tw ? 2u * rem : 2u * (rem - a.tw) - 1u;        // even columns first, then the odd ones
      const uint32_t ok = (uint32_t)(slot < slots) & (uint32_t)(2u * oh0 + py - 1u < a.H) & (uint32_t)(2u * ow0 + px - 1u < a.W);
      if (slot < S2_MAX_SLOTS) pixel_of_slot[slot] = ok ? py * a.W + px : 0xffffffffu;
    }
    __syncthreads();
    // patch: instruction h of wave w fills the 1 KiB block 4h + w = LDS pixels 16 * (4h + w) .. + 15;
    // lane -> pixel + lane / 4, LDS chunk lane % 4, source chunk swizzled (bits 2..3 of the pixel
    // index are bits 4..5 of the lane whatever h and w)
    const uint16_t* origin = a.x + (((int64_t)img * a.H + 2 * (int64_t)oh0) * a.W + 2 * (int64_t)ow0 - (int64_t)a.W - 1) * 32 +
                             8u * ((lane & 3u) ^ ((lane >> 4) & 3u));
    uint32_t a_pixel[S2_NPB];                  // (all table reads first: a DMA request orders later LDS reads behind it)
  #pragma unroll
    for (uint32_t h = 0; h < S2_NPB; ++h) a_pixel[h] = pixel_of_slot[16u * (4u * h + wave) + (lane >> 2)];
  #pragma unroll
    for (uint32_t h = 0; h < S2_NPB; ++h)
      if (h < nph) dma16(a_pixel[h] != 0xffffffffu ? origin + (uint64_t)a_pixel[h] * 32u : zeros, lds_base + (4u * h + wave) * 1024u);
  }
  f32x16 acc[1][2];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[0][j][r] = 0.f;
  // this lane's pixel: LDS index of its tap (0, 0), and where the result goes
  const uint32_t q = 32u * wave + l32;
  const uint32_t ty = q / a.by_tw, tx = q - ty * a.tw;
  const bool mine = q < a.th * a.tw;
  const uint32_t slot0 = mine ? 2u * ty * pw + tx : 0u;
  const int32_t pix[2] = {mine && oh0 + ty < a.Ho && ow0 + tx < a.Wo ? (int32_t)((img * a.Ho + oh0 + ty) * a.Wo + ow0 + tx) : -1, -1};
  // weight fragments: row 32 j + l32 (bits 2..3 the same for both j), depth chunk 4 * tap + 2 * slice + lhi
  const uint32_t w_at = l32 * S2_WPITCH, w_swz = (l32 >> 2) & 3u;

  __builtin_amdgcn_s_waitcnt(vm_wait(0));
  __syncthreads();
  // slice n = 2 * tap + half: the fragments of slice n + 1 are read before the MFMAs of slice n
  u32x4 fp[2], fw[2][2];
  auto frag_load = [&](uint32_t n, uint32_t set) {
    const uint32_t tap = n >> 1, sl = n & 1u;
    const uint32_t r = tap / 3u, t = tap - 3u * r;
    const uint32_t slot = slot0 + r * pw + (t == 1u ? a.tw + 1u : t >> 1);
    fp[set] = *reinterpret_cast<const u32x4*>(smem + slot * 64u + (((2u * sl + lhi) ^ ((slot >> 2) & 3u)) << 4));
    const uint32_t at = w_at + 64u * tap + (((2u * sl + lhi) ^ w_swz) << 4);
    fw[set][0] = *reinterpret_cast<const u32x4*>(wl + at);
    fw[set][1] = *reinterpret_cast<const u32x4*>(wl + at + 32u * S2_WPITCH);
  };
  frag_load(0u, 0u);
#pragma unroll
  for (uint32_t n = 0; n < 18u; ++n) {
    if (n + 1u < 18u) frag_load(n + 1u, (n + 1u) & 1u);
    acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(fw[n & 1u][0]), as_bf16x8(fp[n & 1u]), acc[0][0], 0, 0, 0);
    acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(fw[n & 1u][1]), as_bf16x8(fp[n & 1u]), acc[0][1], 0, 0, 0);
  }
  // every wave is done with the patch: each takes a part of it to stage its results
  __syncthreads();
  store_tile_via_lds<true, 1u>(smem + wave * (OUT_STAGE_BYTES / 2u + 128u), acc, pix, 0u, a.K, a.out_f32, a.y);
}

// ---- 3-channel first layer (c_in == 3, stride 1, c_out % 8 == 0, c_out <= 64) ------------------
//
// Depth 27: the kernel is bound by writing its output (c_out / 3 times the input).  A workgroup
// owns 256 consecutive output pixels (n, oh, ow flattened).  With stride 1 the input pixel of tap
// (r, s) is the output pixel's flattened index + (r-1)*W + (s-1), so the three input strips
// [first - 1 + (r-1)*W, + 260 pixels) hold every operand; they are copied to LDS once, each pixel
// padded to four channels (8 bytes, zeros outside the tensor).  The depth is laid out as
// (r, s, c) with s and c padded to 4: 16 per filter row, one MFMA step per row, and a lane's
// eight operands of a step are two adjacent padded pixels = 16 contiguous, 8-byte aligned bytes
// of LDS (one two-address read), with the taps that fall outside the image masked to zero.  The
// padding positions meet zero weights.  The results are rounded, transposed through LDS and
// written as 16 bytes per lane, 4 KiB contiguous per wave.
constexpr uint32_t C3_PIX = 256, C3_STRIP_PIX = 260;   // 256 + 2 halo pixels + the padded tap s = 3

template <uint32_t NJ>    // 32-channel blocks: c_out <= 32 * NJ
__global__ __launch_bounds__(256) void conv3x3_c3_kernel(ConvArgs a) {
  __shared__ __attribute__((aligned(16))) uint2 strip[3u * C3_STRIP_PIX];
  __shared__ __attribute__((aligned(16))) uint16_t outs[C3_PIX * 32u * NJ];
  const uint32_t bm = blockIdx.x * C3_PIX;
  if (bm >= a.pixels) return;
  const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
  const uint32_t l32 = lane & 31u, lhi = lane >> 5;

  // input strips (H = Ho, W = Wo with stride 1: input and output pixels share their flattened index).
  // All loads of the set-up, strips and weights, are issued before the first of them is used:
  // one trip to memory instead of one per loop iteration.
  const int64_t total = (int64_t)a.pixels;
  constexpr uint32_t STRIP_ITERS = (3u * C3_STRIP_PIX + 255u) / 256u;
  uint32_t sc[STRIP_ITERS][3];
  bool sok[STRIP_ITERS];
#pragma unroll
  for (uint32_t it = 0; it < STRIP_ITERS; ++it) {
    const uint32_t idx = tid + 256u * it;
    const uint32_t r = idx / C3_STRIP_PIX, e = idx - r * C3_STRIP_PIX;
    const int64_t g = (int64_t)bm - 1 + ((int64_t)r - 1) * a.W + e;
    sok[it] = idx < 3u * C3_STRIP_PIX && g >= 0 && g < total;
    const int64_t gc = sok[it] ? g : 0;
#pragma unroll
    for (uint32_t c = 0; c < 3; ++c) sc[it][c] = a.x[gc * 3 + c];
  }

  // The filter (27 values per channel) goes through LDS, in the space the results are staged in
  // later: 27 * c_out loads per workgroup instead of 24 per lane and block of 32 channels.  The
  // CU's address unit handles a load instruction in the same time whatever its width, and with
  // the per-lane gather the kernel was bound by it.
  constexpr uint32_t W_ITERS = (32u * NJ * 27u + 255u) / 256u;
  uint32_t wv[W_ITERS];
#pragma unroll
  for (uint32_t it = 0; it < W_ITERS; ++it) {
    const uint32_t idx = tid + 256u * it;
    wv[it] = a.w[idx < a.K * 27u ? idx : 0u];
  }
#pragma unroll
  for (uint32_t it = 0; it < STRIP_ITERS; ++it) {
    const uint32_t idx = tid + 256u * it;
    if (idx < 3u * C3_STRIP_PIX)
      strip[idx] = sok[it] ? make_uint2(sc[it][0] | (sc[it][1] << 16), sc[it][2]) : make_uint2(0u, 0u);
  }
#pragma unroll
  for (uint32_t it = 0; it < W_ITERS; ++it) {
    const uint32_t idx = tid + 256u * it;
    if (idx < 32u * NJ * 27u) outs[idx] = (uint16_t)(idx < a.K * 27u ? wv[it] : 0u);
  }
  __syncthreads();

  // weight fragments of filter row r: channel 32j + l32, operand e = (s, c) = (2*lhi + e/4, e%4)
  u32x4 fw[3][NJ];
#pragma unroll
  for (uint32_t r = 0; r < 3; ++r)
#pragma unroll
    for (uint32_t j = 0; j < NJ; ++j) {
      const uint32_t ch = 32u * j + l32;
      uint32_t wd[4] = {0u, 0u, 0u, 0u};
#pragma unroll
      for (uint32_t e = 0; e < 8; ++e) {
        const uint32_t t = 2u * lhi + (e >> 2), c = e & 3u;
        const uint32_t ok = (uint32_t)(t < 3u) & (uint32_t)(c < 3u);      // (channels >= c_out hold zeros)
        const uint32_t v = outs[ok ? ch * 27u + r * 9u + t * 3u + c : 0u];
        wd[e >> 1] |= (ok ? v : 0u) << (16u * (e & 1u));
      }
      fw[r][j] = u32x4{wd[0], wd[1], wd[2], wd[3]};
    }

  f32x16 acc[2][NJ];
#pragma unroll
  for (uint32_t i = 0; i < 2; ++i) {
    const uint32_t pl = 64u * wave + 32u * i + l32;            // pixel inside the workgroup's 256
    const uint32_t p = bm + pl;
    const uint32_t rem = p - (p / a.by_plane) * (a.H * a.W);     // (stride 1: Ho = H, Wo = W)
    const uint32_t oh = rem / a.by_wo, ow = rem - oh * a.W;
    uint32_t taps = 0u;
#pragma unroll
    for (int32_t r = 0; r < 3; ++r)
#pragma unroll
      for (int32_t t = 0; t < 3; ++t)
        if (p < a.pixels && (uint32_t)((int32_t)oh + r - 1) < a.H && (uint32_t)((int32_t)ow + t - 1) < a.W)
          taps |= 1u << (3 * r + t);
#pragma unroll
    for (uint32_t j = 0; j < NJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
#pragma unroll
    for (uint32_t r = 0; r < 3; ++r) {
      // taps s = 2*lhi and 2*lhi + 1 of row r: input pixels pl + s - 1 = strip entries pl + s
      const uint2 d0 = strip[r * C3_STRIP_PIX + pl + 2u * lhi];
      const uint2 d1 = strip[r * C3_STRIP_PIX + pl + 2u * lhi + 1u];
      const uint32_t ok0 = (taps >> (3u * r + 2u * lhi)) & 1u;
      const uint32_t ok1 = lhi ? 0u : (taps >> (3u * r + 1u)) & 1u;       // s = 3 is padding
      const uint32_t m0 = 0u - ok0, m1 = 0u - ok1;
      const bf16x8 fp = as_bf16x8(u32x4{d0.x & m0, d0.y & m0, d1.x & m1, d1.y & m1});
#pragma unroll
      for (uint32_t j = 0; j < NJ; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(fw[r][j]), fp, acc[i][j], 0, 0, 0);
    }
  }

  __syncthreads();            // every wave has read the filter out of `outs`
  // ReLU + rounding; transpose through LDS: outs[pixel][channel], c_out values per pixel
  const uint32_t Kc = a.K;
  if (!a.out_f32) {
#pragma unroll
    for (uint32_t i = 0; i < 2; ++i)
#pragma unroll
      for (uint32_t j = 0; j < NJ; ++j)
#pragma unroll
        for (uint32_t g = 0; g < 4; ++g) {
          const uint32_t pl = 64u * wave + 32u * i + l32, ch = 32u * j + 8u * g + 4u * lhi;
          if (ch < Kc) {
            uint2 q;
            q.x = pack_bf16x2(fmaxf(acc[i][j][4u * g], 0.f), fmaxf(acc[i][j][4u * g + 1u], 0.f));
            q.y = pack_bf16x2(fmaxf(acc[i][j][4u * g + 2u], 0.f), fmaxf(acc[i][j][4u * g + 3u], 0.f));
            *reinterpret_cast<uint2*>(&outs[pl * Kc + ch]) = q;
          }
        }
    __syncthreads();
    const uint32_t chunks = C3_PIX * Kc / 8u;                  // 16-byte chunks of the workgroup's output
    uint16_t* y = reinterpret_cast<uint16_t*>(a.y) + (size_t)bm * Kc;
    const uint32_t valid = (min(a.pixels - bm, C3_PIX) * Kc) / 8u;
    for (uint32_t q = tid; q < chunks; q += 256u)
      if (q < valid) *reinterpret_cast<u32x4*>(y + 8u * (size_t)q) = *reinterpret_cast<const u32x4*>(&outs[8u * q]);
  } else {
#pragma unroll
    for (uint32_t i = 0; i < 2; ++i)
#pragma unroll
      for (uint32_t j = 0; j < NJ; ++j)
#pragma unroll
        for (uint32_t g = 0; g < 4; ++g) {
          const uint32_t p = bm + 64u * wave + 32u * i + l32, ch = 32u * j + 8u * g + 4u * lhi;
          if (p < a.pixels && ch < Kc)
            *reinterpret_cast<float4*>(reinterpret_cast<float*>(a.y) + (size_t)p * Kc + ch) =
                make_float4(fmaxf(acc[i][j][4u * g], 0.f), fmaxf(acc[i][j][4u * g + 1u], 0.f),
                            fmaxf(acc[i][j][4u * g + 2u], 0.f), fmaxf(acc[i][j][4u * g + 3u], 0.f));
        }
  }
}

enum Path { PATH_GENERIC, PATH_DMA_128x128, PATH_DMA_256x64, PATH_DMA_64x64, PATH_DMA_KSPLIT, PATH_C3, PATH_PATCH, PATH_S2C32 };

struct Geometry {
  uint32_t Ho, Wo, pixels, bn, tiles_n, total, blocks, threads;
  Path path;
  uint32_t th, tw, tiles_y, tiles_x;   // PATH_PATCH: output tile, tiles per image
};

// Output tile of a patch kernel for an image of h x w output pixels: th * tw <= max_px pixels
// whose input patch ((th + 2) * (tw + 2) pixels at stride 1, (2 th + 1) * (2 tw + 1) at stride 2)
// fits max_slots, such that the fewest tiles cover the image (every tile costs the MFMAs of
// max_px pixels); among those the one with the smallest patch.
void patch_tile(uint32_t h, uint32_t w, uint32_t stride, uint32_t max_px, uint32_t max_slots, uint32_t* th, uint32_t* tw,
                uint32_t max_sides = 0xffffffffu) {      // max_sides: limit on th + tw
  uint64_t best_tiles = ~0ull;
  uint32_t best_slots = 0u;
  *th = *tw = 1u;
  for (uint32_t x = 1u; x <= max_px && x <= w; ++x)
    for (uint32_t y = 1u; y <= max_px / x && y <= h; ++y) {
      const uint32_t slots = stride == 1u ? (x + 2u) * (y + 2u) : (2u * x + 1u) * (2u * y + 1u);
      if (slots > max_slots || x + y > max_sides) break;
      const uint64_t tiles = (uint64_t)((h + y - 1u) / y) * ((w + x - 1u) / x);
      if (tiles < best_tiles || (tiles == best_tiles && slots < best_slots)) {
        best_tiles = tiles;
        best_slots = slots;
        *th = y;
        *tw = x;
      }
    }
}

bool shape_ok(uint32_t batch, uint32_t h, uint32_t w, uint32_t c_in, uint32_t c_out, uint32_t stride) {
  if (batch == 0u || h == 0u || w == 0u || c_in == 0u || c_out == 0u) return false;
  if (stride != 1u && stride != 2u) return false;
  if (h > 16384u || w > 16384u || c_in > 8192u || c_out > 8192u || batch > 65536u) return false;
  const uint64_t ho = (h - 1u) / stride + 1u, wo = (w - 1u) / stride + 1u;
  if ((uint64_t)batch * ho * wo > 0x7fffffffull) return false;
  if ((uint64_t)batch * h * w > 0x7fffffffull) return false;     // pixel indices are 32-bit
  return true;
}

// Which kernel a layer gets, and its launch shape.
//   stride 1, c_in % 64 == 0 and c_out % 8 == 0: the patch kernel, if its tiles (patch_tile) times
//     blocks of 64 channels make at least PT_MIN_TILES workgroups;
//   stride 2, c_in == 32, c_out % 8 == 0 and c_out <= 64: the kernel with the filter and the
//     tile's patch in LDS, if its tiles (at most 128 pixels, th + tw <= 30) make at least
//     S2_MIN_TILES workgroups;
//   else c_in % 32 == 0 and c_out % 8 == 0: DMA-ring kernel; 128 x 128 tiles (256 pixels x 64 channels
//     when c_out <= 64) if that gives at least one workgroup per CU, else 64 x 64 tiles: four
//     waves that split the depth when c_in % 64 == 0, one wave per workgroup otherwise;
//   c_in == 3, stride 1, c_out % 8 == 0, c_out <= 64: the first-layer kernel;
//   anything else: the register-staged kernel.
Geometry geometry(uint32_t batch, uint32_t h, uint32_t w, uint32_t c_in, uint32_t c_out, uint32_t stride,
                  bool allow_fast = true) {
  Geometry g;
  g.Ho = (h - 1u) / stride + 1u;
  g.Wo = (w - 1u) / stride + 1u;
  g.pixels = batch * g.Ho * g.Wo;
  g.threads = CV_THREADS;
  g.th = g.tw = g.tiles_y = g.tiles_x = 0u;
  if (allow_fast && stride == 1u && c_in % 64u == 0u && c_out % 8u == 0u) {
    patch_tile(h, w, 1u, 256u, PT_MAX_SLOTS, &g.th, &g.tw);
    g.tiles_y = (h + g.th - 1u) / g.th;
    g.tiles_x = (w + g.tw - 1u) / g.tw;
    const uint64_t total = (uint64_t)batch * g.tiles_y * g.tiles_x * ((c_out + 63u) / 64u);
    if (total >= PT_MIN_TILES && total <= 0x7fffffffull) {
      g.bn = 64u;
      g.tiles_n = (c_out + 63u) / 64u;
      g.total = (uint32_t)total;
      g.path = PATH_PATCH;
      g.blocks = (g.total + 7u) / 8u * 8u;
      return g;
    }
  }
  if (allow_fast && stride == 2u && c_in == 32u && c_out % 8u == 0u && c_out <= 64u) {
    patch_tile(g.Ho, g.Wo, 2u, 128u, S2_MAX_SLOTS, &g.th, &g.tw, S2_MAX_SIDES);
    g.tiles_y = (g.Ho + g.th - 1u) / g.th;
    g.tiles_x = (g.Wo + g.tw - 1u) / g.tw;
    const uint64_t total = (uint64_t)batch * g.tiles_y * g.tiles_x;
    if (total >= S2_MIN_TILES && total <= 0x7fffffffull) {
      g.bn = 64u;
      g.tiles_n = 1u;
      g.total = (uint32_t)total;
      g.path = PATH_S2C32;
      g.blocks = (g.total + 7u) / 8u * 8u;
      return g;
    }
  }
  if (allow_fast && c_in % 32u == 0u && c_out % 8u == 0u) {
    const uint32_t bmp = c_out > 64u ? 128u : 256u;
    g.bn = c_out > 64u ? 128u : 64u;
    g.tiles_n = (c_out + g.bn - 1u) / g.bn;
    g.total = ((g.pixels + bmp - 1u) / bmp) * g.tiles_n;
    g.path = c_out > 64u ? PATH_DMA_128x128 : PATH_DMA_256x64;
    if (g.total < 256u) {
      g.bn = 64u;
      g.tiles_n = (c_out + 63u) / 64u;
      g.total = ((g.pixels + 63u) / 64u) * g.tiles_n;
      g.path = c_in % 64u == 0u ? PATH_DMA_KSPLIT : PATH_DMA_64x64;
      g.threads = c_in % 64u == 0u ? 256u : 64u;
    }
  } else if (allow_fast && c_in == 3u && stride == 1u && c_out % 8u == 0u && c_out <= 64u) {
    g.bn = c_out;
    g.tiles_n = 1u;
    g.total = (g.pixels + C3_PIX - 1u) / C3_PIX;
    g.path = PATH_C3;
  } else {
    g.bn = c_out <= 64u ? 64u : 128u;
    g.tiles_n = (c_out + g.bn - 1u) / g.bn;
    g.total = ((g.pixels + CV_BM - 1u) / CV_BM) * g.tiles_n;
    g.path = PATH_GENERIC;
  }
  g.blocks = (g.total + 7u) / 8u * 8u;
  return g;
}

// A chain of layers: every layer's kernel and launch shape, and how many ways its depth is split
// across workgroups.  A depth-split layer of at most 96 tiles and c_in >= 512 (the second launch
// costs about 4 us, shallower layers do not win that back) is split further when its fp32
// partial sums fit the idle part of the ping-pong buffers: behind the layer's own bf16 output in
// its destination buffer, or, for the last layer (which writes to `out`), the buffer it does
// not read.  splits = min(16, 512 / tiles, depth tiles / 4, what fits); 1 if that is below 2.
struct LayerPlan {
  Geometry g;
  uint32_t splits;
  uint64_t work_off;     // byte offset of the partial sums in that buffer
  bool in_next;          // this layer is computed inside the next layer's kernel: no launch of its own
};

int plan_chain(const mgb_conv_layer* layers, uint32_t n_layers, uint32_t batch, uint32_t h, uint32_t w,
               bool allow_fast, LayerPlan* plan, uint64_t* weights, uint64_t* act_max, uint64_t* last) {
  *weights = 0; *act_max = 0; *last = 0;
  uint32_t ch = h, cw = w;
  for (uint32_t i = 0; i < n_layers; ++i) {
    const mgb_conv_layer& L = layers[i];
    if (i > 0u && L.c_in != layers[i - 1u].c_out) return MGB_E_INVAL;
    if (!shape_ok(batch, ch, cw, L.c_in, L.c_out, L.stride)) return MGB_E_UNSUPPORTED;
    plan[i].g = geometry(batch, ch, cw, L.c_in, L.c_out, L.stride, allow_fast);
    plan[i].splits = 1u;
    plan[i].work_off = 0u;
    plan[i].in_next = false;
    *weights += 9ull * L.c_in * L.c_out * 2;
    const uint64_t elems = (uint64_t)plan[i].g.pixels * L.c_out;
    if (i + 1u < n_layers) *act_max = *act_max > elems * 2 ? *act_max : elems * 2;
    else *last = elems * 4;
    ch = plan[i].g.Ho;
    cw = plan[i].g.Wo;
  }
  // The 3-channel first layer with 32 output channels in front of a layer that takes the
  // stride-2 kernel for 32 input channels is computed inside that kernel.
  for (uint32_t i = 0; i + 1u < n_layers; ++i)
    plan[i].in_next = plan[i].g.path == PATH_C3 && layers[i].c_out == 32u && plan[i + 1u].g.path == PATH_S2C32;
  for (uint32_t i = 0; i < n_layers; ++i) {
    Geometry& g = plan[i].g;
    if (g.path != PATH_DMA_KSPLIT || g.total > 96u || layers[i].c_in < 512u) continue;
    const uint64_t elems = (uint64_t)g.pixels * layers[i].c_out;
    const bool is_last = i + 1u == n_layers;
    const uint64_t own = is_last ? 0u : (elems * 2 + 255u) / 256u * 256u;
    const uint64_t spare = *act_max > own ? *act_max - own : 0u;
    uint64_t s = 512u / g.total;
    s = s < 16u ? s : 16u;
    const uint64_t nk = 9ull * layers[i].c_in / KS_BK;
    s = s < nk / 4u ? s : nk / 4u;
    s = s < spare / (elems * 4) ? s : spare / (elems * 4);
    if (s < 2u) continue;
    plan[i].splits = (uint32_t)s;
    plan[i].work_off = own;
    g.total *= (uint32_t)s;
    g.blocks = (g.total + 7u) / 8u * 8u;
  }
  return MGB_OK;
}

constexpr uint32_t MAX_LAYERS = 64;

// the depth-64 kernel when c_in allows it and `deep` says so, else the depth-32 kernel: both rings take the same LDS
template <uint32_t WM, uint32_t WN>
hipError_t launch_dma(hipStream_t st, const Geometry& g, const ConvArgs& a, bool deep = false) {
  constexpr uint32_t lds = CD_NST * (64u * WM + 64u * WN) * 64u;
  static_assert(lds == 2u * (64u * WM + 64u * WN) * 128u, "two stages of depth 64 = four of depth 32");
  static std::once_flag once;
  static hipError_t attr = hipSuccess;
  std::call_once(once, [] {
    attr = hipFuncSetAttribute((const void*)conv3x3_dma_kernel<WM, WN>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (attr == hipSuccess)
      attr = hipFuncSetAttribute((const void*)conv3x3_dma64_kernel<WM, WN>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  });
  if (attr != hipSuccess) return attr;
  // (the depth-64 kernel addresses its input with 32-bit offsets)
  const bool fits = (uint64_t)a.batch * a.H * a.W * a.C * 2u + ((uint64_t)a.W + 1u) * a.C * 2u < (1ull << 31);
  if (deep && a.C % 64u == 0u && fits)
    hipLaunchKernelGGL((conv3x3_dma64_kernel<WM, WN>), dim3(g.blocks), dim3(64u * WM * WN), lds, st, a);
  else
    hipLaunchKernelGGL((conv3x3_dma_kernel<WM, WN>), dim3(g.blocks), dim3(64u * WM * WN), lds, st, a);
  return hipSuccess;
}

// `splits` > 1 (depth-split path only): `work` holds splits * pixels * c_out floats
// `w_first`: the layer in front (3 channels -> 32, stride 1, reading `x`) is computed inside this
// layer's kernel; h, wd and c_in describe this layer's input as if it existed.
int launch_layer(hipStream_t st, const uint16_t* x, const uint16_t* w, void* y, uint32_t batch,
                 uint32_t h, uint32_t wd, uint32_t c_in, uint32_t c_out, uint32_t stride,
                 uint32_t out_f32, uint32_t splits = 1u, float* work = nullptr, const uint16_t* w_first = nullptr) {
  // the fast paths move 16 bytes at a time (the probe assumed aligned tensors)
  // (a fused first layer's 3-channel input is read two bytes at a time: any alignment will do)
  const bool aligned = (((w_first ? (uintptr_t)0 : (uintptr_t)x) | (uintptr_t)w | (uintptr_t)y | (uintptr_t)work) & 15u) == 0u;
  Geometry g = geometry(batch, h, wd, c_in, c_out, stride, aligned);
  if (w_first && g.path != PATH_S2C32) {
    mgb_internal_set_error_text("conv chain: a first layer planned into the second layer's kernel, which the second layer's tensors do not allow (alignment)");
    return MGB_E_INVAL;
  }
  if (splits > 1u && (g.path != PATH_DMA_KSPLIT || !work)) splits = 1u;
  g.total *= splits;
  g.blocks = (g.total + 7u) / 8u * 8u;
  ConvArgs a;
  a.x = x; a.w = w; a.y = y;
  a.batch = batch; a.H = h; a.W = wd; a.C = c_in; a.K = c_out; a.stride = stride;
  a.Ho = g.Ho; a.Wo = g.Wo; a.pixels = g.pixels; a.depth = 9u * c_in;
  a.tiles_n = g.tiles_n; a.tiles_total = g.total; a.out_f32 = out_f32;
  a.splits = splits; a.work = work;
  a.th = g.th; a.tw = g.tw; a.tiles_y = g.tiles_y; a.tiles_x = g.tiles_x;
  a.by_tiles_n = fast_div(g.tiles_n);
  a.by_plane = fast_div(g.Ho * g.Wo);
  a.by_wo = fast_div(g.Wo);
  a.by_tiles_x = fast_div(g.tiles_x ? g.tiles_x : 1u);
  a.by_tiles_y = fast_div(g.tiles_y ? g.tiles_y : 1u);
  a.by_pw = fast_div(g.path == PATH_S2C32 ? 2u * g.tw + 1u : g.tw + 2u);
  a.by_tw = fast_div(g.tw ? g.tw : 1u);
  a.w_first = w_first;
  a.by_iw = fast_div(2u * g.tw + 3u);
  hipError_t e = hipSuccess;
  switch (g.path) {
    case PATH_DMA_128x128: e = launch_dma<2, 2>(st, g, a, true); break;
    case PATH_DMA_256x64: e = launch_dma<4, 1>(st, g, a, true); break;
    case PATH_DMA_64x64: e = launch_dma<1, 1>(st, g, a); break;
    case PATH_DMA_KSPLIT: {
      static std::once_flag once;
      static hipError_t attr = hipSuccess;
      std::call_once(once, [] {
        attr = hipFuncSetAttribute((const void*)conv3x3_dma_ksplit_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)KS_LDS);
      });
      e = attr;
      if (e == hipSuccess) {
        hipLaunchKernelGGL(conv3x3_dma_ksplit_kernel, dim3(g.blocks), dim3(256), KS_LDS, st, a);
        if (splits > 1u) {
          const uint32_t quads = g.pixels * (c_out / 4u);
          hipLaunchKernelGGL(conv_split_reduce_kernel, dim3((quads + 255u) / 256u), dim3(256), 0, st, work, y, splits, quads, out_f32);
        }
      }
      break;
    }
    case PATH_PATCH: {
      static std::once_flag once;
      static hipError_t attr = hipSuccess;
      std::call_once(once, [] {
        attr = hipFuncSetAttribute((const void*)conv3x3_patch_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)PT_LDS);
      });
      e = attr;
      if (e == hipSuccess) hipLaunchKernelGGL(conv3x3_patch_kernel, dim3(g.blocks), dim3(256), PT_LDS, st, a);
      break;
    }
    case PATH_S2C32: {
      static std::once_flag once;
      static hipError_t attr = hipSuccess;
      std::call_once(once, [] {
        attr = hipFuncSetAttribute((const void*)conv3x3_s2c32_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)S2_LDS);
        if (attr == hipSuccess)
          attr = hipFuncSetAttribute((const void*)conv3x3_s2c32_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)S2_LDS_FUSED);
      });
      e = attr;
      if (e == hipSuccess) {
        if (w_first) hipLaunchKernelGGL(conv3x3_s2c32_kernel<true>, dim3(g.blocks), dim3(256), S2_LDS_FUSED, st, a);
        else hipLaunchKernelGGL(conv3x3_s2c32_kernel<false>, dim3(g.blocks), dim3(256), S2_LDS, st, a);
      }
      break;
    }
    case PATH_C3:
      if (c_out <= 32u) hipLaunchKernelGGL((conv3x3_c3_kernel<1>), dim3(g.blocks), dim3(CV_THREADS), 0, st, a);
      else hipLaunchKernelGGL((conv3x3_c3_kernel<2>), dim3(g.blocks), dim3(CV_THREADS), 0, st, a);
      break;
    case PATH_GENERIC: {
      const bool vec = c_in % 8u == 0u && (((uintptr_t)x | (uintptr_t)w) & 15u) == 0u;
      if (g.bn == 64u) {
        if (vec) hipLaunchKernelGGL((conv3x3_kernel<64, true>), dim3(g.blocks), dim3(CV_THREADS), 0, st, a);
        else hipLaunchKernelGGL((conv3x3_kernel<64, false>), dim3(g.blocks), dim3(CV_THREADS), 0, st, a);
      } else {
        if (vec) hipLaunchKernelGGL((conv3x3_kernel<128, true>), dim3(g.blocks), dim3(CV_THREADS), 0, st, a);
        else hipLaunchKernelGGL((conv3x3_kernel<128, false>), dim3(g.blocks), dim3(CV_THREADS), 0, st, a);
      }
      break;
    }
  }
  if (e != hipSuccess) {
    mgb_internal_set_error("conv3x3_dma_kernel: dynamic LDS size", e);
    return MGB_E_BACKEND;
  }
  return MGB_OK;
}

}  // namespace

extern "C" {

int mgb_conv3x3_probe(uint32_t batch, uint32_t h, uint32_t w, uint32_t c_in, uint32_t c_out,
                      uint32_t stride, uint64_t* mem_bytes, mgb_dim3* grid, mgb_dim3* block) {
  if (!mem_bytes || !grid || !block) return MGB_E_INVAL;
  if (!shape_ok(batch, h, w, c_in, c_out, stride)) return MGB_E_UNSUPPORTED;
  const Geometry g = geometry(batch, h, w, c_in, c_out, stride);
  *mem_bytes = ((uint64_t)batch * h * w * c_in + 9ull * c_in * c_out + (uint64_t)g.pixels * c_out) * 2;
  *grid = mgb_dim3{g.blocks, 1u, 1u};
  *block = mgb_dim3{g.threads, 1u, 1u};
  return MGB_OK;
}

// workgroups of a layer's kernel that fit one CU (LDS of the ring / the strips; registers of the
// register-staged kernel)
static uint32_t residency_of(const Geometry& g, uint32_t c_out) {
  switch (g.path) {
    case PATH_DMA_128x128: return 2u;                 // 64 KiB ring
    case PATH_DMA_256x64: return 2u;                  // 80 KiB ring
    case PATH_DMA_64x64: return 5u;                   // 32 KiB ring
    case PATH_DMA_KSPLIT: return 2u;                  // 64 KiB ring
    case PATH_C3: return c_out <= 32u ? 7u : 4u;      // 22 / 38 KiB of strips and output staging
    case PATH_GENERIC: return 2u;                     // 162 - 244 registers per lane
    case PATH_PATCH: return 2u;                       // 76 KiB of patch and weight ring
    case PATH_S2C32: return 2u;                       // 74.25 KiB of patch, filter and table
  }
  return 0u;
}

uint32_t mgb_conv3x3_residency(uint32_t batch, uint32_t h, uint32_t w, uint32_t c_in, uint32_t c_out,
                               uint32_t stride) {
  if (!shape_ok(batch, h, w, c_in, c_out, stride)) return 0u;
  return residency_of(geometry(batch, h, w, c_in, c_out, stride), c_out);
}

uint32_t mgb_cnn_residency(const mgb_conv_layer* layers, uint32_t n_layers, uint32_t batch, uint32_t h,
                           uint32_t w) {
  if (!layers || n_layers == 0u || n_layers > MAX_LAYERS) return 0u;
  LayerPlan plan[MAX_LAYERS];
  uint64_t weights, act_max, last;
  if (plan_chain(layers, n_layers, batch, h, w, true, plan, &weights, &act_max, &last) != MGB_OK) return 0u;
  uint32_t blocks = 0, threads = CV_THREADS, res = 0;
  for (uint32_t i = 0; i < n_layers; ++i) {
    const Geometry& g = plan[i].g;
    if (plan[i].in_next) continue;                     // no launch of its own
    if ((uint64_t)g.blocks * g.threads > (uint64_t)blocks * threads) {   // the launch that gives the task its geometry
      blocks = g.blocks;
      threads = g.threads;
      res = residency_of(g, layers[i].c_out);
    }
  }
  return res;
}

int mgb_conv3x3_enqueue(void* stream, const uint16_t* x, const uint16_t* w, void* y, uint32_t batch,
                        uint32_t h, uint32_t wd, uint32_t c_in, uint32_t c_out, uint32_t stride,
                        uint32_t out_f32) {
  if (!x || !w || !y) return MGB_E_INVAL;
  if (!shape_ok(batch, h, wd, c_in, c_out, stride)) return MGB_E_UNSUPPORTED;
  const int rc = launch_layer((hipStream_t)stream, x, w, y, batch, h, wd, c_in, c_out, stride, out_f32);
  if (rc != MGB_OK) return rc;
  return mgb_check_launch("conv3x3_kernel");
}

int mgb_cnn_probe(const mgb_conv_layer* layers, uint32_t n_layers, uint32_t batch, uint32_t h,
                  uint32_t w, uint64_t* mem_bytes, uint64_t* act_bytes, uint64_t* out_bytes,
                  mgb_dim3* grid, mgb_dim3* block) {
  if (!layers || !mem_bytes || !act_bytes || !out_bytes || !grid || !block || n_layers == 0u)
    return MGB_E_INVAL;
  if (n_layers > MAX_LAYERS) return MGB_E_UNSUPPORTED;
  LayerPlan plan[MAX_LAYERS];
  uint64_t weights, act_max, last;
  const int prc = plan_chain(layers, n_layers, batch, h, w, true, plan, &weights, &act_max, &last);
  if (prc != MGB_OK) return prc;
  uint32_t blocks = 0, threads = CV_THREADS;
  const uint64_t input = (uint64_t)batch * h * w * layers[0].c_in * 2;
  for (uint32_t i = 0; i < n_layers; ++i) {
    const Geometry& g = plan[i].g;
    if (plan[i].in_next) continue;                     // no launch of its own
    // launches are stream-ordered: the one with the most waves counts
    if ((uint64_t)g.blocks * g.threads > (uint64_t)blocks * threads) {
      blocks = g.blocks;
      threads = g.threads;
    }
  }
  *act_bytes = act_max;
  *out_bytes = last;
  *mem_bytes = input + weights + 2 * act_max + last;
  *grid = mgb_dim3{blocks, 1u, 1u};
  *block = mgb_dim3{threads, 1u, 1u};
  return MGB_OK;
}

int mgb_cnn_enqueue(void* stream, const mgb_conv_layer* layers, uint32_t n_layers,
                    const uint16_t* x, const uint16_t* const* weights, uint16_t* act0,
                    uint16_t* act1, float* out, uint32_t batch, uint32_t h, uint32_t w) {
  if (!layers || !x || !weights || !out || n_layers == 0u) return MGB_E_INVAL;
  if (n_layers > 1u && (!act0 || !act1 || act0 == act1)) return MGB_E_INVAL;
  uint64_t mem, act, ob;
  mgb_dim3 g, b;
  int rc = mgb_cnn_probe(layers, n_layers, batch, h, w, &mem, &act, &ob, &g, &b);
  if (rc != MGB_OK) return rc;
  for (uint32_t i = 0; i < n_layers; ++i)
    if (!weights[i]) return MGB_E_INVAL;
  LayerPlan plan[MAX_LAYERS];
  uint64_t wb, act_max, lb;
  rc = plan_chain(layers, n_layers, batch, h, w, true, plan, &wb, &act_max, &lb);
  if (rc != MGB_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  const uint16_t* src = x;
  const uint16_t* first_w = nullptr;       // the filter of a layer left to the next layer's kernel
  bool skipped = false;
  uint32_t ch = h, cw = w;
  for (uint32_t i = 0; i < n_layers; ++i) {
    const mgb_conv_layer& L = layers[i];
    const bool last = i + 1u == n_layers;
    uint16_t* pong = (i & 1u) ? act1 : act0;           // the buffer this layer does not read
    void* dst = last ? (void*)out : (void*)pong;
    float* work = plan[i].splits > 1u ? reinterpret_cast<float*>(reinterpret_cast<uint8_t*>(pong) + plan[i].work_off) : nullptr;
    // Planned into the next layer's kernel: that kernel moves 16 bytes at a time, so it takes the
    // two layers only if the next layer's filter and destination are aligned for it; otherwise
    // both run on their own.
    if (plan[i].in_next) {
      const bool next_last = i + 2u == n_layers;
      const void* next_dst = next_last ? (const void*)out : (const void*)(((i + 1u) & 1u) ? act1 : act0);
      skipped = (((uintptr_t)weights[i + 1u] | (uintptr_t)next_dst) & 15u) == 0u;
    } else {
      skipped = false;
    }
    if (skipped) {
      // nothing is launched and nothing written; the next layer reads `src` and writes its own destination
      first_w = weights[i];
    } else {
      rc = launch_layer(st, src, weights[i], dst, batch, ch, cw, L.c_in, L.c_out, L.stride, last ? 1u : 0u,
                        plan[i].splits, work, first_w);
      if (rc != MGB_OK) return rc;
      src = (const uint16_t*)dst;
      first_w = nullptr;
    }
    ch = (ch - 1u) / L.stride + 1u;
    cw = (cw - 1u) / L.stride + 1u;
  }
  return mgb_check_launch("conv3x3_kernel");
}

}  // extern "C"
