// 3x3 convolution + ReLU (padding 1, stride 1 or 2) as an implicit GEMM on the
// bf16 matrix cores, and a chain of such layers run as one task.
//
// GEMM view: rows = output pixels (n, oh, ow), columns = output channels,
// depth = (r, s, c) = 9 * c_in.  Activations are N,H,W,C and weights K,3,3,C,
// so for a fixed filter tap the channel run is contiguous for both operands:
// neither needs a transpose, the A tile is gathered straight from the input
// image (zeros outside it) into LDS, 8 channels per 16-byte load when c_in is
// a multiple of 8, element-wise otherwise (the 3-channel first layer).
// A workgroup of 4 waves (2 x 2) owns 128 pixels x BN channels, depth 64 per
// step.  The late layers of a small batch have only a handful of workgroups, so
// a step's memory latency cannot be hidden by other workgroups: the tiles of
// the next TWO steps are kept in flight in registers while the MFMAs of the
// current step run from LDS.
// Wide layers are MFMA-bound; the first layer and the small late layers of a
// small batch are bandwidth / latency bound.
#include "../../include/mgb.h"
#include "launch_util.h"

#include <hip/hip_runtime.h>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // one 16-byte chunk of 8 bf16

constexpr uint32_t CV_BM = 128, CV_THREADS = 256;

struct ConvArgs {
  const uint16_t* x;
  const uint16_t* w;
  void* y;
  uint32_t batch, H, W, C, K, stride, Ho, Wo;
  uint32_t pixels, depth;      // batch*Ho*Wo, 9*C
  uint32_t tiles_n, tiles_total, out_f32;
};

// 16 bytes of zeros in device memory: the source of every padded / out-of-range operand chunk
__device__ __attribute__((aligned(16))) uint32_t g_zero16[4];

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t w = __float_as_uint(f);
  return (uint16_t)((w + 0x7fffu + ((w >> 16) & 1u)) >> 16);
}

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 q) { return __builtin_bit_cast(bf16x8, q); }

// p if ok (0 or 1) else z, by integer arithmetic: the compiler cannot turn it into a branch
__device__ __forceinline__ const uint16_t* pick(const uint16_t* p, const uint16_t* z, uint32_t ok) {
  const uintptr_t pz = (uintptr_t)z;
  return (const uint16_t*)(pz + (((uintptr_t)p - pz) & (uintptr_t)(0 - (int64_t)ok)));
}

// VEC (c_in % 8 == 0) runs depth 64 per step; the element-wise path (3-channel first layer,
// total depth 27) runs depth 32 per step.
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
    const uint32_t b = pp / (a.Ho * a.Wo);
    const uint32_t rem = pp - b * a.Ho * a.Wo;
    const uint32_t oh = rem / a.Wo, ow = rem - oh * a.Wo;
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

struct Geometry {
  uint32_t Ho, Wo, pixels, bn, tiles_n, total, blocks;
};

bool shape_ok(uint32_t batch, uint32_t h, uint32_t w, uint32_t c_in, uint32_t c_out, uint32_t stride) {
  if (batch == 0u || h == 0u || w == 0u || c_in == 0u || c_out == 0u) return false;
  if (stride != 1u && stride != 2u) return false;
  if (h > 16384u || w > 16384u || c_in > 8192u || c_out > 8192u || batch > 65536u) return false;
  const uint64_t ho = (h - 1u) / stride + 1u, wo = (w - 1u) / stride + 1u;
  if ((uint64_t)batch * ho * wo > 0x7fffffffull) return false;
  if ((uint64_t)batch * h * w > 0x7fffffffull) return false;     // pixel indices are 32-bit
  return true;
}

Geometry geometry(uint32_t batch, uint32_t h, uint32_t w, uint32_t c_out, uint32_t stride) {
  Geometry g;
  g.Ho = (h - 1u) / stride + 1u;
  g.Wo = (w - 1u) / stride + 1u;
  g.pixels = batch * g.Ho * g.Wo;
  g.bn = c_out <= 64u ? 64u : 128u;
  g.tiles_n = (c_out + g.bn - 1u) / g.bn;
  g.total = ((g.pixels + CV_BM - 1u) / CV_BM) * g.tiles_n;
  g.blocks = (g.total + 7u) / 8u * 8u;
  return g;
}

int launch_layer(hipStream_t st, const uint16_t* x, const uint16_t* w, void* y, uint32_t batch,
                 uint32_t h, uint32_t wd, uint32_t c_in, uint32_t c_out, uint32_t stride,
                 uint32_t out_f32) {
  const Geometry g = geometry(batch, h, wd, c_out, stride);
  ConvArgs a;
  a.x = x; a.w = w; a.y = y;
  a.batch = batch; a.H = h; a.W = wd; a.C = c_in; a.K = c_out; a.stride = stride;
  a.Ho = g.Ho; a.Wo = g.Wo; a.pixels = g.pixels; a.depth = 9u * c_in;
  a.tiles_n = g.tiles_n; a.tiles_total = g.total; a.out_f32 = out_f32;
  const bool vec = c_in % 8u == 0u && (((uintptr_t)x | (uintptr_t)w) & 15u) == 0u;
  if (g.bn == 64u) {
    if (vec) hipLaunchKernelGGL((conv3x3_kernel<64, true>), dim3(g.blocks), dim3(CV_THREADS), 0, st, a);
    else hipLaunchKernelGGL((conv3x3_kernel<64, false>), dim3(g.blocks), dim3(CV_THREADS), 0, st, a);
  } else {
    if (vec) hipLaunchKernelGGL((conv3x3_kernel<128, true>), dim3(g.blocks), dim3(CV_THREADS), 0, st, a);
    else hipLaunchKernelGGL((conv3x3_kernel<128, false>), dim3(g.blocks), dim3(CV_THREADS), 0, st, a);
  }
  return MGB_OK;
}

}  // namespace

extern "C" {

int mgb_conv3x3_probe(uint32_t batch, uint32_t h, uint32_t w, uint32_t c_in, uint32_t c_out,
                      uint32_t stride, uint64_t* mem_bytes, mgb_dim3* grid, mgb_dim3* block) {
  if (!mem_bytes || !grid || !block) return MGB_E_INVAL;
  if (!shape_ok(batch, h, w, c_in, c_out, stride)) return MGB_E_UNSUPPORTED;
  const Geometry g = geometry(batch, h, w, c_out, stride);
  *mem_bytes = ((uint64_t)batch * h * w * c_in + 9ull * c_in * c_out + (uint64_t)g.pixels * c_out) * 2;
  *grid = mgb_dim3{g.blocks, 1u, 1u};
  *block = mgb_dim3{CV_THREADS, 1u, 1u};
  return MGB_OK;
}

int mgb_conv3x3_enqueue(void* stream, const uint16_t* x, const uint16_t* w, void* y, uint32_t batch,
                        uint32_t h, uint32_t wd, uint32_t c_in, uint32_t c_out, uint32_t stride,
                        uint32_t out_f32) {
  if (!x || !w || !y) return MGB_E_INVAL;
  if (!shape_ok(batch, h, wd, c_in, c_out, stride)) return MGB_E_UNSUPPORTED;
  launch_layer((hipStream_t)stream, x, w, y, batch, h, wd, c_in, c_out, stride, out_f32);
  return mgb_check_launch("conv3x3_kernel");
}

int mgb_cnn_probe(const mgb_conv_layer* layers, uint32_t n_layers, uint32_t batch, uint32_t h,
                  uint32_t w, uint64_t* mem_bytes, uint64_t* act_bytes, uint64_t* out_bytes,
                  mgb_dim3* grid, mgb_dim3* block) {
  if (!layers || !mem_bytes || !act_bytes || !out_bytes || !grid || !block || n_layers == 0u)
    return MGB_E_INVAL;
  uint64_t weights = 0, act_max = 0, last = 0;
  uint32_t blocks = 0, ch = h, cw = w;
  const uint64_t input = (uint64_t)batch * h * w * layers[0].c_in * 2;
  for (uint32_t i = 0; i < n_layers; ++i) {
    const mgb_conv_layer& L = layers[i];
    if (i > 0u && L.c_in != layers[i - 1u].c_out) return MGB_E_INVAL;
    if (!shape_ok(batch, ch, cw, L.c_in, L.c_out, L.stride)) return MGB_E_UNSUPPORTED;
    const Geometry g = geometry(batch, ch, cw, L.c_out, L.stride);
    weights += 9ull * L.c_in * L.c_out * 2;
    const uint64_t elems = (uint64_t)g.pixels * L.c_out;
    if (i + 1u < n_layers) act_max = act_max > elems * 2 ? act_max : elems * 2;
    else last = elems * 4;
    blocks = blocks > g.blocks ? blocks : g.blocks;   // launches are stream-ordered: the largest counts
    ch = g.Ho;
    cw = g.Wo;
  }
  *act_bytes = act_max;
  *out_bytes = last;
  *mem_bytes = input + weights + 2 * act_max + last;
  *grid = mgb_dim3{blocks, 1u, 1u};
  *block = mgb_dim3{CV_THREADS, 1u, 1u};
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
  hipStream_t st = (hipStream_t)stream;
  const uint16_t* src = x;
  uint32_t ch = h, cw = w;
  for (uint32_t i = 0; i < n_layers; ++i) {
    const mgb_conv_layer& L = layers[i];
    const bool last = i + 1u == n_layers;
    void* dst = last ? (void*)out : (void*)((i & 1u) ? act1 : act0);
    launch_layer(st, src, weights[i], dst, batch, ch, cw, L.c_in, L.c_out, L.stride, last ? 1u : 0u);
    src = (const uint16_t*)dst;
    ch = (ch - 1u) / L.stride + 1u;
    cw = (cw - 1u) / L.stride + 1u;
  }
  return mgb_check_launch("conv3x3_kernel");
}

}  // extern "C"
