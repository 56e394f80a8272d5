// 3x3 convolution + ReLU (padding 1, stride 1 or 2) as an implicit GEMM on the
// bf16 matrix cores, and a chain of such layers run as one task.
//
// GEMM view: rows = output pixels (n, oh, ow), columns = output channels,
// depth = (r, s, c) = 9 * c_in.  Activations are N,H,W,C and weights K,3,3,C,
// so for a fixed filter tap the channel run is contiguous for both operands:
// neither needs a transpose, the A tile is gathered straight from the input
// image (zeros outside it) into LDS, 8 channels per 16-byte load when c_in is
// a multiple of 8, element-wise otherwise (the 3-channel first layer).
// A workgroup of 4 waves owns 128 pixels x BN channels; a wave owns 32 pixels.
// Wide layers are MFMA-bound; the first layer and the small late layers of a
// small batch are bandwidth / launch bound.
#include "../../include/mgb.h"
#include "launch_util.h"

#include <hip/hip_runtime.h>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr uint32_t CV_BM = 128, CV_BK = 32, CV_THREADS = 256;
constexpr uint32_t CV_LD = CV_BK + 8;

union Frag {
  uint4 q;
  uint16_t h[8];
  bf16x8 v;
};

struct ConvArgs {
  const uint16_t* x;
  const uint16_t* w;
  void* y;
  uint32_t batch, H, W, C, K, stride, Ho, Wo;
  uint32_t pixels, depth;      // batch*Ho*Wo, 9*C
  uint32_t tiles_n, tiles_total, out_f32;
};

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t w = __float_as_uint(f);
  return (uint16_t)((w + 0x7fffu + ((w >> 16) & 1u)) >> 16);
}

template <uint32_t BN, bool VEC>
__global__ __launch_bounds__(CV_THREADS) void conv3x3_kernel(ConvArgs a) {
  __shared__ __attribute__((aligned(16))) uint16_t As[2][CV_BM][CV_LD];   // [pixel][k]
  __shared__ __attribute__((aligned(16))) uint16_t Bs[2][BN][CV_LD];      // [channel][k]
  constexpr uint32_t NT = BN / 32u;          // MFMA blocks per wave along the channels
  constexpr uint32_t BCH = BN * 4u / CV_THREADS;   // weight chunks per thread

  const uint32_t per_xcd = (a.tiles_total + 7u) / 8u;
  const uint32_t tile = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
  if ((blockIdx.x >> 3) >= per_xcd || tile >= a.tiles_total) return;
  const uint32_t bm = (tile / a.tiles_n) * CV_BM;
  const uint32_t bn = (tile % a.tiles_n) * BN;

  const uint32_t tid = threadIdx.x;
  const uint32_t lane = tid & 63u, wave = tid >> 6;
  const uint32_t l32 = lane & 31u, lhi = lane >> 5;
  const uint32_t a_row = tid >> 2, ch = tid & 3u;

  // the two pixels this thread gathers for
  int32_t ih0[2], iw0[2];
  size_t img[2];
  bool pv[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const uint32_t p = bm + a_row + 64u * h;
    pv[h] = p < a.pixels;
    const uint32_t pp = pv[h] ? p : 0u;
    const uint32_t b = pp / (a.Ho * a.Wo);
    const uint32_t rem = pp - b * a.Ho * a.Wo;
    const uint32_t oh = rem / a.Wo, ow = rem - oh * a.Wo;
    ih0[h] = (int32_t)(oh * a.stride) - 1;
    iw0[h] = (int32_t)(ow * a.stride) - 1;
    img[h] = (size_t)b * a.H * a.W * a.C;
  }

  Frag ra[2], rb[BCH];
  auto load_tiles = [&](uint32_t k0) {
    const uint32_t k = k0 + 8u * ch;
    if (VEC) {
      // the 8 k-values share one filter tap
      const uint32_t tap = k / a.C, c = k - tap * a.C;
      const int32_t r = (int32_t)(tap / 3u), s = (int32_t)(tap - 3u * (tap / 3u));
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int32_t ih = ih0[h] + r, iw = iw0[h] + s;
        const bool ok = pv[h] && k < a.depth && ih >= 0 && iw >= 0 && ih < (int32_t)a.H && iw < (int32_t)a.W;
        ra[h].q = ok ? *reinterpret_cast<const uint4*>(a.x + img[h] + ((size_t)ih * a.W + iw) * a.C + c)
                     : make_uint4(0, 0, 0, 0);
      }
    } else {
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const uint32_t kk = k + i;
          const uint32_t tap = kk / a.C, c = kk - tap * a.C;
          const int32_t r = (int32_t)(tap / 3u), s = (int32_t)(tap - 3u * (tap / 3u));
          const int32_t ih = ih0[h] + r, iw = iw0[h] + s;
          const bool ok = pv[h] && kk < a.depth && ih >= 0 && iw >= 0 && ih < (int32_t)a.H && iw < (int32_t)a.W;
          ra[h].h[i] = ok ? a.x[img[h] + ((size_t)ih * a.W + iw) * a.C + c] : (uint16_t)0;
        }
    }
#pragma unroll
    for (uint32_t j = 0; j < BCH; ++j) {
      const uint32_t idx = tid + CV_THREADS * j;
      const uint32_t n = bn + (idx >> 2);
      const uint32_t kb = k0 + 8u * (idx & 3u);
      if (VEC) {
        rb[j].q = (n < a.K && kb < a.depth) ? *reinterpret_cast<const uint4*>(a.w + (size_t)n * a.depth + kb)
                                           : make_uint4(0, 0, 0, 0);
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i)
          rb[j].h[i] = (n < a.K && kb + i < a.depth) ? a.w[(size_t)n * a.depth + kb + i] : (uint16_t)0;
      }
    }
  };
  auto store_tiles = [&](uint32_t buf) {
#pragma unroll
    for (int h = 0; h < 2; ++h)
      *reinterpret_cast<uint4*>(&As[buf][a_row + 64u * h][8u * ch]) = ra[h].q;
#pragma unroll
    for (uint32_t j = 0; j < BCH; ++j) {
      const uint32_t idx = tid + CV_THREADS * j;
      *reinterpret_cast<uint4*>(&Bs[buf][idx >> 2][8u * (idx & 3u)]) = rb[j].q;
    }
  };

  f32x16 acc[NT];
#pragma unroll
  for (uint32_t j = 0; j < NT; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;

  const uint32_t nk = (a.depth + CV_BK - 1u) / CV_BK;
  load_tiles(0);
  store_tiles(0);
  __syncthreads();
  for (uint32_t kt = 0; kt < nk; ++kt) {
    const uint32_t buf = kt & 1u;
    if (kt + 1u < nk) load_tiles((kt + 1u) * CV_BK);
#pragma unroll
    for (uint32_t ks = 0; ks < CV_BK; ks += 16u) {
      Frag fa;
      fa.q = *reinterpret_cast<const uint4*>(&As[buf][32u * wave + l32][ks + 8u * lhi]);
#pragma unroll
      for (uint32_t j = 0; j < NT; ++j) {
        Frag fb;
        fb.q = *reinterpret_cast<const uint4*>(&Bs[buf][32u * j + l32][ks + 8u * lhi]);
        acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa.v, fb.v, acc[j], 0, 0, 0);
      }
    }
    if (kt + 1u < nk) store_tiles(buf ^ 1u);
    __syncthreads();
  }

  // ReLU, then bf16 (nearest even) or fp32
#pragma unroll
  for (uint32_t j = 0; j < NT; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const uint32_t p = bm + 32u * wave + 8u * (r >> 2) + 4u * lhi + (r & 3);
      const uint32_t col = bn + 32u * j + l32;
      if (p < a.pixels && col < a.K) {
        const float v = fmaxf(acc[j][r], 0.f);
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
  if ((uint64_t)batch * h * w * c_in > 0xffffffffull * 16ull) return false;
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
