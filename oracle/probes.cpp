// CPU checker for the requirement derivation -- TEST INFRASTRUCTURE ONLY.
//
// A task's probe carries the sum of its device allocations and the geometry
// of its kernel launches (paper Sec. III-A: requirements are read off the
// task's allocation and launch operations; a task with several launches on
// shared buffers is one task, Algorithm 1).  The functions below recompute
// those figures from the published tiling rules of each task kind, written
// out independently of the GPU library.
#include <algorithm>
#include <cstdint>
#include <vector>

namespace {
uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }
// launches are padded to whole rounds over the 8 XCDs
uint64_t round8(uint64_t x) { return ceil_div(x, 8) * 8; }
}  // namespace

extern "C" {

// out = {mem_bytes, grid_x, grid_y, grid_z, block_x, block_y, block_z}

// Jacobi n x n: two fp32 grids.  n % 4 != 0: one column per thread, 256 columns x 8 rows per
// workgroup, one sweep per launch.  n % 4 == 0: sweeps are fused, up to 4 per launch (up to 8
// from n = 2048 on), planned in chunks of 128 sweeps: the fewest launches whose number has the
// parity of the chunk, the sweeps spread evenly over them.  A launch of t <= 4 sweeps: a wave takes a window of 256 columns x 8 output
// rows, windows step by 248 columns (4 stale columns on each side of a window, none next to the
// grid's own boundary).  A launch of t > 4 sweeps: a wave
// takes a strip of 256 columns stepping by 240 (8 stale columns per side) and runs of 40 output
// rows (fewer or more on grids that give less than four rounds of 2048 waves, see below).  Four waves per 256-thread workgroup, grids rounded up to a multiple of 8.  One probe
// covers all launches of the task: its grid is the largest of them.
static uint64_t jacobi_blocks(uint64_t n, uint64_t t) {
  uint64_t halo = t > 4 ? 8 : 4, rows = t > 4 ? 40 : 8;
  // windows start every 256 - 2 * halo columns; the last one is the first that reaches column n - 1
  uint64_t win_c = n <= 256 ? 1 : 1 + ceil_div(n - 256, 256 - 2 * halo);
  if (t > 4) {
    // runs of 40 rows, unless that gives fewer than 4 x 2048 waves: then as many runs per strip
    // as make the waves a whole number (the nearest, at least one) of rounds of 2048
    uint64_t waves = win_c * ceil_div(n - 2, 40);
    if (waves < 4 * 2048) {
      uint64_t rounds = std::max<uint64_t>(1, (waves + 1024) / 2048);
      uint64_t runs = std::max<uint64_t>(1, rounds * 2048 / win_c);
      rows = ceil_div(n - 2, runs);
    }
  }
  uint64_t win_r = ceil_div(n - 2, rows);
  return round8(ceil_div(win_c * win_r, 4));
}
static uint64_t jacobi_chunk_blocks(uint64_t n, uint64_t sweeps, uint64_t maxt) {
  uint64_t launches = ceil_div(sweeps, maxt);
  if (launches % 2 != sweeps % 2) ++launches;
  // the launches get floor(sweeps / launches) sweeps, some of them one more
  uint64_t lo = sweeps / launches, hi = lo + (sweeps % launches != 0 ? 1 : 0);
  return std::max(jacobi_blocks(n, lo), jacobi_blocks(n, hi));
}
void orc_jacobi_probe(uint64_t n, uint64_t iters, uint64_t out[7]) {
  uint64_t wg;
  if (n % 4 != 0) {
    wg = round8(ceil_div(n, 256) * ceil_div(n - 2, 8));
  } else if (iters == 0) {
    wg = jacobi_blocks(n, 4);
  } else {
    uint64_t maxt = n >= 2048 ? 8 : 4;
    wg = jacobi_chunk_blocks(n, iters > 128 ? 128 : iters, maxt);
    if (iters > 128 && iters % 128 != 0) wg = std::max(wg, jacobi_chunk_blocks(n, iters % 128, maxt));
  }
  out[0] = 2 * n * n * 4;
  out[1] = wg; out[2] = 1; out[3] = 1;
  out[4] = 256; out[5] = 1; out[6] = 1;
}
// Workgroups per CU: the window kernels need up to 168 registers per lane (three waves per SIMD),
// the streaming kernels used from 2048 columns on up to 224 (two); the one-sweep kernel is limited
// by the 32 wave slots (8 workgroups of 4 waves).
uint64_t orc_jacobi_residency(uint64_t n) { return n % 4 != 0 ? 8 : (n >= 2048 ? 2 : 3); }

// fp32 GEMM: A, B, C in fp32.  When k is a multiple of 16 and n a multiple of 4 the tile is
// 256 x 256 (256 threads), 128 x 128 (512 threads) or 64 x 64 (256 threads), whichever the
// library's estimate finishes first: a CU works ceil(tiles / 256) tiles off, each taking its area
// over the rate of that tile (153, 150, 143 TFLOP/s; 128 for the small tile when k > 5632), i.e.
// the least ceil(tiles / 256) * tile^2 * (100000 / rate), the larger tile on a tie.  Otherwise
// 128 x 128 with 512 threads.
static uint64_t f32_tile(uint64_t m, uint64_t n, uint64_t k) {
  if (k % 16 != 0 || n % 4 != 0) return 128;
  const uint64_t tile[3] = {256, 128, 64}, inv_rate[3] = {100000ull / 153, 100000ull / 150, 100000ull / (k <= 5632 ? 143 : 128)};
  uint64_t best = 256, best_cost = ~0ull;
  for (int i = 0; i < 3; ++i) {
    uint64_t cost = ceil_div(ceil_div(m, tile[i]) * ceil_div(n, tile[i]), 256) * tile[i] * tile[i] * inv_rate[i];
    if (cost < best_cost) { best_cost = cost; best = tile[i]; }
  }
  return best;
}
void orc_gemm_f32_probe(uint64_t m, uint64_t n, uint64_t k, uint64_t out[7]) {
  out[0] = (m * k + k * n + m * n) * 4;
  uint64_t t = f32_tile(m, n, k);
  out[1] = round8(ceil_div(m, t) * ceil_div(n, t)); out[2] = 1; out[3] = 1;
  out[4] = t == 128 ? 512 : 256; out[5] = 1; out[6] = 1;
}

// bf16 GEMM: bf16 A and B, fp32 C.  When k is a multiple of 32 and n a multiple of 8: one
// 256-thread workgroup per 256 x 256 tile of C, or per 128 x 128 tile if there would be fewer than
// 128 of the big ones; otherwise per 128 x 256 tile.
void orc_gemm_bf16_probe(uint64_t m, uint64_t n, uint64_t k, uint64_t out[7]) {
  out[0] = (m * k + k * n) * 2 + m * n * 4;
  uint64_t wgs;
  if (k % 32 == 0 && n % 8 == 0) {
    wgs = ceil_div(m, 256) * ceil_div(n, 256);
    if (wgs < 128) wgs = ceil_div(m, 128) * ceil_div(n, 128);
  } else {
    wgs = ceil_div(m, 128) * ceil_div(n, 256);
  }
  out[1] = round8(wgs); out[2] = 1; out[3] = 1;
  out[4] = 256; out[5] = 1; out[6] = 1;
}

// One 3x3 conv layer (pad 1): bf16 input, weights and output.  Workgroup shape by layer:
//   stride 1, c_in % 64 == 0 and c_out % 8 == 0: 256 threads per tile of one image's output and
//     64 channels, if that gives at least 128 workgroups.  A tile is th x tw output pixels with
//     th * tw <= 256 whose input patch of (th + 2) x (tw + 2) pixels is at most 352 pixels (44 KiB
//     of LDS at 64 channels); the image is cut into the fewest such tiles;
//   stride 2, c_in == 32, c_out % 8 == 0 and c_out <= 64: 256 threads per tile of one image's output
//     (all channels), if that gives at least 256 workgroups.  A tile is th x tw output pixels with
//     th * tw <= 128 and th + tw <= 30 whose input patch of (2 th + 1) x (2 tw + 1) pixels is at most
//     576 pixels (36 KiB of LDS at 32 channels); the image is cut into the fewest such tiles;
//   else c_in % 32 == 0 and c_out % 8 == 0: 256 threads per 128 pixels x 128 channels (256 x 64 when
//     c_out <= 64); if that gives fewer than 256 workgroups, 64 x 64 tiles instead, with 256
//     threads (the depth split four ways) when c_in % 64 == 0, else 64 threads;
//   c_in == 3, stride 1, c_out % 8 == 0, c_out <= 64: 256 threads per 256 pixels (all channels);
//   otherwise 256 threads per 128 pixels x 64 channels (128 channels when c_out > 64).
static uint64_t patch_tiles_per_image(uint64_t h, uint64_t w, uint64_t stride) {
  const uint64_t max_px = stride == 1 ? 256 : 128, max_patch = stride == 1 ? 352 : 576;
  uint64_t best = ~0ull;
  for (uint64_t ny = 1; ny <= h; ++ny) {                 // ny rows of tiles, each ceil(h / ny) pixels high
    const uint64_t th = ceil_div(h, ny);
    if (th > max_px) continue;
    for (uint64_t nx = 1; nx <= w && ny * nx < best; ++nx) {
      const uint64_t tw = ceil_div(w, nx);
      const uint64_t patch = stride == 1 ? (th + 2) * (tw + 2) : (2 * th + 1) * (2 * tw + 1);
      if (th * tw <= max_px && patch <= max_patch && (stride == 1 || th + tw <= 30)) { best = ny * nx; break; }
    }
  }
  return best;
}

static bool conv_patch_path(uint64_t batch, uint64_t ho, uint64_t wo, uint64_t c_in, uint64_t c_out, uint64_t stride,
                            uint64_t* wgs) {
  if (stride != 1 || c_in % 64 != 0 || c_out % 8 != 0) return false;
  *wgs = batch * patch_tiles_per_image(ho, wo, 1) * ceil_div(c_out, 64);
  return *wgs >= 128;
}

static bool conv_stride2_32_path(uint64_t batch, uint64_t ho, uint64_t wo, uint64_t c_in, uint64_t c_out, uint64_t stride,
                                 uint64_t* wgs) {
  if (stride != 2 || c_in != 32 || c_out % 8 != 0 || c_out > 64) return false;
  *wgs = batch * patch_tiles_per_image(ho, wo, 2);
  return *wgs >= 256;
}

static uint64_t conv_workgroups(uint64_t batch, uint64_t ho, uint64_t wo, uint64_t c_in, uint64_t c_out, uint64_t stride,
                                uint64_t* threads, bool* depth_split) {
  const uint64_t pixels = batch * ho * wo;
  uint64_t wgs;
  *threads = 256;
  *depth_split = false;
  if (conv_patch_path(batch, ho, wo, c_in, c_out, stride, &wgs)) return wgs;
  if (conv_stride2_32_path(batch, ho, wo, c_in, c_out, stride, &wgs)) return wgs;
  if (c_in % 32 == 0 && c_out % 8 == 0) {
    wgs = c_out > 64 ? ceil_div(pixels, 128) * ceil_div(c_out, 128) : ceil_div(pixels, 256) * ceil_div(c_out, 64);
    if (wgs < 256) {
      wgs = ceil_div(pixels, 64) * ceil_div(c_out, 64);
      *depth_split = c_in % 64 == 0;
      *threads = *depth_split ? 256 : 64;
    }
  } else if (c_in == 3 && stride == 1 && c_out % 8 == 0 && c_out <= 64) {
    wgs = ceil_div(pixels, 256);
  } else {
    wgs = ceil_div(pixels, 128) * ceil_div(c_out, c_out <= 64 ? 64 : 128);
  }
  return wgs;
}

void orc_conv3x3_probe(uint64_t batch, uint64_t h, uint64_t w, uint64_t c_in, uint64_t c_out,
                       uint64_t stride, uint64_t out[7]) {
  uint64_t ho = (h + 2 - 3) / stride + 1, wo = (w + 2 - 3) / stride + 1;
  uint64_t pixels = batch * ho * wo;
  out[0] = (batch * h * w * c_in + 9 * c_in * c_out + pixels * c_out) * 2;
  uint64_t threads;
  bool split;
  uint64_t wgs = conv_workgroups(batch, ho, wo, c_in, c_out, stride, &threads, &split);
  out[1] = round8(wgs); out[2] = 1; out[3] = 1;
  out[4] = threads; out[5] = 1; out[6] = 1;
}

// A chain of conv layers run as one task (launches that share buffers are merged into one
// task): footprint = bf16 input + all weights + two ping-pong buffers of the largest
// intermediate activation + the fp32 output of the last layer; geometry = the launch with the
// most threads.
// c[3*i..3*i+2] = {c_in, c_out, stride} of layer i.
//
// A first layer of 3 -> 32 channels at stride 1 in front of a layer that takes the stride-2 kernel for
// 32 input channels has no launch of its own (that kernel computes it on the fly).
//
// Inside a chain a depth-split layer of at most 96 tiles with c_in >= 512 is split further, over
// min(16, 512 / tiles, (9 c_in / 64) / 4) workgroups per tile, as far as the fp32 partial sums fit the
// idle part of a ping-pong buffer (behind the layer's own output rounded up to 256 bytes; the
// whole buffer for the last layer); fewer than 2 means no further split.
void orc_cnn_probe(const uint64_t* c, uint64_t n_layers, uint64_t batch, uint64_t h, uint64_t w,
                   uint64_t out[7]) {
  uint64_t mem = batch * h * w * c[0] * 2, act_max = 0, grid = 0, threads = 256, last = 0;
  uint64_t hh = h, ww = w;
  for (uint64_t i = 0; i < n_layers; ++i) {
    uint64_t ho = (hh - 1) / c[3 * i + 2] + 1, wo = (ww - 1) / c[3 * i + 2] + 1;
    uint64_t elems = batch * ho * wo * c[3 * i + 1];
    mem += 9 * c[3 * i] * c[3 * i + 1] * 2;
    if (i + 1 < n_layers) { if (elems * 2 > act_max) act_max = elems * 2; }
    else last = elems * 4;
    hh = ho; ww = wo;
  }
  hh = h; ww = w;
  for (uint64_t i = 0; i < n_layers; ++i) {
    uint64_t c_in = c[3 * i], c_out = c[3 * i + 1], stride = c[3 * i + 2];
    uint64_t ho = (hh - 1) / stride + 1, wo = (ww - 1) / stride + 1;
    uint64_t pixels = batch * ho * wo, elems = pixels * c_out, th;
    bool split;
    uint64_t wgs = conv_workgroups(batch, ho, wo, c_in, c_out, stride, &th, &split);
    if (c_in == 3 && c_out == 32 && stride == 1 && i + 1 < n_layers) {
      uint64_t s2 = c[3 * i + 5], ho2 = (ho - 1) / s2 + 1, wo2 = (wo - 1) / s2 + 1, next_wgs;
      if (conv_stride2_32_path(batch, ho2, wo2, c[3 * i + 3], c[3 * i + 4], s2, &next_wgs)) { hh = ho; ww = wo; continue; }
    }
    if (split && wgs <= 96 && c_in >= 512) {
      uint64_t own = i + 1 < n_layers ? ceil_div(elems * 2, 256) * 256 : 0;
      uint64_t spare = act_max > own ? act_max - own : 0;
      uint64_t ways = 512 / wgs;
      if (ways > 16) ways = 16;
      if (ways > 9 * c_in / 64 / 4) ways = 9 * c_in / 64 / 4;
      if (ways > spare / (elems * 4)) ways = spare / (elems * 4);
      if (ways >= 2) wgs *= ways;
    }
    if (round8(wgs) * th > grid * threads) { grid = round8(wgs); threads = th; }
    hh = ho; ww = wo;
  }
  out[0] = mem + 2 * act_max + last;
  out[1] = grid; out[2] = 1; out[3] = 1;
  out[4] = threads; out[5] = 1; out[6] = 1;
}

// Workgroups per CU that each kernel's own resources allow (what the probe adds to grid and block).
// A CU has 160 KiB of LDS, 4 SIMDs of 512 registers per lane, 32 wave slots.
//   fp32 GEMM: the DMA kernels keep a four-stage ring of (tile_m + tile_n) x 16 floats; the
//   register-staged one is limited by its 8 waves per workgroup.
uint64_t orc_gemm_f32_residency(uint64_t m, uint64_t n, uint64_t k) {
  if (k % 16 == 0 && n % 4 == 0) {
    uint64_t tile = f32_tile(m, n, k);
    return (160 * 1024) / (4 * (tile + tile) * 16 * 4);
  }
  return 32 / 8;
}
//   bf16 GEMM: ring of (tile_m + tile_n) x 32 bf16 x 4 stages, or (k % 64 == 0) three stages of
//   tile_m x 64 for A beside the four of 32 x tile_n for B; the 256 x 256 kernel also needs all
//   512 registers of a lane; the register-staged kernel 207 registers (2 waves per SIMD, 4-wave groups).
uint64_t orc_gemm_bf16_residency(uint64_t m, uint64_t n, uint64_t k) {
  if (k % 32 == 0 && n % 8 == 0) {
    uint64_t tile = ceil_div(m, 256) * ceil_div(n, 256) < 128 ? 128 : 256;
    if (k % 64 == 0) return (160 * 1024) / (3 * tile * 64 * 2 + 4 * tile * 32 * 2);   // A: three stages 64 deep
    return (160 * 1024) / (4 * (tile + tile) * 32 * 2);
  }
  return 2;
}
//   conv: patch kernel as said there; else ring of (pixels + channels) x 32 bf16 x 4 stages (x 64 bf16 for the depth-split tiles); first-layer kernel: 3 strips of 260 pixels padded to 4 bf16 +
//   256 x c_out' bf16 of output staging (c_out' = c_out rounded up to 32); register-staged: 2.
uint64_t orc_conv3x3_residency(uint64_t batch, uint64_t h, uint64_t w, uint64_t c_in, uint64_t c_out,
                               uint64_t stride) {
  uint64_t ho = (h - 1) / stride + 1, wo = (w - 1) / stride + 1, pixels = batch * ho * wo;
  uint64_t patch_wgs;
  if (conv_patch_path(batch, ho, wo, c_in, c_out, stride, &patch_wgs))
    return (160 * 1024) / (352 * 64 * 2 + 4 * 64 * 64 * 2);      // the patch and four weight tiles of 64 x 64
  if (conv_stride2_32_path(batch, ho, wo, c_in, c_out, stride, &patch_wgs))
    return (160 * 1024) / (576 * 32 * 2 + 64 * 9 * 32 * 2 + 576 * 4);   // the patch, the filter of 64 channels, a table of 576 words
  if (c_in % 32 == 0 && c_out % 8 == 0) {
    uint64_t tp = c_out > 64 ? 128 : 256, tc = c_out > 64 ? 128 : 64;
    uint64_t bk = 32;
    if (ceil_div(pixels, tp) * ceil_div(c_out, tc) < 256) { tp = tc = 64; bk = c_in % 64 == 0 ? 64 : 32; }
    return (160 * 1024) / (4 * (tp + tc) * bk * 2);
  }
  if (c_in == 3 && stride == 1 && c_out % 8 == 0 && c_out <= 64)
    return (160 * 1024) / (3 * 260 * 8 + 256 * ceil_div(c_out, 32) * 32 * 2);
  return 2;
}

// BFS: CSR (n+1 row pointers, m column indices), the level array, two frontier queues of n
// entries (each rounded up to 256 bytes), three frontier bitmaps of one bit per vertex (each
// rounded up to 256 bytes) and a 256-byte control block.  One 512-thread workgroup per 4096
// vertices, at least 8 and at most 512.
static uint64_t bfs_bitmap_bytes(uint64_t n) { return ceil_div(ceil_div(n, 32), 64) * 64 * 4; }
void orc_bfs_probe(uint64_t n, uint64_t m, uint64_t out[7]) {
  uint64_t queue = ceil_div(n * 4, 256) * 256;
  uint64_t wg = ceil_div(n, 4096);
  if (wg < 8) wg = 8;
  if (wg > 512) wg = 512;
  out[0] = (n + 1 + m) * 4 + n * 4 + 256 + 2 * queue + 3 * bfs_bitmap_bytes(n);
  out[1] = round8(wg); out[2] = 1; out[3] = 1;
  out[4] = 512; out[5] = 1; out[6] = 1;
}
// The level kernel keeps 29184 bytes of LDS for staging and, for graphs of up to 2^20 vertices,
// one frontier bitmap; its 128 registers per lane leave room for two 8-wave workgroups per CU.
uint64_t orc_bfs_residency(uint64_t n) {
  uint64_t lds = 29184 + (n <= (1ull << 20) ? bfs_bitmap_bytes(n) : 0);
  uint64_t by_lds = (160 * 1024) / lds, by_regs = 2;
  return by_lds < by_regs ? by_lds : by_regs;
}

}  // extern "C"
