// CPU checker for the requirement derivation -- TEST INFRASTRUCTURE ONLY.
//
// A task's probe carries the sum of its device allocations and the geometry
// of its kernel launches (paper Sec. III-A: requirements are read off the
// task's allocation and launch operations; a task with several launches on
// shared buffers is one task, Algorithm 1).  The functions below recompute
// those figures from the published tiling rules of each task kind, written
// out independently of the GPU library.
#include <cstdint>

namespace {
uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }
// launches are padded to whole rounds over the 8 XCDs
uint64_t round8(uint64_t x) { return ceil_div(x, 8) * 8; }
}  // namespace

extern "C" {

// out = {mem_bytes, grid_x, grid_y, grid_z, block_x, block_y, block_z}

// Jacobi n x n: two fp32 grids.  A workgroup of 256 threads sweeps 16 interior
// rows of a column strip; a thread covers 4 columns when n is a multiple of 4
// (strip = 1024 columns), else 1 column (strip = 256 columns).
void orc_jacobi_probe(uint64_t n, uint64_t out[7]) {
  uint64_t strip = (n % 4 == 0) ? 1024 : 256;
  uint64_t tiles = ceil_div(n, strip) * ceil_div(n - 2, 16);
  out[0] = 2 * n * n * 4;
  out[1] = round8(tiles); out[2] = 1; out[3] = 1;
  out[4] = 256; out[5] = 1; out[6] = 1;
}

// fp32 GEMM: A, B, C in fp32; one 256-thread workgroup per 128 x 128 tile of C.
void orc_gemm_f32_probe(uint64_t m, uint64_t n, uint64_t k, uint64_t out[7]) {
  out[0] = (m * k + k * n + m * n) * 4;
  out[1] = round8(ceil_div(m, 128) * ceil_div(n, 128)); out[2] = 1; out[3] = 1;
  out[4] = 256; out[5] = 1; out[6] = 1;
}

}  // extern "C"
