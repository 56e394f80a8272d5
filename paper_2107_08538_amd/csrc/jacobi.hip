// fp32 5-point Jacobi relaxation, up to four sweeps per kernel launch in the window form
// described first, five to eight in the streaming form (grids of 2048 columns and more).
//
// One sweep per launch is HBM-bound at 8 bytes per cell update (one read and
// one write of every cell).  Fusing T sweeps into a launch divides that traffic
// by about T: a wave loads a window of (JB_ROWS + 2T) rows x 256 columns into
// registers (each lane four adjacent columns, one 16-byte load per row), runs
// T sweeps entirely in registers -- north / south neighbours are the lane's
// own registers, west / east come from the neighbouring lane through a wave
// shuffle -- and stores the JB_ROWS x 248 cells that are still exact.  Cells
// next to a window edge go stale by one cell per sweep, which is why windows
// overlap by four columns (eight when T > 4) and T rows on each side; the fixed outer ring of the
// grid is a true boundary and costs no overlap.  No LDS and no barriers: waves
// are independent.  Eight output rows per window keep the register file small
// enough for three waves per SIMD, which measured faster than taller windows
// with less overlap: once fused the kernel is bound by its vector instructions
// (about 1200 per wave and launch at T = 4, the four sweeps' adds and
// multiplies), not by bandwidth.  A quarter of them were the selects that keep
// the grid's ring fixed; only the windows that touch the ring execute those.
//
// The arithmetic of every update is exactly v = 0.25f * ((N + S) + (W + E)):
// two roundings of pair sums, one rounding of their sum, an exact scaling, no
// FMA can form.  Fusing sweeps changes which wave computes a cell, not what
// is computed, so results are bit-identical to the one-sweep definition.
#include "../../include/mgb.h"
#include "launch_util.h"

#include <hip/hip_runtime.h>

#ifndef JB_ROWS_DEF
#define JB_ROWS_DEF 8
#endif
#ifndef JB_STREAM_MIN_N
#define JB_STREAM_MIN_N 2048     // grids from this many columns on fuse five to eight sweeps (streaming form)
#endif

namespace {

constexpr uint32_t JB_THREADS = 256;          // 4 waves, one window each
constexpr uint32_t JB_ROWS = JB_ROWS_DEF;     // output rows per window
constexpr uint32_t JB_WIN = 256;              // window width in columns (64 lanes x 4)
constexpr uint32_t JB_MAXT = 8;
constexpr uint32_t JS_ROWS = 40;              // output rows per run of the streaming form (large grids)
// Sweeps fused per launch.  Launches of up to four sweeps use the window form below; from 2048
// columns on, launches of five to eight sweeps use the streaming form further down (measured,
// 50 sweeps against windows of four: 2048^2 7 %, 2816^2 20 %, 3584^2 27 %, 4032^2 28 % faster,
// 8192^2 9 %, 16384^2 24 % against windows of six; below about 1900 columns a grid has too few
// strips to fill the device with runs of useful length and is 1-20 % slower that way).
constexpr uint32_t fused_sweeps(uint32_t n) { return n >= JB_STREAM_MIN_N ? JB_MAXT : 4u; }
// columns lost on each side of a window: at least the sweeps of the launch, a multiple of 4 (16-byte alignment)
constexpr uint32_t halo_of(uint32_t t) { return t > 4u ? 8u : 4u; }
constexpr uint32_t step_of(uint32_t halo) { return JB_WIN - 2u * halo; }   // exact columns per window: 248 or 240

// Workgroups are dealt round-robin to the 8 XCDs in launch order; give each
// XCD one contiguous band of windows so that the rows shared by vertically
// adjacent windows meet in the same L2.
__device__ __forceinline__ bool window_of_wave(uint32_t tiles_c, uint32_t tiles_r, uint32_t* tc,
                                               uint32_t* tr) {
  const uint32_t total = tiles_c * tiles_r;
  const uint32_t groups = (total + 3u) / 4u;              // workgroups that have work
  const uint32_t per_xcd = (groups + 7u) / 8u;
  const uint32_t grp = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
  if ((blockIdx.x >> 3) >= per_xcd || grp >= groups) return false;
  const uint32_t w = grp * 4u + (threadIdx.x >> 6);
  if (w >= total) return false;
  *tc = w % tiles_c;
  *tr = w / tiles_c;
  return true;
}

// T sweeps over the window held in `cur` (register rows; row i is grid row g0 + i).  EDGE: the
// window contains cells of the grid's fixed ring, which keep their value.
template <uint32_t T, bool EDGE>
__device__ __forceinline__ void run_sweeps(float4 (&cur)[JB_ROWS + 2u * T], int32_t g0, uint32_t n,
                                           bool first_col, bool last_col) {
  constexpr uint32_t NR = JB_ROWS + 2u * T;
#pragma unroll
  for (uint32_t s = 1; s <= T; ++s) {
    float4 north = cur[s - 1u];                           // value of the row above before this sweep
#pragma unroll
    for (uint32_t i = s; i + s < NR; ++i) {
      const float4 c = cur[i];
      const float4 south = cur[i + 1u];
      const float west = __shfl_up(c.w, 1);
      const float east = __shfl_down(c.x, 1);
      float4 o;
      o.x = 0.25f * ((north.x + south.x) + (west + c.y));
      o.y = 0.25f * ((north.y + south.y) + (c.x + c.z));
      o.z = 0.25f * ((north.z + south.z) + (c.y + c.w));
      o.w = 0.25f * ((north.w + south.w) + (c.z + east));
      if (EDGE) {
        if (first_col) o.x = c.x;                         // the ring keeps its value
        if (last_col) o.w = c.w;
        const int32_t g = g0 + (int32_t)i;
        const bool interior_row = g >= 1 && g <= (int32_t)n - 2;
        cur[i] = interior_row ? o : c;
      } else {
        cur[i] = o;
      }
      north = c;
    }
  }
}

// n % 4 == 0: rows are 16-byte aligned, every lane's four columns are either
// all inside the grid or all outside.
template <uint32_t T>
__global__ __launch_bounds__(JB_THREADS, 3) void jacobi_sweeps(const float* __restrict__ u,
                                                           float* __restrict__ v, uint32_t n,
                                                           uint32_t tiles_c, uint32_t tiles_r) {
  constexpr uint32_t NR = JB_ROWS + 2u * T;               // rows held in registers
  constexpr uint32_t JB_HALO = halo_of(T), JB_STEP = step_of(JB_HALO);
  uint32_t tc, tr;
  if (!window_of_wave(tiles_c, tiles_r, &tc, &tr)) return;
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t w0 = tc * JB_STEP;                       // first column of the window
  const uint32_t c0 = w0 + 4u * lane;                     // this lane's first column
  if (c0 >= n) return;
  const int32_t g0 = 1 + (int32_t)(tr * JB_ROWS) - (int32_t)T;   // grid row of register row 0
  const bool first_col = c0 == 0u, last_col = c0 + 4u == n;

  // load the window; rows above / below the grid do not exist and are never needed
  float4 cur[NR];
#pragma unroll
  for (uint32_t i = 0; i < NR; ++i) {
    const int32_t g = g0 + (int32_t)i;
    const uint32_t gc = (uint32_t)min(max(g, 0), (int32_t)n - 1);
    cur[i] = *reinterpret_cast<const float4*>(u + (size_t)gc * n + c0);
  }

  // Only windows that touch the grid's ring need the per-cell selects that keep the ring fixed;
  // every other window (most of them) runs the plain update, a quarter fewer instructions.
  const bool edge = g0 < 1 || g0 + (int32_t)NR - 1 > (int32_t)n - 2 || tc == 0u || w0 + JB_WIN >= n;
  if (edge) run_sweeps<T, true>(cur, g0, n, first_col, last_col);
  else run_sweeps<T, false>(cur, g0, n, first_col, last_col);

  // store what is still exact: not the JB_HALO columns next to a window edge (an edge that is
  // the grid's own boundary loses nothing), rows JB_ROWS of this window that are interior
  const bool left_ok = tc == 0u || 4u * lane >= JB_HALO;
  const bool right_ok = c0 + 4u <= w0 + JB_WIN - JB_HALO || w0 + JB_WIN >= n;
  if (left_ok && right_ok) {
#pragma unroll
    for (uint32_t i = T; i < T + JB_ROWS; ++i) {
      const int32_t g = g0 + (int32_t)i;
      if (g <= (int32_t)n - 2) *reinterpret_cast<float4*>(v + (size_t)g * n + c0) = cur[i];
    }
  }
}


// ---- streaming form ----------------------------------------------------------------------
// A wave owns a strip of 256 columns and walks down `rows` output rows of it.  Row g of the
// input enters at the top of a pipeline of T stages; stage s holds the two rows it saw last and
// turns (row g - s - 1, row g - s, row g - s + 1) after s - 1 sweeps into row g - s after s
// sweeps, so each input row costs T row updates and one row leaves the bottom per step: no row
// is recomputed except the 2T that warm the pipeline up at the start of a run.  The state is 2T
// rows (8T registers per lane), input rows are requested JS_PF steps before they are used.
constexpr uint32_t JS_PF = 6;                 // rows in flight per lane = steps per pass of the loop

// The neighbouring lane's value as a DPP wave shift: an operand modifier of the add that uses it,
// not an instruction of its own.  Lane 0 / lane 63 have no such neighbour and get zero; what they
// compute from it lies in the strip's halo.
__device__ __forceinline__ float from_lane_below(float x) {      // lane l gets lane l - 1's value
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x138, 0xF, 0xF, true));
}
__device__ __forceinline__ float from_lane_above(float x) {      // lane l gets lane l + 1's value
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x130, 0xF, 0xF, true));
}

// JS_PF steps of a run, starting with input row g_first + jb.  COLS: the strip touches the
// grid's left or right ring column, whose cells keep their value.  ROWS: some row produced in
// these steps may be the grid's top or bottom ring row (or lie outside the grid): tested per row.
template <uint32_t T, bool COLS, bool ROWS>
__device__ __forceinline__ void stream_steps(float4 (&h)[T][2], float4 (&pf)[JS_PF], const float* __restrict__ col,
                                             float* __restrict__ v, uint32_t n, uint32_t c0, int32_t g_first,
                                             int32_t jb, int32_t r0, int32_t g_last, bool first_col,
                                             bool last_col, bool col_ok) {
  // The products by 0.25 must stay products: fused into the next stage's add they would round
  // differently when they underflow.
#pragma clang fp contract(off)
#pragma unroll
  for (uint32_t k = 0; k < JS_PF; ++k) {
    const int32_t g_in = g_first + jb + (int32_t)k;
    float4 newest = pf[k];
    // rows outside the grid are never needed, but they are requested: clamp them into it
    pf[k] = *reinterpret_cast<const float4*>(col + (size_t)min(max(g_in + (int32_t)JS_PF, 0), (int32_t)n - 1) * n);
#pragma unroll
    for (uint32_t s = 1; s <= T; ++s) {
      const float4 north = h[s - 1u][0], c = h[s - 1u][1], south = newest;
      float4 o;
      const int32_t g = g_in - (int32_t)s;                // the row this stage produces (wave-uniform)
      if (ROWS && (g <= 0 || g >= (int32_t)n - 1)) {
        o = c;                                            // the ring keeps its value
      } else {
        const float west = from_lane_below(c.w);
        const float east = from_lane_above(c.x);
        o.x = 0.25f * ((north.x + south.x) + (west + c.y));
        o.y = 0.25f * ((north.y + south.y) + (c.x + c.z));
        o.z = 0.25f * ((north.z + south.z) + (c.y + c.w));
        o.w = 0.25f * ((north.w + south.w) + (c.z + east));
        if (COLS) {
          if (first_col) o.x = c.x;
          if (last_col) o.w = c.w;
        }
      }
      h[s - 1u][0] = c;
      h[s - 1u][1] = south;
      newest = o;
    }
    const int32_t g_out = g_in - (int32_t)T;
    if (g_out >= r0 && g_out <= g_last && col_ok) *reinterpret_cast<float4*>(v + (size_t)g_out * n + c0) = newest;
  }
}

template <uint32_t T, bool COLS>
__device__ __forceinline__ void stream_run(const float* __restrict__ u, float* __restrict__ v, uint32_t n,
                                           uint32_t c0, int32_t r0, int32_t g_last, bool first_col,
                                           bool last_col, bool col_ok) {
  const int32_t g_first = r0 - (int32_t)T;                  // first input row of the run
  const int32_t steps = g_last - r0 + 1 + 2 * (int32_t)T;   // input rows r0 - T .. g_last + T
  const float* col = u + c0;
  float4 h[T][2];
#pragma unroll
  for (uint32_t s = 0; s < T; ++s) h[s][0] = h[s][1] = make_float4(0.f, 0.f, 0.f, 0.f);
  float4 pf[JS_PF];
#pragma unroll
  for (uint32_t k = 0; k < JS_PF; ++k)
    pf[k] = *reinterpret_cast<const float4*>(col + (size_t)min(max(g_first + (int32_t)k, 0), (int32_t)n - 1) * n);
  for (int32_t jb = 0; jb < steps; jb += (int32_t)JS_PF) {
    // rows produced in this pass: g_first + jb - T (last stage, first step) .. g_first + jb + JS_PF - 2
    const bool ring_rows = g_first + jb - (int32_t)T <= 0 || g_first + jb + (int32_t)JS_PF - 2 >= (int32_t)n - 1;
    if (ring_rows) stream_steps<T, COLS, true>(h, pf, col, v, n, c0, g_first, jb, r0, g_last, first_col, last_col, col_ok);
    else stream_steps<T, COLS, false>(h, pf, col, v, n, c0, g_first, jb, r0, g_last, first_col, last_col, col_ok);
  }
}

template <uint32_t T>
__global__ __launch_bounds__(JB_THREADS) void jacobi_stream(const float* __restrict__ u, float* __restrict__ v,
                                                            uint32_t n, uint32_t tiles_c, uint32_t tiles_r,
                                                            uint32_t rows) {
  constexpr uint32_t JB_HALO = halo_of(T), JB_STEP = step_of(JB_HALO);
  uint32_t tc, tr;
  if (!window_of_wave(tiles_c, tiles_r, &tc, &tr)) return;
  // (the run is the same for the whole wave: said so, the tests on its rows are scalar)
  tr = (uint32_t)__builtin_amdgcn_readfirstlane((int)tr);
  tc = (uint32_t)__builtin_amdgcn_readfirstlane((int)tc);
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t w0 = tc * JB_STEP;
  const uint32_t c0 = w0 + 4u * lane;
  if (c0 >= n) return;
  const int32_t r0 = 1 + (int32_t)(tr * rows);
  const int32_t g_last = min(r0 + (int32_t)rows - 1, (int32_t)n - 2);
  const bool first_col = c0 == 0u, last_col = c0 + 4u == n;
  const bool left_ok = tc == 0u || 4u * lane >= JB_HALO;
  const bool right_ok = c0 + 4u <= w0 + JB_WIN - JB_HALO || w0 + JB_WIN >= n;
  const bool col_ok = left_ok && right_ok;
  // only strips next to the grid's left / right ring pay for keeping it (two selects per row
  // update); the top and bottom ring rows are tested for in the passes that can meet them
  if (tc == 0u || w0 + JB_WIN >= n) stream_run<T, true>(u, v, n, c0, r0, g_last, first_col, last_col, col_ok);
  else stream_run<T, false>(u, v, n, c0, r0, g_last, first_col, last_col, col_ok);
}

// any n: one column per thread.
__global__ __launch_bounds__(JB_THREADS) void jacobi_sweep_v1(const float* __restrict__ u,
                                                             float* __restrict__ v, uint32_t n,
                                                             uint32_t tiles_x, uint32_t tiles_y) {
  const uint32_t total = tiles_x * tiles_y;
  const uint32_t per_xcd = (total + 7u) / 8u;
  const uint32_t tile = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
  if ((blockIdx.x >> 3) >= per_xcd || tile >= total) return;
  const uint32_t tx = tile % tiles_x, ty = tile / tiles_x;
  const uint32_t c = tx * JB_THREADS + threadIdx.x;
  const uint32_t r0 = 1u + ty * JB_ROWS;
  if (c == 0u || c + 1u >= n) return;
  const uint32_t r1 = min(r0 + JB_ROWS, n - 1u);
  const float* p = u + (size_t)(r0 - 1u) * n + c;
  float north = p[0];
  p += n;
  float centre = p[0];
  for (uint32_t r = r0; r < r1; ++r) {
    const float south = p[n];
    v[(size_t)r * n + c] = 0.25f * ((north + south) + (p[-1] + p[1]));
    north = centre;
    centre = south;
    p += n;
  }
}

struct Geometry {
  uint32_t tiles_x, tiles_y, blocks;
  bool vec4;
};

Geometry geometry(uint32_t n, uint32_t JB_HALO) {
  const uint32_t JB_STEP = step_of(JB_HALO);
  Geometry g;
  g.vec4 = (n % 4u) == 0u;
  if (g.vec4) {
    // windows step by 248 (240) columns; a window next to the grid's ring loses nothing on that
    // side, so the last window is the first one that reaches the right edge
    g.tiles_x = n <= JB_WIN ? 1u : 1u + (n - JB_WIN + JB_STEP - 1u) / JB_STEP;
    g.tiles_y = (n - 2u + JB_ROWS - 1u) / JB_ROWS;
    const uint32_t groups = (g.tiles_x * g.tiles_y + 3u) / 4u;       // four windows per workgroup
    g.blocks = ((groups + 7u) / 8u) * 8u;                             // whole rounds over the 8 XCDs
  } else {
    g.tiles_x = (n + JB_THREADS - 1u) / JB_THREADS;
    g.tiles_y = (n - 2u + JB_ROWS - 1u) / JB_ROWS;
    g.blocks = ((g.tiles_x * g.tiles_y + 7u) / 8u) * 8u;
  }
  return g;
}

// Split `iters` sweeps into launches of 1..maxt sweeps: the fewest launches whose number has the
// parity of iters (the buffers swap once per launch and the result must end in buffer
// iters % 2), the sweeps spread evenly over them.
uint32_t plan_launches(uint32_t iters, uint32_t maxt, uint32_t* plan, uint32_t cap) {
  if (iters == 0u) return 0u;
  uint32_t launches = (iters + maxt - 1u) / maxt;
  if (launches % 2u != iters % 2u) ++launches;            // then launches < iters: every launch still gets a sweep
  if (launches > cap) launches = cap;                     // callers plan chunks that fit
  const uint32_t base = iters / launches, extra = iters % launches;
  for (uint32_t i = 0; i < launches; ++i) plan[i] = base + (i < extra ? 1u : 0u);
  return launches;
}

// workgroups of a launch of t sweeps
// Output rows per run of the streaming form.  Its waves live as long as the launch and a SIMD
// holds two of them (registers), so what counts is that every SIMD gets the same number: with
// fewer than four rounds of 2048 waves at JS_ROWS rows per run, the rows are chosen to make the
// waves a whole number of such rounds (4096^2: 35 rows, 17 strips x 117 runs = 1989 waves).
uint32_t stream_rows(uint32_t n, uint32_t strips) {
  const uint32_t waves = strips * ((n - 2u + JS_ROWS - 1u) / JS_ROWS);
  if (waves >= 4u * 2048u) return JS_ROWS;
  uint32_t rounds = (waves + 1024u) / 2048u;
  if (rounds == 0u) rounds = 1u;
  uint32_t runs = rounds * 2048u / strips;
  if (runs == 0u) runs = 1u;
  return (n - 2u + runs - 1u) / runs;
}

uint32_t blocks_of(uint32_t n, uint32_t t, uint32_t* tiles_x, uint32_t* tiles_y, uint32_t* rows) {
  const Geometry g = geometry(n, halo_of(t));
  *tiles_x = g.tiles_x;
  *tiles_y = g.tiles_y;
  if (!g.vec4 || t <= 4u) return g.blocks;
  *rows = stream_rows(n, g.tiles_x);
  *tiles_y = (n - 2u + *rows - 1u) / *rows;                           // runs per strip
  const uint32_t groups = (g.tiles_x * *tiles_y + 3u) / 4u;             // four strips' runs per workgroup
  return ((groups + 7u) / 8u) * 8u;
}

template <uint32_t T>
void launch_sweeps(hipStream_t st, const float* src, float* dst, uint32_t n) {
  uint32_t tiles_x, tiles_y, rows = 0;
  const uint32_t blocks = blocks_of(n, T, &tiles_x, &tiles_y, &rows);
  if constexpr (T <= 4u)
    hipLaunchKernelGGL(jacobi_sweeps<T>, dim3(blocks), dim3(JB_THREADS), 0, st, src, dst, n, tiles_x, tiles_y);
  else
    hipLaunchKernelGGL(jacobi_stream<T>, dim3(blocks), dim3(JB_THREADS), 0, st, src, dst, n, tiles_x, tiles_y,
                       rows);
}

}  // namespace

extern "C" {

int mgb_jacobi_probe(uint32_t n, uint32_t iters, uint64_t* mem_bytes, mgb_dim3* grid,
                     mgb_dim3* block) {
  (void)iters;
  if (!mem_bytes || !grid || !block) return MGB_E_INVAL;
  if (n < 3u || n > 65536u) return MGB_E_UNSUPPORTED;
  // the largest grid among the task's launches (one probe covers them all).  Sweeps are planned
  // in chunks of 128: every chunk but the last has the plan of the first.
  uint32_t blocks = geometry(n, 4u).blocks;
  if (n % 4u == 0u && iters != 0u) {
    blocks = 0u;
    const uint32_t chunks[2] = {iters > 128u ? 128u : iters, iters > 128u ? iters % 128u : 0u};
    for (uint32_t c = 0; c < 2u; ++c) {
      uint32_t plan[64], tx, ty, rows;
      const uint32_t np = chunks[c] ? plan_launches(chunks[c], fused_sweeps(n), plan, 64u) : 0u;
      for (uint32_t i = 0; i < np; ++i) {
        const uint32_t b = blocks_of(n, plan[i], &tx, &ty, &rows);
        if (b > blocks) blocks = b;
      }
    }
  }
  *mem_bytes = 2ull * n * n * sizeof(float);
  *grid = mgb_dim3{blocks, 1u, 1u};
  *block = mgb_dim3{JB_THREADS, 1u, 1u};
  return MGB_OK;
}

// workgroups a CU holds (one workgroup's four waves go to the four SIMDs): the window kernels
// take up to 168 registers per lane (three waves per SIMD), the streaming kernels of grids from
// 2048 columns on up to 224 (two); the one-sweep kernel for n % 4 != 0 is limited by the 32 wave
// slots alone
uint32_t mgb_jacobi_residency(uint32_t n) {
  if (n < 3u || n > 65536u) return 0u;
  if (n % 4u != 0u) return 8u;
  return n >= JB_STREAM_MIN_N ? 2u : 3u;
}

uint32_t mgb_jacobi_launch_count(uint32_t n, uint32_t iters) {
  if (n < 3u || n > 65536u) return 0u;
  if (n % 4u != 0u) return iters;
  uint32_t total = 0, done = 0;
  while (done < iters) {
    uint32_t plan[64];
    const uint32_t chunk = iters - done > 128u ? 128u : iters - done;
    total += plan_launches(chunk, fused_sweeps(n), plan, 64u);
    done += chunk;
  }
  return total;
}

int mgb_jacobi_enqueue(void* stream, float* u0, float* u1, uint32_t n, uint32_t iters) {
  if (!u0 || !u1 || u0 == u1) return MGB_E_INVAL;
  if (n < 3u || n > 65536u) return MGB_E_UNSUPPORTED;
  if (((uintptr_t)u0 | (uintptr_t)u1) & 15u) return MGB_E_INVAL;
  const Geometry g = geometry(n, 4u);
  hipStream_t st = (hipStream_t)stream;
  const float* src = u0;
  float* dst = u1;
  if (!g.vec4) {
    for (uint32_t t = 0; t < iters; ++t) {
      hipLaunchKernelGGL(jacobi_sweep_v1, dim3(g.blocks), dim3(JB_THREADS), 0, st, src, dst, n,
                         g.tiles_x, g.tiles_y);
      float* tmp = const_cast<float*>(src);
      src = dst;
      dst = tmp;
    }
    return mgb_check_launch("jacobi_sweep");
  }
  uint32_t done = 0;
  while (done < iters) {
    uint32_t plan[64];
    const uint32_t chunk = iters - done > 128u ? 128u : iters - done;   // even chunks keep the parity rule
    const uint32_t np = plan_launches(chunk, fused_sweeps(n), plan, 64u);
    for (uint32_t i = 0; i < np; ++i) {
      switch (plan[i]) {
        case 1: launch_sweeps<1>(st, src, dst, n); break;
        case 2: launch_sweeps<2>(st, src, dst, n); break;
        case 3: launch_sweeps<3>(st, src, dst, n); break;
        case 4: launch_sweeps<4>(st, src, dst, n); break;
        case 5: launch_sweeps<5>(st, src, dst, n); break;
        case 6: launch_sweeps<6>(st, src, dst, n); break;
        case 7: launch_sweeps<7>(st, src, dst, n); break;
        default: launch_sweeps<8>(st, src, dst, n); break;
      }
      float* tmp = const_cast<float*>(src);
      src = dst;
      dst = tmp;
    }
    done += chunk;
  }
  return mgb_check_launch("jacobi_sweeps");
}

}  // extern "C"
