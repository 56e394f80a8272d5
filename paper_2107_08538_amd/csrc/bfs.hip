// Level-synchronous BFS on a CSR graph with a frontier queue.
//
// HBM / latency bound: per traversed edge one 4-byte column read and one
// 4-byte probe of level[] (a random access), per frontier vertex two row_ptr
// reads and one queue slot.  One kernel per level; a wave takes 64 frontier
// vertices at a time and spreads their adjacency lists evenly over its lanes
// (prefix sum of the degrees, each lane finds the owner of "its" edge by
// binary search), so lanes stay busy whatever the degree distribution.  Newly
// reached vertices are claimed with one compare-and-swap on level[] (levels
// are unique, so the result does not depend on who wins) and appended to the
// next queue with one atomic per wave: ballot of the winners, leader reserves
// popcount slots, each winner writes at its rank.
//
// The host does not know the depth in advance: it enqueues a batch of level
// kernels whose grids do not depend on the frontier size (the kernels read the
// size from device memory and exit at once on an empty frontier), then reads
// the per-level counters back once per batch.
#include "../../include/mgb.h"
#include "launch_util.h"

#include <hip/hip_runtime.h>

namespace {

constexpr uint32_t BFS_THREADS = 256;
constexpr uint32_t BFS_WAVES = BFS_THREADS / 64;
constexpr uint32_t BFS_BATCH = 16;            // levels per host round trip (even: keeps queue parity)

struct Work {                                  // layout of the caller's scratch buffer
  uint32_t* counts;                            // BFS_BATCH + 1 frontier sizes, + 1 spare
  int32_t* queue[2];                           // n entries each
};

__host__ __device__ inline uint64_t counts_bytes() { return 256; }

Work carve(void* work, uint32_t n) {
  Work w;
  char* p = (char*)work;
  w.counts = (uint32_t*)p;
  p += counts_bytes();
  w.queue[0] = (int32_t*)p;
  p += ((uint64_t)n * 4 + 255) / 256 * 256;
  w.queue[1] = (int32_t*)p;
  return w;
}

__global__ __launch_bounds__(BFS_THREADS) void bfs_init(int32_t* __restrict__ level, uint32_t n,
                                                       uint32_t source, int32_t* __restrict__ q0,
                                                       uint32_t* __restrict__ counts) {
  const uint32_t stride = gridDim.x * BFS_THREADS;
  for (uint32_t v = blockIdx.x * BFS_THREADS + threadIdx.x; v < n; v += stride)
    level[v] = (v == source) ? 0 : -1;
  if (blockIdx.x == 0 && threadIdx.x <= BFS_BATCH) counts[threadIdx.x] = threadIdx.x == 0 ? 1u : 0u;
  if (blockIdx.x == 0 && threadIdx.x == 0) q0[0] = (int32_t)source;
}

// start of the next batch: its first frontier is the last one of the previous batch
__global__ void bfs_roll(uint32_t* __restrict__ counts) {
  const uint32_t t = threadIdx.x;
  uint32_t carry = counts[BFS_BATCH];
  __syncthreads();
  if (t <= BFS_BATCH) counts[t] = t == 0 ? carry : 0u;
}

__global__ __launch_bounds__(BFS_THREADS) void bfs_level(const int32_t* __restrict__ row_ptr,
                                                        const int32_t* __restrict__ col_idx,
                                                        int32_t* __restrict__ level,
                                                        const int32_t* __restrict__ q_in,
                                                        int32_t* __restrict__ q_out,
                                                        const uint32_t* __restrict__ cnt_in,
                                                        uint32_t* __restrict__ cnt_out,
                                                        int32_t next_level) {
  __shared__ uint32_t s_excl[BFS_WAVES][64];
  __shared__ int32_t s_start[BFS_WAVES][64];
  const uint32_t n_in = *cnt_in;
  if (n_in == 0u) return;
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  const uint32_t gwave = blockIdx.x * BFS_WAVES + wave;
  const uint32_t wave_stride = gridDim.x * BFS_WAVES * 64u;

  for (uint32_t base = gwave * 64u; base < n_in; base += wave_stride) {
    int32_t start = 0;
    uint32_t deg = 0;
    if (base + lane < n_in) {
      const int32_t v = q_in[base + lane];
      start = row_ptr[v];
      deg = (uint32_t)(row_ptr[v + 1] - start);
    }
    // inclusive prefix sum of the degrees across the wave
    uint32_t incl = deg;
#pragma unroll
    for (uint32_t off = 1; off < 64u; off <<= 1) {
      const uint32_t up = __shfl_up(incl, off);
      if (lane >= off) incl += up;
    }
    const uint32_t total = __shfl(incl, 63);
    s_excl[wave][lane] = incl - deg;
    s_start[wave][lane] = start;
    __builtin_amdgcn_wave_barrier();

    for (uint32_t e0 = 0; e0 < total; e0 += 64u) {
      const uint32_t e = e0 + lane;
      bool won = false;
      int32_t nb = 0;
      if (e < total) {
        // owner = last lane whose exclusive prefix is <= e
        uint32_t lo = 0, hi = 63;
#pragma unroll
        for (int it = 0; it < 6; ++it) {
          const uint32_t mid = (lo + hi + 1u) >> 1;
          if (s_excl[wave][mid] <= e) lo = mid; else hi = mid - 1u;
        }
        nb = col_idx[s_start[wave][lo] + (int32_t)(e - s_excl[wave][lo])];
        if (level[nb] < 0) won = atomicCAS(&level[nb], -1, next_level) == -1;
      }
      const uint64_t winners = __ballot(won);
      if (winners != 0ull) {
        uint32_t slot = 0;
        if (lane == 0u) slot = atomicAdd(cnt_out, (uint32_t)__popcll(winners));
        slot = __shfl(slot, 0);
        if (won) q_out[slot + __popcll(winners & ((1ull << lane) - 1ull))] = nb;
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
}

uint32_t blocks_for(uint32_t n) {
  uint32_t b = (n + 2047u) / 2048u;
  if (b < 8u) b = 8u;
  if (b > 1024u) b = 1024u;
  return (b + 7u) / 8u * 8u;
}

}  // namespace

extern "C" {

uint64_t mgb_bfs_work_bytes(uint32_t n) {
  return counts_bytes() + 2ull * (((uint64_t)n * 4 + 255) / 256 * 256);
}

int mgb_bfs_probe(uint32_t n, uint64_t m, uint64_t* mem_bytes, mgb_dim3* grid, mgb_dim3* block) {
  if (!mem_bytes || !grid || !block) return MGB_E_INVAL;
  if (n == 0u || n > 0x7fffffffu || m > 0x7fffffffull) return MGB_E_UNSUPPORTED;
  *mem_bytes = ((uint64_t)n + 1 + m) * 4 + (uint64_t)n * 4 + mgb_bfs_work_bytes(n);
  *grid = mgb_dim3{blocks_for(n), 1u, 1u};
  *block = mgb_dim3{BFS_THREADS, 1u, 1u};
  return MGB_OK;
}

int mgb_bfs_enqueue(void* stream, const int32_t* row_ptr, const int32_t* col_idx, uint32_t n,
                    uint32_t source, int32_t* level, void* work, uint32_t* depth) {
  if (!row_ptr || !col_idx || !level || !work) return MGB_E_INVAL;
  if (n == 0u || n > 0x7fffffffu || source >= n) return MGB_E_INVAL;
  if ((uintptr_t)work & 255u) return MGB_E_INVAL;
  hipStream_t st = (hipStream_t)stream;
  const Work w = carve(work, n);
  const uint32_t blocks = blocks_for(n);
  hipLaunchKernelGGL(bfs_init, dim3(blocks), dim3(BFS_THREADS), 0, st, level, n, source, w.queue[0],
                     w.counts);
  uint32_t levels_done = 0;
  uint32_t host_counts[BFS_BATCH + 1];
  for (;;) {
    for (uint32_t j = 0; j < BFS_BATCH; ++j)
      hipLaunchKernelGGL(bfs_level, dim3(blocks), dim3(BFS_THREADS), 0, st, row_ptr, col_idx, level,
                         w.queue[j & 1u], w.queue[(j + 1u) & 1u], w.counts + j, w.counts + j + 1u,
                         (int32_t)(levels_done + j + 1u));
    int rc = mgb_check_launch("bfs_level");
    if (rc != MGB_OK) return rc;
    hipError_t e = hipMemcpyAsync(host_counts, w.counts, sizeof host_counts, hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) {
      mgb_internal_set_error("bfs counter read-back", e);
      return MGB_E_BACKEND;
    }
    // host_counts[j] = size of the frontier at depth levels_done + j
    uint32_t j = 0;
    while (j <= BFS_BATCH && host_counts[j] != 0u) ++j;
    if (j <= BFS_BATCH) {                       // an empty frontier was reached
      if (depth) *depth = levels_done + j;      // number of non-empty levels (source level included)
      return MGB_OK;
    }
    levels_done += BFS_BATCH;
    if (levels_done >= n) return MGB_OK;        // cannot happen: depth < n
    hipLaunchKernelGGL(bfs_roll, dim3(1), dim3(64), 0, st, w.counts);
  }
}

}  // extern "C"
