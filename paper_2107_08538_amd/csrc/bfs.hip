// Level-synchronous, direction-optimising BFS on a CSR graph.
//
// HBM / latency bound: per traversed edge one 4-byte column read and one
// 4-byte probe of level[] (a random access), per frontier vertex two row_ptr
// reads and one queue slot.  One kernel per level, which picks its direction
// from the frontier size it finds in device memory:
//   * top-down (small frontiers): a wave takes up to 64 frontier vertices and
//     spreads their adjacency lists evenly over its lanes (prefix sum of the
//     degrees, each lane finds the owner of "its" edge by binary search in
//     LDS), four edges per lane in flight.  Newly reached vertices are claimed
//     with one compare-and-swap on level[] (levels are unique, so the result
//     does not depend on who wins);
//   * bottom-up (frontier large against what is still unvisited): one thread
//     per unvisited vertex scans its own adjacency list until it meets a
//     vertex of the current level; no atomics on level[], early exit.
// Either way the new frontier is appended to the next queue with one atomic
// per wave: ballot of the winners, the leader reserves popcount slots, each
// winner writes at its rank among the winners.
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
constexpr uint32_t BFS_BATCH = 12;            // levels per host round trip (even: keeps queue parity)
constexpr uint32_t BFS_CUM = BFS_BATCH + 1;   // control word: vertices reached before this batch's first frontier
constexpr uint32_t BFS_UNROLL = 4;            // edges per lane in flight (top-down)
constexpr uint32_t BFS_STAGE = 512;           // per-wave LDS staging of discovered vertices

struct Work {                                  // layout of the caller's scratch buffer
  uint32_t* ctrl;                              // [0..BATCH] frontier sizes of the batch, [BFS_CUM] see above
  int32_t* queue[2];                           // n entries each
};

__host__ __device__ inline uint64_t ctrl_bytes() { return 256; }

Work carve(void* work, uint32_t n) {
  Work w;
  char* p = (char*)work;
  w.ctrl = (uint32_t*)p;
  p += ctrl_bytes();
  w.queue[0] = (int32_t*)p;
  p += ((uint64_t)n * 4 + 255) / 256 * 256;
  w.queue[1] = (int32_t*)p;
  return w;
}

__global__ __launch_bounds__(BFS_THREADS) void bfs_init(int32_t* __restrict__ level, uint32_t n,
                                                       uint32_t source, int32_t* __restrict__ q0,
                                                       uint32_t* __restrict__ ctrl) {
  const uint32_t stride = gridDim.x * BFS_THREADS;
  for (uint32_t v = blockIdx.x * BFS_THREADS + threadIdx.x; v < n; v += stride)
    level[v] = (v == source) ? 0 : -1;
  if (blockIdx.x == 0 && threadIdx.x <= BFS_CUM) ctrl[threadIdx.x] = threadIdx.x == 0 ? 1u : 0u;
  if (blockIdx.x == 0 && threadIdx.x == 0) q0[0] = (int32_t)source;
}

// start of the next batch: its first frontier is the last one of the previous batch
__global__ void bfs_roll(uint32_t* __restrict__ ctrl) {
  const uint32_t t = threadIdx.x;
  uint32_t carry = ctrl[BFS_BATCH];
  uint32_t cum = ctrl[BFS_CUM];
  for (uint32_t i = 0; i < BFS_BATCH; ++i) cum += ctrl[i];
  __syncthreads();
  if (t <= BFS_BATCH) ctrl[t] = t == 0 ? carry : 0u;
  if (t == BFS_CUM) ctrl[t] = cum;
}

// Frontier staging.  Atomics on one address (the queue tail) serialise at about 13 ns each on
// this device, so a level that discovers hundreds of thousands of vertices cannot afford one
// tail update per wave step.  Each wave collects what it discovers in its own LDS buffer
// (ballot -> rank among the winners -> LDS slot); a full buffer is copied out with one tail
// update, and whatever is left when the workgroup is done goes out with ONE tail update for
// the whole workgroup.
struct Stage {
  int32_t* buf;        // this wave's LDS buffer, BFS_STAGE entries
  uint32_t count;      // entries in it (wave-uniform)
};

__device__ __forceinline__ void stage_flush(Stage& st, int32_t* __restrict__ q_out,
                                            uint32_t* __restrict__ tail, uint32_t lane) {
  uint32_t slot = 0;
  if (lane == 0u) slot = atomicAdd(tail, st.count);
  slot = __shfl(slot, 0);
  for (uint32_t i = lane; i < st.count; i += 64u) q_out[slot + i] = st.buf[i];
  st.count = 0;
}

__device__ __forceinline__ void stage_append(Stage& st, bool won, int32_t v,
                                             int32_t* __restrict__ q_out,
                                             uint32_t* __restrict__ tail, uint32_t lane) {
  const uint64_t winners = __ballot(won);
  if (winners == 0ull) return;
  const uint32_t k = (uint32_t)__popcll(winners);
  if (st.count + k > BFS_STAGE) stage_flush(st, q_out, tail, lane);
  if (won) st.buf[st.count + __popcll(winners & ((1ull << lane) - 1ull))] = v;
  st.count += k;
}

__global__ __launch_bounds__(BFS_THREADS) void bfs_level(const int32_t* __restrict__ row_ptr,
                                                        const int32_t* __restrict__ col_idx,
                                                        int32_t* __restrict__ level,
                                                        const int32_t* __restrict__ q_in,
                                                        int32_t* __restrict__ q_out,
                                                        uint32_t* __restrict__ ctrl, uint32_t j,
                                                        int32_t next_level, uint32_t n,
                                                        uint32_t symmetric) {
  __shared__ uint32_t s_excl[BFS_WAVES][64];
  __shared__ int32_t s_start[BFS_WAVES][64];
  __shared__ int32_t s_stage[BFS_WAVES][BFS_STAGE];
  __shared__ uint32_t s_cnt[BFS_WAVES];
  __shared__ uint32_t s_base;
  const uint32_t n_in = ctrl[j];
  if (n_in == 0u) return;
  uint32_t reached = ctrl[BFS_CUM];
  for (uint32_t i = 0; i <= j; ++i) reached += ctrl[i];
  const uint32_t unvisited = n - reached;
  if (unvisited == 0u) return;
  uint32_t* cnt_out = ctrl + j + 1u;
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  const uint32_t gwave = blockIdx.x * BFS_WAVES + wave;
  const uint32_t total_waves = gridDim.x * BFS_WAVES;
  Stage stage{&s_stage[wave][0], 0u};

  // Top-down touches about n_in * (m/n) edges; bottom-up makes every unvisited vertex look at
  // about n/n_in neighbours before it meets the frontier.  Go bottom-up when the first is larger.
  const float m = (float)row_ptr[n];      // number of stored (directed) edges
  const float td_cost = (float)n_in * (float)n_in * m;
  const float bu_cost = (float)unvisited * (float)n * (float)n;
  // (bottom-up reads a vertex's stored edges as its in-edges: only right for a symmetric graph)
  if (symmetric != 0u && td_cost > bu_cost) {
    // bottom-up: two vertices per lane and four neighbours per step in flight, so that the
    // dependent column -> level reads of different vertices and neighbours overlap
    const int32_t cur = next_level - 1;
    for (uint32_t v0 = gwave * 128u; v0 < n; v0 += total_waves * 128u) {
      int32_t e[2], e1[2];
      bool open[2], found[2];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const uint32_t v = v0 + 64u * u + lane;
        open[u] = v < n && level[v] < 0;
        found[u] = false;
        e[u] = e1[u] = 0;
      }
#pragma unroll
      for (int u = 0; u < 2; ++u)
        if (open[u]) {
          const uint32_t v = v0 + 64u * u + lane;
          e[u] = row_ptr[v];
          e1[u] = row_ptr[v + 1u];
        }
      while (__any((open[0] && e[0] < e1[0]) || (open[1] && e[1] < e1[1]))) {
        int32_t nb[2][4];
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int i = 0; i < 4; ++i) nb[u][i] = (open[u] && e[u] + i < e1[u]) ? col_idx[e[u] + i] : -1;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          bool hit = false;
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (nb[u][i] >= 0) hit |= level[nb[u][i]] == cur;
          if (hit) { found[u] = true; open[u] = false; }
          e[u] += 4;
        }
      }
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const uint32_t v = v0 + 64u * u + lane;
        if (found[u]) level[v] = next_level;
        stage_append(stage, found[u], (int32_t)v, q_out, cnt_out, lane);
      }
    }
  } else {

  // top-down.  Small frontiers are split into chunks of fewer than 64 vertices so that
  // every wave of the grid gets some of the edges.
  uint32_t chunk = (n_in + total_waves - 1u) / total_waves;
  if (chunk > 64u) chunk = 64u;
  for (uint32_t base = gwave * chunk; base < n_in; base += total_waves * chunk) {
    int32_t start = 0;
    uint32_t deg = 0;
    if (lane < chunk && base + lane < n_in) {
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

    for (uint32_t e0 = 0; e0 < total; e0 += 64u * BFS_UNROLL) {
      int32_t nb[BFS_UNROLL];
      bool live[BFS_UNROLL];
#pragma unroll
      for (uint32_t u = 0; u < BFS_UNROLL; ++u) {
        const uint32_t e = e0 + 64u * u + lane;
        live[u] = e < total;
        nb[u] = 0;
        if (live[u]) {
          // owner = last lane whose exclusive prefix is <= e
          uint32_t lo = 0, hi = 63;
#pragma unroll
          for (int it = 0; it < 6; ++it) {
            const uint32_t mid = (lo + hi + 1u) >> 1;
            if (s_excl[wave][mid] <= e) lo = mid; else hi = mid - 1u;
          }
          nb[u] = col_idx[s_start[wave][lo] + (int32_t)(e - s_excl[wave][lo])];
        }
      }
      int32_t seen[BFS_UNROLL];
#pragma unroll
      for (uint32_t u = 0; u < BFS_UNROLL; ++u) seen[u] = live[u] ? level[nb[u]] : 0;
#pragma unroll
      for (uint32_t u = 0; u < BFS_UNROLL; ++u) {
        bool won = false;
        if (live[u] && seen[u] < 0) won = atomicCAS(&level[nb[u]], -1, next_level) == -1;
        stage_append(stage, won, nb[u], q_out, cnt_out, lane);
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
  }

  // what is still staged leaves with one tail update per workgroup
  if (lane == 0u) s_cnt[wave] = stage.count;
  __syncthreads();
  if (threadIdx.x == 0u) {
    uint32_t tot = 0;
    for (uint32_t w = 0; w < BFS_WAVES; ++w) tot += s_cnt[w];
    s_base = tot ? atomicAdd(cnt_out, tot) : 0u;
  }
  __syncthreads();
  uint32_t off = s_base;
  for (uint32_t w = 0; w < wave; ++w) off += s_cnt[w];
  for (uint32_t i = lane; i < stage.count; i += 64u) q_out[off + i] = stage.buf[i];
}

// one workgroup per 1024 vertices, between 8 and 2048 workgroups
uint32_t blocks_for(uint32_t n) {
  uint32_t b = (n + 1023u) / 1024u;
  if (b < 8u) b = 8u;
  if (b > 2048u) b = 2048u;
  return (b + 7u) / 8u * 8u;
}

}  // namespace

extern "C" {

uint64_t mgb_bfs_work_bytes(uint32_t n) {
  return ctrl_bytes() + 2ull * (((uint64_t)n * 4 + 255) / 256 * 256);
}

int mgb_bfs_probe(uint32_t n, uint64_t m, uint64_t* mem_bytes, mgb_dim3* grid, mgb_dim3* block) {
  if (!mem_bytes || !grid || !block) return MGB_E_INVAL;
  if (n == 0u || n > 0x7fffffffu || m > 0x7fffffffull) return MGB_E_UNSUPPORTED;
  *mem_bytes = ((uint64_t)n + 1 + m) * 4 + (uint64_t)n * 4 + mgb_bfs_work_bytes(n);
  *grid = mgb_dim3{blocks_for(n), 1u, 1u};
  *block = mgb_dim3{BFS_THREADS, 1u, 1u};
  return MGB_OK;
}

static int bfs_run(void* stream, const int32_t* row_ptr, const int32_t* col_idx, uint32_t n,
                   uint32_t source, int32_t* level, void* work, uint32_t* depth, uint32_t symmetric) {
  if (!row_ptr || !col_idx || !level || !work) return MGB_E_INVAL;
  if (n == 0u || n > 0x7fffffffu || source >= n) return MGB_E_INVAL;
  if ((uintptr_t)work & 255u) return MGB_E_INVAL;
  hipStream_t st = (hipStream_t)stream;
  const Work w = carve(work, n);
  const uint32_t blocks = blocks_for(n);
  hipLaunchKernelGGL(bfs_init, dim3(blocks), dim3(BFS_THREADS), 0, st, level, n, source, w.queue[0],
                     w.ctrl);
  uint32_t levels_done = 0;
  uint32_t host_counts[BFS_BATCH + 1];
  for (;;) {
    for (uint32_t j = 0; j < BFS_BATCH; ++j)
      hipLaunchKernelGGL(bfs_level, dim3(blocks), dim3(BFS_THREADS), 0, st, row_ptr, col_idx, level,
                         w.queue[j & 1u], w.queue[(j + 1u) & 1u], w.ctrl, j,
                         (int32_t)(levels_done + j + 1u), n, symmetric);
    int rc = mgb_check_launch("bfs_level");
    if (rc != MGB_OK) return rc;
    hipError_t e = hipMemcpyAsync(host_counts, w.ctrl, sizeof host_counts, hipMemcpyDeviceToHost, st);
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
    hipLaunchKernelGGL(bfs_roll, dim3(1), dim3(64), 0, st, w.ctrl);
  }
}

int mgb_bfs_enqueue(void* stream, const int32_t* row_ptr, const int32_t* col_idx, uint32_t n,
                    uint32_t source, int32_t* level, void* work, uint32_t* depth) {
  return bfs_run(stream, row_ptr, col_idx, n, source, level, work, depth, 1u);
}

int mgb_bfs_directed_enqueue(void* stream, const int32_t* row_ptr, const int32_t* col_idx, uint32_t n,
                             uint32_t source, int32_t* level, void* work, uint32_t* depth) {
  return bfs_run(stream, row_ptr, col_idx, n, source, level, work, depth, 0u);
}

}  // extern "C"
