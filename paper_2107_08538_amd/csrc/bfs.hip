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
//   * bottom-up (frontier large against what is still unvisited): one lane
//     per unvisited vertex scans its own adjacency list until it meets a
//     vertex of the current frontier; no atomics on level[], early exit.
//     Frontier membership is a bitmap (one bit per vertex, three of them in
//     rotation: read / written / cleared by a level); for graphs of up to
//     2^20 vertices every workgroup first copies it into LDS (128 KiB), so
//     the probes - the bulk of the work - never leave the CU.  On the level
//     where the frontier explodes (three quarters of a 256-vertex span still
//     unvisited) the span's rows are read edge-parallel instead, as one
//     contiguous piece of col_idx, and each vertex tests its row's bits.  Top-down
//     levels set the bits of what they discover with one more atomic each;
//     bottom-up levels own whole bitmap words and store them.
// Either way the new frontier is staged per wave in LDS (ballot of the winners,
// each winner writes at its rank among them) and appended to the next queue
// with one atomic on the queue tail per workgroup, or per full staging buffer.
//
// The host does not know the depth in advance: it enqueues a batch of level
// kernels whose grids do not depend on the frontier size (the kernels read the
// size from device memory and exit at once on an empty frontier), then reads
// the per-level counters back once per batch (8 levels, then 4, 8, 16, then 32 at a
// time; the read-back polls the stream rather than sleeping on it).
#include "../../include/mgb.h"
#include "launch_util.h"

#include <hip/hip_runtime.h>

#include <chrono>
#include <mutex>
#include <type_traits>

namespace {

constexpr uint32_t BFS_THREADS = 512;
constexpr uint32_t BFS_WAVES = BFS_THREADS / 64;
constexpr uint32_t BFS_BATCH0 = 8;            // levels before the first host round trip
constexpr uint32_t BFS_BATCH1 = 4;            // levels of the second batch, doubled after each
constexpr uint32_t BFS_BATCH = 32;            // up to this many (all even: keeps queue parity)
constexpr uint32_t BFS_CUM = BFS_BATCH + 1;   // control word: vertices reached before this batch's first frontier
constexpr uint32_t BFS_BU_SPAN = 256;         // vertices a wave scans per bottom-up pass (4 per lane)
constexpr uint32_t BFS_BU_UNROLL = 8;         // neighbours per unvisited vertex in flight (bottom-up)
constexpr uint32_t BFS_LDS_BITS = 1u << 20;   // the frontier bitmap is kept in LDS up to this many vertices
constexpr float BFS_TD_WEIGHT = 4.f;          // LDS bitmap: cost of a top-down edge (probe + claim) against reading one unvisited vertex's row
struct __attribute__((packed, aligned(4))) Int4 { int32_t v[4]; };   // four consecutive column indices
static_assert(BFS_BU_UNROLL % 4u == 0u, "neighbours are fetched four at a time");
constexpr uint32_t BFS_DENSE_BITS = BFS_BU_SPAN * 32u;   // edges of a span read edge-parallel (one bit each in the list's LDS)
constexpr uint32_t BFS_DENSE_BATCH = 16;      // loads per lane in flight on that path
static_assert((BFS_DENSE_BITS / 64u) % BFS_DENSE_BATCH == 0u, "whole batches fit the bit array");
constexpr uint32_t BFS_UNROLL = 4;            // edges per lane in flight (top-down)
constexpr uint32_t BFS_STAGE = 512;           // per-wave LDS staging of discovered vertices

typedef int32_t i32x4_u __attribute__((ext_vector_type(4), aligned(4)));

struct Work {                                  // layout of the caller's scratch buffer
  uint32_t* ctrl;                              // [0..BATCH] frontier sizes of the batch, [BFS_CUM] see above
  int32_t* queue[2];                           // n entries each
  uint32_t* bitmap[3];                         // one bit per vertex each
  uint32_t words;                              // 32-bit words per bitmap (a multiple of 64)
};

constexpr uint64_t ctrl_bytes() { return 256; }
constexpr uint64_t work_bytes(uint64_t n) {
  return ctrl_bytes() + 2ull * ((n * 4 + 255) / 256 * 256) + 3ull * (((n + 31) / 32 + 63) / 64 * 64) * 4;
}

// Scratch of the entry point that allocates nothing: queues, bitmaps and counters of one
// traversal of up to BFS_STATIC_MAX_N vertices, held by every device the library runs on until
// the process ends.  In host code this name is only a handle for hipGetSymbolAddress: the
// device address it yields (one per device) is what kernels and copies are given.
constexpr uint32_t BFS_STATIC_MAX_N = 1u << 22;
constexpr uint64_t BFS_STATIC_BYTES = work_bytes(BFS_STATIC_MAX_N);      // 33.5 MiB
__device__ __align__(256) unsigned char scratch[BFS_STATIC_BYTES];
constexpr int BFS_MAX_DEVICES = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[BFS_MAX_DEVICES] = {};

Work carve(void* work, uint32_t n) {
  Work w;
  char* p = (char*)work;
  w.ctrl = (uint32_t*)p;
  p += ctrl_bytes();
  w.queue[0] = (int32_t*)p;
  p += ((uint64_t)n * 4 + 255) / 256 * 256;
  w.queue[1] = (int32_t*)p;
  p += ((uint64_t)n * 4 + 255) / 256 * 256;
  w.words = (uint32_t)((((uint64_t)n + 31) / 32 + 63) / 64 * 64);
  for (int i = 0; i < 3; ++i) {
    w.bitmap[i] = (uint32_t*)p;
    p += (uint64_t)w.words * 4;
  }
  return w;
}

__global__ __launch_bounds__(BFS_THREADS) void bfs_init(int32_t* __restrict__ level, uint32_t n,
                                                       uint32_t source, int32_t* __restrict__ q0,
                                                       uint32_t* __restrict__ ctrl,
                                                       uint32_t* __restrict__ bitmaps, uint32_t words) {
  const uint32_t stride = gridDim.x * BFS_THREADS;
  for (uint32_t v = blockIdx.x * BFS_THREADS + threadIdx.x; v < n; v += stride)
    level[v] = (v == source) ? 0 : -1;
  // the three bitmaps are contiguous; the first is the frontier of level 0
  for (uint32_t i = blockIdx.x * BFS_THREADS + threadIdx.x; i < 3u * words; i += stride)
    bitmaps[i] = i == (source >> 5) ? 1u << (source & 31u) : 0u;
  if (blockIdx.x == 0 && threadIdx.x <= BFS_CUM) ctrl[threadIdx.x] = threadIdx.x == 0 ? 1u : 0u;
  if (blockIdx.x == 0 && threadIdx.x == 0) q0[0] = (int32_t)source;
}

// start of the next batch: its first frontier is the last one of the previous batch of nb levels
__global__ void bfs_roll(uint32_t* __restrict__ ctrl, uint32_t nb) {
  const uint32_t t = threadIdx.x;
  uint32_t carry = ctrl[nb];
  uint32_t cum = ctrl[BFS_CUM];
  for (uint32_t i = 0; i < nb; ++i) cum += ctrl[i];
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

__global__ __launch_bounds__(BFS_THREADS, 2) void bfs_level(const int32_t* __restrict__ row_ptr,
                                                        const int32_t* __restrict__ col_idx,
                                                        int32_t* __restrict__ level,
                                                        const int32_t* __restrict__ q_in,
                                                        int32_t* __restrict__ q_out,
                                                        uint32_t* __restrict__ ctrl, uint32_t j,
                                                        int32_t next_level, uint32_t n,
                                                        uint32_t symmetric,
                                                        const uint32_t* __restrict__ bm_in,
                                                        uint32_t* __restrict__ bm_out,
                                                        uint32_t* __restrict__ bm_clr, uint32_t words) {
  extern __shared__ __attribute__((aligned(16))) uint32_t s_bitmap[];   // `words` entries when n <= BFS_LDS_BITS, else none
  __shared__ uint32_t s_excl[BFS_WAVES][64];
  __shared__ int32_t s_start[BFS_WAVES][64];
  __shared__ int32_t s_stage[BFS_WAVES][BFS_STAGE];
  __shared__ int32_t s_list[BFS_WAVES][BFS_BU_SPAN];
  __shared__ uint32_t s_out[BFS_WAVES][BFS_BU_SPAN / 32u];
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
  // the bitmap this level's successor will write must be empty by then
  if (symmetric != 0u)
    for (uint32_t i = blockIdx.x * BFS_THREADS + threadIdx.x; i < words; i += gridDim.x * BFS_THREADS) bm_clr[i] = 0u;
  const bool in_lds = n <= BFS_LDS_BITS;

  // Top-down touches about n_in * (m/n) edges, each a random probe of level[] and, for most, an
  // atomic claim.  Bottom-up reads level[] once and the row of every unvisited vertex; with the
  // bitmap in LDS its probes are almost free, otherwise an unvisited vertex makes about n/n_in
  // of them through L2 before it meets the frontier.  Go bottom-up when top-down costs more.
  const int32_t m_edges = row_ptr[n];     // number of stored (directed) edges
  const float m = (float)m_edges;
  const float td_edges_n = (float)n_in * m;                     // top-down edges, times n
  const bool bottom_up = in_lds ? BFS_TD_WEIGHT * td_edges_n > (float)unvisited * (float)n
                                : td_edges_n * (float)n_in > (float)unvisited * (float)n * (float)n;
  // (bottom-up reads a vertex's stored edges as its in-edges: only right for a symmetric graph)
  if (symmetric != 0u && bottom_up && m_edges >= (int32_t)BFS_BU_UNROLL) {
    // Most vertices are already reached when this direction pays, so a wave first packs the
    // unvisited ones of its span into LDS (coalesced level reads, ballot ranks) and then works on
    // full lanes: one unvisited vertex per lane, eight of its neighbours in flight per step,
    // until one of them is in the frontier or the list ends.
    // (a handful of unvisited vertices do not pay for the copy: they probe the bitmap in memory)
    const bool copy = in_lds && (uint64_t)unvisited * 64u >= n;
    if (copy) {
      typedef uint32_t Quad __attribute__((ext_vector_type(4)));
      const Quad* src = reinterpret_cast<const Quad*>(bm_in);
      Quad* dst = reinterpret_cast<Quad*>(s_bitmap);
      // (eight loads in flight per lane: written as a plain loop the compiler waits for each
      // load before its LDS store, sixteen memory round trips for the 128 KiB bitmap)
      const uint32_t quads = words / 4u;          // > 0, a multiple of 16
      for (uint32_t base = 0; base < quads; base += 8u * BFS_THREADS) {
        Quad t[8];            // (lanes past the end copy the last quad once more: no branches)
#pragma unroll
        for (uint32_t k = 0; k < 8u; ++k) t[k] = src[min(base + k * BFS_THREADS + threadIdx.x, quads - 1u)];
#pragma unroll
        for (uint32_t k = 0; k < 8u; ++k) dst[min(base + k * BFS_THREADS + threadIdx.x, quads - 1u)] = t[k];
      }
      __syncthreads();
    }
    // (two instantiations of the loop: a pointer that may be LDS or memory would turn every probe
    // into a flat load)
    // The loads below are unconditional (indices clamped into the arrays, results masked): a
    // load under a per-lane condition becomes a branch, and the compiler then waits for every
    // load before it issues the next.
    int32_t* list = &s_list[wave][0];
    const int32_t last_block = m_edges - (int32_t)BFS_BU_UNROLL;   // >= 0: see the choice of direction
    // one round for the first NQ * 64 entries of the list: NQ vertices per lane, eight neighbours
    // of each in flight
    auto rounds = [&](auto lds_probe, auto nq_tag, uint32_t v0, uint32_t cnt) {
      constexpr bool LDS_PROBE = decltype(lds_probe)::value;
      constexpr uint32_t NQ = decltype(nq_tag)::value;
      int32_t vq[NQ], e[NQ], e1[NQ];
      bool open[NQ], found[NQ];
#pragma unroll
      for (uint32_t q = 0; q < NQ; ++q) {
        open[q] = 64u * q + lane < cnt;
        vq[q] = list[min(64u * q + lane, BFS_BU_SPAN - 1u)];
        if (!open[q]) vq[q] = 0;
        found[q] = false;
      }
#pragma unroll
      for (uint32_t q = 0; q < NQ; ++q) {
        e[q] = row_ptr[vq[q]];
        e1[q] = row_ptr[vq[q] + 1];
      }
#pragma unroll
      for (uint32_t q = 0; q < NQ; ++q) open[q] = open[q] && e[q] < e1[q];
      for (;;) {
        bool any_open = false;
#pragma unroll
        for (uint32_t q = 0; q < NQ; ++q) any_open |= open[q];
        if (!__any(any_open)) break;
        // (16-byte loads that need only 4-byte alignment: a lane's eight neighbours are two memory
        // instructions instead of eight, and it is the number of cache-line requests of these
        // row-per-lane gathers, not their bytes, that bounds this loop)
        int32_t nb[NQ][BFS_BU_UNROLL], b0[NQ];
#pragma unroll
        for (uint32_t q = 0; q < NQ; ++q) {
          b0[q] = min(e[q], last_block);
#pragma unroll
          for (uint32_t i = 0; i < BFS_BU_UNROLL; i += 4u) {
            const Int4 four = *reinterpret_cast<const Int4*>(col_idx + b0[q] + (int32_t)i);
#pragma unroll
            for (uint32_t k = 0; k < 4u; ++k) nb[q][i + k] = four.v[k];
          }
        }
        uint32_t word[NQ][BFS_BU_UNROLL];
#pragma unroll
        for (uint32_t q = 0; q < NQ; ++q)
#pragma unroll
          for (uint32_t i = 0; i < BFS_BU_UNROLL; ++i)
            word[q][i] = LDS_PROBE ? s_bitmap[(uint32_t)nb[q][i] >> 5] : bm_in[(uint32_t)nb[q][i] >> 5];
#pragma unroll
        for (uint32_t q = 0; q < NQ; ++q) {
          uint32_t hit = 0u;
#pragma unroll
          for (uint32_t i = 0; i < BFS_BU_UNROLL; ++i)
            hit |= (word[q][i] >> ((uint32_t)nb[q][i] & 31u)) &
                   (uint32_t)(b0[q] + (int32_t)i >= e[q] && b0[q] + (int32_t)i < e1[q]);
          hit &= (uint32_t)open[q];
          e[q] += (int32_t)BFS_BU_UNROLL;
          found[q] = found[q] || hit != 0u;
          open[q] = open[q] && hit == 0u && e[q] < e1[q];
        }
      }
#pragma unroll
      for (uint32_t q = 0; q < NQ; ++q) {
        if (found[q]) {
          level[vq[q]] = next_level;
          atomicOr(&s_out[wave][((uint32_t)vq[q] - v0) >> 5], 1u << ((uint32_t)vq[q] & 31u));
        }
        stage_append(stage, found[q], vq[q], q_out, cnt_out, lane);
      }
    };
    // (two instantiations per width: a pointer that may be LDS or memory would turn every probe
    // into a flat load)
    // While most vertices are still unvisited (the level on which the frontier explodes) the
    // rows of a span are one almost contiguous piece of col_idx.  A span of which at least three
    // quarters are unvisited is then read edge-parallel: lane l takes edges l, 64 + l, ... of the
    // piece (coalesced, no dependent rounds, up to 16 loads in flight), a ballot per load leaves
    // one bit per edge in LDS (the list's storage: 8192 bits), and each unvisited vertex tests
    // the bits of its own row.  Rows of visited vertices are read too and their bits ignored.
    const bool dense_level = (uint64_t)unvisited * 4u >= (uint64_t)n * 3u;
    auto scan = [&](auto lds_probe) {
    constexpr bool LDS_PROBE = decltype(lds_probe)::value;
    constexpr uint32_t Q = BFS_BU_SPAN / 64u;
    for (uint32_t v0 = gwave * BFS_BU_SPAN; v0 < n; v0 += total_waves * BFS_BU_SPAN) {
      int32_t lv[Q], row0[Q], row1[Q];
#pragma unroll
      for (uint32_t u = 0; u < Q; ++u) lv[u] = level[min(v0 + 64u * u + lane, n - 1u)];
#pragma unroll
      for (uint32_t u = 0; u < Q; ++u) {
        row0[u] = row1[u] = 0;
        if (dense_level) {                 // uniform over the grid
          const uint32_t v = min(v0 + 64u * u + lane, n - 1u);
          row0[u] = row_ptr[v];
          row1[u] = row_ptr[v + 1u];
        }
      }
      const int32_t piece_end = dense_level ? row_ptr[min(v0 + BFS_BU_SPAN, n)] : 0;
      uint32_t cnt = 0;
      bool unv[Q];
      uint64_t unv_mask[Q];
#pragma unroll
      for (uint32_t u = 0; u < Q; ++u) {
        unv[u] = lv[u] < 0 && v0 + 64u * u + lane < n;
        unv_mask[u] = __ballot(unv[u]);
        cnt += (uint32_t)__popcll(unv_mask[u]);
      }
      bool dense = false;
      int32_t bit0 = 0;                    // the piece of col_idx: [bit0, piece_end), bit0 a multiple of 64
      if (dense_level && cnt * 4u >= BFS_BU_SPAN * 3u) {
        bit0 = __builtin_amdgcn_readfirstlane(row0[0]) & ~63;
        dense = piece_end - bit0 <= (int32_t)BFS_DENSE_BITS;
      }
      if (dense) {
        uint32_t* hits = reinterpret_cast<uint32_t*>(list);
        const uint32_t loads = (uint32_t)(piece_end - bit0 + 63) >> 6;      // <= BFS_DENSE_BITS / 64
        // (the next batch's loads are issued before this batch is probed)
        int32_t nb[BFS_DENSE_BATCH], ahead[BFS_DENSE_BATCH];
#pragma unroll
        for (uint32_t i = 0; i < BFS_DENSE_BATCH; ++i)
          ahead[i] = col_idx[min((uint32_t)bit0 + i * 64u + lane, (uint32_t)m_edges - 1u)];
        for (uint32_t r0 = 0; r0 < loads; r0 += BFS_DENSE_BATCH) {
          uint32_t word[BFS_DENSE_BATCH];
#pragma unroll
          for (uint32_t i = 0; i < BFS_DENSE_BATCH; ++i) nb[i] = ahead[i];
#pragma unroll
          for (uint32_t i = 0; i < BFS_DENSE_BATCH; ++i)
            ahead[i] = col_idx[min((uint32_t)bit0 + (r0 + BFS_DENSE_BATCH + i) * 64u + lane, (uint32_t)m_edges - 1u)];
#pragma unroll
          for (uint32_t i = 0; i < BFS_DENSE_BATCH; ++i)
            word[i] = LDS_PROBE ? s_bitmap[(uint32_t)nb[i] >> 5] : bm_in[(uint32_t)nb[i] >> 5];
#pragma unroll
          for (uint32_t i = 0; i < BFS_DENSE_BATCH; ++i) {
            const uint64_t hit = __ballot(((word[i] >> ((uint32_t)nb[i] & 31u)) & 1u) != 0u);
            if (lane == 0u) {
              hits[2u * (r0 + i)] = (uint32_t)hit;
              hits[2u * (r0 + i) + 1u] = (uint32_t)(hit >> 32);
            }
          }
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (uint32_t u = 0; u < Q; ++u) {
          bool found = false;
          const uint32_t s = (uint32_t)(row0[u] - bit0), t = (uint32_t)(row1[u] - bit0);
          if (unv[u] && s < t) {
            const uint32_t w0 = s >> 5, w1 = (t - 1u) >> 5;
            uint32_t any = 0u;
            for (uint32_t w = w0; w <= w1; ++w) {
              uint32_t m = 0xffffffffu;
              if (w == w0) m &= 0xffffffffu << (s & 31u);
              if (w == w1) m &= 0xffffffffu >> (31u - ((t - 1u) & 31u));
              any |= hits[w] & m;
            }
            found = any != 0u;
          }
          const int32_t v = (int32_t)(v0 + 64u * u + lane);
          if (found) level[v] = next_level;
          const uint64_t fm = __ballot(found);
          if (lane == 0u) {
            s_out[wave][2u * u] = (uint32_t)fm;
            s_out[wave][2u * u + 1u] = (uint32_t)(fm >> 32);
          }
          stage_append(stage, found, v, q_out, cnt_out, lane);
        }
      } else {
        uint32_t at = 0;
#pragma unroll
        for (uint32_t u = 0; u < Q; ++u) {
          if (unv[u]) list[at + __popcll(unv_mask[u] & ((1ull << lane) - 1ull))] = (int32_t)(v0 + 64u * u + lane);
          at += (uint32_t)__popcll(unv_mask[u]);
        }
        if (lane < BFS_BU_SPAN / 32u) s_out[wave][lane] = 0u;
        __builtin_amdgcn_wave_barrier();
        if (cnt > 128u) rounds(lds_probe, std::integral_constant<uint32_t, 4>{}, v0, cnt);
        else if (cnt > 64u) rounds(lds_probe, std::integral_constant<uint32_t, 2>{}, v0, cnt);
        else if (cnt > 0u) rounds(lds_probe, std::integral_constant<uint32_t, 1>{}, v0, cnt);
      }
      __builtin_amdgcn_wave_barrier();
      // the span's bitmap words belong to this wave alone (v0 is a multiple of 256)
      if (lane < BFS_BU_SPAN / 32u && (v0 >> 5) + lane < words) bm_out[(v0 >> 5) + lane] = s_out[wave][lane];
    }
    };
    if (copy) scan(std::true_type{}); else scan(std::false_type{});
  } else {

  // top-down.  Small frontiers are split into chunks of fewer than 64 vertices so that
  // every wave of the grid gets some of the edges.
  const bool look_first = (uint64_t)reached * 8u >= n;       // uniform over the grid
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
      // (unconditional loads, edge index clamped and the result masked: see bottom-up)
      int32_t nb[BFS_UNROLL];
      bool live[BFS_UNROLL];
#pragma unroll
      for (uint32_t u = 0; u < BFS_UNROLL; ++u) {
        const uint32_t e = min(e0 + 64u * u + lane, total - 1u);
        live[u] = e0 + 64u * u + lane < total;
        // owner = last lane whose exclusive prefix is <= e
        uint32_t lo = 0, hi = 63;
#pragma unroll
        for (int it = 0; it < 6; ++it) {
          const uint32_t mid = (lo + hi + 1u) >> 1;
          const bool up = s_excl[wave][mid] <= e;
          lo = up ? mid : lo;
          hi = up ? hi : mid - 1u;
        }
        nb[u] = col_idx[s_start[wave][lo] + (int32_t)(e - s_excl[wave][lo])];
      }
      // (while few vertices are reached nearly every neighbour is new: the claim goes out at once,
      // without the round trip of looking first)
      int32_t seen[BFS_UNROLL];
#pragma unroll
      for (uint32_t u = 0; u < BFS_UNROLL; ++u) seen[u] = -1;
      if (look_first) {
#pragma unroll
        for (uint32_t u = 0; u < BFS_UNROLL; ++u) seen[u] = level[nb[u]];
      }
#pragma unroll
      for (uint32_t u = 0; u < BFS_UNROLL; ++u) {
        bool won = false;
        if (live[u] && seen[u] < 0) won = atomicCAS(&level[nb[u]], -1, next_level) == -1;
        if (won && symmetric != 0u) atomicOr(&bm_out[(uint32_t)nb[u] >> 5], 1u << ((uint32_t)nb[u] & 31u));
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

// one workgroup per 4096 vertices, between 8 and 512 workgroups
uint32_t blocks_for(uint32_t n) {
  uint32_t b = (n + 4095u) / 4096u;
  if (b < 8u) b = 8u;
  if (b > 512u) b = 512u;
  return (b + 7u) / 8u * 8u;
}

// dynamic LDS of a level kernel: the frontier bitmap, when it fits
uint32_t lds_bitmap_bytes(uint32_t n, uint32_t words, uint32_t symmetric) {
  return symmetric != 0u && n <= BFS_LDS_BITS ? words * 4u : 0u;
}

}  // namespace

extern "C" {

uint64_t mgb_bfs_work_bytes(uint32_t n) {
  return work_bytes(n);
}

// workgroups of the level kernel that fit one CU: LDS (the frontier bitmap on top of the
// kernel's own 29184 bytes of staging) or registers (the launch bounds hold the kernel to 128
// vector registers per lane: four waves per SIMD, two workgroups of eight waves per CU)
uint32_t mgb_bfs_residency(uint32_t n) {
  if (n == 0u || n > 0x7fffffffu) return 0u;
  const uint32_t words = (uint32_t)((((uint64_t)n + 31) / 32 + 63) / 64 * 64);
  const uint32_t by_lds = (160u * 1024u) / (29184u + lds_bitmap_bytes(n, words, 1u));
  const uint32_t by_regs = 2u;
  return by_lds < by_regs ? by_lds : by_regs;
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
  const uint32_t lds = lds_bitmap_bytes(n, w.words, symmetric);
  static std::once_flag once;
  static hipError_t attr = hipSuccess;
  std::call_once(once, [] {
    attr = hipFuncSetAttribute((const void*)bfs_level, hipFuncAttributeMaxDynamicSharedMemorySize, (int)(BFS_LDS_BITS / 8u));
  });
  if (attr != hipSuccess) {
    mgb_internal_set_error("bfs_level: dynamic LDS size", attr);
    return MGB_E_BACKEND;
  }
  hipLaunchKernelGGL(bfs_init, dim3(blocks), dim3(BFS_THREADS), 0, st, level, n, source, w.queue[0],
                     w.ctrl, w.bitmap[0], w.words);
  uint32_t levels_done = 0, nb = BFS_BATCH0;
  uint32_t host_counts[BFS_BATCH + 1];
  for (;;) {
    for (uint32_t j = 0; j < nb; ++j) {
      const uint32_t lv = levels_done + j;             // bitmap lv % 3 holds frontier lv
      hipLaunchKernelGGL(bfs_level, dim3(blocks), dim3(BFS_THREADS), lds, st, row_ptr, col_idx, level,
                         w.queue[j & 1u], w.queue[(j + 1u) & 1u], w.ctrl, j, (int32_t)(lv + 1u), n,
                         symmetric, w.bitmap[lv % 3u], w.bitmap[(lv + 1u) % 3u], w.bitmap[(lv + 2u) % 3u],
                         w.words);
    }
    int rc = mgb_check_launch("bfs_level");
    if (rc != MGB_OK) return rc;
    hipError_t e = hipMemcpyAsync(host_counts, w.ctrl, (nb + 1u) * sizeof(uint32_t), hipMemcpyDeviceToHost, st);
    // The traversal is a few hundred microseconds of GPU work: poll for the counters instead of
    // sleeping on the stream (a blocking wait wakes up tens of microseconds late), and fall back
    // to the blocking wait if they are not there after a few milliseconds (a deep or huge graph).
    if (e == hipSuccess) {
      const auto t0 = std::chrono::steady_clock::now();
      for (;;) {
        e = hipStreamQuery(st);
        if (e != hipErrorNotReady) break;
        if (std::chrono::steady_clock::now() - t0 > std::chrono::milliseconds(3)) {
          e = hipStreamSynchronize(st);
          break;
        }
      }
      (void)hipGetLastError();     // "not ready" is an answer, not an error to find at the next launch check
    }
    if (e != hipSuccess) {
      mgb_internal_set_error("bfs counter read-back", e);
      return MGB_E_BACKEND;
    }
    // host_counts[j] = size of the frontier at depth levels_done + j
    uint32_t j = 0;
    while (j <= nb && host_counts[j] != 0u) ++j;
    if (j <= nb) {                              // an empty frontier was reached
      if (depth) *depth = levels_done + j;      // number of non-empty levels (source level included)
      return MGB_OK;
    }
    levels_done += nb;
    if (levels_done >= n) return MGB_OK;        // cannot happen: depth < n
    hipLaunchKernelGGL(bfs_roll, dim3(1), dim3(64), 0, st, w.ctrl, nb);
    // A random graph that is not done after eight levels is nearly done (its frontier peaked two or
    // three levels ago): a short second batch spares it a dozen empty launches; a deep graph pays
    // one more round trip on its way to batches of 32
    nb = levels_done == BFS_BATCH0 ? BFS_BATCH1 : (nb < BFS_BATCH ? nb * 2u : nb);
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

// The traversal of mgb_bfs_enqueue with the work area in the library's static device array.
int mgb_bfs_enqueue_static(void* stream, const int32_t* row_ptr, const int32_t* col_idx, uint32_t n,
                           uint32_t source, int32_t* level, uint32_t* depth) {
  if (n > BFS_STATIC_MAX_N) {
    mgb_internal_set_error_text("mgb_bfs_enqueue_static: more than 2^22 vertices do not fit the static work area");
    return MGB_E_TOO_BIG;
  }
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= BFS_MAX_DEVICES) {
    mgb_internal_set_error("mgb_bfs_enqueue_static: hipGetDevice", e == hipSuccess ? hipErrorInvalidDevice : e);
    return MGB_E_BACKEND;
  }
  void* work = nullptr;
  {
    // once per device, with that device current: every device holds its own copy of the array
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
      void* p = nullptr;
      e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (e != hipSuccess || !p) {
        mgb_internal_set_error("mgb_bfs_enqueue_static: hipGetSymbolAddress", e == hipSuccess ? hipErrorInvalidSymbol : e);
        return MGB_E_BACKEND;
      }
      g_scratch_ptr[dev] = p;
    }
    work = g_scratch_ptr[dev];
  }
  // nothing to clear here: bfs_init writes the counters, the first queue entry and all three
  // bitmaps before any level kernel reads them, whatever the previous call left behind
  return bfs_run(stream, row_ptr, col_idx, n, source, level, work, depth, 1u);
}

}  // extern "C"
