// Worker pool that pushes a batch of described tasks through the scheduler (the experimental
// set-up of Sec. V-A of the paper: jobs sit in a queue, a pool of workers each takes a job, runs
// it to its end and pulls the next; jobs are either all queued at the start or arrive over time).
//
// A job here is a task descriptor: which of the library's task kinds, its device buffers and its
// shape.  A worker derives the job's requirements with the kind's probe (footprint = sum of its
// allocations, geometry = its largest launch, Sec. III-A), announces them (mgb_task_probe_ex),
// waits for a placement if it has to, enqueues the kind's kernels on the placement's stream, hands
// the resources back and waits for the kernels.  Everything goes through the public entry points;
// the pool adds no policy.  It exists so that the hand-over between two tasks is a few
// microseconds of native code rather than an interpreter's thread switch.
#include "../../include/mgb.h"
#include "launch_util.h"

#include <algorithm>
#include <atomic>
#include <chrono>
#include <cstring>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

namespace {

uint64_t clock_ns() {
  return (uint64_t)std::chrono::duration_cast<std::chrono::nanoseconds>(
             std::chrono::steady_clock::now().time_since_epoch())
      .count();
}

struct Probe {
  uint64_t mem = 0;
  mgb_dim3 grid{}, block{};
  uint32_t wg_per_cu = 0;
};

int derive(const mgb_task_desc& t, Probe* p) {
  const uint32_t* d = t.dim;
  switch (t.kind) {
    case MGB_TASK_JACOBI:
      p->wg_per_cu = mgb_jacobi_residency(d[0]);
      return mgb_jacobi_probe(d[0], d[1], &p->mem, &p->grid, &p->block);
    case MGB_TASK_GEMM_F32:
      p->wg_per_cu = mgb_gemm_f32_residency(d[0], d[1], d[2]);
      return mgb_gemm_f32_probe(d[0], d[1], d[2], &p->mem, &p->grid, &p->block);
    case MGB_TASK_GEMM_BF16:
      p->wg_per_cu = mgb_gemm_bf16_residency(d[0], d[1], d[2]);
      return mgb_gemm_bf16_probe(d[0], d[1], d[2], &p->mem, &p->grid, &p->block);
    case MGB_TASK_BFS:
      p->wg_per_cu = mgb_bfs_residency(d[0]);
      return mgb_bfs_probe(d[0], t.count, &p->mem, &p->grid, &p->block);
    case MGB_TASK_CNN: {
      uint64_t act = 0, out = 0;
      p->wg_per_cu = mgb_cnn_residency(t.layers, (uint32_t)t.count, d[0], d[1], d[2]);
      return mgb_cnn_probe(t.layers, (uint32_t)t.count, d[0], d[1], d[2], &p->mem, &act, &out, &p->grid, &p->block);
    }
    case MGB_TASK_CUSTOM:
      if (!t.ptr[0]) return MGB_E_INVAL;
      p->mem = t.count;
      p->grid = mgb_dim3{d[0], 1u, 1u};
      p->block = mgb_dim3{d[1], 1u, 1u};
      p->wg_per_cu = d[2];
      return MGB_OK;
    default:
      return MGB_E_INVAL;
  }
}

struct Launch {
  const mgb_task_desc* t;
  uint32_t aux;
};

int enqueue(void* stream, void* user) {
  Launch* l = (Launch*)user;
  const mgb_task_desc& t = *l->t;
  const uint32_t* d = t.dim;
  void* const* p = t.ptr;
  switch (t.kind) {
    case MGB_TASK_JACOBI:
      return mgb_jacobi_enqueue(stream, (float*)p[0], (float*)p[1], d[0], d[1]);
    case MGB_TASK_GEMM_F32:
      return mgb_gemm_f32_enqueue(stream, (const float*)p[0], (const float*)p[1], (float*)p[2], d[0], d[1], d[2]);
    case MGB_TASK_GEMM_BF16:
      return mgb_gemm_bf16_enqueue(stream, (const uint16_t*)p[0], (const uint16_t*)p[1], (float*)p[2], d[0], d[1], d[2]);
    case MGB_TASK_BFS:
      return mgb_bfs_enqueue(stream, (const int32_t*)p[0], (const int32_t*)p[1], d[0], d[1], (int32_t*)p[2], p[3], &l->aux);
    case MGB_TASK_CNN:
      return mgb_cnn_enqueue(stream, t.layers, (uint32_t)t.count, (const uint16_t*)p[0], t.weights, (uint16_t*)p[1],
                             (uint16_t*)p[2], (float*)p[3], d[0], d[1], d[2]);
    case MGB_TASK_CUSTOM:
      return ((int (*)(void*, void*))p[0])(stream, p[1]);
    default:
      return MGB_E_INVAL;
  }
}

}  // namespace

extern "C" int mgb_pool_run(mgb_sched* s, const mgb_task_desc* tasks, uint32_t n, uint32_t n_workers,
                            uint32_t flags, mgb_pool_result* results, uint64_t* start_ns) {
  if (!s || (!tasks && n) || (!results && n)) return MGB_E_INVAL;
  if (n == 0u) return MGB_OK;
  if (n_workers == 0u || n_workers > 1024u) return MGB_E_INVAL;
  n_workers = std::min(n_workers, n);
  const bool arrivals = (flags & MGB_POOL_ARRIVALS) != 0u;
  const bool on_stream = (flags & MGB_POOL_RELEASE_ON_STREAM) != 0u;
  std::vector<Probe> probes(n);
  for (uint32_t i = 0; i < n; ++i) {
    std::memset(&results[i], 0, sizeof results[i]);
    const int rc = derive(tasks[i], &probes[i]);
    if (rc != MGB_OK) return rc;                 // nothing has run
  }
  // jobs are taken in arrival order (ties: in the order given)
  std::vector<uint32_t> order(n);
  for (uint32_t i = 0; i < n; ++i) order[i] = i;
  if (arrivals)
    std::stable_sort(order.begin(), order.end(),
                     [&](uint32_t a, uint32_t b) { return tasks[a].arrival_ns < tasks[b].arrival_ns; });
  std::vector<mgb_placement> placed(n);
  std::vector<int> probe_rc(n, MGB_OK);
  const uint64_t t0 = clock_ns();
  if (start_ns) *start_ns = t0;
  // all jobs queued at the start and a worker for each: the probes go out in the order given,
  // before anything runs, so that the queue the scheduler sees is the batch queue
  const bool pre_probed = !arrivals && n_workers >= n;
  if (pre_probed)
    for (uint32_t i = 0; i < n; ++i) {
      results[i].arrival_ns = t0;
      probe_rc[i] = mgb_task_probe_ex(s, tasks[i].task_id, probes[i].mem, probes[i].grid, probes[i].block,
                                      probes[i].wg_per_cu, &placed[i]);
    }
  std::atomic<uint32_t> cursor{0};
  std::mutex err_mu;
  std::string first_error;

  auto run_one = [&](uint32_t i) {
    mgb_pool_result& r = results[i];
    int rc;
    if (pre_probed) {
      rc = probe_rc[i];
    } else {
      r.arrival_ns = t0 + (arrivals ? tasks[i].arrival_ns : 0u);
      if (arrivals) {
        // (a sleep overshoots by 50-100 us: sleep short of the arrival, then yield up to it)
        for (;;) {
          const uint64_t now = clock_ns();
          if (now >= r.arrival_ns) break;
          const uint64_t left = r.arrival_ns - now;
          if (left > 400000u) std::this_thread::sleep_for(std::chrono::nanoseconds(left - 200000u));
          else std::this_thread::yield();
        }
      }
      rc = mgb_task_probe_ex(s, tasks[i].task_id, probes[i].mem, probes[i].grid, probes[i].block,
                             probes[i].wg_per_cu, &placed[i]);
    }
    if (rc == MGB_WAIT) rc = mgb_task_wait(s, placed[i].ticket, -1, &placed[i]);
    r.ticket = placed[i].ticket;
    if (rc != MGB_OK) {                          // MGB_E_OOM under the memory-blind policy: the job is lost
      r.status = rc;
      return;
    }
    Launch l{&tasks[i], 0u};
    rc = mgb_task_launch(s, r.ticket, enqueue, &l);
    int rc2;
    if (on_stream) {
      rc2 = mgb_task_complete_on_stream(s, r.ticket);
      const int rc3 = mgb_task_sync(s, r.ticket, nullptr);
      if (rc2 == MGB_OK) rc2 = rc3;
    } else {
      rc2 = mgb_task_sync(s, r.ticket, nullptr);
      const int rc3 = mgb_task_complete(s, r.ticket);
      if (rc2 == MGB_OK) rc2 = rc3;
    }
    r.status = rc != MGB_OK ? rc : rc2;
    r.aux = l.aux;
    if (r.status == MGB_E_BACKEND) {
      std::lock_guard<std::mutex> lk(err_mu);
      if (first_error.empty()) first_error = mgb_last_error();
    }
  };
  auto worker = [&](uint32_t w) {
    if (pre_probed) {
      run_one(w);
      return;
    }
    for (;;) {
      const uint32_t k = cursor.fetch_add(1u);
      if (k >= n) return;
      run_one(order[k]);
    }
  };
  std::vector<std::thread> pool;
  pool.reserve(n_workers);
  for (uint32_t w = 0; w < n_workers; ++w) pool.emplace_back(worker, w);
  for (std::thread& th : pool) th.join();
  // what the scheduler recorded of each task
  int worst = MGB_OK;
  for (uint32_t i = 0; i < n; ++i) {
    mgb_pool_result& r = results[i];
    if (r.ticket != 0u && mgb_task_records(s, r.ticket, &r.record, 1) == 1 && r.record.ticket == r.ticket) {
      if (r.status == MGB_E_OOM) r.record.status = MGB_E_OOM;
    } else {
      r.record.status = r.status == MGB_OK ? MGB_WAIT : r.status;
    }
    if (r.status < 0 && r.status != MGB_E_OOM && worst == MGB_OK) worst = r.status;
  }
  if (worst == MGB_E_BACKEND && !first_error.empty()) mgb_internal_set_error_text(first_error.c_str());
  return worst;
}
