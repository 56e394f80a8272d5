// Host-only stress of the scheduler core, the lazy runtime and the multi-process front end on the
// null backend: many threads, random probes / waits / cancels / growths / completions, shared
// runtimes and shared connections.  Built with ThreadSanitizer (and with AddressSanitizer +
// UBSan) by tests/test_sanitizers_host.py; a data race, a leak or a failed check fails the test.
#include "../../include/mgb.h"
#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <thread>
#include <vector>
#include <unistd.h>
#include <string>

// The worker pool dispatches to the task kernels, which are GPU code and not part of this build:
// stand-ins that refuse every shape (the pool is driven with caller-defined jobs below).
extern "C" {
uint32_t mgb_jacobi_residency(uint32_t) { return 0; }
uint32_t mgb_gemm_f32_residency(uint32_t, uint32_t, uint32_t) { return 0; }
uint32_t mgb_gemm_bf16_residency(uint32_t, uint32_t, uint32_t) { return 0; }
uint32_t mgb_bfs_residency(uint32_t) { return 0; }
uint32_t mgb_cnn_residency(const mgb_conv_layer*, uint32_t, uint32_t, uint32_t, uint32_t) { return 0; }
int mgb_jacobi_probe(uint32_t, uint32_t, uint64_t*, mgb_dim3*, mgb_dim3*) { return MGB_E_UNSUPPORTED; }
int mgb_gemm_f32_probe(uint32_t, uint32_t, uint32_t, uint64_t*, mgb_dim3*, mgb_dim3*) { return MGB_E_UNSUPPORTED; }
int mgb_gemm_bf16_probe(uint32_t, uint32_t, uint32_t, uint64_t*, mgb_dim3*, mgb_dim3*) { return MGB_E_UNSUPPORTED; }
int mgb_bfs_probe(uint32_t, uint64_t, uint64_t*, mgb_dim3*, mgb_dim3*) { return MGB_E_UNSUPPORTED; }
int mgb_cnn_probe(const mgb_conv_layer*, uint32_t, uint32_t, uint32_t, uint32_t, uint64_t*, uint64_t*, uint64_t*, mgb_dim3*,
                  mgb_dim3*) { return MGB_E_UNSUPPORTED; }
int mgb_jacobi_enqueue(void*, float*, float*, uint32_t, uint32_t) { return MGB_E_UNSUPPORTED; }
int mgb_gemm_f32_enqueue(void*, const float*, const float*, float*, uint32_t, uint32_t, uint32_t) { return MGB_E_UNSUPPORTED; }
int mgb_gemm_bf16_enqueue(void*, const uint16_t*, const uint16_t*, float*, uint32_t, uint32_t, uint32_t) { return MGB_E_UNSUPPORTED; }
int mgb_bfs_enqueue(void*, const int32_t*, const int32_t*, uint32_t, uint32_t, int32_t*, void*, uint32_t*) { return MGB_E_UNSUPPORTED; }
int mgb_cnn_enqueue(void*, const mgb_conv_layer*, uint32_t, const uint16_t*, const uint16_t* const*, uint16_t*, uint16_t*, float*,
                    uint32_t, uint32_t, uint32_t) { return MGB_E_UNSUPPORTED; }
}

#include <hip/hip_runtime.h>
int mgb_internal_tag_partition(hipStream_t, uint32_t, uint32_t) { return 0; }   // (defined beside the GPU diagnostics)

static std::atomic<int> fails{0};
static std::atomic<int> custom_calls{0};
static int custom_enqueue(void*, void*) { ++custom_calls; return 0; }
#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "CHECK failed %s:%d %s\n", __FILE__, __LINE__, #c); ++fails; } } while (0)

int main() {
  mgb_device_desc d;
  mgb_device_desc_default(&d);
  d.backend = MGB_BACKEND_NULL;
  d.granule_cus = 8;
  d.mem_cap_bytes = 100000;
  d.max_running = 16;
  for (uint32_t pol : {MGB_POLICY_HARD, MGB_POLICY_SOFT, MGB_POLICY_SERIAL}) {
    d.policy = pol;
    mgb_sched* s = nullptr;
    CHECK(mgb_sched_create(&d, &s) == MGB_OK);
    std::vector<std::thread> th;
    for (int k = 0; k < 8; ++k)
      th.emplace_back([&, k] {
        std::mt19937 rng(100 + k);
        for (int i = 0; i < 400; ++i) {
          mgb_placement pl;
          uint64_t mem = 1 + rng() % 30000;
          mgb_dim3 g{(uint32_t)(1 + rng() % 4000), 1, 1}, b{(uint32_t)(64u << (rng() % 4)), 1, 1};
          int rc = mgb_task_probe_ex(s, k * 10000 + i, mem, g, b, rng() % 3, &pl);
          if (rc == MGB_WAIT) {
            uint64_t t = pl.ticket;
            if (rng() % 5 == 0) {
              rc = mgb_task_wait(s, t, 1000, &pl);
              if (rc == MGB_TIMEOUT) {
                if (mgb_task_cancel(s, t) == MGB_OK) continue;
                rc = mgb_task_wait(s, t, -1, &pl);
              }
            } else {
              rc = mgb_task_wait(s, t, -1, &pl);
            }
          }
          CHECK(rc == MGB_OK);
          if (rc != MGB_OK) continue;
          if (rng() % 4 == 0) (void)mgb_task_grow(s, pl.ticket, rng() % 2000);
          mgb_stats st;
          CHECK(mgb_sched_stats(s, &st) == MGB_OK);
          uint64_t behind[8];
          CHECK(mgb_task_deps(s, pl.ticket, behind, 8) >= 0);
          // a third of the releases are ordered on the "device"; some of those are never waited for
          const uint32_t how = rng() % 6;
          if (how < 2) {
            CHECK(mgb_task_launch(s, pl.ticket, custom_enqueue, nullptr) == MGB_OK);
            CHECK(mgb_task_complete_on_stream(s, pl.ticket) == MGB_OK);
            if (how == 0) CHECK(mgb_task_sync(s, pl.ticket, nullptr) == MGB_OK);
          } else {
            CHECK(mgb_task_complete(s, pl.ticket) == MGB_OK);
          }
          mgb_task_record one;
          CHECK(mgb_task_records(s, pl.ticket, &one, 1) == 1 && one.ticket == pl.ticket);
        }
      });
    for (auto& t : th) t.join();
    mgb_stats st;
    CHECK(mgb_sched_stats(s, &st) == MGB_OK);
    CHECK(st.free_bytes == d.mem_cap_bytes && st.n_running == 0 && st.n_waiting == 0);
    CHECK(mgb_sched_destroy(s) == MGB_OK);
  }
  // worker pool: three pools at once on one scheduler, caller-defined jobs
  {
    d.policy = MGB_POLICY_HARD;
    mgb_sched* s = nullptr;
    CHECK(mgb_sched_create(&d, &s) == MGB_OK);
    std::vector<std::thread> th;
    for (int k = 0; k < 3; ++k)
      th.emplace_back([&, k] {
        std::mt19937 rng(900 + k);
        const uint32_t n = 60;
        std::vector<mgb_task_desc> jobs(n);
        std::vector<mgb_pool_result> res(n);
        for (uint32_t i = 0; i < n; ++i) {
          jobs[i] = mgb_task_desc{};
          jobs[i].kind = MGB_TASK_CUSTOM;
          jobs[i].task_id = k * 1000 + i;
          jobs[i].arrival_ns = (rng() % 2000) * 1000ull;
          jobs[i].count = 1 + rng() % 30000;
          jobs[i].ptr[0] = (void*)custom_enqueue;
          jobs[i].dim[0] = 1 + rng() % 4000;
          jobs[i].dim[1] = 64u << (rng() % 4);
        }
        const uint32_t flags = (k == 0 ? 0u : MGB_POOL_ARRIVALS) | (k == 2 ? 0u : MGB_POOL_RELEASE_ON_STREAM);
        CHECK(mgb_pool_run(s, jobs.data(), n, k == 0 ? n : 7, flags, res.data(), nullptr) == MGB_OK);
        for (uint32_t i = 0; i < n; ++i) CHECK(res[i].status == MGB_OK && res[i].record.status == MGB_OK);
        mgb_summary sum;
        std::vector<mgb_task_record> recs(n);
        for (uint32_t i = 0; i < n; ++i) recs[i] = res[i].record;
        CHECK(mgb_accounting(recs.data(), n, nullptr, nullptr, &sum) == MGB_OK && sum.n_done == n);
      });
    for (auto& t : th) t.join();
    mgb_stats st;
    CHECK(mgb_sched_stats(s, &st) == MGB_OK);
    CHECK(st.free_bytes == d.mem_cap_bytes && st.n_running == 0 && st.n_waiting == 0);
    CHECK(mgb_sched_destroy(s) == MGB_OK);
  }
  // lazy runtime: threads share one runtime
  {
    d.policy = MGB_POLICY_HARD;
    d.mem_cap_bytes = 40000;
    mgb_sched* s = nullptr;
    CHECK(mgb_sched_create(&d, &s) == MGB_OK);
    mgb_lazy* z = nullptr;
    CHECK(mgb_lazy_create(s, &z) == MGB_OK);
    std::vector<std::thread> th;
    for (int k = 0; k < 6; ++k)
      th.emplace_back([&, k] {
        std::mt19937 rng(7 + k);
        std::vector<uint8_t> buf(8000, (uint8_t)k), out(8000);
        for (int i = 0; i < 150; ++i) {
          uint64_t a = 0, b = 0;
          uint64_t na = 1000 + rng() % 7000, nb = 1000 + rng() % 7000;
          CHECK(mgb_lazy_malloc(z, na, &a) == MGB_OK);
          CHECK(mgb_lazy_malloc(z, nb, &b) == MGB_OK);
          CHECK(mgb_lazy_memcpy_h2d(z, a, buf.data(), na) == MGB_OK);
          CHECK(mgb_lazy_memset(z, b, 3, nb) == MGB_OK);
          uint64_t args[2] = {a, b};
          void* real[2];
          mgb_placement pl;
          int rc = mgb_lazy_launch_prepare(z, k * 1000 + i, args, 2, mgb_dim3{8, 1, 1}, mgb_dim3{64, 1, 1}, 0, -1, real, &pl);
          CHECK(rc == MGB_OK);
          if (rc == MGB_OK) {
            ((uint8_t*)real[1])[0] = ((uint8_t*)real[0])[0];
            CHECK(mgb_lazy_memcpy_d2h(z, out.data(), b, nb) == MGB_OK);
            CHECK(out[0] == (uint8_t)k && (nb < 2 || out[1] == 3));
          }
          CHECK(mgb_lazy_free(z, a) == MGB_OK);
          CHECK(mgb_lazy_free(z, b) == MGB_OK);
        }
      });
    for (auto& t : th) t.join();
    CHECK(mgb_lazy_destroy(z) == MGB_OK);
    CHECK(mgb_sched_destroy(s) == MGB_OK);
  }
  // front end: server + client connections in this process, two threads per connection
  {
    d.mem_cap_bytes = 30000;
    mgb_sched* s = nullptr;
    CHECK(mgb_sched_create(&d, &s) == MGB_OK);
    std::string name = "tsan" + std::to_string((long)getpid());
    mgb_server* sv = nullptr;
    CHECK(mgb_server_start(s, name.c_str(), 4, &sv) == MGB_OK);
    std::vector<mgb_client*> cl(3, nullptr);
    for (auto& c : cl) CHECK(mgb_client_connect(name.c_str(), &c) == MGB_OK);
    std::vector<std::thread> th;
    for (int k = 0; k < 6; ++k)
      th.emplace_back([&, k] {
        mgb_client* c = cl[k % 3];
        std::mt19937 rng(50 + k);
        for (int i = 0; i < 120; ++i) {
          mgb_placement pl;
          int rc = mgb_client_probe(c, k * 1000 + i, 1 + rng() % 12000, mgb_dim3{(uint32_t)(1 + rng() % 500), 1, 1}, mgb_dim3{256, 1, 1}, 0, &pl);
          if (rc == MGB_WAIT) rc = mgb_client_wait(c, pl.ticket, -1, &pl);
          CHECK(rc == MGB_OK);
          if (rc == MGB_OK) CHECK(mgb_client_complete(c, pl.ticket) == MGB_OK);
        }
      });
    for (auto& t : th) t.join();
    for (auto& c : cl) CHECK(mgb_client_disconnect(c) == MGB_OK);
    CHECK(mgb_server_stop(sv) == MGB_OK);
    CHECK(mgb_sched_destroy(s) == MGB_OK);
  }
  std::printf("stress done, %d failed checks\n", fails.load());
  return fails.load() ? 1 : 0;
}
