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

static std::atomic<int> fails{0};
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
          CHECK(mgb_task_complete(s, pl.ticket) == MGB_OK);
        }
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
