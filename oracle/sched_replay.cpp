// CPU checker for the scheduler's decisions -- TEST INFRASTRUCTURE ONLY.
//
// Replays the *inputs* of an event trace (probes with their arguments,
// completions, cancellations, in their logged total order) through an
// independent implementation of the admission / partition policy and
// regenerates every *decision* (admit with which compute granules and CU mask,
// wait, reject, what is free afterwards).  Shares no code with the library.
//
// What the policy is (paper Sec. III-B, Algorithm 2 and Algorithm 3, and the
// remark in Sec. IV that resources freed by a finished task are offered to the
// tasks still waiting), restated for one device whose compute is handed out
// in granules of CUs instead of per-SM thread-block slots:
//   * memory is a hard constraint: a task is admitted only if its footprint
//     is no larger than the free bytes;
//   * HARD compute (Algorithm 2): the task's thread blocks must all be
//     resident at once; the number of CUs that needs follows from the
//     per-CU limits on resident waves and workgroups; the task gets that many
//     CUs exclusively, or it waits.  Partitions are buddy blocks: the demand
//     in granules is rounded up to a power of two b and the task receives the
//     lowest-indexed free run of b granules that starts at a multiple of b;
//   * SOFT compute (Algorithm 3): compute never blocks; the task is put on
//     the least-loaded compute (here: the aligned block of b granules with
//     the smallest total of in-use waves, lowest index first) and its waves
//     are added to the load of those granules;
//   * at most max_running tasks are resident at a time when that field is
//     non-zero (every resident task holds one hardware queue);
//   * CG (the core-to-GPU-ratio baseline of Sec. IV): up to max_running tasks
//     share the whole device and memory is NOT consulted; a task whose
//     footprint does not fit at the moment it is let in is the job that would
//     have died of an out-of-memory error: it is rejected with E_OOM and
//     counted, never run;
//   * SERIAL (single-assignment baseline, Sec. IV): one task owns the whole
//     device at a time;
//   * a resident task may ask for more memory (GROW): granted iff the bytes are free at that
//     moment, refused (never queued) otherwise; they return with the task's release;
//   * on every release the waiting tasks are retried in arrival order.
#include <cstdint>
#include <cstring>
#include <vector>
#include <algorithm>

namespace {

enum { IN_PROBE = 0, IN_COMPLETE = 1, IN_CANCEL = 2, IN_GROW = 3 };
enum { D_ADMIT = 1, D_WAIT = 2, D_REJECT = 3, D_RELEASE = 4, D_CANCELLED = 5, D_GROWN = 6 };
enum { POL_HARD = 0, POL_SOFT = 1, POL_SERIAL = 2, POL_CG = 3 };
enum { Q_BACKFILL = 0, Q_FIFO = 1 };
enum { E_INVAL = -1, E_TOO_BIG = -2, E_UNKNOWN_TICKET = -3, E_BAD_STATE = -4, E_BUSY = -5, E_OOM = -8 };

struct Task {
  uint64_t ticket, task_id, mem, waves;
  uint32_t demand;      // granules wanted
  uint32_t granted;     // granule bitmap once admitted
  uint64_t share;       // SOFT: waves charged to each granted granule
  bool running;
};

}  // namespace

extern "C" {

struct orc_device {
  uint64_t cap_bytes;
  uint32_t n_cu, granule_cus, wave_size, max_waves_per_cu, max_wg_per_cu, policy, queue_mode;
  uint32_t max_running;   // 0 = no limit
};

struct orc_input {
  uint32_t kind;        // IN_*
  uint32_t wg_per_cu;   // PROBE: workgroups per CU the task's own resources allow, 0 = not known
  uint64_t id;          // PROBE: task id; COMPLETE / CANCEL: ticket
  uint64_t mem;
  uint32_t grid[3], block[3];
};

struct orc_decision {
  uint32_t in_index;    // which input event produced it
  uint32_t kind;        // D_*
  uint64_t ticket;
  uint64_t task_id;
  uint64_t free_bytes;  // after the decision
  uint32_t granule_mask;
  uint32_t free_granules;  // bitmap after the decision (HARD / SERIAL), else all-free map
  uint32_t demand;
  int32_t code;         // reject reason, else 0
  uint32_t cu_mask[8];
};

// granules demanded by a launch geometry: how many CUs are needed to hold all
// workgroups at once given the per-CU wave and workgroup limits.
uint32_t orc_demand_ex(const orc_device* dev, const uint32_t grid[3], const uint32_t block[3],
                       uint32_t wg_per_cu_task, uint64_t* waves_out);

uint32_t orc_demand(const orc_device* dev, const uint32_t grid[3], const uint32_t block[3],
                    uint64_t* waves_out) {
  return orc_demand_ex(dev, grid, block, 0, waves_out);
}

uint32_t orc_demand_ex(const orc_device* dev, const uint32_t grid[3], const uint32_t block[3],
                       uint32_t wg_per_cu_task, uint64_t* waves_out) {
  uint64_t W = (uint64_t)grid[0] * grid[1] * grid[2];
  uint64_t T = (uint64_t)block[0] * block[1] * block[2];
  uint64_t wpw = (T + dev->wave_size - 1) / dev->wave_size;
  uint64_t per_cu = dev->max_waves_per_cu / wpw;
  if (per_cu > dev->max_wg_per_cu) per_cu = dev->max_wg_per_cu;
  if (wg_per_cu_task != 0 && per_cu > wg_per_cu_task) per_cu = wg_per_cu_task;
  if (per_cu < 1) per_cu = 1;
  uint64_t cus = (W + per_cu - 1) / per_cu;
  if (cus > dev->n_cu) cus = dev->n_cu;
  if (waves_out) *waves_out = W * wpw;
  return (uint32_t)((cus + dev->granule_cus - 1) / dev->granule_cus);
}

// Returns the number of decisions written (at most `cap`), or -1 if `cap` was too small.
int64_t orc_sched_replay(const orc_device* dev, const orc_input* in, uint64_t n_in,
                         orc_decision* out, uint64_t cap) {
  const uint32_t G = dev->n_cu / dev->granule_cus;
  const uint32_t all = G >= 32 ? 0xffffffffu : ((1u << G) - 1u);
  uint64_t free_bytes = dev->cap_bytes;
  uint32_t free_map = all;
  std::vector<uint64_t> load(G, 0);
  std::vector<Task> live;       // running and waiting tasks
  std::vector<uint64_t> waitq;  // tickets in arrival order
  uint64_t next_ticket = 0;
  uint64_t n_out = 0;
  bool overflow = false;

  auto find = [&](uint64_t ticket) -> Task* {
    for (auto& t : live)
      if (t.ticket == ticket) return &t;
    return nullptr;
  };
  auto emit = [&](uint32_t idx, uint32_t kind, const Task* t, uint32_t gmask, int32_t code,
                  uint64_t task_id) {
    if (n_out >= cap) { overflow = true; return; }
    orc_decision& d = out[n_out++];
    std::memset(&d, 0, sizeof d);
    d.in_index = idx;
    d.kind = kind;
    d.ticket = t ? t->ticket : 0;
    d.task_id = t ? t->task_id : task_id;
    d.free_bytes = free_bytes;
    d.granule_mask = gmask;
    d.free_granules = free_map;
    d.demand = t ? t->demand : 0;
    d.code = code;
    for (uint32_t g = 0; g < G; ++g)
      if (gmask >> g & 1u)
        for (uint32_t c = 0; c < dev->granule_cus; ++c) {
          uint32_t bit = g * dev->granule_cus + c;
          d.cu_mask[bit / 32] |= 1u << (bit % 32);
        }
  };
  uint32_t n_running = 0;
  bool crashed = false;                  // set by try_admit under CG when the task would have run out of memory
  auto try_admit = [&](Task& t) -> bool {
    crashed = false;
    if (dev->policy == POL_CG) {
      if (dev->max_running != 0 && n_running >= dev->max_running) return false;
      if (t.mem > free_bytes) { crashed = true; return false; }
      free_bytes -= t.mem;
      t.granted = all;
      t.running = true;
      ++n_running;
      return true;
    }
    if (t.mem > free_bytes) return false;
    if (dev->max_running != 0 && n_running >= dev->max_running) return false;
    uint32_t b = 1;                      // block size: demand rounded up to a power of two
    while (b < t.demand) b <<= 1;
    if (b > G) b = G;                    // a device whose granule count is not a power of two
    uint32_t pick = 0;
    if (dev->policy == POL_SOFT) {
      uint64_t best_load = 0;
      bool have = false;
      for (uint32_t start = 0; start + b <= G; start += b) {
        uint64_t sum = 0;
        for (uint32_t g = start; g < start + b; ++g) sum += load[g];
        if (!have || sum < best_load) {
          have = true;
          best_load = sum;
          pick = (b >= 32 ? 0xffffffffu : ((1u << b) - 1u)) << start;
        }
      }
      if (!have) return false;
      t.share = (t.waves + b - 1) / b;
      for (uint32_t g = 0; g < G; ++g)
        if (pick >> g & 1u) load[g] += t.share;
    } else {
      bool have = false;
      for (uint32_t start = 0; start + b <= G && !have; start += b) {
        uint32_t block = (b >= 32 ? 0xffffffffu : ((1u << b) - 1u)) << start;
        if ((free_map & block) == block) {
          pick = block;
          have = true;
        }
      }
      if (!have) return false;
      free_map &= ~pick;
    }
    free_bytes -= t.mem;
    t.granted = pick;
    t.running = true;
    ++n_running;
    return true;
  };
  auto rescan = [&](uint32_t idx) {
    size_t i = 0;
    while (i < waitq.size()) {
      Task* t = find(waitq[i]);
      if (try_admit(*t)) {
        waitq.erase(waitq.begin() + i);
        emit(idx, D_ADMIT, t, t->granted, 0, 0);
      } else if (crashed) {
        emit(idx, D_REJECT, t, 0, E_OOM, 0);
        uint64_t ticket = t->ticket;
        waitq.erase(waitq.begin() + i);
        live.erase(std::find_if(live.begin(), live.end(), [&](const Task& x) { return x.ticket == ticket; }));
      } else if (dev->queue_mode == Q_FIFO) {
        break;
      } else {
        ++i;
      }
    }
  };

  for (uint64_t e = 0; e < n_in; ++e) {
    const orc_input& ev = in[e];
    const uint32_t idx = (uint32_t)e;
    if (ev.kind == IN_PROBE) {
      uint64_t W = (uint64_t)ev.grid[0] * ev.grid[1] * ev.grid[2];
      uint64_t T = (uint64_t)ev.block[0] * ev.block[1] * ev.block[2];
      if (W == 0 || T == 0 || T > 1024) { emit(idx, D_REJECT, nullptr, 0, E_INVAL, ev.id); continue; }
      if (ev.mem > dev->cap_bytes) { emit(idx, D_REJECT, nullptr, 0, E_TOO_BIG, ev.id); continue; }
      Task t{};
      t.ticket = ++next_ticket;
      t.task_id = ev.id;
      t.mem = ev.mem;
      t.demand = orc_demand_ex(dev, ev.grid, ev.block, ev.wg_per_cu, &t.waves);
      if (dev->policy == POL_SERIAL) t.demand = G;
      live.push_back(t);
      Task& ref = live.back();
      bool blocked_by_queue = dev->queue_mode == Q_FIFO && !waitq.empty();
      if (!blocked_by_queue && try_admit(ref)) {
        emit(idx, D_ADMIT, &ref, ref.granted, 0, 0);
      } else if (!blocked_by_queue && crashed) {
        emit(idx, D_REJECT, &ref, 0, E_OOM, 0);
        live.pop_back();
      } else {
        waitq.push_back(ref.ticket);
        emit(idx, D_WAIT, &ref, 0, 0, 0);
      }
    } else if (ev.kind == IN_COMPLETE) {
      Task* t = find(ev.id);
      if (!t) { emit(idx, D_REJECT, nullptr, 0, E_UNKNOWN_TICKET, 0); continue; }
      if (!t->running) { emit(idx, D_REJECT, t, 0, E_BAD_STATE, 0); continue; }
      free_bytes += t->mem;
      if (dev->policy == POL_CG) {
        // nothing to give back but the memory: the device is shared as a whole
      } else if (dev->policy == POL_SOFT) {
        for (uint32_t g = 0; g < G; ++g)
          if (t->granted >> g & 1u) load[g] -= t->share;
      } else {
        free_map |= t->granted;
      }
      --n_running;
      emit(idx, D_RELEASE, t, t->granted, 0, 0);
      uint64_t ticket = t->ticket;
      live.erase(std::find_if(live.begin(), live.end(), [&](const Task& x) { return x.ticket == ticket; }));
      rescan(idx);
    } else if (ev.kind == IN_CANCEL) {
      Task* t = find(ev.id);
      if (!t) { emit(idx, D_REJECT, nullptr, 0, E_UNKNOWN_TICKET, 0); continue; }
      if (t->running) { emit(idx, D_REJECT, t, 0, E_BAD_STATE, 0); continue; }
      emit(idx, D_CANCELLED, t, 0, 0, 0);
      uint64_t ticket = t->ticket;
      waitq.erase(std::find(waitq.begin(), waitq.end(), ticket));
      live.erase(std::find_if(live.begin(), live.end(), [&](const Task& x) { return x.ticket == ticket; }));
      rescan(idx);
    } else if (ev.kind == IN_GROW) {
      Task* t = find(ev.id);
      if (!t) { emit(idx, D_REJECT, nullptr, 0, E_UNKNOWN_TICKET, 0); continue; }
      if (!t->running) { emit(idx, D_REJECT, t, 0, E_BAD_STATE, 0); continue; }
      if (ev.mem > free_bytes) { emit(idx, D_REJECT, t, 0, E_BUSY, 0); continue; }
      free_bytes -= ev.mem;
      t->mem += ev.mem;
      emit(idx, D_GROWN, t, t->granted, 0, 0);
    } else {
      emit(idx, D_REJECT, nullptr, 0, E_INVAL, ev.id);
    }
  }
  return overflow ? -1 : (int64_t)n_out;
}

}  // extern "C"
