// Scheduler core: memory ledger, CU-granule partitioner, wait queue, event
// trace, and the stream backend behind placements.
//
// One device, one mutex.  The policy follows Sec. III-B of the paper
// (Algorithm 2: memory and compute both hard; Algorithm 3: memory hard,
// compute placed by load) with the device's SMs replaced by granules of CUs
// that are handed out exclusively (HARD) and realised as CU-masked streams.
//
// Partitions are buddy blocks (power-of-two runs of granules, aligned to their
// size).  That keeps the set of CU masks small (15 for the default 8 granules
// of 32 CUs, 63 for 32 granules of 8), which matters because a masked stream is
// a hardware queue: creating one costs milliseconds, and beyond about 24 live
// queues the device time-slices them and every launch slows down a hundredfold.
// The library therefore keeps few masked streams alive, reuses them by mask,
// never lets more than max_running tasks be resident, creates the masks of the
// large blocks up front, and creates the others on first use with the scheduler
// lock released, so that only the task that needs a new queue waits for it.
//
// A release can be ordered on the device instead of being observed by the host
// (mgb_task_complete_on_stream): the ledger is credited as soon as the task's
// last kernel is enqueued, and whoever is admitted into what it held starts
// behind the task's stop event (hipStreamWaitEvent), so that in device time a
// granule still has one owner and the bytes one user, while the hand-over
// between two tasks costs the device nothing.
#include "../../include/mgb.h"
#include "launch_util.h"

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <condition_variable>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <deque>
#include <mutex>
#include <string>
#include <unordered_map>
#include <vector>

namespace {

thread_local std::string g_last_error;

void set_error(const char* what, hipError_t e) {
  g_last_error = std::string(what) + ": " + hipGetErrorString(e);
}

uint64_t now_ns() {
  return (uint64_t)std::chrono::duration_cast<std::chrono::nanoseconds>(
             std::chrono::steady_clock::now().time_since_epoch())
      .count();
}

// Live masked streams of the whole process.  Launch cost is flat up to 24 live queues and
// jumps from ~15 us to milliseconds at 28 (measured), and the process also owns the queues of
// its ordinary streams, so idle streams are destroyed (least recently used first) before the
// count would pass kStreamsAlive; only streams of resident tasks may push it higher.
constexpr uint32_t kStreamsAlive = 20;
// Trace records kept per scheduler (120 bytes each); at the cap the older half is dropped.
constexpr size_t kTraceCap = 1u << 20;
std::atomic<uint32_t> g_live_streams{0};

// Draining: released through mgb_task_complete_on_stream, its kernels possibly still running;
// holds nothing in the ledger, only its timing events, until mgb_task_sync retires it.
enum class State { Waiting, Running, Draining };

struct Dep {
  uint64_t ticket;     // the draining task whose stop event orders the start
  hipEvent_t ev;       // (nullptr with the null backend)
  hipStream_t stream;  // the stream that task ran on: a successor on the same stream is ordered already
};

struct Task {
  uint64_t ticket = 0, task_id = 0, mem = 0, waves = 0, share = 0;
  uint32_t demand = 0, granted = 0;
  mgb_dim3 grid{}, block{};
  State state = State::Waiting;
  hipStream_t stream = nullptr;
  hipEvent_t ev_start = nullptr, ev_stop = nullptr;
  bool launched = false;
  std::vector<Dep> deps;        // draining tasks this one must start behind
  bool deps_issued = false;     // the waits are on the task's stream
  bool syncing = false;         // draining: a thread is waiting for its stop event and will retire it
};

// What is known of a task from its probe to its end (mgb_task_records).
struct Record {
  mgb_task_record r;
};

}  // namespace

void mgb_internal_set_error(const char* what, hipError_t e) { set_error(what, e); }
void mgb_internal_set_error_text(const char* text) { g_last_error = text; }

struct mgb_sched {
  mgb_device_desc d{};
  uint32_t G = 0;            // number of granules
  uint32_t all_mask = 0;
  std::mutex mu;
  std::condition_variable cv;
  uint64_t free_bytes = 0;
  uint32_t free_map = 0;
  std::vector<uint64_t> load;                 // SOFT: in-use waves per granule
  std::unordered_map<uint64_t, Task> tasks;   // live tasks by ticket
  std::deque<uint64_t> waitq;                 // tickets in arrival order
  uint64_t next_ticket = 0;
  uint32_t n_running_now = 0;
  bool oom = false;                          // try_admit: CG task that would have run out of memory
  std::vector<uint64_t> crashed;             // tickets rejected while queued, until their waiter collects them
  // A thread blocked in mgb_task_wait sleeps on a condition variable of its own, registered here
  // under its ticket, so that a release wakes only the waiters it admits (with one shared
  // variable every release woke all of them, and the admitted one queued for the lock behind the
  // rest).  A second thread waiting on the same ticket uses the shared variable `cv`.
  std::unordered_map<uint64_t, std::condition_variable*> waiters;
  uint32_t shared_waiters = 0;
  void wake(uint64_t ticket) {
    auto w = waiters.find(ticket);
    if (w != waiters.end()) w->second->notify_one();
    if (shared_waiters != 0u) cv.notify_all();
  }
  std::vector<mgb_trace_rec> trace;          // records trace_base .. trace_base + size - 1
  uint64_t trace_base = 0;                   // seq of trace[0]: the oldest records are dropped at kTraceCap
  // backend: idle masked streams (mask, stream, when last used), idle timing events
  struct IdleStream { uint32_t mask; hipStream_t stream; uint64_t stamp; };
  std::vector<IdleStream> idle_streams;
  std::unordered_map<hipStream_t, uint32_t> stream_users;   // bound streams -> resident tasks on them
  uint64_t stamp = 0;
  // idle timing events.  A start event only ever measures time, so it is created without the
  // system-scope fence (the record then does not flush and invalidate the caches in front of the
  // task's first kernel); a stop event is also what mgb_task_sync and successors wait for and keeps it.
  std::vector<hipEvent_t> idle_start_events, idle_stop_events;
  uint32_t n_streams = 0;   // created so far
  uint32_t n_alive = 0;     // created and not destroyed
  // stream-ordered releases: per granule the draining task that owned it last (exclusive
  // policies), and every draining task with the bytes it may still be using
  std::vector<Dep> gran_pending;
  struct MemPending { uint64_t ticket; hipEvent_t ev; uint64_t mem; hipStream_t stream; };
  std::vector<MemPending> mem_pending;
  uint64_t pending_mem = 0;
  hipEvent_t epoch = nullptr;                 // device-clock origin of gpu_start_ms / gpu_stop_ms
  bool tag_partitions = false;                // MGB_TAG_PARTITIONS: a marker kernel in front of every task
  // one record per ticket (tickets record_base + 1 ...); the older half is dropped at kTraceCap
  std::deque<mgb_task_record> records;
  uint64_t record_base = 0;
  mgb_task_record* record_of(uint64_t ticket) {
    if (ticket <= record_base || ticket - record_base > records.size()) return nullptr;
    return &records[ticket - record_base - 1];
  }

  // Device-side ordering of a task admitted just now (ledger already debited; free_before = the
  // free bytes before the debit).  Exclusive compute: behind the last draining owner of each of
  // its granules.  Memory: if the task needed bytes that draining tasks may still be using,
  // behind all of them.
  void collect_deps(Task& t, uint64_t free_before) {
    t.deps.clear();
    auto add = [&](uint64_t ticket, hipEvent_t ev, hipStream_t st) {
      for (const Dep& d0 : t.deps)
        if (d0.ticket == ticket) return;
      t.deps.push_back({ticket, ev, st});
    };
    if (d.policy == MGB_POLICY_HARD || d.policy == MGB_POLICY_SERIAL)
      for (uint32_t g = 0; g < G; ++g)
        if ((t.granted >> g & 1u) && gran_pending[g].ticket != 0u)
          add(gran_pending[g].ticket, gran_pending[g].ev, gran_pending[g].stream);
    if (d.policy != MGB_POLICY_CG && pending_mem != 0u && t.mem > free_before - std::min(free_before, pending_mem))
      for (const MemPending& m : mem_pending) add(m.ticket, m.ev, m.stream);
  }

  // A draining task's kernels are known to have finished: nothing needs to start behind it any more.
  void forget_pending(uint64_t ticket) {
    for (Dep& g : gran_pending)
      if (g.ticket == ticket) g = Dep{0, nullptr, nullptr};
    for (size_t i = 0; i < mem_pending.size(); ++i)
      if (mem_pending[i].ticket == ticket) {
        pending_mem -= mem_pending[i].mem;
        mem_pending.erase(mem_pending.begin() + (long)i);
        break;
      }
    for (auto& kv : tasks) {
      Task& o = kv.second;
      if (o.deps_issued) continue;
      for (size_t i = 0; i < o.deps.size(); ++i)
        if (o.deps[i].ticket == ticket) {
          o.deps.erase(o.deps.begin() + (long)i);
          break;
        }
    }
  }

  void cu_mask_of(uint32_t gmask, uint32_t out[8]) const {
    std::memset(out, 0, 8 * sizeof(uint32_t));
    for (uint32_t g = 0; g < G; ++g) {
      if (!(gmask >> g & 1u)) continue;
      for (uint32_t c = 0; c < d.granule_cus; ++c) {
        uint32_t bit = g * d.granule_cus + c;
        out[bit >> 5] |= 1u << (bit & 31);
      }
    }
  }

  uint64_t log(uint32_t kind, const Task* t, uint64_t task_id, uint64_t ticket, uint64_t mem,
               mgb_dim3 grid, mgb_dim3 block, uint32_t gmask, int32_t code, uint64_t cause) {
    if (trace.size() >= kTraceCap) {
      trace.erase(trace.begin(), trace.begin() + (long)(kTraceCap / 2));
      trace_base += kTraceCap / 2;
    }
    mgb_trace_rec r;
    std::memset(&r, 0, sizeof r);
    r.seq = trace_base + trace.size();
    r.t_ns = now_ns();
    r.task_id = t ? t->task_id : task_id;
    r.ticket = t ? t->ticket : ticket;
    r.mem_bytes = t ? t->mem : mem;
    r.free_bytes = free_bytes;
    r.kind = kind;
    r.code = code;
    r.granule_mask = gmask;
    r.free_granules = free_map;
    r.demand = t ? t->demand : 0;
    r.cause_seq = (uint32_t)cause;
    r.grid = t ? t->grid : grid;
    r.block = t ? t->block : block;
    cu_mask_of(gmask, r.cu_mask);
    trace.push_back(r);
    if (t)
      if (mgb_task_record* a = record_of(t->ticket)) {
        if (kind == MGB_EV_ADMIT) {
          a->admit_ns = r.t_ns;
          a->granule_mask = gmask;
        } else if (kind == MGB_EV_RELEASE) {
          a->release_ns = r.t_ns;
          if (a->done_ns == 0u) a->done_ns = r.t_ns;
          a->mem_bytes = t->mem;
          a->status = MGB_OK;
        } else if (kind == MGB_EV_CANCELLED) {
          a->status = MGB_TIMEOUT;
          a->release_ns = a->done_ns = r.t_ns;
        } else if (kind == MGB_EV_REJECT && code == MGB_E_OOM) {
          a->status = MGB_E_OOM;
          a->release_ns = a->done_ns = r.t_ns;
        }
      }
    return r.seq;
  }

  static uint32_t block_bits(uint32_t b) { return b >= 32u ? 0xffffffffu : ((1u << b) - 1u); }

  // Memory first (hard in every policy), then the resident-task limit, then compute.
  // Compute is granted in buddy blocks: demand rounded up to a power of two b, block = b
  // granules starting at a multiple of b.
  bool try_admit(Task& t) {
    oom = false;
    const uint64_t free_before = free_bytes;
    if (d.policy == MGB_POLICY_CG) {
      // ratio-limited packing that never looks at memory (Sec. IV): the task that does not fit
      // when it is let in is the one that would have crashed; it is reported, not run
      if (d.max_running != 0u && n_running_now >= d.max_running) return false;
      if (t.mem > free_bytes) {
        oom = true;
        return false;
      }
      free_bytes -= t.mem;
      t.granted = all_mask;
      t.state = State::Running;
      ++n_running_now;
      collect_deps(t, free_before);
      return true;
    }
    if (t.mem > free_bytes) return false;
    if (d.max_running != 0u && n_running_now >= d.max_running) return false;
    uint32_t b = 1;
    while (b < t.demand) b <<= 1;
    if (b > G) b = G;
    uint32_t pick = 0;
    if (d.policy == MGB_POLICY_SOFT) {
      // never blocks on compute: the aligned block carrying the fewest in-use waves,
      // the lower block winning ties
      uint64_t best = 0;
      for (uint32_t start = 0; start + b <= G; start += b) {
        uint64_t sum = 0;
        for (uint32_t g = start; g < start + b; ++g) sum += load[g];
        if (pick == 0u || sum < best) {
          best = sum;
          pick = block_bits(b) << start;
        }
      }
      t.share = (t.waves + b - 1) / b;
      for (uint32_t g = 0; g < G; ++g)
        if (pick >> g & 1u) load[g] += t.share;
    } else {
      for (uint32_t start = 0; start + b <= G; start += b) {
        const uint32_t block = block_bits(b) << start;
        if ((free_map & block) == block) {
          pick = block;
          break;
        }
      }
      if (pick == 0u) return false;
      free_map &= ~pick;
    }
    free_bytes -= t.mem;
    t.granted = pick;
    t.state = State::Running;
    ++n_running_now;
    collect_deps(t, free_before);
    return true;
  }

  void release(Task& t) {
    free_bytes += t.mem;
    --n_running_now;
    if (d.policy == MGB_POLICY_CG) return;
    if (d.policy == MGB_POLICY_SOFT) {
      for (uint32_t g = 0; g < G; ++g)
        if (t.granted >> g & 1u) load[g] -= t.share;
    } else {
      free_map |= t.granted;
    }
  }

  // Offer what is free to the waiters, oldest first.
  bool rescan(uint64_t cause) {
    bool any = false;
    for (size_t i = 0; i < waitq.size();) {
      Task& t = tasks[waitq[i]];
      if (try_admit(t)) {
        waitq.erase(waitq.begin() + (long)i);
        log(MGB_EV_ADMIT, &t, 0, 0, 0, {}, {}, t.granted, 0, cause);
        wake(t.ticket);
        any = true;
      } else if (oom) {
        log(MGB_EV_REJECT, &t, 0, 0, 0, {}, {}, 0, MGB_E_OOM, cause);
        crashed.push_back(t.ticket);
        wake(t.ticket);
        tasks.erase(waitq[i]);
        waitq.erase(waitq.begin() + (long)i);
        any = true;                                   // its waiter must wake up and collect the error
      } else if (d.queue_mode == MGB_QUEUE_FIFO) {
        break;
      } else {
        ++i;
      }
    }
    return any;
  }

  // ---- backend -----------------------------------------------------------
  // Create a masked stream.  Touches no scheduler state: callable without the lock.
  int create_stream(uint32_t gmask, hipStream_t* out) {
    uint32_t cu[8];
    cu_mask_of(gmask, cu);
    hipError_t e = hipSetDevice(d.device);
    if (e == hipSuccess) e = hipExtStreamCreateWithCUMask(out, 8, cu);
    if (e != hipSuccess) {
      set_error("hipExtStreamCreateWithCUMask", e);
      *out = nullptr;
      return MGB_E_BACKEND;
    }
    ++g_live_streams;
    return MGB_OK;
  }

  // Give the task a stream of its mask and two timing events.  A cached idle stream is taken
  // under the lock.  On a miss at the process's limit of live queues, a task whose mask is
  // already in use by a resident task (overlapping placements: SOFT, CG) runs behind that task
  // on its queue, the same CUs, in order, instead of paying for a new queue; otherwise the queue
  // is created (the least recently used idle one destroyed first when at the limit) with the
  // lock released: those runtime calls take milliseconds and only this task should wait for them.
  int bind_stream(Task& t, std::unique_lock<std::mutex>& lk) {
    if (d.backend != MGB_BACKEND_HIP) return MGB_OK;
    Task* tp = &t;
    if (!tp->stream) {
      for (size_t i = 0; i < idle_streams.size(); ++i)
        if (idle_streams[i].mask == tp->granted) {
          tp->stream = idle_streams[i].stream;
          idle_streams.erase(idle_streams.begin() + (long)i);
          stream_users[tp->stream] = 1;
          break;
        }
    }
    if (!tp->stream && g_live_streams.load() >= kStreamsAlive) {
      hipStream_t share = nullptr;
      uint32_t fewest = 0;
      for (auto& kv : tasks) {
        const Task& o = kv.second;
        if (&o == tp || !o.stream || o.state != State::Running || o.granted != tp->granted) continue;
        const uint32_t users = stream_users[o.stream];
        if (!share || users < fewest) {
          share = o.stream;
          fewest = users;
        }
      }
      if (share) {
        tp->stream = share;
        ++stream_users[share];
      }
    }
    if (!tp->stream) {
      hipStream_t victim = nullptr;
      if (!idle_streams.empty() && g_live_streams.load() >= kStreamsAlive) {
        // least recently used, but never a stream on which a released-on-stream task may still run
        // (successors compare stream handles to tell whether they are ordered behind it already)
        auto named = [&](hipStream_t st) {
          for (const MemPending& m : mem_pending)
            if (m.stream == st) return true;
          return false;
        };
        size_t v = idle_streams.size();
        for (size_t i = 0; i < idle_streams.size(); ++i)
          if (!named(idle_streams[i].stream) && (v == idle_streams.size() || idle_streams[i].stamp < idle_streams[v].stamp)) v = i;
        if (v != idle_streams.size()) {
          victim = idle_streams[v].stream;
          idle_streams.erase(idle_streams.begin() + (long)v);
        }
      }
      const uint32_t mask = tp->granted;
      const uint64_t ticket = tp->ticket;
      lk.unlock();
      if (victim) {
        (void)hipStreamDestroy(victim);
        --g_live_streams;
      }
      hipStream_t st = nullptr;
      const int rc = create_stream(mask, &st);
      lk.lock();
      if (rc != MGB_OK) return rc;
      ++n_streams;
      auto it = tasks.find(ticket);
      if (it == tasks.end()) {                       // the task went away meanwhile: keep the queue for later
        idle_streams.push_back({mask, st, ++stamp});
        return MGB_E_UNKNOWN_TICKET;
      }
      tp = &it->second;
      tp->stream = st;
      stream_users[st] = 1;
    }
    for (int which = 0; which < 2; ++which) {
      hipEvent_t* ev = which == 0 ? &tp->ev_start : &tp->ev_stop;
      std::vector<hipEvent_t>& pool = which == 0 ? idle_start_events : idle_stop_events;
      if (*ev) continue;
      if (!pool.empty()) {
        *ev = pool.back();
        pool.pop_back();
      } else {
        hipError_t e = hipEventCreateWithFlags(ev, which == 0 ? hipEventDisableSystemFence : hipEventDefault);
        if (e != hipSuccess) {
          set_error("hipEventCreate", e);
          return MGB_E_BACKEND;
        }
      }
    }
    // start behind the draining tasks whose granules or bytes this one took over
    if (!tp->deps_issued) {
      for (const Dep& dep : tp->deps) {
        if (!dep.ev || dep.stream == tp->stream) continue;      // (its own stream runs in order anyway)
        hipError_t e = hipStreamWaitEvent(tp->stream, dep.ev, 0);
        if (e != hipSuccess) {
          set_error("hipStreamWaitEvent", e);
          return MGB_E_BACKEND;
        }
      }
      tp->deps_issued = true;
    }
    return MGB_OK;
  }

  void unbind_stream(Task& t, bool keep_events = false) {
    if (t.stream && --stream_users[t.stream] == 0u) {
      stream_users.erase(t.stream);
      idle_streams.push_back({t.granted, t.stream, ++stamp});
    }
    t.stream = nullptr;
    if (keep_events) return;
    if (t.ev_start) idle_start_events.push_back(t.ev_start);
    if (t.ev_stop) idle_stop_events.push_back(t.ev_stop);
    t.ev_start = t.ev_stop = nullptr;
  }

  // The body of mgb_task_complete: input record, release, re-pack.  Lock held.
  // on_stream: the task's kernels may still be running; it stays behind as a draining task and
  // whatever takes over its granules or bytes is ordered behind its stop event.
  int complete_locked(uint64_t ticket, bool on_stream = false) {
    uint64_t cause = log(MGB_EV_COMPLETE, nullptr, 0, ticket, 0, {}, {}, 0, 0, 0);
    trace.back().cause_seq = (uint32_t)cause;
    auto it = tasks.find(ticket);
    // (a draining task has been released already: to the ledger, and to whoever replays the
    // trace, its ticket no longer exists)
    if (it == tasks.end() || it->second.state == State::Draining) {
      log(MGB_EV_REJECT, nullptr, 0, ticket, 0, {}, {}, 0, MGB_E_UNKNOWN_TICKET, cause);
      return MGB_E_UNKNOWN_TICKET;
    }
    Task& t = it->second;
    if (t.state != State::Running) {
      log(MGB_EV_REJECT, &t, 0, 0, 0, {}, {}, 0, MGB_E_BAD_STATE, cause);
      return MGB_E_BAD_STATE;
    }
    release(t);
    log(MGB_EV_RELEASE, &t, 0, 0, 0, {}, {}, t.granted, 0, cause);
    if (on_stream) {
      hipEvent_t ev = t.launched ? t.ev_stop : nullptr;
      if (t.launched || d.backend != MGB_BACKEND_HIP) {      // (never launched on a device: nothing to wait for)
        if (d.policy == MGB_POLICY_HARD || d.policy == MGB_POLICY_SERIAL)
          for (uint32_t g = 0; g < G; ++g)
            if (t.granted >> g & 1u) gran_pending[g] = Dep{ticket, ev, t.stream};
        mem_pending.push_back({ticket, ev, t.mem, t.stream});
        pending_mem += t.mem;
      }
      unbind_stream(t, true);
      t.state = State::Draining;
      if (mgb_task_record* a = record_of(ticket)) a->done_ns = 0;      // set when its work is seen finished
    } else {
      unbind_stream(t);
      tasks.erase(it);
    }
    rescan(cause);                              // wakes whom it admits
    return MGB_OK;
  }

  // A draining task's work has finished (the caller waited for its stop event): drop it.
  void retire(uint64_t ticket) {
    auto it = tasks.find(ticket);
    if (it == tasks.end() || it->second.state != State::Draining) return;
    forget_pending(ticket);
    Task& t = it->second;
    if (t.ev_start) idle_start_events.push_back(t.ev_start);
    if (t.ev_stop) idle_stop_events.push_back(t.ev_stop);
    tasks.erase(it);
  }

  // Hand an admitted task to its caller.  If the backend cannot give it a stream the placement
  // is useless: the task is completed on the caller's behalf (the trace shows an ordinary
  // completion right after the admission) and the error is returned with nothing held.
  int fill(Task& t, mgb_placement* out, std::unique_lock<std::mutex>& lk) {
    out->ticket = t.ticket;
    out->granule_mask = t.granted;
    out->n_granules = t.demand;
    cu_mask_of(t.granted, out->cu_mask);
    const uint64_t ticket = t.ticket;
    int rc = bind_stream(t, lk);                     // may release and retake the lock
    auto it = tasks.find(ticket);
    out->stream = it == tasks.end() ? nullptr : (void*)it->second.stream;
    if (rc != MGB_OK) {
      if (it != tasks.end()) (void)complete_locked(ticket);
      std::memset(out, 0, sizeof *out);
    }
    return rc;
  }
};

unsigned mgb_internal_backend(const mgb_sched* s) { return s->d.backend; }
int mgb_internal_device(const mgb_sched* s) { return s->d.device; }

extern "C" {

const char* mgb_last_error(void) { return g_last_error.c_str(); }

void mgb_device_desc_default(mgb_device_desc* out) {
  if (!out) return;
  std::memset(out, 0, sizeof *out);
  out->mem_cap_bytes = 288ull * 1000 * 1000 * 1000;
  out->n_cu = 256;
  out->granule_cus = 32;
  out->wave_size = 64;
  out->max_waves_per_cu = 32;
  out->max_wg_per_cu = 32;
  out->policy = MGB_POLICY_HARD;
  out->queue_mode = MGB_QUEUE_BACKFILL;
  out->backend = MGB_BACKEND_HIP;
  out->device = 0;
  out->max_running = 8;
}

int mgb_sched_create(const mgb_device_desc* desc, mgb_sched** out) {
  if (!desc || !out) return MGB_E_INVAL;
  *out = nullptr;
  const mgb_device_desc& d = *desc;
  if (d.n_cu == 0 || d.granule_cus == 0 || d.n_cu % d.granule_cus != 0) return MGB_E_INVAL;
  if (d.n_cu > 256 || d.n_cu / d.granule_cus > 32) return MGB_E_INVAL;
  if (d.wave_size == 0 || d.max_waves_per_cu == 0 || d.max_wg_per_cu == 0) return MGB_E_INVAL;
  if (d.policy > MGB_POLICY_CG || d.queue_mode > MGB_QUEUE_FIFO) return MGB_E_INVAL;
  if (d.policy == MGB_POLICY_CG && d.max_running == 0u) return MGB_E_INVAL;   // CG is defined by its ratio
  if (d.backend > MGB_BACKEND_HIP) return MGB_E_INVAL;
  if (d.backend == MGB_BACKEND_HIP) {
    // a mask must keep at least one CU in each of the 8 XCDs
    if (d.granule_cus % 8 != 0) return MGB_E_INVAL;
    int count = 0;
    hipError_t e = hipGetDeviceCount(&count);
    if (e != hipSuccess || d.device < 0 || d.device >= count) {
      set_error("hipGetDeviceCount", e == hipSuccess ? hipErrorInvalidDevice : e);
      return MGB_E_BACKEND;
    }
    hipDeviceProp_t p;
    e = hipGetDeviceProperties(&p, d.device);
    if (e != hipSuccess) {
      set_error("hipGetDeviceProperties", e);
      return MGB_E_BACKEND;
    }
    if ((uint32_t)p.multiProcessorCount != d.n_cu) {
      g_last_error = "device CU count does not match descriptor n_cu";
      return MGB_E_BACKEND;
    }
  }
  mgb_sched* s = new (std::nothrow) mgb_sched;
  if (!s) return MGB_E_BACKEND;
  s->d = d;
  s->G = d.n_cu / d.granule_cus;
  s->all_mask = s->G >= 32 ? 0xffffffffu : ((1u << s->G) - 1u);
  s->free_bytes = d.mem_cap_bytes;
  s->free_map = s->all_mask;
  s->load.assign(s->G, 0);
  s->gran_pending.assign(s->G, Dep{0, nullptr, nullptr});
  s->tag_partitions = std::getenv("MGB_TAG_PARTITIONS") != nullptr;
  if (d.backend == MGB_BACKEND_HIP) {
    hipError_t e = hipSetDevice(d.device);
    if (e == hipSuccess) e = hipEventCreate(&s->epoch);
    if (e == hipSuccess) e = hipEventRecord(s->epoch, nullptr);
    if (e == hipSuccess) e = hipEventSynchronize(s->epoch);
    if (e != hipSuccess) {
      set_error("hipEventRecord (clock origin)", e);
      delete s;
      return MGB_E_BACKEND;
    }
    // the masks of the large blocks (whole device, halves, quarters) are created now, not on
    // the first task that needs them; SERIAL and CG only ever grant the whole device
    const bool whole_only = d.policy == MGB_POLICY_SERIAL || d.policy == MGB_POLICY_CG;
    for (uint32_t b = s->G; b >= 1u && b * 4u >= s->G && (b == s->G || !whole_only); b >>= 1)
      for (uint32_t start = 0; start + b <= s->G; start += b) {
        hipStream_t st = nullptr;
        if (s->create_stream(mgb_sched::block_bits(b) << start, &st) != MGB_OK) {
          mgb_sched_destroy(s);
          return MGB_E_BACKEND;
        }
        ++s->n_streams;
        s->idle_streams.push_back({mgb_sched::block_bits(b) << start, st, ++s->stamp});
      }
  }
  *out = s;
  return MGB_OK;
}

int mgb_sched_destroy(mgb_sched* s) {
  if (!s) return MGB_E_INVAL;
  {
    std::lock_guard<std::mutex> lk(s->mu);
    for (auto& kv : s->tasks)
      if (kv.second.state != State::Draining) return MGB_E_BUSY;
    // draining tasks nobody waited for: their kernels must be done before their events go
    for (auto& kv : s->tasks) {
      Task& t = kv.second;
      if (t.launched && t.ev_stop) (void)hipEventSynchronize(t.ev_stop);
      if (t.ev_start) (void)hipEventDestroy(t.ev_start);
      if (t.ev_stop) (void)hipEventDestroy(t.ev_stop);
    }
    s->tasks.clear();
    if (s->epoch) (void)hipEventDestroy(s->epoch);
    for (auto& is : s->idle_streams) {
      (void)hipStreamDestroy(is.stream);
      --g_live_streams;
    }
    for (hipEvent_t e : s->idle_start_events) (void)hipEventDestroy(e);
    for (hipEvent_t e : s->idle_stop_events) (void)hipEventDestroy(e);
    s->idle_streams.clear();
    s->idle_start_events.clear();
    s->idle_stop_events.clear();
  }
  delete s;
  return MGB_OK;
}

int mgb_task_probe(mgb_sched* s, uint64_t task_id, uint64_t mem_bytes, mgb_dim3 grid,
                   mgb_dim3 block, mgb_placement* out) {
  return mgb_task_probe_ex(s, task_id, mem_bytes, grid, block, 0u, out);
}

int mgb_task_probe_ex(mgb_sched* s, uint64_t task_id, uint64_t mem_bytes, mgb_dim3 grid,
                      mgb_dim3 block, uint32_t wg_per_cu_task, mgb_placement* out) {
  if (!s || !out) return MGB_E_INVAL;
  std::memset(out, 0, sizeof *out);
  std::unique_lock<std::mutex> lk(s->mu);
  uint64_t cause = s->log(MGB_EV_PROBE, nullptr, task_id, 0, mem_bytes, grid, block, 0, 0, 0);
  s->trace.back().cause_seq = (uint32_t)cause;
  s->trace.back().demand = wg_per_cu_task;           // input records carry what the caller passed
  const uint64_t W = (uint64_t)grid.x * grid.y * grid.z;
  const uint64_t T = (uint64_t)block.x * block.y * block.z;
  if (W == 0 || T == 0 || T > 1024) {
    s->log(MGB_EV_REJECT, nullptr, task_id, 0, mem_bytes, grid, block, 0, MGB_E_INVAL, cause);
    return MGB_E_INVAL;
  }
  if (mem_bytes > s->d.mem_cap_bytes) {
    s->log(MGB_EV_REJECT, nullptr, task_id, 0, mem_bytes, grid, block, 0, MGB_E_TOO_BIG, cause);
    return MGB_E_TOO_BIG;
  }
  // residency-based compute demand (per-CU wave and workgroup limits, and what the task's own
  // registers and LDS allow if the probe says so)
  const uint64_t waves_per_wg = (T + s->d.wave_size - 1) / s->d.wave_size;
  uint64_t wg_per_cu = s->d.max_waves_per_cu / waves_per_wg;
  wg_per_cu = std::min<uint64_t>(wg_per_cu, s->d.max_wg_per_cu);
  if (wg_per_cu_task != 0u) wg_per_cu = std::min<uint64_t>(wg_per_cu, wg_per_cu_task);
  wg_per_cu = std::max<uint64_t>(1, wg_per_cu);
  const uint64_t cus = std::min<uint64_t>(s->d.n_cu, (W + wg_per_cu - 1) / wg_per_cu);
  Task t;
  t.ticket = ++s->next_ticket;
  t.task_id = task_id;
  t.mem = mem_bytes;
  t.waves = W * waves_per_wg;
  t.demand = (uint32_t)((cus + s->d.granule_cus - 1) / s->d.granule_cus);
  if (s->d.policy == MGB_POLICY_SERIAL) t.demand = s->G;
  t.grid = grid;
  t.block = block;
  Task& ref = s->tasks.emplace(t.ticket, t).first->second;
  {
    if (s->records.size() >= kTraceCap) {
      s->records.erase(s->records.begin(), s->records.begin() + (long)(kTraceCap / 2));
      s->record_base += kTraceCap / 2;
    }
    mgb_task_record a;
    std::memset(&a, 0, sizeof a);
    a.ticket = t.ticket;
    a.task_id = task_id;
    a.mem_bytes = mem_bytes;
    a.probe_ns = s->trace.back().t_ns;
    a.demand = t.demand;
    a.status = MGB_WAIT;                          // not finished yet
    s->records.push_back(a);
  }
  const bool behind_queue = s->d.queue_mode == MGB_QUEUE_FIFO && !s->waitq.empty();
  if (!behind_queue && s->try_admit(ref)) {
    s->log(MGB_EV_ADMIT, &ref, 0, 0, 0, {}, {}, ref.granted, 0, cause);
    return s->fill(ref, out, lk);
  }
  if (!behind_queue && s->oom) {
    s->log(MGB_EV_REJECT, &ref, 0, 0, 0, {}, {}, 0, MGB_E_OOM, cause);
    s->tasks.erase(ref.ticket);
    return MGB_E_OOM;
  }
  s->waitq.push_back(ref.ticket);
  s->log(MGB_EV_QUEUED, &ref, 0, 0, 0, {}, {}, 0, 0, cause);
  out->ticket = ref.ticket;
  out->n_granules = ref.demand;
  return MGB_WAIT;
}

int mgb_task_wait(mgb_sched* s, uint64_t ticket, int64_t timeout_ns, mgb_placement* out) {
  if (!s || !out) return MGB_E_INVAL;
  std::unique_lock<std::mutex> lk(s->mu);
  auto admitted = [&]() {
    auto it = s->tasks.find(ticket);
    return it == s->tasks.end() || it->second.state == State::Running;
  };
  auto collect_crash = [&]() {
    auto c = std::find(s->crashed.begin(), s->crashed.end(), ticket);
    if (c == s->crashed.end()) return false;
    s->crashed.erase(c);
    return true;
  };
  if (collect_crash()) return MGB_E_OOM;
  if (s->tasks.find(ticket) == s->tasks.end()) return MGB_E_UNKNOWN_TICKET;
  std::condition_variable own;
  const bool first = s->waiters.emplace(ticket, &own).second;
  std::condition_variable& on = first ? own : s->cv;
  if (!first) ++s->shared_waiters;
  bool in_time = true;
  if (timeout_ns < 0) on.wait(lk, admitted);
  else in_time = on.wait_for(lk, std::chrono::nanoseconds(timeout_ns), admitted);
  if (first) s->waiters.erase(ticket);
  else --s->shared_waiters;
  if (!in_time) return MGB_TIMEOUT;
  auto it = s->tasks.find(ticket);
  if (it == s->tasks.end()) return collect_crash() ? MGB_E_OOM : MGB_E_UNKNOWN_TICKET;  // rejected / cancelled meanwhile
  return s->fill(it->second, out, lk);
}

int mgb_task_cancel(mgb_sched* s, uint64_t ticket) {
  if (!s) return MGB_E_INVAL;
  std::lock_guard<std::mutex> lk(s->mu);
  uint64_t cause = s->log(MGB_EV_CANCEL, nullptr, 0, ticket, 0, {}, {}, 0, 0, 0);
  s->trace.back().cause_seq = (uint32_t)cause;
  auto it = s->tasks.find(ticket);
  if (it == s->tasks.end() || it->second.state == State::Draining) {
    s->log(MGB_EV_REJECT, nullptr, 0, ticket, 0, {}, {}, 0, MGB_E_UNKNOWN_TICKET, cause);
    return MGB_E_UNKNOWN_TICKET;
  }
  if (it->second.state != State::Waiting) {
    s->log(MGB_EV_REJECT, &it->second, 0, 0, 0, {}, {}, 0, MGB_E_BAD_STATE, cause);
    return MGB_E_BAD_STATE;
  }
  s->log(MGB_EV_CANCELLED, &it->second, 0, 0, 0, {}, {}, 0, 0, cause);
  s->waitq.erase(std::find(s->waitq.begin(), s->waitq.end(), ticket));
  s->tasks.erase(it);
  s->wake(ticket);                              // a thread waiting for the cancelled task learns of it
  s->rescan(cause);
  return MGB_OK;
}

int mgb_task_grow(mgb_sched* s, uint64_t ticket, uint64_t extra_bytes) {
  if (!s) return MGB_E_INVAL;
  std::lock_guard<std::mutex> lk(s->mu);
  uint64_t cause = s->log(MGB_EV_GROW, nullptr, 0, ticket, extra_bytes, {}, {}, 0, 0, 0);
  s->trace.back().cause_seq = (uint32_t)cause;
  auto it = s->tasks.find(ticket);
  if (it == s->tasks.end() || it->second.state == State::Draining) {
    s->log(MGB_EV_REJECT, nullptr, 0, ticket, extra_bytes, {}, {}, 0, MGB_E_UNKNOWN_TICKET, cause);
    return MGB_E_UNKNOWN_TICKET;
  }
  Task& t = it->second;
  if (t.state != State::Running) {
    s->log(MGB_EV_REJECT, &t, 0, 0, 0, {}, {}, 0, MGB_E_BAD_STATE, cause);
    return MGB_E_BAD_STATE;
  }
  if (extra_bytes > s->free_bytes) {
    s->log(MGB_EV_REJECT, &t, 0, 0, 0, {}, {}, 0, MGB_E_BUSY, cause);
    return MGB_E_BUSY;
  }
  // bytes that released-on-stream tasks may still be using: what the task enqueues from now on
  // starts behind them
  if (s->pending_mem != 0u && extra_bytes > s->free_bytes - std::min(s->free_bytes, s->pending_mem))
    for (const mgb_sched::MemPending& m : s->mem_pending) {
      bool have = false;
      for (const Dep& d0 : t.deps) have = have || d0.ticket == m.ticket;
      if (have) continue;
      t.deps.push_back({m.ticket, m.ev, m.stream});
      if (t.deps_issued && t.stream && m.ev && m.stream != t.stream) (void)hipStreamWaitEvent(t.stream, m.ev, 0);
    }
  s->free_bytes -= extra_bytes;
  t.mem += extra_bytes;
  s->log(MGB_EV_GROWN, &t, 0, 0, 0, {}, {}, t.granted, 0, cause);
  return MGB_OK;
}

int mgb_task_launch(mgb_sched* s, uint64_t ticket, int (*enqueue)(void* stream, void* user),
                    void* user) {
  if (!s || !enqueue) return MGB_E_INVAL;
  hipStream_t stream = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  bool hip = false;
  uint32_t granted = 0;
  {
    std::unique_lock<std::mutex> lk(s->mu);
    auto it = s->tasks.find(ticket);
    if (it == s->tasks.end()) return MGB_E_UNKNOWN_TICKET;
    if (it->second.state != State::Running) return MGB_E_BAD_STATE;
    hip = s->d.backend == MGB_BACKEND_HIP;
    if (hip) {
      int rc = s->bind_stream(it->second, lk);
      if (rc != MGB_OK) return rc;
      it = s->tasks.find(ticket);
      if (it == s->tasks.end()) return MGB_E_UNKNOWN_TICKET;
    }
    stream = it->second.stream;
    e0 = it->second.ev_start;
    e1 = it->second.ev_stop;
    it->second.launched = true;
    granted = it->second.granted;
  }
  if (hip && s->tag_partitions && granted != 0u) {
    uint32_t first = 0, count = 0;
    while (!(granted >> first & 1u)) ++first;
    for (uint32_t g = 0; g < 32u; ++g) count += granted >> g & 1u;
    (void)mgb_internal_tag_partition(stream, first, count);
  }
  if (hip) {
    hipError_t e = hipSetDevice(s->d.device);
    if (e == hipSuccess) e = hipEventRecord(e0, stream);
    if (e != hipSuccess) {
      set_error("hipEventRecord", e);
      return MGB_E_BACKEND;
    }
  }
  int rc = enqueue((void*)stream, user);
  if (hip) {
    hipError_t e = hipEventRecord(e1, stream);
    if (e != hipSuccess) {
      set_error("hipEventRecord", e);
      return MGB_E_BACKEND;
    }
  }
  return rc;
}

int mgb_task_sync(mgb_sched* s, uint64_t ticket, double* gpu_ms) {
  if (!s) return MGB_E_INVAL;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  bool launched = false, draining = false;
  {
    std::lock_guard<std::mutex> lk(s->mu);
    auto it = s->tasks.find(ticket);
    if (it == s->tasks.end()) return MGB_E_UNKNOWN_TICKET;
    if (it->second.state == State::Waiting) return MGB_E_BAD_STATE;
    draining = it->second.state == State::Draining;
    if (draining) {
      // one thread waits for a draining task and forgets it; its events go back to the pool then
      if (it->second.syncing) return MGB_E_BAD_STATE;
      it->second.syncing = true;
    }
    e0 = it->second.ev_start;
    e1 = it->second.ev_stop;
    launched = it->second.launched;
  }
  if (gpu_ms) *gpu_ms = 0.0;
  double ms = 0.0, t_start = 0.0, t_stop = 0.0;
  int rc = MGB_OK;
  if (s->d.backend == MGB_BACKEND_HIP && launched) {
    hipError_t e = hipEventSynchronize(e1);
    float f = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&f, e0, e1);
    ms = f;
    if (e == hipSuccess) e = hipEventElapsedTime(&f, s->epoch, e0);
    t_start = f;
    if (e == hipSuccess) e = hipEventElapsedTime(&f, s->epoch, e1);
    t_stop = f;
    if (e != hipSuccess) {
      set_error("mgb_task_sync: wait for / read the task's events", e);
      rc = MGB_E_BACKEND;
    }
  }
  const uint64_t seen = now_ns();
  std::lock_guard<std::mutex> lk(s->mu);
  if (rc == MGB_OK) {
    if (mgb_task_record* a = s->record_of(ticket)) {
      a->gpu_ms = ms;
      a->gpu_start_ms = t_start;
      a->gpu_stop_ms = t_stop;
      a->done_ns = seen;
    }
    if (gpu_ms) *gpu_ms = ms;
  }
  if (draining) s->retire(ticket);              // (also after a failed wait: nothing more can be learnt)
  return rc;
}

int mgb_task_complete(mgb_sched* s, uint64_t ticket) {
  if (!s) return MGB_E_INVAL;
  std::lock_guard<std::mutex> lk(s->mu);
  return s->complete_locked(ticket);
}

int mgb_task_complete_on_stream(mgb_sched* s, uint64_t ticket) {
  if (!s) return MGB_E_INVAL;
  std::lock_guard<std::mutex> lk(s->mu);
  return s->complete_locked(ticket, true);
}

int64_t mgb_task_deps(mgb_sched* s, uint64_t ticket, uint64_t* out, uint64_t cap) {
  if (!s || (!out && cap)) return MGB_E_INVAL;
  std::lock_guard<std::mutex> lk(s->mu);
  auto it = s->tasks.find(ticket);
  if (it == s->tasks.end()) return MGB_E_UNKNOWN_TICKET;
  if (it->second.state != State::Running) return MGB_E_BAD_STATE;
  const std::vector<Dep>& deps = it->second.deps;
  for (size_t i = 0; i < deps.size() && i < cap; ++i) out[i] = deps[i].ticket;
  return (int64_t)deps.size();
}

int64_t mgb_task_records(mgb_sched* s, uint64_t first_ticket, mgb_task_record* out, uint64_t cap) {
  if (!s || (!out && cap)) return MGB_E_INVAL;
  std::lock_guard<std::mutex> lk(s->mu);
  if (first_ticket <= s->record_base) first_ticket = s->record_base + 1;
  const uint64_t at = first_ticket - s->record_base - 1;
  if (at >= s->records.size()) return 0;
  const uint64_t n = std::min<uint64_t>(cap, s->records.size() - at);
  for (uint64_t i = 0; i < n; ++i) out[i] = s->records[at + i];
  return (int64_t)n;
}

int mgb_accounting(const mgb_task_record* recs, uint64_t n, const uint64_t* arrival_ns,
                   const double* ref_gpu_ms, mgb_summary* out) {
  if (!out || (!recs && n)) return MGB_E_INVAL;
  std::memset(out, 0, sizeof *out);
  uint64_t first = 0, last = 0;
  double turn_sum = 0.0, wait_sum = 0.0, slow_sum = 0.0;
  uint64_t n_slow = 0;
  for (uint64_t i = 0; i < n; ++i) {
    const mgb_task_record& r = recs[i];
    if (r.status == MGB_E_OOM) { ++out->n_crashed; continue; }
    if (r.status != MGB_OK) { ++out->n_unfinished; continue; }
    const uint64_t arr = arrival_ns ? arrival_ns[i] : r.probe_ns;
    if (r.done_ns < arr || r.admit_ns < r.probe_ns) return MGB_E_INVAL;
    const double turn = 1e-6 * (double)(r.done_ns - arr), wait = 1e-6 * (double)(r.admit_ns - r.probe_ns);
    if (out->n_done == 0u || arr < first) first = arr;
    if (out->n_done == 0u || r.done_ns > last) last = r.done_ns;
    ++out->n_done;
    turn_sum += turn;
    wait_sum += wait;
    if (turn > out->max_turnaround_ms) out->max_turnaround_ms = turn;
    if (wait > out->max_wait_ms) out->max_wait_ms = wait;
    out->gpu_busy_ms += r.gpu_ms;
    if (ref_gpu_ms && ref_gpu_ms[i] > 0.0) {
      const double sl = r.gpu_ms / ref_gpu_ms[i] - 1.0;
      if (n_slow == 0u || sl > out->max_slowdown) out->max_slowdown = sl;
      slow_sum += sl;
      ++n_slow;
    }
  }
  if (out->n_done != 0u) {
    out->makespan_ms = 1e-6 * (double)(last - first);
    out->tasks_per_s = last > first ? (double)out->n_done / (1e-9 * (double)(last - first)) : 0.0;
    out->mean_turnaround_ms = turn_sum / (double)out->n_done;
    out->mean_wait_ms = wait_sum / (double)out->n_done;
  }
  if (n_slow != 0u) out->mean_slowdown = slow_sum / (double)n_slow;
  return MGB_OK;
}

int mgb_sched_stats(mgb_sched* s, mgb_stats* out) {
  if (!s || !out) return MGB_E_INVAL;
  std::lock_guard<std::mutex> lk(s->mu);
  out->free_bytes = s->free_bytes;
  out->free_granules = s->free_map;
  out->n_waiting = (uint32_t)s->waitq.size();
  out->n_running = s->n_running_now;
  out->n_streams = s->n_streams;
  out->n_events = s->trace_base + s->trace.size();
  return MGB_OK;
}

int64_t mgb_trace_read(mgb_sched* s, uint64_t first, mgb_trace_rec* out, uint64_t cap) {
  if (!s || (!out && cap)) return MGB_E_INVAL;
  std::lock_guard<std::mutex> lk(s->mu);
  if (first < s->trace_base) first = s->trace_base;            // older records were dropped
  if (first - s->trace_base >= s->trace.size()) return 0;
  const uint64_t at = first - s->trace_base;
  uint64_t n = std::min<uint64_t>(cap, s->trace.size() - at);
  std::memcpy(out, s->trace.data() + at, n * sizeof(mgb_trace_rec));
  return (int64_t)n;
}

int mgb_trace_dump(mgb_sched* s, const char* path) {
  if (!s || !path) return MGB_E_INVAL;
  std::lock_guard<std::mutex> lk(s->mu);
  FILE* f = std::fopen(path, "w");
  if (!f) return MGB_E_INVAL;
  for (const mgb_trace_rec& r : s->trace) {
    std::fprintf(f,
                 "{\"seq\":%llu,\"t_ns\":%llu,\"kind\":%u,\"task_id\":%llu,\"ticket\":%llu,"
                 "\"mem_bytes\":%llu,\"free_bytes\":%llu,\"code\":%d,\"granule_mask\":%u,"
                 "\"free_granules\":%u,\"demand\":%u,\"cause_seq\":%u,\"grid\":[%u,%u,%u],"
                 "\"block\":[%u,%u,%u],\"cu_mask\":[%u,%u,%u,%u,%u,%u,%u,%u]}\n",
                 (unsigned long long)r.seq, (unsigned long long)r.t_ns, r.kind,
                 (unsigned long long)r.task_id, (unsigned long long)r.ticket,
                 (unsigned long long)r.mem_bytes, (unsigned long long)r.free_bytes, r.code,
                 r.granule_mask, r.free_granules, r.demand, r.cause_seq, r.grid.x, r.grid.y,
                 r.grid.z, r.block.x, r.block.y, r.block.z, r.cu_mask[0], r.cu_mask[1],
                 r.cu_mask[2], r.cu_mask[3], r.cu_mask[4], r.cu_mask[5], r.cu_mask[6],
                 r.cu_mask[7]);
  }
  std::fclose(f);
  return MGB_OK;
}

}  // extern "C"
