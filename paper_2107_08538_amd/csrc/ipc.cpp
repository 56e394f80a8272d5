// Multi-process front end (Sec. IV of the paper: independent processes talk to the scheduler
// over shared memory).
//
// The scheduler lives in one process (the server; it only takes decisions, so it can run on the
// null backend and never touch the device).  Every other process is a client: it claims a slot
// in a POSIX shared-memory segment, writes a request (probe / wait / cancel / grow / complete),
// posts the slot's request semaphore and sleeps on its response semaphore.  One server thread
// per slot executes the request against the in-process scheduler; a wait for admission blocks
// that thread, not the others.  A placement comes back as a CU mask: the client builds its own
// CU-masked stream from it (a hardware queue belongs to the process that created it), so no
// device handle ever crosses a process boundary.
//
// A client that dies without giving its tasks back would hold memory and CUs for ever: each
// slot thread checks, whenever it has been idle for a moment, that the owner's process still
// exists, and otherwise withdraws its queued probes and completes its resident tasks.
#include "../../include/mgb.h"
#include "launch_util.h"

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <fcntl.h>
#include <semaphore.h>
#include <signal.h>
#include <sys/mman.h>
#include <sys/stat.h>
#include <time.h>
#include <unistd.h>

#include <atomic>
#include <chrono>
#include <cerrno>
#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <new>
#include <string>
#include <thread>
#include <vector>

namespace {

constexpr uint64_t kMagic = 0x4d47422d49504331ull;   // "MGB-IPC1"
constexpr uint32_t kMaxSlots = 64;

enum Op : uint32_t { OP_PROBE = 1, OP_WAIT, OP_CANCEL, OP_GROW, OP_COMPLETE, OP_STATS, OP_BYE };

struct Slot {
  std::atomic<uint32_t> owner;   // 0 = free, else the client's process id
  sem_t req, resp;
  uint32_t op;
  int32_t rc;
  uint32_t wg_per_cu;
  uint64_t task_id, ticket, bytes;
  int64_t timeout_ns;
  mgb_dim3 grid, block;
  mgb_placement placement;       // the stream field stays NULL: streams are made by the client
  mgb_stats stats;
};

struct Segment {
  uint64_t magic;
  uint32_t n_slots;
  std::atomic<uint32_t> stopping;
  int32_t server_pid;
  mgb_device_desc desc;
  Slot slots[1];
};

size_t segment_bytes(uint32_t n_slots) { return sizeof(Segment) + (size_t)(n_slots - 1u) * sizeof(Slot); }

timespec deadline_in(long ms) {
  timespec ts;
  clock_gettime(CLOCK_REALTIME, &ts);
  ts.tv_nsec += (ms % 1000) * 1000000L;
  ts.tv_sec += ms / 1000 + ts.tv_nsec / 1000000000L;
  ts.tv_nsec %= 1000000000L;
  return ts;
}

bool process_alive(uint32_t pid) { return ::kill((pid_t)pid, 0) == 0 || errno != ESRCH; }

std::string shm_name(const char* name) { return std::string("/mgb.") + name; }

}  // namespace

struct mgb_server {
  mgb_sched* s = nullptr;
  std::string name;
  Segment* seg = nullptr;
  size_t bytes = 0;
  std::vector<std::thread> threads;
  std::vector<std::vector<uint64_t>> held;   // per slot: tickets of its live tasks (slot thread only)
  std::atomic<uint64_t> reclaimed{0};

  void forget(uint32_t i, uint64_t ticket) {
    auto& v = held[i];
    for (size_t k = 0; k < v.size(); ++k)
      if (v[k] == ticket) {
        v.erase(v.begin() + (long)k);
        return;
      }
  }
  // the owner of slot i is gone: withdraw what it queued, finish what it ran
  void reclaim(uint32_t i) {
    for (uint64_t t : held[i])
      if (mgb_task_cancel(s, t) != MGB_OK) (void)mgb_task_complete(s, t);
    reclaimed += held[i].size();
    held[i].clear();
    // a request the dead client never posted, or an answer it never collected, must not greet
    // the slot's next owner
    while (sem_trywait(&seg->slots[i].req) == 0) {}
    while (sem_trywait(&seg->slots[i].resp) == 0) {}
    seg->slots[i].owner.store(0);
  }
  void serve(uint32_t i) {
    Slot& sl = seg->slots[i];
    while (!seg->stopping.load()) {
      timespec ts = deadline_in(100);
      if (sem_timedwait(&sl.req, &ts) != 0) {
        const uint32_t owner = sl.owner.load();
        if (owner != 0u && !process_alive(owner)) reclaim(i);
        continue;
      }
      if (seg->stopping.load()) break;
      switch (sl.op) {
        case OP_PROBE:
          sl.rc = mgb_task_probe_ex(s, sl.task_id, sl.bytes, sl.grid, sl.block, sl.wg_per_cu, &sl.placement);
          if (sl.rc == MGB_OK || sl.rc == MGB_WAIT) held[i].push_back(sl.placement.ticket);
          break;
        case OP_WAIT: {
          // in slices, so that a client that died while waiting is noticed
          int64_t left = sl.timeout_ns;
          const int64_t slice = 100 * 1000 * 1000;
          for (;;) {
            const int64_t step = (sl.timeout_ns < 0 || left > slice) ? slice : left;
            sl.rc = mgb_task_wait(s, sl.ticket, step, &sl.placement);
            if (sl.rc != MGB_TIMEOUT) break;
            if (sl.timeout_ns >= 0 && (left -= step) <= 0) break;
            if (seg->stopping.load() || !process_alive(sl.owner.load())) break;
          }
          if (sl.rc == MGB_E_OOM || sl.rc == MGB_E_UNKNOWN_TICKET) forget(i, sl.ticket);
          break;
        }
        case OP_CANCEL:
          sl.rc = mgb_task_cancel(s, sl.ticket);
          if (sl.rc == MGB_OK) forget(i, sl.ticket);
          break;
        case OP_GROW:
          sl.rc = mgb_task_grow(s, sl.ticket, sl.bytes);
          break;
        case OP_COMPLETE:
          sl.rc = mgb_task_complete(s, sl.ticket);
          if (sl.rc == MGB_OK) forget(i, sl.ticket);
          break;
        case OP_STATS:
          sl.rc = mgb_sched_stats(s, &sl.stats);
          break;
        case OP_BYE:
          // (the client gives the slot up itself once it has this answer: were the slot freed
          // here, a client connecting right now could take it and read this answer as its own)
          sl.rc = held[i].empty() ? MGB_OK : MGB_E_BUSY;
          break;
        default:
          sl.rc = MGB_E_INVAL;
      }
      sl.placement.stream = nullptr;
      sem_post(&sl.resp);
    }
  }
};

struct mgb_client;
namespace {
// Takes the connection for one request.  A mutex is not fair: a waiter that takes it again at
// once for its next slice could starve everybody else, so other requests announce themselves
// and the waiter stays away while any are announced.
struct Turn {
  explicit Turn(mgb_client* c);
  ~Turn();
  mgb_client* c;
};
}  // namespace

struct mgb_client {
  Segment* seg = nullptr;
  size_t bytes = 0;
  uint32_t slot = 0;
  std::mutex mu;                                   // one request at a time per connection
  std::atomic<int> callers{0};                     // threads inside or queued for a request other than a wait slice
  std::map<std::vector<uint32_t>, hipStream_t> streams;   // CU mask -> this process's masked stream

  int gone() {
    mgb_internal_set_error_text("the scheduler process has gone away");
    return MGB_E_BACKEND;
  }
  int call(Op op) {
    Slot& sl = seg->slots[slot];
    if (seg->stopping.load()) return gone();
    sl.op = op;
    sem_post(&sl.req);
    for (;;) {
      timespec ts = deadline_in(500);
      const bool woke = sem_timedwait(&sl.resp, &ts) == 0;
      if (seg->stopping.load() || !process_alive((uint32_t)seg->server_pid)) return gone();
      if (woke) return sl.rc;
    }
  }
};

namespace {
Turn::Turn(mgb_client* cl) : c(cl) {
  ++c->callers;
  c->mu.lock();
}
Turn::~Turn() {
  c->mu.unlock();
  --c->callers;
}
}  // namespace

extern "C" {

int mgb_server_start(mgb_sched* s, const char* name, uint32_t n_slots, mgb_server** out) {
  if (!s || !name || !out || n_slots == 0u || n_slots > kMaxSlots || std::strlen(name) > 200) return MGB_E_INVAL;
  *out = nullptr;
  const std::string path = shm_name(name);
  const int fd = shm_open(path.c_str(), O_CREAT | O_EXCL | O_RDWR, 0600);
  if (fd < 0) {
    mgb_internal_set_error_text(errno == EEXIST ? "a scheduler segment of that name exists already" : "shm_open failed");
    return errno == EEXIST ? MGB_E_BUSY : MGB_E_BACKEND;
  }
  const size_t bytes = segment_bytes(n_slots);
  void* p = MAP_FAILED;
  if (ftruncate(fd, (off_t)bytes) == 0) p = mmap(nullptr, bytes, PROT_READ | PROT_WRITE, MAP_SHARED, fd, 0);
  close(fd);
  if (p == MAP_FAILED) {
    shm_unlink(path.c_str());
    mgb_internal_set_error_text("mapping the scheduler segment failed");
    return MGB_E_BACKEND;
  }
  mgb_server* sv = new (std::nothrow) mgb_server;
  if (!sv) {
    munmap(p, bytes);
    shm_unlink(path.c_str());
    return MGB_E_BACKEND;
  }
  sv->s = s;
  sv->name = path;
  sv->bytes = bytes;
  sv->seg = new (p) Segment;
  sv->seg->n_slots = n_slots;
  sv->seg->stopping.store(0);
  sv->seg->server_pid = (int32_t)getpid();
  std::memset(&sv->seg->desc, 0, sizeof sv->seg->desc);
  sv->held.resize(n_slots);
  for (uint32_t i = 0; i < n_slots; ++i) {
    Slot& sl = sv->seg->slots[i];
    new (&sl.owner) std::atomic<uint32_t>(0);
    sem_init(&sl.req, 1, 0);
    sem_init(&sl.resp, 1, 0);
  }
  sv->seg->magic = kMagic;                          // last: a client that sees it sees the rest
  for (uint32_t i = 0; i < n_slots; ++i) sv->threads.emplace_back([sv, i] { sv->serve(i); });
  *out = sv;
  return MGB_OK;
}

int mgb_server_stop(mgb_server* sv) {
  if (!sv) return MGB_E_INVAL;
  sv->seg->stopping.store(1);
  for (uint32_t i = 0; i < sv->seg->n_slots; ++i) sem_post(&sv->seg->slots[i].req);
  for (auto& t : sv->threads) t.join();
  for (uint32_t i = 0; i < sv->seg->n_slots; ++i) {
    sem_post(&sv->seg->slots[i].resp);              // a client caught mid-call sees `stopping`
  }
  shm_unlink(sv->name.c_str());
  munmap(sv->seg, sv->bytes);
  delete sv;
  return MGB_OK;
}

uint64_t mgb_server_reclaimed(mgb_server* sv) { return sv ? sv->reclaimed.load() : 0; }

int mgb_client_connect(const char* name, mgb_client** out) {
  if (!name || !out) return MGB_E_INVAL;
  *out = nullptr;
  const std::string path = shm_name(name);
  const int fd = shm_open(path.c_str(), O_RDWR, 0600);
  if (fd < 0) {
    mgb_internal_set_error_text("no scheduler segment of that name");
    return MGB_E_BACKEND;
  }
  struct stat st;
  void* p = MAP_FAILED;
  if (fstat(fd, &st) == 0 && (size_t)st.st_size >= sizeof(Segment))
    p = mmap(nullptr, (size_t)st.st_size, PROT_READ | PROT_WRITE, MAP_SHARED, fd, 0);
  close(fd);
  if (p == MAP_FAILED) {
    mgb_internal_set_error_text("mapping the scheduler segment failed");
    return MGB_E_BACKEND;
  }
  Segment* seg = (Segment*)p;
  if (seg->magic != kMagic || (size_t)st.st_size < segment_bytes(seg->n_slots) || seg->stopping.load()) {
    munmap(p, (size_t)st.st_size);
    mgb_internal_set_error_text("not a live scheduler segment");
    return MGB_E_BACKEND;
  }
  const uint32_t pid = (uint32_t)getpid();
  for (uint32_t i = 0; i < seg->n_slots; ++i) {
    uint32_t expect = 0;
    if (seg->slots[i].owner.compare_exchange_strong(expect, pid)) {
      mgb_client* c = new (std::nothrow) mgb_client;
      if (!c) {
        seg->slots[i].owner.store(0);
        munmap(p, (size_t)st.st_size);
        return MGB_E_BACKEND;
      }
      c->seg = seg;
      c->bytes = (size_t)st.st_size;
      c->slot = i;
      *out = c;
      return MGB_OK;
    }
  }
  munmap(p, (size_t)st.st_size);
  return MGB_E_BUSY;                                // every slot is taken
}

int mgb_client_disconnect(mgb_client* c) {
  if (!c) return MGB_E_INVAL;
  {
    std::lock_guard<std::mutex> lk(c->mu);
    const int rc = c->call(OP_BYE);                 // MGB_E_BACKEND: the server is gone, nothing left to tell it
    if (rc == MGB_E_BUSY) return rc;                // tasks still held: complete or cancel them first
    if (rc == MGB_OK) c->seg->slots[c->slot].owner.store(0);   // answer collected: the slot is free again
    for (auto& kv : c->streams) (void)hipStreamDestroy(kv.second);
    c->streams.clear();
    munmap(c->seg, c->bytes);
  }
  delete c;
  return MGB_OK;
}

int mgb_client_probe(mgb_client* c, uint64_t task_id, uint64_t mem_bytes, mgb_dim3 grid, mgb_dim3 block,
                     uint32_t wg_per_cu, mgb_placement* out) {
  if (!c || !out) return MGB_E_INVAL;
  Turn turn(c);
  Slot& sl = c->seg->slots[c->slot];
  sl.task_id = task_id;
  sl.bytes = mem_bytes;
  sl.grid = grid;
  sl.block = block;
  sl.wg_per_cu = wg_per_cu;
  const int rc = c->call(OP_PROBE);
  *out = sl.placement;
  return rc;
}

// A connection carries one request at a time, and a wait for admission ends only when some task
// is completed - possibly by another thread of this process, over this connection.  The wait
// therefore goes to the server in slices of 2 ms and gives the connection up between them (a
// task admitted between two slices is found admitted by the next one at once).
int mgb_client_wait(mgb_client* c, uint64_t ticket, int64_t timeout_ns, mgb_placement* out) {
  if (!c || !out) return MGB_E_INVAL;
  const int64_t slice = 2 * 1000 * 1000;
  int64_t left = timeout_ns;
  for (;;) {
    const int64_t step = (timeout_ns < 0 || left > slice) ? slice : left;
    int rc;
    {
      std::lock_guard<std::mutex> lk(c->mu);
      Slot& sl = c->seg->slots[c->slot];
      sl.ticket = ticket;
      sl.timeout_ns = step;
      rc = c->call(OP_WAIT);
      *out = sl.placement;
    }
    if (rc != MGB_TIMEOUT) return rc;
    if (timeout_ns >= 0 && (left -= step) <= 0) return MGB_TIMEOUT;
    while (c->callers.load() > 0) std::this_thread::sleep_for(std::chrono::microseconds(50));
  }
}

static int ticket_call(mgb_client* c, Op op, uint64_t ticket, uint64_t bytes) {
  if (!c) return MGB_E_INVAL;
  Turn turn(c);
  Slot& sl = c->seg->slots[c->slot];
  sl.ticket = ticket;
  sl.bytes = bytes;
  return c->call(op);
}

int mgb_client_cancel(mgb_client* c, uint64_t ticket) { return ticket_call(c, OP_CANCEL, ticket, 0); }
int mgb_client_grow(mgb_client* c, uint64_t ticket, uint64_t extra_bytes) { return ticket_call(c, OP_GROW, ticket, extra_bytes); }
int mgb_client_complete(mgb_client* c, uint64_t ticket) { return ticket_call(c, OP_COMPLETE, ticket, 0); }

int mgb_client_stats(mgb_client* c, mgb_stats* out) {
  if (!c || !out) return MGB_E_INVAL;
  Turn turn(c);
  const int rc = c->call(OP_STATS);
  *out = c->seg->slots[c->slot].stats;
  return rc;
}

int mgb_client_stream(mgb_client* c, const mgb_placement* placement, void** stream) {
  if (!c || !placement || !stream) return MGB_E_INVAL;
  std::vector<uint32_t> key(placement->cu_mask, placement->cu_mask + 8);
  // Mask bit i selects a CU of XCD (i mod 8).  A mask that leaves one of the 8 XCDs without a CU is
  // never handed to the runtime (creating a stream with a one-bit mask ended in a crash inside the
  // runtime, on the host); a server on the null backend may legally grant such masks (granules of
  // 1, 2 or 4 CUs), so the check belongs here.
  uint32_t residues = 0;
  for (uint32_t w : key) residues |= (w | w >> 8 | w >> 16 | w >> 24) & 0xffu;
  if (residues != 0xffu) {
    mgb_internal_set_error_text("mgb_client_stream: the CU mask leaves an XCD without a CU");
    return MGB_E_INVAL;
  }
  Turn turn(c);
  auto it = c->streams.find(key);
  if (it == c->streams.end()) {
    hipStream_t st = nullptr;
    hipError_t e = hipExtStreamCreateWithCUMask(&st, 8, key.data());
    if (e != hipSuccess) {
      mgb_internal_set_error("hipExtStreamCreateWithCUMask", e);
      return MGB_E_BACKEND;
    }
    it = c->streams.emplace(key, st).first;
  }
  *stream = (void*)it->second;
  return MGB_OK;
}

}  // extern "C"
