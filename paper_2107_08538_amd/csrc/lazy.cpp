// Lazy runtime (Sec. III-A of the paper, "Lazy Runtime").
//
// A program whose allocations, copies and kernel launches sit in different
// functions cannot be given a probe by static analysis alone.  Its device
// memory calls are redirected here instead: an allocation only hands out a
// pseudo address, copies and fills to that address are recorded (with their
// bytes) in the object's queue, and nothing touches the device until a kernel
// launch is prepared.  At that point the memory objects the kernel names are
// known, so the task's footprint is known: the probe goes to the scheduler, and
// once a placement is granted the objects are allocated, their queues replayed
// in order on the task's stream, and the pseudo addresses translated.
//
// Launches that share a memory object belong to one task (Algorithm 1 merges
// such unit tasks; here the merge happens as the launches arrive): a launch
// whose objects are already on the device joins their task, memory it adds is
// asked for with mgb_task_grow, and a launch that touches objects of two tasks
// fuses them (the later stream waits for the other).  A task ends when its last
// memory object is freed, which is when its tickets are completed.
//
// With the null backend "device memory" is host memory, so all of the above can
// be exercised without a GPU.
#include "../../include/mgb.h"
#include "launch_util.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <map>
#include <memory>
#include <mutex>
#include <set>
#include <vector>

namespace {

constexpr uint64_t kTag = 0xA5ull << 56;       // pseudo address = tag | object id << 40 | offset
constexpr uint64_t kOffMask = (1ull << 40) - 1;
constexpr uint32_t kMaxObjects = 1u << 16;

enum OpKind { OP_H2D, OP_MEMSET };
struct Op {
  OpKind kind;
  uint64_t offset, bytes;
  int value;                       // OP_MEMSET
  std::vector<uint8_t> data;       // OP_H2D: the bytes as they were when the copy was called
};

struct LTask {
  std::vector<uint64_t> tickets;   // scheduler tickets (more than one after a fusion)
  std::vector<void*> streams;      // their streams; streams[0] is the task's stream
  std::set<uint32_t> objs;
};

struct Obj {
  uint64_t bytes = 0;
  std::vector<Op> queue;           // recorded while unbound
  void* real = nullptr;            // device (or, null backend, host) memory once bound
  std::shared_ptr<LTask> task;     // owner once bound
};

}  // namespace

struct mgb_lazy {
  mgb_sched* s = nullptr;
  bool hip = false;
  int device = 0;
  std::mutex mu;
  std::map<uint32_t, Obj> objs;
  uint32_t next_id = 1;
  mgb_lazy_stats st{};

  Obj* lookup(uint64_t pseudo, uint32_t* id, uint64_t* off) {
    if ((pseudo & (0xFFull << 56)) != kTag) return nullptr;
    const uint32_t i = (uint32_t)((pseudo >> 40) & 0xFFFFu);
    auto it = objs.find(i);
    if (it == objs.end()) return nullptr;
    *id = i;
    *off = pseudo & kOffMask;
    return &it->second;
  }

  int backend_error(const char* what, hipError_t e) {
    mgb_internal_set_error(what, e);
    return MGB_E_BACKEND;
  }

  int dev_alloc(uint64_t bytes, void** out) {
    const uint64_t n = bytes ? bytes : 1;
    if (!hip) {
      *out = std::aligned_alloc(256, (n + 255) / 256 * 256);
      return *out ? MGB_OK : MGB_E_BACKEND;
    }
    hipError_t e = hipSetDevice(device);
    if (e == hipSuccess) e = hipMalloc(out, n);
    return e == hipSuccess ? MGB_OK : backend_error("hipMalloc", e);
  }
  void dev_free(void* p) {
    if (!p) return;
    if (!hip) std::free(p);
    else (void)hipFree(p);
  }
  int stream_sync(void* stream) {
    if (!hip) return MGB_OK;
    hipError_t e = hipStreamSynchronize((hipStream_t)stream);
    return e == hipSuccess ? MGB_OK : backend_error("hipStreamSynchronize", e);
  }
  // one recorded (or immediate) operation on bound memory, in stream order
  int apply(void* stream, uint8_t* base, OpKind kind, uint64_t off, uint64_t bytes, int value, const void* src) {
    if (bytes == 0) return MGB_OK;
    if (!hip) {
      if (kind == OP_H2D) std::memcpy(base + off, src, bytes);
      else std::memset(base + off, value, bytes);
      return MGB_OK;
    }
    hipError_t e = kind == OP_H2D ? hipMemcpyAsync(base + off, src, bytes, hipMemcpyHostToDevice, (hipStream_t)stream)
                                  : hipMemsetAsync(base + off, value, bytes, (hipStream_t)stream);
    return e == hipSuccess ? MGB_OK : backend_error(kind == OP_H2D ? "hipMemcpyAsync" : "hipMemsetAsync", e);
  }
  // make `first` wait for everything enqueued so far on `other`
  int order_after(void* first, void* other) {
    if (!hip || first == other) return MGB_OK;
    hipEvent_t ev;
    hipError_t e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventRecord(ev, (hipStream_t)other);
    if (e == hipSuccess) e = hipStreamWaitEvent((hipStream_t)first, ev, 0);
    (void)hipEventDestroy(ev);    // released once the recorded work has completed
    return e == hipSuccess ? MGB_OK : backend_error("hipStreamWaitEvent", e);
  }
  // the task has lost its last object: drain its streams and give its tickets back
  int finish(const std::shared_ptr<LTask>& t) {
    int rc = MGB_OK;
    for (void* st : t->streams) {
      const int r = stream_sync(st);
      if (r != MGB_OK) rc = r;
    }
    for (uint64_t tk : t->tickets) {
      const int r = mgb_task_complete(s, tk);
      if (r != MGB_OK) rc = r;
    }
    --st.n_tasks;
    return rc;
  }
};

extern "C" {

int mgb_lazy_create(mgb_sched* s, mgb_lazy** out) {
  if (!s || !out) return MGB_E_INVAL;
  mgb_lazy* z = new (std::nothrow) mgb_lazy;
  if (!z) return MGB_E_BACKEND;
  z->s = s;
  z->hip = mgb_internal_backend(s) == MGB_BACKEND_HIP;
  z->device = mgb_internal_device(s);
  *out = z;
  return MGB_OK;
}

int mgb_lazy_destroy(mgb_lazy* z) {
  if (!z) return MGB_E_INVAL;
  {
    std::lock_guard<std::mutex> lk(z->mu);
    if (!z->objs.empty()) return MGB_E_BUSY;
  }
  delete z;
  return MGB_OK;
}

int mgb_lazy_malloc(mgb_lazy* z, uint64_t bytes, uint64_t* pseudo) {
  if (!z || !pseudo) return MGB_E_INVAL;
  if (bytes > kOffMask) return MGB_E_TOO_BIG;
  std::lock_guard<std::mutex> lk(z->mu);
  if (z->objs.size() >= kMaxObjects - 1u) return MGB_E_BUSY;
  while (z->next_id == 0u || z->objs.count(z->next_id)) z->next_id = (z->next_id + 1u) & (kMaxObjects - 1u);
  const uint32_t id = z->next_id;
  z->next_id = (z->next_id + 1u) & (kMaxObjects - 1u);
  z->objs[id].bytes = bytes;
  ++z->st.n_objects;
  *pseudo = kTag | ((uint64_t)id << 40);
  return MGB_OK;
}

static int write_op(mgb_lazy* z, uint64_t pseudo, OpKind kind, const void* src, int value, uint64_t bytes) {
  std::lock_guard<std::mutex> lk(z->mu);
  uint32_t id;
  uint64_t off;
  Obj* o = z->lookup(pseudo, &id, &off);
  if (!o) return MGB_E_UNKNOWN_TICKET;
  if (off > o->bytes || bytes > o->bytes - off) return MGB_E_INVAL;
  if (o->real) {
    // already on the device: executed now, in order with the task's kernels, and complete on
    // return as the call it stands in for would be
    void* stream = o->task->streams[0];
    int rc = z->apply(stream, (uint8_t*)o->real, kind, off, bytes, value, src);
    if (rc == MGB_OK) rc = z->stream_sync(stream);
    return rc;
  }
  Op op;
  op.kind = kind;
  op.offset = off;
  op.bytes = bytes;
  op.value = value;
  if (kind == OP_H2D) {
    op.data.assign((const uint8_t*)src, (const uint8_t*)src + bytes);
    z->st.staged_bytes += bytes;
  }
  o->queue.push_back(std::move(op));
  ++z->st.recorded_ops;
  return MGB_OK;
}

int mgb_lazy_memcpy_h2d(mgb_lazy* z, uint64_t dst_pseudo, const void* src_host, uint64_t bytes) {
  if (!z || (!src_host && bytes)) return MGB_E_INVAL;
  return write_op(z, dst_pseudo, OP_H2D, src_host, 0, bytes);
}

int mgb_lazy_memset(mgb_lazy* z, uint64_t dst_pseudo, int value, uint64_t bytes) {
  if (!z) return MGB_E_INVAL;
  return write_op(z, dst_pseudo, OP_MEMSET, nullptr, value, bytes);
}

int mgb_lazy_launch_prepare(mgb_lazy* z, uint64_t task_id, const uint64_t* pseudo_args, uint32_t n_args,
                            mgb_dim3 grid, mgb_dim3 block, uint32_t wg_per_cu, int64_t timeout_ns,
                            void** real_args, mgb_placement* placement) {
  if (!z || !pseudo_args || !real_args || !placement || n_args == 0u) return MGB_E_INVAL;
  std::unique_lock<std::mutex> lk(z->mu);
  // the memory objects the kernel names
  std::vector<uint32_t> ids(n_args);
  std::vector<uint64_t> offs(n_args);
  std::vector<uint32_t> fresh;                       // not yet on the device, each once
  std::vector<std::shared_ptr<LTask>> owners;        // tasks whose objects are named, each once
  uint64_t extra = 0;
  auto classify = [&]() {
    fresh.clear();
    owners.clear();
    extra = 0;
    for (uint32_t i = 0; i < n_args; ++i) {
      Obj* o = z->lookup(pseudo_args[i], &ids[i], &offs[i]);
      if (!o || offs[i] > o->bytes) return false;
      if (o->real) {
        if (std::find(owners.begin(), owners.end(), o->task) == owners.end()) owners.push_back(o->task);
      } else if (std::find(fresh.begin(), fresh.end(), ids[i]) == fresh.end()) {
        fresh.push_back(ids[i]);
        extra += o->bytes;
      }
    }
    return true;
  };
  if (!classify()) return MGB_E_UNKNOWN_TICKET;
  std::shared_ptr<LTask> task;
  if (owners.empty()) {
    // a new task: its footprint is what the kernel's objects add up to
    mgb_placement pl;
    int rc = mgb_task_probe_ex(z->s, task_id, extra, grid, block, wg_per_cu, &pl);
    if (rc == MGB_WAIT) {
      // The wait may be long and ends only when some task gives resources back, which other
      // threads do through this runtime (mgb_lazy_free): wait with the runtime unlocked, then
      // look at the objects again.  If another thread freed or bound one of them meanwhile the
      // footprint that was admitted is no longer this launch's: give the placement back.
      const uint64_t ticket = pl.ticket;
      const uint64_t asked = extra;
      lk.unlock();
      rc = mgb_task_wait(z->s, ticket, timeout_ns, &pl);
      // (a release may have admitted the task between the end of the wait and the withdrawal: then
      // the scheduler refuses to cancel a resident task, and the placement is this launch's after all)
      if (rc == MGB_TIMEOUT && mgb_task_cancel(z->s, ticket) == MGB_E_BAD_STATE) rc = mgb_task_wait(z->s, ticket, 0, &pl);
      lk.lock();
      if (rc == MGB_OK && (!classify() || !owners.empty() || extra != asked)) {
        (void)mgb_task_complete(z->s, ticket);
        return MGB_E_BAD_STATE;
      }
    }
    if (rc != MGB_OK) return rc;
    task = std::make_shared<LTask>();
    task->tickets.push_back(pl.ticket);
    task->streams.push_back(pl.stream);
    ++z->st.n_tasks;
    *placement = pl;
  } else {
    // joins the task(s) that own its objects; the oldest ticket's task absorbs the others
    std::sort(owners.begin(), owners.end(),
              [](const std::shared_ptr<LTask>& a, const std::shared_ptr<LTask>& b) { return a->tickets[0] < b->tickets[0]; });
    task = owners[0];
    // (the stream order first: if it fails nothing has been debited, and an order that a refused
    // growth leaves behind is harmless)
    for (size_t k = 1; k < owners.size(); ++k)
      for (void* st : owners[k]->streams) {
        const int rc = z->order_after(task->streams[0], st);
        if (rc != MGB_OK) return rc;
      }
    if (extra) {
      const int rc = mgb_task_grow(z->s, task->tickets[0], extra);
      if (rc != MGB_OK) return rc;                   // MGB_E_BUSY: nothing has changed, the caller may retry
    }
    for (size_t k = 1; k < owners.size(); ++k) {
      const std::shared_ptr<LTask>& other = owners[k];
      for (uint32_t id : other->objs) {
        z->objs[id].task = task;
        task->objs.insert(id);
      }
      task->tickets.insert(task->tickets.end(), other->tickets.begin(), other->tickets.end());
      task->streams.insert(task->streams.end(), other->streams.begin(), other->streams.end());
      other->objs.clear();
      --z->st.n_tasks;
    }
    std::memset(placement, 0, sizeof *placement);
    placement->ticket = task->tickets[0];
    placement->stream = task->streams[0];
  }
  // bind: allocate, replay each queue in its recorded order
  void* stream = task->streams[0];
  size_t done = 0;
  int rc = MGB_OK;
  for (; done < fresh.size() && rc == MGB_OK; ++done) {
    Obj& o = z->objs[fresh[done]];
    rc = z->dev_alloc(o.bytes, &o.real);
    if (rc != MGB_OK) break;
    for (const Op& op : o.queue) {
      rc = z->apply(stream, (uint8_t*)o.real, op.kind, op.offset, op.bytes, op.value, op.data.data());
      if (rc != MGB_OK) break;
      ++z->st.replayed_ops;
    }
    if (rc != MGB_OK) {
      z->dev_free(o.real);
      o.real = nullptr;
      break;
    }
    o.task = task;
    task->objs.insert(fresh[done]);
    ++z->st.n_bound;
  }
  if (rc == MGB_OK) rc = z->stream_sync(stream);     // the recorded bytes may go once the copies have read them
  if (rc != MGB_OK) {
    // undo what this call bound; a task that was created here ends here
    for (size_t k = 0; k < done; ++k) {
      Obj& o = z->objs[fresh[k]];
      z->dev_free(o.real);
      o.real = nullptr;
      o.task.reset();
      task->objs.erase(fresh[k]);
      --z->st.n_bound;
    }
    if (owners.empty()) (void)z->finish(task);
    return rc;
  }
  for (uint32_t id : fresh) {
    Obj& o = z->objs[id];
    for (const Op& op : o.queue) z->st.staged_bytes -= op.data.size();
    o.queue.clear();
    o.queue.shrink_to_fit();
  }
  for (uint32_t i = 0; i < n_args; ++i) real_args[i] = (uint8_t*)z->objs[ids[i]].real + offs[i];
  return MGB_OK;
}

int mgb_lazy_memcpy_d2h(mgb_lazy* z, void* dst_host, uint64_t src_pseudo, uint64_t bytes) {
  if (!z || (!dst_host && bytes)) return MGB_E_INVAL;
  std::lock_guard<std::mutex> lk(z->mu);
  uint32_t id;
  uint64_t off;
  Obj* o = z->lookup(src_pseudo, &id, &off);
  if (!o) return MGB_E_UNKNOWN_TICKET;
  if (off > o->bytes || bytes > o->bytes - off) return MGB_E_INVAL;
  if (bytes == 0) return MGB_OK;
  if (!o->real) {
    // never used by a kernel so far: what the copy would read is what the recorded writes left
    // in [off, off + bytes), in their order (bytes nobody wrote read as zero)
    uint8_t* dst = (uint8_t*)dst_host;
    std::memset(dst, 0, bytes);
    for (const Op& op : o->queue) {
      const uint64_t lo = std::max(op.offset, off), hi = std::min(op.offset + op.bytes, off + bytes);
      if (lo >= hi) continue;
      if (op.kind == OP_H2D) std::memcpy(dst + (lo - off), op.data.data() + (lo - op.offset), hi - lo);
      else std::memset(dst + (lo - off), op.value, hi - lo);
    }
    return MGB_OK;
  }
  if (!z->hip) {
    std::memcpy(dst_host, (uint8_t*)o->real + off, bytes);
    return MGB_OK;
  }
  void* stream = o->task->streams[0];
  hipError_t e = hipMemcpyAsync(dst_host, (uint8_t*)o->real + off, bytes, hipMemcpyDeviceToHost, (hipStream_t)stream);
  if (e != hipSuccess) return z->backend_error("hipMemcpyAsync", e);
  return z->stream_sync(stream);
}

int mgb_lazy_free(mgb_lazy* z, uint64_t pseudo) {
  if (!z) return MGB_E_INVAL;
  std::lock_guard<std::mutex> lk(z->mu);
  uint32_t id;
  uint64_t off;
  Obj* o = z->lookup(pseudo, &id, &off);
  if (!o || off != 0) return MGB_E_UNKNOWN_TICKET;
  int rc = MGB_OK;
  if (o->real) {
    std::shared_ptr<LTask> task = o->task;
    rc = z->stream_sync(task->streams[0]);
    z->dev_free(o->real);
    task->objs.erase(id);
    --z->st.n_bound;
    if (task->objs.empty()) {
      const int r = z->finish(task);
      if (rc == MGB_OK) rc = r;
    }
  } else {
    for (const Op& op : o->queue) z->st.staged_bytes -= op.data.size();
  }
  z->objs.erase(id);
  --z->st.n_objects;
  return rc;
}

int mgb_lazy_stats_get(mgb_lazy* z, mgb_lazy_stats* out) {
  if (!z || !out) return MGB_E_INVAL;
  std::lock_guard<std::mutex> lk(z->mu);
  *out = z->st;
  return MGB_OK;
}

}  // extern "C"
