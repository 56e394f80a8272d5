"""Test infrastructure only (imported by tests, the smoke check and the bench's CPU leg; never by
the product path).

Plain-Python model of task construction (Sec. III-A of the paper):

* ``build_gpu_tasks``  -- Algorithm 1: every kernel launch is a unit task (its memory objects,
  allocations, grid, block); unit tasks that share a memory object are merged.  The pass is written
  in the algorithm's order; because one pass only merges the units that share an object *with the
  unit it started from*, it is repeated on its own output until no two tasks share an object
  (sharing is meant to be transitive: tasks that share memory must not be placed apart).
* ``LazyModel``        -- the meaning of a program's device-memory calls and kernel launches when
  every call is executed at once on plain byte arrays (the semantics the lazy runtime has to
  preserve), together with what the lazy runtime must tell the scheduler: one probe per new task
  (footprint = bytes of the objects the launch names), one growth per launch that brings new
  objects into an existing task, one completion per ticket when a task's last object is freed.
"""
import numpy as np


def _merge(units):
    out = dict(memobjs=set(), allocs={}, launches=[])
    for u in units:
        out["memobjs"] |= set(u["memobjs"])
        out["allocs"].update(u["allocs"])
        out["launches"] += list(u["launches"])
    out["launches"].sort()
    return out


def _one_pass(units):
    """Algorithm 1's second loop, as stated."""
    tasks = []
    visited = [False] * len(units)
    for i, u1 in enumerate(units):
        if visited[i]:
            continue
        union = []
        visited[i] = True
        for j, u2 in enumerate(units):
            if visited[j]:
                continue
            if set(u1["memobjs"]) & set(u2["memobjs"]):
                if not union:
                    union.append(u1)
                union.append(u2)
                visited[j] = True
        tasks.append(_merge([u1]) if not union else _merge(union))
    return tasks


def waves_of(grid, block, wave=64):
    g = int(grid[0]) * int(grid[1]) * int(grid[2])
    b = int(block[0]) * int(block[1]) * int(block[2])
    return g * -(-b // wave)


def build_gpu_tasks(launches):
    """launches: list of dict(memobjs=[names], allocs={name: bytes}, grid=(..), block=(..)).
    Returns the merged tasks in order of their first launch: dict(memobjs, mem_bytes, launches
    (indices), grid, block) where grid / block are those of the task's largest launch."""
    units = [dict(memobjs=set(l["memobjs"]), allocs=dict(l["allocs"]), launches=[i]) for i, l in enumerate(launches)]
    tasks = _one_pass(units)
    while True:
        again = _one_pass(tasks)
        if len(again) == len(tasks):
            break
        tasks = again
    out = []
    for t in sorted(tasks, key=lambda t: t["launches"][0]):
        big = max(t["launches"], key=lambda i: (waves_of(launches[i]["grid"], launches[i]["block"]), -i))
        out.append(dict(memobjs=set(t["memobjs"]), mem_bytes=sum(t["allocs"].values()), launches=t["launches"],
                        grid=tuple(launches[big]["grid"]), block=tuple(launches[big]["block"])))
    return out


class LazyModel:
    """Eager execution of a program's device calls + the scheduler traffic they imply."""

    def __init__(self, kernels):
        self.kernels = kernels            # name -> fn(list of uint8 views starting at each argument, params)
        self.mem = {}                     # handle -> uint8 array (unwritten bytes are zero)
        self.task_of = {}                 # handle -> task index, once a launch has used the object
        self.tasks = []                   # per task: dict(objs=set, tickets=[ticket numbers], alive)
        self.next_handle = 0
        self.next_ticket = 0
        self.sched_inputs = []            # ("probe", task_id, mem, grid, block) | ("grow", ticket, extra) | ("complete", ticket)
        self.launch_task = []             # first ticket of the task every launch ran in

    def malloc(self, nbytes):
        h = self.next_handle
        self.next_handle += 1
        self.mem[h] = np.zeros(nbytes, dtype=np.uint8)
        return h

    def memcpy_h2d(self, h, off, data):
        data = np.frombuffer(bytes(data), dtype=np.uint8)
        self.mem[h][off:off + data.size] = data

    def memset(self, h, off, value, n):
        self.mem[h][off:off + n] = value & 0xFF

    def launch(self, task_id, kernel, args, grid, block, params=None):
        handles = []
        for h, _ in args:
            if h not in handles:
                handles.append(h)
        fresh = [h for h in handles if h not in self.task_of]
        owners = sorted({self.task_of[h] for h in handles if h in self.task_of},
                        key=lambda t: self.tasks[t]["tickets"][0])
        extra = sum(self.mem[h].size for h in fresh)
        if not owners:
            self.next_ticket += 1
            self.tasks.append(dict(objs=set(), tickets=[self.next_ticket]))
            t = len(self.tasks) - 1
            self.sched_inputs.append(("probe", task_id, extra, tuple(grid), tuple(block)))
        else:
            t = owners[0]
            if extra:
                self.sched_inputs.append(("grow", self.tasks[t]["tickets"][0], extra))
            for o in owners[1:]:
                for h in self.tasks[o]["objs"]:
                    self.task_of[h] = t
                self.tasks[t]["objs"] |= self.tasks[o]["objs"]
                self.tasks[t]["tickets"] += self.tasks[o]["tickets"]
                self.tasks[o]["objs"] = set()
        for h in fresh:
            self.task_of[h] = t
            self.tasks[t]["objs"].add(h)
        self.launch_task.append(self.tasks[t]["tickets"][0])
        self.kernels[kernel]([self.mem[h][off:] for h, off in args], params)

    def memcpy_d2h(self, h, off, n):
        return self.mem[h][off:off + n].tobytes()

    def free(self, h):
        del self.mem[h]
        if h in self.task_of:
            t = self.task_of.pop(h)
            self.tasks[t]["objs"].discard(h)
            if not self.tasks[t]["objs"]:
                for tk in self.tasks[t]["tickets"]:
                    self.sched_inputs.append(("complete", tk))
