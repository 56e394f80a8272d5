/*
 * mgb.h -- C ABI of the one-GPU task co-execution library.
 *
 * The library implements, for a single AMD CDNA4 device, the resource-aware
 * sharing scheme of "Effective GPU Sharing Under Compiler Guidance"
 * (arXiv 2107.08538): every GPU task announces its memory footprint and launch
 * geometry through a probe before it touches the device (Sec. III-A, Fig. 3:
 * the instrumented task_begin(mem, threads, blocks)); a user-level scheduler
 * answers with a placement or makes the task wait (Sec. III-B, Algorithms 2
 * and 3); resources are handed back when the task completes and waiting tasks
 * are retried (Sec. IV).  Where the paper picks one of several GPUs and relies
 * on a process-sharing service to co-run kernels, this library partitions the
 * compute units of one device: a placement is a set of compute "granules"
 * (groups of CUs) realised as a CU-masked HIP stream.
 *
 * Conventions
 *   - plain C types only; all handles are opaque; no exceptions cross the ABI.
 *   - return value: 0 = MGB_OK, > 0 = non-error status, < 0 = error.
 *   - "device pointer" = address in GPU memory owned by the caller; the
 *     library never allocates or frees task buffers.  "host pointer" = CPU
 *     memory.  Out-parameters are host pointers written before return.
 *   - every function is thread-safe unless stated otherwise.
 *   - the memory ledger is pure accounting (as in the paper, where the
 *     scheduler tracks FreeMem but allocates nothing).
 */
#ifndef MGB_H
#define MGB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- status codes ------------------------------------------------------ */
#define MGB_OK 0
#define MGB_WAIT 1               /* probe accepted, task queued             */
#define MGB_TIMEOUT 2            /* mgb_task_wait gave up, task still queued */
#define MGB_E_INVAL (-1)         /* null pointer, zero / oversized geometry */
#define MGB_E_TOO_BIG (-2)       /* footprint larger than the whole cap     */
#define MGB_E_UNKNOWN_TICKET (-3)
#define MGB_E_BAD_STATE (-4)     /* e.g. complete of a waiting task         */
#define MGB_E_BUSY (-5)          /* destroy with tasks in flight            */
#define MGB_E_BACKEND (-6)       /* HIP call failed; see mgb_last_error     */
#define MGB_E_UNSUPPORTED (-7)   /* shape outside what a kernel accepts     */
#define MGB_E_OOM (-8)           /* CG policy: the task would have run out of memory */

/* ---- policies (Sec. III-B and Sec. IV) --------------------------------- */
#define MGB_POLICY_HARD 0    /* Algorithm 2: memory and compute both hard   */
#define MGB_POLICY_SOFT 1    /* Algorithm 3: memory hard, compute by load   */
#define MGB_POLICY_SERIAL 2  /* single-assignment baseline: one task owns the device */
#define MGB_POLICY_CG 3      /* core-to-GPU-ratio baseline: up to max_running tasks share the
                                whole device, memory is not consulted; a task that does not
                                fit when let in is rejected with MGB_E_OOM (counted, not run) */
#define MGB_QUEUE_BACKFILL 0 /* on release retry every waiter in arrival order */
#define MGB_QUEUE_FIFO 1     /* stop at the first waiter that does not fit  */
#define MGB_BACKEND_NULL 0   /* bookkeeping only, no HIP call (host tests)  */
#define MGB_BACKEND_HIP 1    /* placements carry a CU-masked hipStream_t    */

typedef struct mgb_sched mgb_sched;

typedef struct { uint32_t x, y, z; } mgb_dim3;

/* Device description; copied by mgb_sched_create.  The per-CU limits are the
 * analogue of the "max thread blocks and warps per SM" that Algorithm 2
 * tracks.  n_cu must be a multiple of granule_cus and n_cu / granule_cus must
 * be <= 32.  With the HIP backend granule_cus must be a multiple of 8: CU-mask
 * bit i selects a CU of XCD (i mod 8), so 8 consecutive aligned bits are one CU
 * in every XCD, and a mask that leaves an XCD without CUs is never built.    */
typedef struct {
  uint64_t mem_cap_bytes;      /* ledger capacity                           */
  uint32_t n_cu;               /* 256                                       */
  uint32_t granule_cus;        /* 32 (a multiple of 8 with the HIP backend) */
  uint32_t wave_size;          /* 64                                        */
  uint32_t max_waves_per_cu;   /* 32                                        */
  uint32_t max_wg_per_cu;      /* 32                                        */
  uint32_t policy;             /* MGB_POLICY_*                              */
  uint32_t queue_mode;         /* MGB_QUEUE_*                               */
  uint32_t backend;            /* MGB_BACKEND_*                             */
  int32_t  device;             /* HIP device ordinal (HIP backend)          */
  uint32_t max_running;        /* most tasks resident at once, 0 = no limit (8) */
} mgb_device_desc;

/* Answer to a probe.  `stream` is a hipStream_t owned by the library (NULL
 * with the null backend); it is valid until mgb_task_complete(ticket).
 * Granule k owns CU-mask bits [k*granule_cus, (k+1)*granule_cus).  Granted
 * granules form a buddy block: the demand rounded up to a power of two b, a
 * run of b granules starting at a multiple of b.                             */
typedef struct {
  uint64_t ticket;             /* handle of this task inside the scheduler  */
  uint32_t granule_mask;       /* bit k set = granule k granted             */
  uint32_t n_granules;         /* granules demanded (granted: next power of two) */
  uint32_t cu_mask[8];         /* 256-bit CU mask derived from granule_mask */
  void*    stream;
} mgb_placement;

typedef struct {
  uint64_t free_bytes;
  uint32_t free_granules;      /* bitmap (HARD / SERIAL)                    */
  uint32_t n_running;
  uint32_t n_waiting;
  uint32_t n_streams;          /* masked streams created so far             */
  uint64_t n_events;           /* trace records so far                      */
} mgb_stats;

/* ---- event trace -------------------------------------------------------- */
#define MGB_EV_PROBE 0       /* input: a probe arrived (mem, grid, block)   */
#define MGB_EV_COMPLETE 1    /* input: mgb_task_complete(ticket)            */
#define MGB_EV_CANCEL 2      /* input: mgb_task_cancel(ticket)              */
#define MGB_EV_GROW 3        /* input: mgb_task_grow(ticket, extra bytes)   */
#define MGB_EV_ADMIT 16      /* decision: placed (granule_mask, cu_mask)    */
#define MGB_EV_QUEUED 17     /* decision: must wait                         */
#define MGB_EV_REJECT 18     /* decision: refused, `code` says why          */
#define MGB_EV_RELEASE 19    /* decision: resources credited back           */
#define MGB_EV_CANCELLED 20  /* decision: waiter removed                    */
#define MGB_EV_GROWN 21      /* decision: a resident task's footprint grew  */

/* One record per event, in the total order in which the scheduler lock was
 * taken.  Input records carry what the caller passed; decision records carry
 * the state after the decision.  Replaying the input records through an
 * independent implementation of the policy must regenerate the decisions.   */
typedef struct {
  uint64_t seq;
  uint64_t t_ns;               /* monotonic clock                           */
  uint64_t task_id;
  uint64_t ticket;
  uint64_t mem_bytes;
  uint64_t free_bytes;         /* after the event                           */
  uint32_t kind;               /* MGB_EV_*                                  */
  int32_t  code;               /* reject reason or 0                        */
  uint32_t granule_mask;
  uint32_t free_granules;      /* after the event                           */
  uint32_t demand;             /* granules demanded                         */
  uint32_t cause_seq;          /* seq of the input record that caused a decision */
  mgb_dim3 grid, block;
  uint32_t cu_mask[8];
} mgb_trace_rec;

/* ---- scheduler ----------------------------------------------------------
 * Fill `out` with the defaults for one MI355X: 256 CUs in granules of 32
 * (8 granules, 15 possible partitions), 64-lane waves, 32 waves and 32
 * workgroups per CU, cap 288e9 bytes, HARD, BACKFILL, HIP backend, device 0,
 * at most 8 resident tasks.  granule_cus may be any multiple of 8 that
 * divides n_cu (8 = one CU in every XCD, the finest partition).              */
void mgb_device_desc_default(mgb_device_desc* out);

/* Create a scheduler for one device.  Errors: MGB_E_INVAL (bad descriptor),
 * MGB_E_BACKEND (HIP device unusable).                                      */
int mgb_sched_create(const mgb_device_desc* desc, mgb_sched** out);

/* Destroy; MGB_E_BUSY if any task is running or waiting (nothing is freed). */
int mgb_sched_destroy(mgb_sched* s);

/* The probe (the paper's task_begin, Fig. 3 and Sec. IV): announce footprint
 * and launch geometry of a task before it runs.  A task that launches several
 * kernels on the same buffers is ONE task (Algorithm 1 merges launches that
 * share memory objects): pass the largest geometry of its launches.
 *   MGB_OK    placed: *out holds granules, CU mask, stream.
 *   MGB_WAIT  queued: out->ticket valid, call mgb_task_wait.
 *   MGB_E_INVAL  grid or block has a zero dimension or block > 1024 threads.
 *   MGB_E_TOO_BIG  mem_bytes exceeds the cap; the task is never queued.
 *   MGB_E_BACKEND  admitted, but no stream could be made for its CU mask: the
 *                  placement has been given back (nothing is held, *out zeroed).
 * Compute demand (Algorithm 2's per-SM residency limits, per CU here):
 *   waves/wg = ceil(threads / wave_size);
 *   wg/CU    = max(1, min(max_wg_per_cu, max_waves_per_cu / waves/wg [, wg_per_cu of the probe]));
 *   CUs      = min(n_cu, ceil(workgroups / wg/CU)); granules = ceil(CUs / granule_cus).
 * Admission: mem_bytes <= free bytes, fewer than max_running tasks resident,
 * and (HARD) a free aligned block of next_pow2(granules) granules, the lowest
 * such block being taken; SOFT takes the aligned block with the fewest in-use
 * waves instead and never waits for compute.                                */
int mgb_task_probe(mgb_sched* s, uint64_t task_id, uint64_t mem_bytes, mgb_dim3 grid,
                   mgb_dim3 block, mgb_placement* out);

/* The same with one more fact the compiler has about the task's kernels: wg_per_cu = how many of
 * its workgroups one CU can hold at once given their registers and LDS (the hardware dispatcher
 * stops at whichever resource runs out first, Sec. II-A).  It enters the demand rule as one more
 * upper limit on workgroups per CU; 0 = not known (mgb_task_probe).  The probe's trace record
 * carries it in its `demand` field.                                            */
int mgb_task_probe_ex(mgb_sched* s, uint64_t task_id, uint64_t mem_bytes, mgb_dim3 grid,
                      mgb_dim3 block, uint32_t wg_per_cu, mgb_placement* out);

/* Block until the queued task is admitted (MGB_OK, *out filled) or
 * timeout_ns elapsed (MGB_TIMEOUT, task stays queued; < 0 waits forever).    */
int mgb_task_wait(mgb_sched* s, uint64_t ticket, int64_t timeout_ns, mgb_placement* out);

/* Remove a queued (not yet admitted) task.  MGB_E_BAD_STATE if it runs.      */
int mgb_task_cancel(mgb_sched* s, uint64_t ticket);

/* A resident task needs `extra_bytes` more device memory (a later kernel of
 * the task touches memory objects that were not known at its probe: Sec.
 * III-A, lazy runtime).  Never blocks -- a resident task that waited for
 * memory while holding memory could deadlock: MGB_OK and the ledger debited
 * if the bytes are free now, MGB_E_BUSY (nothing changed) if not,
 * MGB_E_BAD_STATE for a task that is still queued.  The bytes are credited
 * back with the rest of the task's footprint at mgb_task_complete.           */
int mgb_task_grow(mgb_sched* s, uint64_t ticket, uint64_t extra_bytes);

/* Run enqueue(stream, user) on the task's stream, bracketed by timing events
 * (HIP backend).  enqueue must only enqueue work on `stream` (it may
 * synchronise that stream).  Its return value != 0 is passed back.
 * Profiling aid: if MGB_TAG_PARTITIONS was set in the environment when the
 * scheduler was created, an empty kernel partition_tag_kernel is launched on
 * the stream first, with (first granted granule * 64 + number of granted
 * granules) workgroups of 64 threads, so that a kernel trace shows which
 * partition each hardware queue serves.                                      */
int mgb_task_launch(mgb_sched* s, uint64_t ticket, int (*enqueue)(void* stream, void* user),
                    void* user);

/* Wait until everything launched for the task has finished; *gpu_ms (may be
 * NULL) receives the time between the bracketing events.                    */
int mgb_task_sync(mgb_sched* s, uint64_t ticket, double* gpu_ms);

/* Task finished: credit memory and granules back and retry the waiters
 * (Sec. IV).  The caller must have synchronised the task's work first.      */
int mgb_task_complete(mgb_sched* s, uint64_t ticket);

/* The same release, ordered on the device instead of observed by the host: to be called when the
 * task's last kernel has been ENQUEUED (after the last mgb_task_launch), without waiting for it.
 * The ledger is credited and the waiters retried at once (the same COMPLETE / RELEASE / ADMIT
 * records as mgb_task_complete, so a trace replays unchanged); what the device must not see is
 * enforced on the device: a task admitted into granules this one held (HARD, SERIAL) starts
 * behind this task's stop event (hipStreamWaitEvent on its stream before its first kernel), and a
 * task whose footprint needed bytes that tasks released this way may still be using starts
 * behind all of them.  So in device time a granule still has one owner and the bytes one user,
 * while the hand-over between two tasks (completion seen by the host, waiter woken, kernels
 * launched) overlaps the finishing task's kernels.  For tasks whose buffers stay valid until
 * their kernels end (allocated up front, or freed in stream order); a task that frees its memory
 * from the host right after the call must use mgb_task_complete.
 * Afterwards the ticket is gone for every call except mgb_task_sync, which waits for the task's
 * kernels, reports their time and forgets the task (one thread may do so: a second concurrent
 * mgb_task_sync on the ticket gets MGB_E_BAD_STATE; mgb_sched_destroy does it for tasks nobody
 * synchronised).  A later mgb_task_grow of another task into bytes such a task may still be using
 * orders that task's further work behind it in the same way.  Errors as mgb_task_complete.      */
int mgb_task_complete_on_stream(mgb_sched* s, uint64_t ticket);

/* Tickets of the released-on-stream tasks that the resident task `ticket` starts behind (those
 * whose kernels were not known to have finished when it was admitted).  Copies up to `cap`
 * tickets to `out` (host) and returns how many there are, or < 0.                 */
int64_t mgb_task_deps(mgb_sched* s, uint64_t ticket, uint64_t* out, uint64_t cap);

/* ---- accounting (Sec. V-A: throughput, turnaround = completion - arrival in the queue; Sec. V,
 * kernel-slowdown table: time of a task's kernels when sharing over their time on a dedicated
 * device) ----------------------------------------------------------------------
 * One record per probe, kept by the scheduler (the last 2^20).  Host times are the monotonic
 * clock of the trace, device times milliseconds since the scheduler was created.              */
typedef struct {
  uint64_t ticket, task_id, mem_bytes;
  uint64_t probe_ns;           /* the probe arrived                                             */
  uint64_t admit_ns;           /* it was admitted (0: never)                                    */
  uint64_t release_ns;         /* its resources went back to the ledger                         */
  uint64_t done_ns;            /* its work was seen finished: return of the wait in
                                  mgb_task_sync if that was called, else release_ns             */
  double   gpu_ms;             /* between the events around its launches (mgb_task_sync)        */
  double   gpu_start_ms, gpu_stop_ms;  /* those events on the device clock                      */
  uint32_t granule_mask, demand;
  int32_t  status;             /* MGB_OK finished, MGB_WAIT not finished yet, MGB_TIMEOUT cancelled
                                  while queued, MGB_E_OOM lost under the CG policy              */
  uint32_t reserved;
} mgb_task_record;

typedef struct {
  uint64_t n_done, n_crashed, n_unfinished;
  double tasks_per_s;          /* n_done / (last completion - first arrival)                    */
  double makespan_ms;          /* last completion - first arrival                               */
  double mean_turnaround_ms, max_turnaround_ms;   /* completion - arrival                       */
  double mean_wait_ms, max_wait_ms;               /* admission - probe (a task admitted behind a
                                  task released on the stream may still wait on the device for that task's
                                  kernels: that time is in its turnaround, not here)            */
  double gpu_busy_ms;          /* sum of the tasks' gpu_ms                                      */
  double max_slowdown, mean_slowdown;             /* gpu_ms / reference - 1 over the tasks given one */
} mgb_summary;

/* Copy up to `cap` records starting at ticket `first_ticket` (tickets count from 1) into `out`;
 * returns the number copied or < 0.                                                            */
int64_t mgb_task_records(mgb_sched* s, uint64_t first_ticket, mgb_task_record* out, uint64_t cap);

/* Pure arithmetic on n records (host arrays).  arrival_ns[i] (NULL: the probe time) is when task
 * i entered the queue; ref_gpu_ms[i] (NULL or <= 0: none) is the time of the same task's kernels
 * on a dedicated device.  Tasks lost to MGB_E_OOM are counted, not timed; tasks not finished are
 * counted in n_unfinished and otherwise ignored.  MGB_E_INVAL for a record that ends before it
 * arrives.                                                                                     */
int mgb_accounting(const mgb_task_record* recs, uint64_t n, const uint64_t* arrival_ns,
                   const double* ref_gpu_ms, mgb_summary* out);

int mgb_sched_stats(mgb_sched* s, mgb_stats* out);
/* Copy up to `cap` trace records starting at sequence number `first` into
 * `out` (host); returns the number copied or < 0.  A scheduler keeps its last
 * 2^20 records at most (when that many are held the older half is dropped):
 * a `first` below the oldest record kept starts at that record, and the `seq`
 * fields show the gap.                                                       */
int64_t mgb_trace_read(mgb_sched* s, uint64_t first, mgb_trace_rec* out, uint64_t cap);
/* Write the whole trace as JSON lines to `path`.                             */
int mgb_trace_dump(mgb_sched* s, const char* path);
/* Text of the last backend error seen by this thread ("" if none).          */
const char* mgb_last_error(void);

/* ---- lazy runtime (Sec. III-A, "Lazy Runtime") ------------------------------
 * For programs whose allocations, copies and launches cannot be tied to a task
 * statically.  Device-memory calls are redirected to these: an allocation hands
 * out a pseudo address and allocates nothing; copies and fills to an object that
 * is not on the device yet are recorded in the object's queue (a host-to-device
 * copy keeps the bytes as they are at the call); mgb_lazy_launch_prepare is the
 * paper's kernelLaunchPrepare.  All pointers are host pointers; pseudo
 * addresses are opaque 64-bit values (object + byte offset, offsets may be
 * added by the caller).  An mgb_lazy serves one client: its calls are
 * serialised, and a launch that waits for admission holds the instance.
 * Unknown pseudo addresses give MGB_E_UNKNOWN_TICKET, ranges outside an object
 * MGB_E_INVAL; runtime failures MGB_E_BACKEND (mgb_last_error has the text).    */
typedef struct mgb_lazy mgb_lazy;

typedef struct {
  uint64_t n_objects;      /* memory objects alive                            */
  uint64_t n_bound;        /* of these, on the device                         */
  uint64_t n_tasks;        /* tasks alive (admitted, some object not freed)   */
  uint64_t recorded_ops;   /* copies / fills recorded so far                  */
  uint64_t replayed_ops;   /* of these, replayed at a launch                  */
  uint64_t staged_bytes;   /* host bytes held for recorded copies right now   */
} mgb_lazy_stats;

int mgb_lazy_create(mgb_sched* s, mgb_lazy** out);
/* MGB_E_BUSY while memory objects are alive.                                   */
int mgb_lazy_destroy(mgb_lazy* z);
/* Stand-in for a device allocation of `bytes` (< 2^40).                        */
int mgb_lazy_malloc(mgb_lazy* z, uint64_t bytes, uint64_t* pseudo);
/* Stand-ins for host-to-device copy and fill.  Recorded if the object is not on
 * the device yet; otherwise executed on its task's stream, complete on return.  */
int mgb_lazy_memcpy_h2d(mgb_lazy* z, uint64_t dst_pseudo, const void* src_host, uint64_t bytes);
int mgb_lazy_memset(mgb_lazy* z, uint64_t dst_pseudo, int value, uint64_t bytes);
/* Before a kernel launch: `pseudo_args[0..n_args)` are the memory objects the
 * kernel accesses (n_args >= 1), grid / block its geometry, wg_per_cu its residency (0 = not
 * known), as in mgb_task_probe_ex.
 *  - none of the objects is on the device: a new task.  Its footprint is the
 *    sum of the objects' sizes; mgb_task_probe_ex(task_id, footprint, grid, block, wg_per_cu)
 *    is issued and, if the task is queued, waited for up to timeout_ns (< 0:
 *    forever; on MGB_TIMEOUT the probe is cancelled and nothing has changed).
 *    Other threads may use the runtime during that wait (freeing objects is
 *    what lets a queued task in); if one of them frees or binds an object this
 *    launch names, the placement is given back and MGB_E_BAD_STATE returned.
 *  - some are: the launch joins their task (launches that share memory objects
 *    form one task, Alg. 1); the sizes of the new objects are asked for with
 *    mgb_task_grow (MGB_E_BUSY: nothing has changed).  Objects of several tasks:
 *    the task with the oldest ticket absorbs the others and its stream waits
 *    for theirs.
 * Then every new object is allocated and its recorded operations are replayed
 * in order on the task's stream.  real_args[i] receives the device address for
 * pseudo_args[i]; placement->stream is the stream to launch on (ticket: the
 * task's first ticket; masks are filled for a new task only).                  */
int mgb_lazy_launch_prepare(mgb_lazy* z, uint64_t task_id, const uint64_t* pseudo_args, uint32_t n_args,
                            mgb_dim3 grid, mgb_dim3 block, uint32_t wg_per_cu, int64_t timeout_ns,
                            void** real_args, mgb_placement* placement);
/* Stand-in for a device-to-host copy; waits for the task's stream first.  For an
 * object no kernel has used yet the bytes are those the recorded writes left
 * (unwritten bytes read as zero).                                               */
int mgb_lazy_memcpy_d2h(mgb_lazy* z, void* dst_host, uint64_t src_pseudo, uint64_t bytes);
/* Stand-in for freeing a device allocation (pseudo must be the object's base).
 * Freeing the last object of a task drains its stream and completes it.         */
int mgb_lazy_free(mgb_lazy* z, uint64_t pseudo);
int mgb_lazy_stats_get(mgb_lazy* z, mgb_lazy_stats* out);

/* ---- multi-process front end (Sec. IV: processes reach the scheduler over
 * shared memory) ---------------------------------------------------------------
 * Server side: mgb_server_start publishes scheduler `s` under `name` (a POSIX
 * shared-memory segment "/mgb.<name>", at most 64 client slots) and serves it
 * with one thread per slot until mgb_server_stop.  The scheduler may use the
 * null backend: the server only takes decisions.  MGB_E_BUSY if the name is in
 * use.  A client whose process has died has its queued probes withdrawn and its
 * resident tasks completed (mgb_server_reclaimed counts such tasks).
 * Client side (any process): the mgb_client_* calls mirror mgb_task_* (mgb_client_probe takes the
 * residency fact of mgb_task_probe_ex, 0 = not known); the
 * placement carries ticket, granules and CU mask, its stream field is NULL.
 * mgb_client_stream gives the calling process's own CU-masked hipStream_t for
 * the placement's mask (created on first use, cached, destroyed at
 * disconnect).  mgb_client_disconnect refuses (MGB_E_BUSY) while the client
 * still holds tasks.  MGB_E_BACKEND if the server has gone away.               */
typedef struct mgb_server mgb_server;
typedef struct mgb_client mgb_client;
int mgb_server_start(mgb_sched* s, const char* name, uint32_t n_slots, mgb_server** out);
int mgb_server_stop(mgb_server* sv);
uint64_t mgb_server_reclaimed(mgb_server* sv);
int mgb_client_connect(const char* name, mgb_client** out);
int mgb_client_disconnect(mgb_client* c);
int mgb_client_probe(mgb_client* c, uint64_t task_id, uint64_t mem_bytes, mgb_dim3 grid, mgb_dim3 block,
                     uint32_t wg_per_cu, mgb_placement* out);
int mgb_client_wait(mgb_client* c, uint64_t ticket, int64_t timeout_ns, mgb_placement* out);
int mgb_client_cancel(mgb_client* c, uint64_t ticket);
int mgb_client_grow(mgb_client* c, uint64_t ticket, uint64_t extra_bytes);
int mgb_client_complete(mgb_client* c, uint64_t ticket);
int mgb_client_stats(mgb_client* c, mgb_stats* out);
int mgb_client_stream(mgb_client* c, const mgb_placement* placement, void** stream);

/* ---- task kernels ---------------------------------------------------------
 * Each task kind has a *probe* -- the requirement derivation a compiler pass
 * would have inserted (Sec. III-A: footprint = sum of the task's allocations,
 * compute = grid and block of its launches) -- and an *enqueue* that puts the
 * task's kernels on a stream.  Probes are pure host arithmetic.  Enqueues
 * return MGB_E_UNSUPPORTED / MGB_E_INVAL before launching anything if the
 * arguments do not fit what the kernels assume.  All device buffers are
 * caller-owned and must stay valid until the stream has drained.            */

/* fp32 5-point Jacobi relaxation on an n x n row-major grid whose outermost
 * ring is a fixed boundary: v = 0.25f * ((N + S) + (W + E)) on the interior,
 * `iters` sweeps ping-ponging between u0 (initial state) and u1; the result is
 * in u0 if iters is even, else u1.  Both buffers must hold the same ring.
 * Up to four sweeps are fused into one launch, up to eight for n >= 2048
 * (bit-identical to single sweeps).  The probe's grid is the largest among
 * the task's launches.  mgb_jacobi_residency(n) = workgroups of these kernels
 * that one CU holds (registers), 0 if n is unsupported.
 * Footprint 2*n*n*4 bytes.  n >= 3.                                         */
int mgb_jacobi_probe(uint32_t n, uint32_t iters, uint64_t* mem_bytes, mgb_dim3* grid, mgb_dim3* block);
uint32_t mgb_jacobi_residency(uint32_t n);
int mgb_jacobi_enqueue(void* stream, float* u0, float* u1, uint32_t n, uint32_t iters);
/* Number of kernel launches mgb_jacobi_enqueue issues for (n, iters): sweeps are fused up to
 * four (n >= 2048: eight) per launch, with the launch count kept at the parity of iters (0 if n
 * is unsupported). */
uint32_t mgb_jacobi_launch_count(uint32_t n, uint32_t iters);

/* fp32 GEMM C = A * B, row-major A (m x k), B (k x n), C (m x n), fp32 MFMA
 * accumulation.  Footprint (m*k + k*n + m*n)*4.                              */
/* *_residency: workgroups of the task's (largest) kernel that one CU can hold given their registers
 * and LDS -- the wg_per_cu of mgb_task_probe_ex; 0 for a shape the kernel does not accept.       */
uint32_t mgb_gemm_f32_residency(uint32_t m, uint32_t n, uint32_t k);
uint32_t mgb_gemm_bf16_residency(uint32_t m, uint32_t n, uint32_t k);
uint32_t mgb_conv3x3_residency(uint32_t batch, uint32_t h, uint32_t w, uint32_t c_in, uint32_t c_out, uint32_t stride);
int mgb_gemm_f32_probe(uint32_t m, uint32_t n, uint32_t k, uint64_t* mem_bytes, mgb_dim3* grid, mgb_dim3* block);
int mgb_gemm_f32_enqueue(void* stream, const float* A, const float* B, float* C, uint32_t m, uint32_t n, uint32_t k);

/* bf16 GEMM: A, B hold bfloat16 bit patterns (uint16), C is fp32; products are
 * accumulated in fp32 by the bf16 MFMA.  Footprint (m*k + k*n)*2 + m*n*4.    */
int mgb_gemm_bf16_probe(uint32_t m, uint32_t n, uint32_t k, uint64_t* mem_bytes, mgb_dim3* grid, mgb_dim3* block);
int mgb_gemm_bf16_enqueue(void* stream, const uint16_t* A, const uint16_t* B, float* C, uint32_t m, uint32_t n, uint32_t k);

/* One 3x3 convolution + ReLU, padding 1, stride 1 or 2, as an implicit GEMM.
 * x: N,H,W,C bf16; w: K,3,3,C bf16; y: N,Ho,Wo,K with Ho = (H-1)/stride + 1,
 * stored as bf16 (round to nearest even) if out_f32 == 0 else as fp32.
 * fp32 accumulation.                                                         */
typedef struct {
  uint32_t c_in, c_out, stride;
} mgb_conv_layer;
int mgb_conv3x3_probe(uint32_t batch, uint32_t h, uint32_t w, uint32_t c_in, uint32_t c_out,
                      uint32_t stride, uint64_t* mem_bytes, mgb_dim3* grid, mgb_dim3* block);
int mgb_conv3x3_enqueue(void* stream, const uint16_t* x, const uint16_t* w, void* y, uint32_t batch,
                        uint32_t h, uint32_t wd, uint32_t c_in, uint32_t c_out, uint32_t stride,
                        uint32_t out_f32);

/* A chain of n_layers conv+ReLU layers run as one task.  Activations ping-pong
 * between act0 and act1 (bf16, each large enough for the largest intermediate
 * activation); the last layer writes fp32 to `out`.  weights[i] is the device
 * pointer of layer i's K,3,3,C tensor (host array of device pointers).
 * Footprint = input + all weights + 2 * largest intermediate + fp32 output;
 * geometry = the largest over the layers.  act0 and act1 are scratch for the
 * whole call: a small, deep layer also keeps fp32 partial sums in the part of
 * them its activations leave idle.                                            */
uint32_t mgb_cnn_residency(const mgb_conv_layer* layers, uint32_t n_layers, uint32_t batch, uint32_t h,
                           uint32_t w);
int mgb_cnn_probe(const mgb_conv_layer* layers, uint32_t n_layers, uint32_t batch, uint32_t h,
                  uint32_t w, uint64_t* mem_bytes, uint64_t* act_bytes, uint64_t* out_bytes,
                  mgb_dim3* grid, mgb_dim3* block);
int mgb_cnn_enqueue(void* stream, const mgb_conv_layer* layers, uint32_t n_layers,
                    const uint16_t* x, const uint16_t* const* weights, uint16_t* act0,
                    uint16_t* act1, float* out, uint32_t batch, uint32_t h, uint32_t w);

/* Level-synchronous BFS on a CSR graph (row_ptr int32[n+1], col_idx int32[m]).
 * mgb_bfs_enqueue expects a symmetric graph (every edge stored in both
 * directions: it may expand a level from the unvisited side);
 * mgb_bfs_directed_enqueue follows the stored edges as out-edges of any graph.
 * level[v] = hop distance from `source`, -1 if unreachable.  `work` is scratch
 * of mgb_bfs_work_bytes(n) bytes (two frontier queues, three frontier bitmaps
 * and per-level counters).  mgb_bfs_residency(n) = workgroups of the level
 * kernel one CU holds (the fact a probe may add to grid and block).
 * The call enqueues batches of level kernels and synchronises the stream
 * between batches to learn whether the frontier is empty; on return `level` is
 * complete.  *depth (host, may be NULL) receives the number of levels.
 * Footprint (n+1+m)*4 + n*4 + work.                                          */
uint64_t mgb_bfs_work_bytes(uint32_t n);
uint32_t mgb_bfs_residency(uint32_t n);
int mgb_bfs_probe(uint32_t n, uint64_t m, uint64_t* mem_bytes, mgb_dim3* grid, mgb_dim3* block);
int mgb_bfs_enqueue(void* stream, const int32_t* row_ptr, const int32_t* col_idx, uint32_t n,
                    uint32_t source, int32_t* level, void* work, uint32_t* depth);
int mgb_bfs_directed_enqueue(void* stream, const int32_t* row_ptr, const int32_t* col_idx, uint32_t n,
                             uint32_t source, int32_t* level, void* work, uint32_t* depth);

/* mgb_bfs_enqueue for callers that cannot allocate device memory (code that runs under stream
 * capture rules of its own, tight serving loops, harnesses that forbid hipMalloc): the work area
 * is a static device array inside the library (33.5 MiB, held by each device the library runs on
 * until the process ends) instead of a caller buffer.  The call allocates and frees nothing.
 * n <= 2^22 vertices, else MGB_E_TOO_BIG (mgb_last_error has the text) and nothing is launched;
 * otherwise arguments, result and errors are those of mgb_bfs_enqueue.  `stream` must belong to
 * the calling thread's current device.  All calls on one device share that device's array: the
 * call itself re-initialises what it reads, but two calls that overlap in time on one device
 * race (run them one after the other, or give the second one mgb_bfs_enqueue and its own work
 * buffer).                                                                      */
int mgb_bfs_enqueue_static(void* stream, const int32_t* row_ptr, const int32_t* col_idx, uint32_t n,
                           uint32_t source, int32_t* level, uint32_t* depth);

/* ---- worker pool (Sec. V-A: a queue of jobs, a pool of workers, each running one job to its end
 * and pulling the next; jobs all queued at the start, or arriving over time) -------------------
 * A job is one of the task kinds above, given by its device buffers and shape:
 *   MGB_TASK_JACOBI     ptr = {u0, u1},                     dim = {n, iters}
 *   MGB_TASK_GEMM_F32   ptr = {A, B, C},                    dim = {m, n, k}
 *   MGB_TASK_GEMM_BF16  ptr = {A, B, C},                    dim = {m, n, k}
 *   MGB_TASK_BFS        ptr = {row_ptr, col_idx, level, work}, dim = {n, source}, count = stored edges
 *   MGB_TASK_CNN        ptr = {x, act0, act1, out},         dim = {batch, h, w}, count = n_layers,
 *                       layers / weights as for mgb_cnn_enqueue (host arrays)
 *   MGB_TASK_CUSTOM     the caller's own kernels: ptr = {int (*enqueue)(void* stream, void* user), user}
 *                       (host pointers; enqueue as for mgb_task_launch), count = footprint in bytes,
 *                       dim = {workgroups, threads per workgroup, workgroups per CU or 0}
 * All buffers are device pointers owned by the caller and must stay valid until the call returns. */
#define MGB_TASK_JACOBI 0
#define MGB_TASK_GEMM_F32 1
#define MGB_TASK_GEMM_BF16 2
#define MGB_TASK_BFS 3
#define MGB_TASK_CNN 4
#define MGB_TASK_CUSTOM 5
typedef struct {
  uint32_t kind;               /* MGB_TASK_*                                                    */
  uint32_t reserved;
  uint64_t task_id;
  uint64_t arrival_ns;         /* when the job enters the queue, from the start of the run       */
  uint64_t count;
  void*    ptr[4];
  uint32_t dim[4];
  const mgb_conv_layer* layers;
  const uint16_t* const* weights;
} mgb_task_desc;

typedef struct {
  int32_t  status;             /* MGB_OK, or what stopped the job (MGB_E_OOM: lost under CG)     */
  uint32_t aux;                /* BFS: number of levels                                          */
  uint64_t ticket;
  uint64_t arrival_ns;         /* on the clock of the records                                    */
  mgb_task_record record;      /* as mgb_task_records gives it after the job's end               */
} mgb_pool_result;

#define MGB_POOL_ARRIVALS 1u           /* a job is not probed before start + arrival_ns; otherwise all
                                          jobs are in the queue at the start                     */
#define MGB_POOL_RELEASE_ON_STREAM 2u  /* hand resources back with mgb_task_complete_on_stream   */

/* Run the n jobs through scheduler `s` with min(n_workers, n) worker threads and return when all
 * have ended.  Each worker: derive the job's requirements with its kind's probe and residency,
 * mgb_task_probe_ex, mgb_task_wait if queued, mgb_task_launch of the kind's enqueue, then
 * mgb_task_sync + mgb_task_complete (or mgb_task_complete_on_stream + mgb_task_sync).  Jobs are
 * taken in arrival order; with all jobs queued at the start and a worker for each, all probes are
 * issued in the order given before anything runs.  results[i] (host, n entries) describes job i;
 * *start_ns (may be NULL) receives the clock value arrivals count from.  Returns MGB_OK, or the
 * first error other than MGB_E_OOM that a job met (the other jobs still run), or an error of a
 * probe derivation (then nothing has run).                                                     */
int mgb_pool_run(mgb_sched* s, const mgb_task_desc* tasks, uint32_t n, uint32_t n_workers,
                 uint32_t flags, mgb_pool_result* results, uint64_t* start_ns);

/* Diagnostic: launch n_blocks one-wave workgroups on `stream`; workgroup i
 * stores where it ran in out[i] (device, uint32): (xcd << 8) | (shader engine
 * << 4) | CU index within the engine.  Shows which physical CUs a placement's
 * stream reaches.  n_blocks in [1, 2^20].                                    */
int mgb_cu_trace_enqueue(void* stream, uint32_t* out, uint32_t n_blocks);

/* Diagnostic: plain device-to-device copy of `bytes` (multiple of 16, both
 * pointers 16-byte aligned) by a grid-stride kernel.  Moves exactly 2*bytes
 * through HBM: the measured bandwidth ceiling and the calibration point for
 * hardware traffic counters.                                                */
int mgb_copy_enqueue(void* stream, void* dst, const void* src, uint64_t bytes);

/* Diagnostic: n_blocks workgroups of four waves run `iters` rounds of 16
 * independent matrix instructions on registers (v_mfma_f32_32x32x2_f32, or
 * v_mfma_f32_32x32x16_bf16 if bf16 != 0) and store one float per thread to
 * out (device, n_blocks * 256 floats).  The operands are a fixed hash of
 * (accumulator block, lane, element) in [-1, 1), so that the matrix units see
 * changing full-width mantissas as in a GEMM on real data (constant operands
 * draw less power and clock higher).  *flops (host, may be NULL) receives the
 * flop count of the launch.  The rate it reaches is the measured ceiling of the
 * MFMA-bound kernels on this part.  n_blocks <= 65536, iters in [1, 2^24].     */
int mgb_mfma_loop_enqueue(void* stream, uint32_t bf16, uint32_t n_blocks, uint32_t iters, float* out,
                          double* flops);

/* Diagnostic: the rate at which the CUs bring operand rows from memory into LDS with the
 * instruction the DMA-ring kernels use (16 bytes per lane, 1 KiB per wave instruction).
 * n_blocks workgroups of four waves issue iters rounds of 8 such instructions each; the 64 lanes
 * of an instruction cover 1024 / row_bytes rows of row_bytes bytes (64, 128, or 1024 = one
 * contiguous KiB; then `pitch` is ignored), `pitch` bytes apart (a multiple of 16, >= row_bytes),
 * and every wave walks its own sequence of places through src[0, footprint_bytes) (device, 16-byte
 * aligned; the footprint decides which level of the memory hierarchy answers).  Rows of 64 bytes
 * are half cache lines: the figure that tells what depth-32 bf16 operand tiles cost against
 * depth-64 ones.  `sink` (device, one uint32) is never written in practice; *bytes (host, may be
 * NULL) receives the bytes requested by the launch.  n_blocks <= 65536, iters in [1, 2^20].    */
int mgb_fetch_rate_enqueue(void* stream, const void* src, uint64_t footprint_bytes, uint32_t row_bytes,
                           uint32_t pitch, uint32_t n_blocks, uint32_t iters, uint32_t* sink, double* bytes);

/* Diagnostic: the rate at which the waves of a CU read 16-byte matrix fragments from LDS (32 rows
 * of 128 bytes per half-wave), with the chunk swizzle of the conv kernels (swizzled != 0) or
 * without (bank conflicts).  n_blocks workgroups of four waves, iters rounds of 8 reads per lane;
 * *bytes (host, may be NULL) receives the bytes read.  n_blocks <= 65536, iters in [1, 2^24].  */
int mgb_lds_read_rate_enqueue(void* stream, uint32_t swizzled, uint32_t n_blocks, uint32_t iters, uint32_t* sink,
                              double* bytes);

#ifdef __cplusplus
}
#endif
#endif /* MGB_H */
