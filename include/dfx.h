/*
 * dfx -- preemptive daemon-kernel collectives for one MI355X (gfx950).
 *
 * A C ABI for the hot path of the deadlock-free collective library of
 * arXiv 2303.06324 (DFCCL): a daemon kernel polls a submission queue (SQ),
 * executes ring collectives as chunked reduce/copy primitives through
 * flag-guarded FIFOs ("connectors") in HBM, preempts a collective whose
 * primitive spins past its stickiness-adjusted threshold (context save /
 * switch / restore) and posts completions to a completion queue (CQ).
 *
 * R virtual ranks ("vranks") share ONE GPU: vrank r is a set of workgroups of
 * the one daemon grid, with its own SQ, CQ, task queues and contexts; only the
 * connectors are shared between neighbouring vranks.
 *
 * All pointers are plain pointers.  "device" = memory of the GPU the context
 * was created on, "host" = ordinary process memory.  No function throws; every
 * function returns DFX_OK (0) or a negative dfx_status.  Functions taking a
 * rank are thread-safe against calls for OTHER ranks (one submitter per SQ at
 * a time: Sec. 5, "single-producer multi-consumer"); dfx_init, dfx_prepare,
 * dfx_start, dfx_stop and dfx_finalize must not run concurrently with
 * anything else on the same context.
 */
#ifndef DFX_H
#define DFX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dfx_ctx dfx_ctx; /* opaque, library-owned */

/* The collectives of Sec. 4.1.  DFX_REDUCE: a chain that ends at the root (rank root+1 sends, the ranks
   after it combine and forward, the root combines and keeps); only the root's recv buffer is written. */
typedef enum { DFX_ALLREDUCE = 0, DFX_ALLGATHER = 1, DFX_REDUCESCATTER = 2, DFX_BROADCAST = 3, DFX_REDUCE = 4 } dfx_kind;
typedef enum { DFX_F32 = 0, DFX_BF16 = 1, DFX_F16 = 2, DFX_I32 = 3 } dfx_dtype;
/* Sec. 4.1 "reducing function", evaluated at every hop as partial (op) own, the partial that arrived
   first.  Sum and product round once per hop in the storage type (16-bit types: widen to fp32, operate,
   round to nearest even; int32 wraps).  Maximum / minimum pass on the partial if it is strictly greater
   (smaller), else the own value, bit for bit; NaN inputs are not supported. */
typedef enum { DFX_SUM = 0, DFX_PROD = 1, DFX_MAX = 2, DFX_MIN = 3 } dfx_op;

typedef enum {
  DFX_OK = 0,
  DFX_ERR_INVALID_ARG = -1,
  DFX_ERR_NOT_PREPARED = -2,
  DFX_ERR_BUSY = -3,      /* this (rank, coll_id) is already outstanding */
  DFX_ERR_SQ_FULL = -4,   /* retry: the slot is reusable once every workgroup has read it (Sec. 5) */
  DFX_ERR_TIMEOUT = -5,   /* wait deadline passed, or the in-kernel watchdog fired */
  DFX_ERR_HIP = -6,       /* a HIP runtime call failed; see dfx_last_hip_error */
  DFX_ERR_NO_RESOURCES = -7, /* grid does not fit the GPU / connector pool exhausted */
  DFX_ERR_ABORTED = -8,   /* the daemon was aborted; context must be finalized */
  DFX_ERR_TOO_LARGE = -9  /* dfx_collective_noalloc: beyond the sizes its static scratch memory is laid out for */
} dfx_status;

/* One completion.  In the paper the CQE carries only the collective's ID (Sec. 5); the invocation
   number is added here so that repeated runs of one ID can be told apart. */
typedef struct {
  uint32_t coll_id;
  uint32_t seq; /* how many times this (rank, coll_id) had been submitted before this invocation */
} dfx_cqe;

/* Tunables.  Zero-initialise, call dfx_config_default, then override fields. */
typedef struct {
  uint32_t struct_bytes;   /* sizeof(dfx_config) the caller was compiled with */
  uint32_t max_channels;   /* workgroups per vrank; daemon grid = nranks * max_channels (Sec. 5: launched with the largest grid) */
  uint32_t max_colls;      /* coll_id range [0, max_colls); also task-queue capacity (<= 4096) */
  uint32_t sq_depth;       /* SQ ring entries per vrank (power of two; default 1024: a burst of a thousand submissions does not wait for the daemon) */
  uint32_t cq_slots;       /* CQ slot-array length per vrank (Sec. 5 "optimized CQ") */
  uint32_t nslots;         /* K: slots per connector FIFO, >= 2 (a fused recv+send ring cannot run on 1) */
  uint32_t slot_bytes;     /* S: bytes per FIFO slot and channel, multiple of 16 (default 256 KiB).  A slice is
                              at most this long.  The chains take shorter slices, because their last rank starts
                              R-1 slices after the first: a broadcast about 2R per channel share, a reduce 4R,
                              of 32 KiB or more (reduce: at most 64 KiB); a broadcast with direct steps has no
                              slots and its slices may reach 2 S.  dfx_coll_info reports the slice length */
  uint32_t chan_min_bytes; /* a collective uses C = clamp(ceil(ringChunkBytes / chan_min_bytes), 1, max_channels) channels */
  /* The four spin_* fields shape the thresholds of passes that poll every queue entry in turn, as Alg. 1 is
     written: queues shorter than scan_min, or every queue with scan_min = 0.  A pass that began with a readiness
     scan visits only entries found runnable and waits at most spin_min polls on each; there the order of the
     visits (focus_bytes, order_policy) does what the adjusted thresholds are for. */
  uint32_t spin_init;      /* initial spin threshold (poll attempts) at the task-queue front (Sec. 4.3) */
  uint32_t spin_min;       /* thr(pos) = max(spin_min, spin_init >> pos) */
  uint32_t spin_max;       /* cap after boosting */
  uint32_t spin_boost;     /* thr *= spin_boost after a primitive succeeds (Sec. 6.4: twentyfold) */
  uint32_t preempt;        /* 0 = never abort a wait (the non-preemptive negative control) */
  uint32_t watchdog_ms;    /* in-kernel: work queued but no progress for this long => error + daemon exit */
  uint32_t quit_idle_us;   /* voluntary quit (Sec. 4.4): a workgroup leaves after this long without a
                              successful primitive or SQE fetch; 0 = stay resident until dfx_stop.  While the daemon
                              is resident a device-wide synchronisation, a kernel that needs the whole device, and
                              work of another stream that the runtime has put on the daemon's hardware queue (streams
                              share a few of them; a synchronous copy of results to the host has been seen to) wait
                              until it leaves: keep this above 0 unless the process does nothing else on the device */
  uint32_t sq_in_device;   /* 0: SQ in pinned host memory (the paper's placement);
                              1: SQ in fine-grained device memory written by the host through the PCIe BAR;
                              2: choose 1 when the device reports a large BAR, else 0 */
  uint32_t wg_map;         /* 0 (default): workgroup = channel*nranks + rank; 1: workgroup = rank*max_channels + channel */
  uint32_t order_policy;   /* 0 = FIFO ordering, 1 = priority ordering (Sec. 4.3): a fetched collective joins the queue
                              behind those of equal or higher priority, a scanned pass ranks the runnable collectives by
                              priority first, and the pass looks again (SQ probe, scan, ranking) after at most 32 KiB of
                              posted work and keeps one fold step in flight instead of two, so that an urgent collective waits for
                              little that was chosen before it came */
  uint32_t trace;          /* 1 = record context-switch latency samples (two clock reads per switch);
                              2 = also time the save / load parts and the wait / data / publish phases;
                              3 = phases as in 2, and the trace holds one sample per executed primitive
                                  instead of one per switch (see dfx_trace_read) */
  uint32_t fetch_batch;    /* SQEs a workgroup may fetch in a row when its queue is empty or stuck; 0 = all available */
  uint64_t pool_bytes;     /* device memory reserved for connectors of all prepared collectives (default 4 GiB) */
  uint32_t scan_min;       /* a pass over a task queue of at least this many entries starts with a readiness
                              scan (64 entries polled at once, one per lane) and visits only runnable
                              entries; 0 = never scan, poll every entry in turn as Alg. 1 is written */
  uint32_t chan_spread;    /* 1: a collective that uses fewer channels than max_channels starts at workgroup
                              (coll_id * channels) mod max_channels of its rank, so that many small
                              collectives spread over the grid; 0: every collective starts at workgroup 0
                              (small collectives all share the first task queues: the single-queue
                              setting of Sec. 2.3) */
  uint32_t cq_mode;        /* completion-queue variant (Sec. 5 "Optimizing CQ"): 0 = optimized CQ, one
                              system-scope CAS of the id into a free slot (default); 1 = vanilla ring buffer
                              (reserve, entry, fence, in-order tail update); 2 = optimized ring buffer (id and
                              position in one 64-bit atomic write, validated by the poller against its head) */
  uint32_t sq_eager;       /* 1 (default): a workgroup probes the SQ before every pass over its queue; 0: only when
                              its queue is empty or a whole pass made no progress (FIFO ordering as Sec. 4.3 words it) */
  uint32_t window;         /* slices of a collective are taken in windows of this many (1, 2 or 4; halved until it
                              is below nslots, which a ring of fused recv+send primitives needs to stay live):
                              primitive p of every slice of the window, then primitive p+1 ..., so that the
                              hop latency of one slice hides behind the data of another.  1 = the whole
                              primitive sequence slice after slice */
  uint32_t focus_bytes;    /* stickiness across ranks (the aim of Sec. 4.3's threshold adjustment): when not 0, a scanned
                              pass over a queue of at most 64 entries visits the runnable collectives
                              furthest-along first and ends once it has handed the movers this many bytes, so
                              that all ranks carry the same few collectives through instead of advancing all
                              of them side by side (whose FIFO slots together outgrow the memory-side cache);
                              0 = every runnable collective once per pass, in queue order */
  uint32_t direct;         /* 1 (default): collectives of at least direct_min_bytes (all-reduce, broadcast,
                              reduce: per rank; all-gather, reduce-scatter: all R blocks, which must be
                              16-byte multiples) take direct steps, since all buffers lie in one HBM.  The
                              opening send of an all-reduce, a reduce-scatter or a reduce chain only raises
                              the connector's counter and the next rank reads that
                              chunk from this rank's send buffer; in the gather steps (of an
                              all-reduce, an all-gather, a broadcast) a rank writes a chunk to its recv buffer
                              only and raises the counter, and the next rank reads it there; a last step waits
                              until the next rank has read everything before the completion is posted.  0:
                              every step goes through a FIFO slot, as the primitive table of Sec. 4.2 has it */
  uint32_t direct_min_bytes; /* default 2 MiB: below it the extra step costs more than the saved writes (the measured
                              break-even of an all-reduce per rank and of an all-gather in all; a reduce-scatter
                              takes the direct steps from twice this value in all, a broadcast or reduce from a
                              quarter of it per rank); 0 = every
                              all-reduce, broadcast and reduce, every all-gather and reduce-scatter of
                              16-byte-multiple blocks */
  uint32_t fold_max_bytes; /* default 64 MiB: an all-reduce of fewer bytes per rank runs in fold steps instead of ring steps.
                              The 2R-1 ring steps depend on one another and cost a few microseconds each whatever the
                              size, and a short message gives a channel one slice, so nothing hides them; with all
                              buffers in one HBM two steps that wait on all ranks at once do the same work: (1) when
                              every rank has submitted, rank r combines chunk r out of all R send buffers in the ring's
                              own order (x[r+1] (op) ... (op) x[r]: same association, same bits) and writes the result
                              into chunk r of all R recv buffers; (2) when every rank has done so, it posts the
                              completion (every input read once, every output written once).  Each step is a bounded
                              wait (Sec. 4.2) followed by the data, preempted like any primitive.  From this size on the
                              ring through the connectors' FIFOs keeps its movers busy and is what runs.  0 = off */
  uint32_t fold_slice_bytes; /* a collective in fold steps takes its share of a channel in slices of at most this many bytes
                              per source, one mover job each (16-byte multiple), so that what is ahead of an urgent
                              collective under priority ordering is short; 0 (default) = one slice, the whole share
                              (with 32 KiB slices under priority ordering the urgent bucket of the bench's staggered
                              study completes after 0.52-0.68 ms instead of 0.63-0.78 ms and the whole run takes 8 % longer) */
  uint32_t reserved0;      /* keeps the struct a multiple of 8 bytes; must be 0 */
} dfx_config;

/* Aggregated over the workgroups of one vrank since dfx_init. */
typedef struct {
  uint64_t preemptions;    /* waits that hit their spin threshold (context switches) */
  uint64_t ctx_loads;      /* context loads from HBM into an LDS active slot */
  uint64_t ctx_slot_hits;  /* loads avoided because the collective's LDS slot already held the context */
  uint64_t ctx_saves;      /* dynamic-context saves to HBM */
  uint64_t lazy_skips;     /* preemptions that skipped the save (nothing had progressed) */
  uint64_t polls;          /* poll attempts in wait phases */
  uint64_t prims;          /* primitives (slices) executed */
  uint64_t sqe_fetched;
  uint64_t cqe_posted;
  uint64_t max_taskq;      /* largest task-queue length seen by any workgroup */
  uint64_t passes;         /* traversals of the task queue */
  uint64_t quits;          /* voluntary quits */
  uint64_t launches;       /* daemon launches (whole context, not per rank) */
  uint64_t switch_samples; /* context-switch latency samples available */
  double switch_us_p50;    /* abort decision -> first poll of the next collective */
  double switch_us_p99;
  double switch_us_mean;
  double save_us_mean;     /* the save part of a switch */
  double load_us_mean;     /* the load part of a switch */
  double wait_us;          /* with trace >= 2: time in successful wait phases, summed over the vrank's workgroups */
  double data_us;          /* ... in data phases (first mover wave: job taken until its stores are drained) */
  double publish_us;       /* ... between the last mover wave's drain and its counter updates */
  uint64_t scan_skips;     /* queue entries a readiness scan found not runnable (no context load, no spin) */
  double cqe_us;           /* time spent writing CQEs (first to last host-memory operation), summed; always counted */
  double advance_us_mean;  /* with trace = 2: the part of a switch between the save and the load (retiring finished jobs, next queue entry) */
  double setup_us_mean;    /* with trace = 2: the part after the load (thresholds, the primitive's descriptor) up to the first poll */
  double clock_read_us;    /* with trace = 1 or 2: what one read of the wall clock costs the scheduler (a switch sample holds two
                              reads, a split sample five) */
  double sqe_us;           /* time the vrank's workgroups spent fetching SQEs (entry seen -> run of up to 64 entries read,
                              cooked into contexts, queued), summed over workgroups; always counted.  Every workgroup reads
                              every entry of its vrank: divide by sqe_fetched for the time per entry and workgroup */
} dfx_stats_t;

/* Fill *cfg with defaults (struct_bytes set). cfg: host, caller-owned. */
int dfx_config_default(dfx_config* cfg);

/*
 * Create a context for nranks vranks on the current HIP device (= nranks x dfcclInit, Sec. 3.2).
 * cfg: host, may be NULL (defaults).  hip_stream: a hipStream_t (default priority) that the
 * library uses ONLY for the daemon kernel; nothing else may be enqueued on it (work queued
 * behind a resident daemon would never start).  Allocates SQ, CQ, context buffers, counters
 * and the connector pool; all are library-owned and freed by dfx_finalize.
 * Several contexts may exist on one device, but their daemons take turns: a context's daemon is not
 * started while another context's is in flight on the same device (that one leaves after
 * quit_idle_us without work, or at dfx_stop; with quit_idle_us = 0 only at dfx_stop), and the calls
 * that wait for completions start it as soon as the device is free.
 * Errors: INVALID_ARG (nranks < 1 or > 64, bad cfg), NO_RESOURCES (grid cannot be co-resident), HIP.
 */
int dfx_init(dfx_ctx** out, int nranks, const dfx_config* cfg, void* hip_stream);

/*
 * Register collective coll_id on every vrank (= dfcclRegister* on each rank of the device set,
 * Sec. 3.2): fixes kind, element count, dtype, op (ignored by all-gather and broadcast), root
 * (broadcast and reduce) and priority (larger =
 * more urgent; only used by the priority order policy), assigns its connectors (exclusive to
 * this collective, Sec. 4.5) and its channel count.  May be called while the daemon runs.
 * count: all-reduce / broadcast / reduce: elements per rank; all-gather: elements each rank contributes
 * (recv buffers hold nranks*count); reduce-scatter: elements each rank receives (send buffers
 * hold nranks*count).  Errors: INVALID_ARG (id out of range or already prepared, unknown enum),
 * NO_RESOURCES (connector pool exhausted).
 */
int dfx_prepare(dfx_ctx* ctx, int coll_id, dfx_kind kind, size_t count, dfx_dtype dtype, dfx_op op,
                int root, int priority);

/*
 * Invoke a prepared collective on one vrank (= dfcclRun*, Sec. 3.2): writes one SQE and returns
 * at once; starts the daemon if it is not running (Sec. 4.4 event-driven start).
 * sendbuf, recvbuf: device, caller-owned, 16-byte aligned, valid and unmodified (sendbuf) /
 * unread (recvbuf) until this rank's CQE for the invocation; they may differ between
 * invocations of one coll_id (Sec. 4.2) and must not overlap each other, except that an all-reduce may
 * run in place (recvbuf == sendbuf).
 * Errors: INVALID_ARG, NOT_PREPARED, BUSY, SQ_FULL (retry), ABORTED, HIP.
 * Unless dfx_set_callback has started the poller thread, completions wait in the CQ (cq_slots entries per vrank) until
 * dfx_poll / dfx_wait / dfx_wait_all take them, or until a dfx_submit on that vrank finds the SQ full
 * and moves them to the host-side list itself.  A vrank whose CQ is full stops making progress.
 */
int dfx_submit(dfx_ctx* ctx, int rank, int coll_id, const void* sendbuf, void* recvbuf);

/*
 * One invocation of coll_id on every vrank in a single call (vrank order 0 .. nranks-1):
 * sendbufs / recvbufs: host arrays of nranks device pointers.  The same as nranks dfx_submit calls,
 * minus nranks-1 trips through the caller's language binding; for the single-process setting in which
 * one thread drives all vranks, and with all entries made visible together (their bodies, one store fence,
 * their generation words).  All or nothing: returns DFX_OK when every vrank's entry is in its SQ, else the first
 * status that is not OK with no vrank submitted (a full SQ is retried for up to timeout_ns first).
 */
int dfx_submit_all(dfx_ctx* ctx, int coll_id, const void* const* sendbufs, void* const* recvbufs, uint64_t timeout_ns);

/*
 * Submit n collectives of one vrank in the given order (a burst of dfcclRun* calls, e.g. the
 * gradient buckets of one backward pass): element i is dfx_submit(ctx, rank, coll_ids[i],
 * sendbufs[i], recvbufs[i]), made visible to the daemon in runs of up to 32 entries (the bodies of a run, one
 * store fence, its generation words).  A full SQ is retried until timeout_ns has passed.  The three arrays
 * are host arrays of n entries, read only during the call; the buffers they point to are device
 * memory under the rules of dfx_submit.  Returns how many were submitted (n on success, fewer on
 * timeout or on an error after the first), or the negative status of the first submission.
 */
int dfx_submit_many(dfx_ctx* ctx, int rank, int n, const int* coll_ids, const void* const* sendbufs,
                    void* const* recvbufs, uint64_t timeout_ns);

/*
 * dfx_submit_many with a pause before every entry: delays_ns[i] nanoseconds of busy waiting precede
 * entry i (host array of n values, or NULL for none).  For workloads whose submissions are staggered
 * in time, driven from native threads rather than from an interpreter loop.
 */
int dfx_submit_many_paced(dfx_ctx* ctx, int rank, int n, const int* coll_ids, const void* const* sendbufs,
                          void* const* recvbufs, const uint64_t* delays_ns, uint64_t timeout_ns);

/*
 * Take up to max completions of one vrank (the poller's job, Sec. 3.1).  out: host.
 * Returns the number of CQEs written to out (>= 0) or a negative status.  Restarts a daemon
 * that quit voluntarily while work is outstanding.
 */
int dfx_poll(dfx_ctx* ctx, int rank, dfx_cqe* out, int max);

/*
 * Callback delivery (Sec. 3.1: the poller thread reads CQEs and runs the callback bound to the
 * collective).  With fn != NULL the library starts one poller thread that drains the CQs of all
 * vranks, restarts a daemon that quit while work is outstanding, and calls fn(user, rank, coll_id,
 * seq) once per completion, outside any library lock (fn may submit).  Completions delivered this
 * way are not returned by dfx_poll any more; dfx_wait / dfx_wait_all keep working.  fn == NULL stops
 * and joins the thread.  fn runs on the poller thread; user is passed through untouched.
 */
typedef void (*dfx_callback)(void* user, int rank, uint32_t coll_id, uint32_t seq);
int dfx_set_callback(dfx_ctx* ctx, dfx_callback fn, void* user);

/*
 * Block until the latest invocation of coll_id on rank has completed, or timeout_ns passed
 * (TIMEOUT; the context stays usable).  Consumes that CQE; other CQEs seen meanwhile stay
 * available to dfx_poll.  If the daemon reported a watchdog error: TIMEOUT, and the context is
 * aborted.
 */
int dfx_wait(dfx_ctx* ctx, int rank, int coll_id, uint64_t timeout_ns);

/* Block until every submission made so far on every vrank has completed (CQEs are consumed). */
int dfx_wait_all(dfx_ctx* ctx, uint64_t timeout_ns);

/* Launch the daemon now if it is not running (normally implicit in dfx_submit). */
int dfx_start(dfx_ctx* ctx);

/*
 * Post an exit SQE to every vrank (Sec. 4.4 "exiting SQE") and wait until the daemon grid has
 * drained.  Outstanding collectives keep their saved contexts and resume at the next start.
 */
int dfx_stop(dfx_ctx* ctx);

/* Counters of one vrank; out: host. Safe while the daemon runs (values may lag). */
int dfx_stats(dfx_ctx* ctx, int rank, dfx_stats_t* out);

/* Geometry the library chose for a prepared collective (for tests and the bench). */
int dfx_coll_info(dfx_ctx* ctx, int coll_id, uint32_t* nchan, uint32_t* slot_bytes, uint32_t* rounds,
                  uint32_t* nprim);

/* Raw trace samples of one workgroup (0 <= wg < nranks * max_channels), oldest first while fewer than
   4096 have been written (a ring afterwards); valid once the daemon has stopped or quit.  With
   trace = 1 or 2 a sample is one context switch: bits 0-15 total ticks, and with trace = 2 bits 16-27 save,
   28-39 queue advance, 40-51 load, 52-63 set-up ticks (each saturating).  With trace = 3 a sample is one executed primitive (the breakdown of Sec. 6.3 per
   workgroup): bits 0-31 low word of the wall clock when its data phase began, 32-47 ticks the data
   phase took (saturating), 48-59 collective id (low 12 bits), 60-63 index in the primitive sequence
   (low 4 bits), or 15 for a wait phase that ended in preemption (then the two times are those of
   the wait); switch-latency statistics are not collected in that mode.  *tick_us: microseconds
   per tick.  out, tick_us: host.  Returns the number of samples copied, or a negative error. */
int dfx_trace_read(dfx_ctx* ctx, uint32_t wg, uint64_t* out, uint32_t max, double* tick_us);

/* Milliseconds the last completed daemon launch spent on the GPU (HIP events on the daemon's
   stream), and how many launches have completed; 0 launches => *ms = 0. out pointers: host. */
int dfx_last_launch_ms(dfx_ctx* ctx, float* ms, uint64_t* launches_done);

/* = nranks x dfcclDestroy: dfx_stop, then free everything. ABORTED if work was still outstanding
   (it is dropped).  ctx is invalid afterwards in every case. */
int dfx_finalize(dfx_ctx* ctx);

/* hipError_t of the last failing HIP call on this context, as an int. */
int dfx_last_hip_error(dfx_ctx* ctx);

/* hipError_t of the HIP call that made the last dfx_init in this process fail (0 if none). */
int dfx_last_init_error(void);

const char* dfx_strerror(int status);

/* Identifier of the sources this library was built from (a hash of the kernel and host sources, this
   header and the compiler flags, baked in at build time): lets a loader notice a library that is
   older than the sources beside it.  Points to static storage. */
const char* dfx_build_id(void);

/* Measurement aid, not part of the method: copy `bytes` (multiple of 16) from src to dst (both
   device) with a plain grid-stride kernel on hip_stream (NULL = the null stream) and wait.  Its
   known traffic calibrates the profiler's HBM byte counters; with ms != NULL (host) the kernel is
   timed with HIP events on that stream, which gives the copy bandwidth the chip reaches. */
int dfx_copy_calibrate(const void* src, void* dst, size_t bytes, void* hip_stream, float* ms);

/*
 * Self-check of the kernel's index arithmetic, on the host, without a GPU (the kernel and this call compile the
 * same functions).  For collective (kind, count, dtype, op, root, coll_id) among nranks vranks under cfg (NULL =
 * defaults) and workgroup map wg_map it enumerates every workgroup of the grid and verifies that (i) the map is
 * a bijection between workgroups and (rank, channel) and every channel of the collective is served by exactly
 * one workgroup per rank, (ii) both ends of every connector (Sec. 4.1) resolve to the same flag line and the same
 * slots, inside the collective's connector block, (iii) along every workgroup's walk through its primitive
 * sequence (Sec. 4.2: slices x primitives, in windows) every read and write stays inside the send / recv buffer,
 * the neighbour's buffer or the connector's slots, the writes to each recv buffer tile it exactly once, and every
 * edge carries as many slices as its receiver takes.  wg_map 2 = the labelling "XCD = (rank + channel) mod 8",
 * which the kernel does not offer, kept here so that the check covers it.  msg (host, may be NULL): receives a
 * description of the first violation.  Returns DFX_OK, or DFX_ERR_INVALID_ARG with msg filled.
 */
int dfx_check_geometry(int nranks, const dfx_config* cfg, dfx_kind kind, size_t count, dfx_dtype dtype, dfx_op op,
                       int root, int coll_id, uint32_t wg_map, char* msg, size_t msg_bytes);

/*
 * For callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  One invocation of one collective on every vrank -- what dfx_init + dfx_prepare + dfx_submit_all do
 * with memory they allocate -- with everything the daemon kernel needs beyond the caller's buffers (SQ, CQ,
 * counters, saved contexts, connector flag lines and slots) in a static device array of the library:
 * 32.5 MiB per GPU the library runs on, held until the process ends.  The call allocates nothing (no hipMalloc,
 * hipFree, stream, event or host allocation) and only enqueues work on hip_stream (NULL = the null stream): a
 * kernel that clears the array's control part, one that writes the submission entries, the daemon kernel
 * (nranks x min(32, 256 / nranks) workgroups, which leaves by itself when every vrank's completion is posted)
 * and one that writes the outcome.  It returns when the work is enqueued; the results are in recvbufs once the
 * stream has reached the end of that work.
 * nranks: 1 .. 64.  kind / count / dtype / op / root: as for dfx_prepare; same values, bit for bit, as the
 * context path.  sendbufs / recvbufs: host arrays of nranks device pointers (read during the call), the buffers
 * under the rules of dfx_submit.  status_dev: device, 4 bytes, may be NULL; written at the end: 0 = completed,
 * 0x100 | code = the in-kernel watchdog or an internal check fired, 0x200 = a completion is missing.
 * Limits: no per-rank buffer (send or recv) above DFX_NOALLOC_MAX_BYTES => DFX_ERR_TOO_LARGE.
 * Every call on a GPU uses that GPU's one array: calls that overlap on one GPU race (also from different
 * streams or threads); a call is refused with DFX_ERR_BUSY while a context's daemon is in flight on the device,
 * and no context's daemon may be started on the device before the call's work has finished.
 * Errors: INVALID_ARG, TOO_LARGE, BUSY, NO_RESOURCES (the grid cannot be co-resident on this device), HIP.
 */
#define DFX_NOALLOC_MAX_BYTES (1ull << 30)
int dfx_collective_noalloc(int nranks, dfx_kind kind, size_t count, dfx_dtype dtype, dfx_op op, int root,
                           const void* const* sendbufs, void* const* recvbufs, uint32_t* status_dev, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* DFX_H */
