// Host side of the dfx C ABI: SQ/CQ management, collective registration, event-driven daemon
// start, completion polling.  The "CPU part" of the paper's Fig. 3 (Sec. 3.1), for R virtual
// ranks in one process.  No computation of the collectives happens here.
#include <hip/hip_runtime.h>
#include <immintrin.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <deque>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

#include "../../include/dfx.h"
#include "dfx_internal.h"
#include "dfx_geometry.h"

// defined next to the kernels
hipError_t dfx_daemon_occupancy(int* blocks_per_cu);
hipError_t dfx_daemon_launch(uint32_t nwg, hipStream_t stream, const DfxDaemonArgs& a);
hipError_t dfx_copy_launch(const void* src, void* dst, size_t bytes, hipStream_t stream);

namespace {

struct CollInfo {
  bool prepared = false;
  DfxStatic tmpl;   // everything but buffers, seq and ready
};

struct RankState {
  std::mutex mu;
  uint64_t sq_tail = 0;                 // entries written to this rank's SQ
  std::vector<uint32_t> sub;            // per coll: submissions so far
  std::vector<uint32_t> done;           // per coll: completions seen
  std::deque<dfx_cqe> ready;            // completions not yet handed to the caller
  uint64_t cq_head = 0;                 // ring-buffer CQ variants: entries consumed
  std::atomic<uint64_t> n_sub{0}, n_cqe{0};
};

}  // namespace

struct dfx_ctx {
  dfx_config cfg;
  int R = 0;
  int device = 0;
  uint32_t nwg = 0;
  uint32_t sq_shift = 0;
  hipStream_t stream = nullptr;      // daemon stream
  bool own_stream = false;
  hipStream_t side = nullptr;        // private non-blocking stream for small copies
  hipEvent_t ev_start = nullptr, ev_stop = nullptr;
  bool launched = false;             // a launch has been enqueued whose end was not yet observed
  uint64_t launches = 0, launches_done = 0;
  float last_ms = 0.f;
  double tick_us = 0.01;             // wall_clock64 tick in microseconds
  std::mutex launch_mu;
  std::atomic<bool> aborted{false};
  int last_hip = 0;
  bool sq_device = false;
  uint32_t fifo_coherent = 1;        // connector accesses: 1 = device-coherent (sc1), 0 = cached + agent-scope fences

  // host-visible memory
  void* qmem_sq = nullptr;           // SQ ring + host_ctl (pinned host or fine-grained device)
  size_t qmem_sq_bytes = 0;
  void* qmem_cq = nullptr;           // CQ slot arrays (pinned host)
  DfxSqSlot* sq = nullptr;
  uint32_t* host_ctl = nullptr;
  uint64_t* cq = nullptr;
  uint64_t* cq_ctl = nullptr;        // ring bookkeeping of the ring-buffer CQ variants (same allocation as cq)
  uint32_t* sq_freed = nullptr;      // [R][sq_depth] generation of the last entry every workgroup has read (same allocation as cq)
  // device memory
  uint32_t* sq_readers = nullptr;
  uint32_t* done_cnt = nullptr;
  uint32_t* dev_ctl = nullptr;
  uint8_t* pool = nullptr;
  DfxCtxEntry* ctxbuf = nullptr;
  DfxWgState* wgstate = nullptr;
  uint16_t* taskq_store = nullptr;
  uint64_t* trace = nullptr;
  void* pinned_tmp = nullptr;        // staging for stats reads
  size_t pinned_tmp_bytes = 0;

  uint64_t pool_used = 0;
  std::vector<CollInfo> colls;
  std::vector<RankState*> ranks;

  // callback delivery
  std::thread poller;
  std::atomic<bool> poller_run{false};
  std::atomic<bool> user_stopped{false};   // dfx_stop was the last word: the poller thread does not restart the daemon
  dfx_callback cb = nullptr;
  void* cb_user = nullptr;
};

namespace {

#define HIPCHK(ctx, call)                        \
  do {                                           \
    hipError_t e_ = (call);                      \
    if (e_ != hipSuccess) {                      \
      (ctx)->last_hip = (int)e_;                 \
      return DFX_ERR_HIP;                        \
    }                                            \
  } while (0)

int g_init_hip_error = 0;   // hipError_t of the last failing call inside dfx_init

inline uint64_t now_ns() {
  return (uint64_t)std::chrono::duration_cast<std::chrono::nanoseconds>(
             std::chrono::steady_clock::now().time_since_epoch()).count();
}

inline uint32_t elem_bytes(int dt) { return (dt == DFX_F32 || dt == DFX_I32) ? 4u : 2u; }
inline uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }
inline uint64_t round_up(uint64_t a, uint64_t b) { return ceil_div(a, b) * b; }
inline bool is_pow2(uint32_t x) { return x && !(x & (x - 1)); }

// Fine-grained device memory that a kernel has read is not given back to the driver while the
// process lives (memory handed out after such a free has been seen to hold wrong values): a
// context's SQ goes to this list instead and the next context of the same size takes it over.
struct ParkedSq { int device; size_t bytes; void* ptr; };
std::mutex g_parked_mu;
std::vector<ParkedSq> g_parked_sq;

void* take_parked_sq(int device, size_t bytes) {
  std::lock_guard<std::mutex> lk(g_parked_mu);
  for (size_t i = 0; i < g_parked_sq.size(); ++i)
    if (g_parked_sq[i].device == device && g_parked_sq[i].bytes == bytes) {
      void* p = g_parked_sq[i].ptr;
      g_parked_sq.erase(g_parked_sq.begin() + (long)i);
      return p;
    }
  return nullptr;
}

void free_all(dfx_ctx* c) {
  if (c->qmem_sq) {
    if (c->sq_device) {
      std::lock_guard<std::mutex> lk(g_parked_mu);
      g_parked_sq.push_back({c->device, c->qmem_sq_bytes, c->qmem_sq});
    } else (void)hipHostFree(c->qmem_sq);
  }
  if (c->qmem_cq) (void)hipHostFree(c->qmem_cq);
  if (c->pinned_tmp) (void)hipHostFree(c->pinned_tmp);
  void* dev[] = {c->sq_readers, c->done_cnt, c->dev_ctl, c->pool, c->ctxbuf, c->wgstate, c->taskq_store, c->trace};
  for (void* p : dev) if (p) (void)hipFree(p);
  if (c->ev_start) (void)hipEventDestroy(c->ev_start);
  if (c->ev_stop) (void)hipEventDestroy(c->ev_stop);
  if (c->side) (void)hipStreamDestroy(c->side);
  if (c->own_stream && c->stream) (void)hipStreamDestroy(c->stream);
  for (RankState* r : c->ranks) delete r;
  delete c;
}

// Observe the end of the last launch, if it ended.  Caller holds launch_mu.
// Returns true if no daemon launch is in flight afterwards.
int reap_locked(dfx_ctx* c, bool* idle) {
  *idle = true;
  if (!c->launched) return DFX_OK;
  hipError_t q = hipEventQuery(c->ev_stop);
  if (q == hipErrorNotReady) { *idle = false; return DFX_OK; }
  if (q != hipSuccess) { c->last_hip = (int)q; return DFX_ERR_HIP; }
  c->launched = false;
  c->launches_done++;
  float ms = 0.f;
  if (hipEventElapsedTime(&ms, c->ev_start, c->ev_stop) == hipSuccess) c->last_ms = ms;
  // the grid has drained: a plain copy on the private stream is safe
  uint32_t* ctl = (uint32_t*)c->pinned_tmp;
  HIPCHK(c, hipMemcpyAsync(ctl, c->dev_ctl, DC_N * sizeof(uint32_t), hipMemcpyDeviceToHost, c->side));
  HIPCHK(c, hipStreamSynchronize(c->side));
  if (ctl[DC_ABORT]) c->aborted.store(true);
  return DFX_OK;
}

int launch_locked(dfx_ctx* c) {
  DfxDaemonArgs a;
  memset(&a, 0, sizeof(a));
  a.sq = c->sq; a.cq = c->cq; a.host_ctl = c->host_ctl;
  a.sq_readers = c->sq_readers; a.done_cnt = c->done_cnt; a.dev_ctl = c->dev_ctl;
  a.pool = c->pool; a.ctxbuf = c->ctxbuf; a.wgstate = c->wgstate; a.taskq_store = c->taskq_store; a.trace = c->trace;
  a.R = (uint32_t)c->R; a.cmax = c->cfg.max_channels; a.max_colls = c->cfg.max_colls;
  a.sq_depth = c->cfg.sq_depth; a.sq_shift = c->sq_shift; a.cq_slots = c->cfg.cq_slots;
  a.spin_init = c->cfg.spin_init; a.spin_min = c->cfg.spin_min; a.spin_max = c->cfg.spin_max;
  a.spin_boost = c->cfg.spin_boost; a.preempt = c->cfg.preempt;
  a.wg_map = c->cfg.wg_map; a.order_policy = c->cfg.order_policy; a.trace_on = c->cfg.trace;
  a.fetch_batch = c->cfg.fetch_batch ? c->cfg.fetch_batch : 0xffffffffu;
  a.fifo_coherent = c->fifo_coherent;
  a.watchdog_ticks = (uint64_t)((double)c->cfg.watchdog_ms * 1000.0 / c->tick_us);
  a.quit_ticks = (uint64_t)((double)c->cfg.quit_idle_us / c->tick_us);
  a.nwg = c->nwg;
  a.cq_ctl = c->cq_ctl; a.sq_freed = c->sq_freed; a.cq_mode = c->cfg.cq_mode; a.sq_eager = c->cfg.sq_eager; a.window = c->cfg.window; a.sq_local = c->sq_device ? 1u : 0u; a.focus_bytes = c->cfg.focus_bytes;
  // Priority ordering looks again (SQ probe, scan, ranking) after 32 KiB of posted work at most: an urgent
  // collective that arrives waits for less work that was chosen before it was there.
  if (c->cfg.order_policy == 1 && a.focus_bytes > (32u << 10)) a.focus_bytes = 32u << 10;
  a.scan_min = c->cfg.scan_min;
  a.chan_spread = c->cfg.chan_spread;
  a.epoch = (uint32_t)(c->launches + 1);
  // quit votes and the quit flag belong to one launch
  HIPCHK(c, hipMemsetAsync(c->dev_ctl + DC_QUIT, 0, 2 * sizeof(uint32_t), c->stream));
  HIPCHK(c, hipEventRecord(c->ev_start, c->stream));
  HIPCHK(c, dfx_daemon_launch(c->nwg, c->stream, a));
  HIPCHK(c, hipEventRecord(c->ev_stop, c->stream));
  c->launched = true;
  c->launches++;
  return DFX_OK;
}

// One daemon grid per device at a time.  A grid fills the compute units and every workgroup of it
// spins on flags that its other workgroups write, so two grids that each got part of the device
// would wait for each other until their watchdogs fire.  The contexts of a process therefore take
// turns: a launch is put off while the daemon of another context on the same device is still in
// flight (it leaves when it has been idle for quit_idle_us, or at dfx_stop), and every call that
// waits for completions comes back here.  Lock order: a context's launch_mu, then the slot.
struct DeviceSlot {
  std::mutex mu;
  dfx_ctx* owner = nullptr;
  hipEvent_t until = nullptr;   // the owner's ev_stop: not ready while its grid is in flight
};
constexpr int kMaxDevices = 64;
DeviceSlot g_slot[kMaxDevices];

void release_slot(dfx_ctx* c) {
  DeviceSlot& s = g_slot[c->device % kMaxDevices];
  std::lock_guard<std::mutex> lk(s.mu);
  if (s.owner == c) { s.owner = nullptr; s.until = nullptr; }
}

// Event-driven start (Sec. 4.4): make sure a daemon is running or queued.
int ensure_running(dfx_ctx* c) {
  std::lock_guard<std::mutex> lk(c->launch_mu);
  bool idle = false;
  int rc = reap_locked(c, &idle);
  if (rc != DFX_OK) return rc;
  if (c->aborted.load()) return DFX_ERR_ABORTED;
  if (!idle) return DFX_OK;
  DeviceSlot& s = g_slot[c->device % kMaxDevices];
  std::lock_guard<std::mutex> lk2(s.mu);
  if (s.owner && s.owner != c) {
    if (hipEventQuery(s.until) == hipErrorNotReady) return DFX_OK;   // another context's turn
    s.owner = nullptr;
  }
  rc = launch_locked(c);
  if (rc == DFX_OK) { s.owner = c; s.until = c->ev_stop; }
  return rc;
}

bool outstanding(dfx_ctx* c) {
  for (RankState* r : c->ranks)
    if (r->n_cqe.load(std::memory_order_relaxed) < r->n_sub.load(std::memory_order_relaxed)) return true;
  return false;
}

// Writing an SQE has two halves (the caller holds the rank's mutex): the body goes into the slot `ahead` entries
// behind the tail, and -- after a store fence -- the generation word, which the daemon looks for, makes it
// visible.  Several bodies may be written before one fence and their generation words after it, so a burst
// costs two fences in all instead of two per entry (behind the PCIe BAR a fence is a third of a microsecond).
bool sqe_slot_free(dfx_ctx* c, int rank, uint32_t ahead) {
  RankState* rs = c->ranks[rank];
  const uint32_t D = c->cfg.sq_depth;
  const uint64_t at = rs->sq_tail + ahead;
  // The slot last held the entry of one generation back; the last workgroup to read that one wrote
  // its generation into host memory.  Nothing is read from the SQ itself: it may lie behind the
  // PCIe BAR, where a load costs a microsecond.
  const uint32_t gen_before = (uint32_t)(at >> c->sq_shift);
  volatile uint32_t* freed = &c->sq_freed[(size_t)rank * D + (at & (D - 1))];
  if (ahead >= D || *freed != gen_before) return false;   // not yet read by every workgroup of the rank
  std::atomic_thread_fence(std::memory_order_acquire);
  return true;
}
void sqe_write_body(dfx_ctx* c, int rank, uint32_t ahead, const DfxStatic& e) {
  RankState* rs = c->ranks[rank];
  const uint32_t D = c->cfg.sq_depth;
  DfxSqSlot* slot = &c->sq[(size_t)rank * D + ((rs->sq_tail + ahead) & (D - 1))];
  DfxStatic tmp = e;
  tmp.ready = 0;
  // six 16-byte stores, the last one without its last word (the generation)
  const __m128i* src = (const __m128i*)&tmp;
  __m128i* dst = (__m128i*)&slot->e;
  for (int i = 0; i < 5; ++i) _mm_storeu_si128(dst + i, _mm_loadu_si128(src + i));
  uint32_t* lastw = (uint32_t*)(dst + 5);
  const uint32_t* lasts = (const uint32_t*)(src + 5);
  lastw[0] = lasts[0]; lastw[1] = lasts[1]; lastw[2] = lasts[2];
}
void sqe_fence() {
  std::atomic_thread_fence(std::memory_order_release);
  _mm_sfence();   // orders write-combined stores when the SQ lives behind the PCIe BAR
}
// generation words of the `n` bodies written at the tail, in order; the tail moves on
void sqe_publish(dfx_ctx* c, int rank, uint32_t n) {
  RankState* rs = c->ranks[rank];
  const uint32_t D = c->cfg.sq_depth;
  for (uint32_t k = 0; k < n; ++k) {
    DfxSqSlot* slot = &c->sq[(size_t)rank * D + (rs->sq_tail & (D - 1))];
    volatile uint32_t* ready = &slot->e.ready;
    *ready = (uint32_t)(rs->sq_tail >> c->sq_shift) + 1u;
    rs->sq_tail++;
  }
}

// Write one SQE (caller holds the rank's mutex).
int push_sqe(dfx_ctx* c, int rank, const DfxStatic& e) {
  if (!sqe_slot_free(c, rank, 0)) return DFX_ERR_SQ_FULL;
  sqe_write_body(c, rank, 0, e);
  sqe_fence();
  sqe_publish(c, rank, 1);
  _mm_sfence();
  return DFX_OK;
}

// Move every completion of a rank that has arrived into its ready list (caller holds the rank's mutex).
void drain_cq(dfx_ctx* c, int rank) {
  RankState* rs = c->ranks[rank];
  volatile uint64_t* q = c->cq + (size_t)rank * c->cfg.cq_slots;
  auto take = [&](uint32_t coll, uint32_t seq) {
    dfx_cqe e;
    e.coll_id = coll;
    e.seq = seq;
    if (e.coll_id < rs->done.size()) rs->done[e.coll_id]++;
    rs->ready.push_back(e);
    rs->n_cqe.fetch_add(1, std::memory_order_relaxed);
  };
  if (c->cfg.cq_mode == 0) {
    // optimized CQ: scan the slots, take the valid ones and mark them writable
    for (uint32_t i = 0; i < c->cfg.cq_slots; ++i) {
      uint64_t v = q[i];
      if (!(v >> 63)) continue;
      std::atomic_thread_fence(std::memory_order_acquire);
      q[i] = 0;
      take((uint32_t)(v & 0xffffffffu), (uint32_t)((v >> 32) & 0x7fffffffu));
    }
    return;
  }
  volatile uint64_t* ctl = c->cq_ctl + (size_t)rank * DFX_CQ_CTL_WORDS;
  const uint64_t head0 = rs->cq_head;
  if (c->cfg.cq_mode == 1) {
    // vanilla ring: everything below the producers' tail is complete
    const uint64_t tail = ctl[8];
    std::atomic_thread_fence(std::memory_order_acquire);
    for (; rs->cq_head < tail; ++rs->cq_head) {
      const uint64_t v = q[rs->cq_head % c->cfg.cq_slots];
      take((uint32_t)(v & 0xffffffffu), (uint32_t)((v >> 32) & 0x7fffffffu));
    }
  } else {
    // optimized ring: the entry at the head is valid when the position written into it is head + 1;
    // the invocation number is the host's own count (one invocation of an id is outstanding at a time)
    for (;;) {
      const uint64_t v = q[rs->cq_head % c->cfg.cq_slots];
      if ((uint32_t)(v >> 32) != (uint32_t)(rs->cq_head + 1)) break;
      std::atomic_thread_fence(std::memory_order_acquire);
      const uint32_t coll = (uint32_t)(v & 0xffffu);
      take(coll, coll < rs->done.size() ? rs->done[coll] : 0u);
      ++rs->cq_head;
    }
  }
  if (rs->cq_head != head0) {
    std::atomic_thread_fence(std::memory_order_release);
    ctl[16] = rs->cq_head;   // room for the producers
  }
}

// Geometry of one collective under a configuration: ring chunk, channels, slice length, rounds, primitive
// count, whether it takes direct steps, and the bytes of connector memory it needs (flag lines first, then
// the slots).  Shared by dfx_prepare and the entry point that brings its own static memory.
int plan_collective(const dfx_config& cfg, int nranks, int coll_id, dfx_kind kind, size_t count, dfx_dtype dtype, dfx_op op,
                    int root, int priority, uint64_t conn_off, DfxStatic* out, uint64_t* conn_bytes_out) {
  if ((int)kind < 0 || (int)kind > 4 || (int)dtype < 0 || (int)dtype > 3 || (int)op < 0 || (int)op > 3) return DFX_ERR_INVALID_ARG;
  const bool rooted = (kind == DFX_BROADCAST || kind == DFX_REDUCE);
  if (rooted && (root < 0 || root >= nranks)) return DFX_ERR_INVALID_ARG;
  if (priority < -32768 || priority > 32767) return DFX_ERR_INVALID_ARG;
  if (count > (1ull << 40)) return DFX_ERR_INVALID_ARG;

  const uint64_t R = (uint64_t)nranks;
  const uint32_t eb = elem_bytes(dtype);
  const uint64_t per16 = 16 / eb;
  // ring chunk: all-reduce cuts the message into R contiguous chunks of ceil(N/R) elements
  // rounded up to 16 bytes; the other kinds move blocks of `count`
  // Fold steps (see dfx_config.fold_max_bytes): every kind whose largest per-rank buffer is below the limit; the blocks
  // of an all-gather / reduce-scatter must be 16-byte multiples (they are read with 16-byte vectors where they lie).
  const uint64_t largest_bytes = (kind == DFX_ALLGATHER || kind == DFX_REDUCESCATTER) ? count * eb * R : count * eb;
  const bool blocks_ok = !(kind == DFX_ALLGATHER || kind == DFX_REDUCESCATTER) || (count * eb) % 16 == 0;
  // (a reduce's fold step has one look-up more than it has ranks, one per lane of the scheduler wavefront: at most 63 ranks)
  const bool fold = R > 1 && cfg.fold_max_bytes && largest_bytes < cfg.fold_max_bytes && blocks_ok && !(kind == DFX_REDUCE && R > 63);
  uint64_t block = count;
  // (a reduce in fold steps is cut into chunks like an all-reduce: rank r combines chunk r into the root's buffer)
  if ((kind == DFX_ALLREDUCE || (kind == DFX_REDUCE && fold)) && R > 1) block = round_up(ceil_div(count, R), per16);
  const uint64_t block_bytes = block * eb;
  uint64_t C = ceil_div(std::max<uint64_t>(block_bytes, 1), cfg.chan_min_bytes);
  C = std::min<uint64_t>(std::max<uint64_t>(C, 1), cfg.max_channels);
  uint64_t part = round_up(std::max<uint64_t>(ceil_div(block, C), 1), per16);
  C = std::max<uint64_t>(1, ceil_div(block, part));   // drop channels that would be empty
  // direct steps of a broadcast: every rank writes its recv buffer only and the next one reads it there
  // (measured break-even points: the rings at direct_min_bytes, a reduce-scatter at twice that, the chains at a quarter)
  const bool bc_direct = kind == DFX_BROADCAST && R > 1 && !fold && cfg.direct && count * eb >= cfg.direct_min_bytes / 4;
  uint64_t slice_cap = cfg.slot_bytes;
  if (rooted && R > 1 && !fold) {
    // A chain's last rank starts R-1 slices after its first, so a chain wants shorter slices than a
    // ring, where all ranks start at once: measured best (R = 8, 2 - 256 MiB) are about 2R slices per
    // channel share for the broadcast and 4R for the reduce, of no less than 32 KiB; the reduce, whose
    // every hop goes through a slot, gains nothing beyond 64 KiB, while the direct broadcast uses no
    // slots and may take slices of twice the slot size.
    const uint64_t lo = std::min<uint64_t>(32u << 10, cfg.slot_bytes);
    const uint64_t hi = kind == DFX_BROADCAST ? (bc_direct ? std::min<uint64_t>(2ull * cfg.slot_bytes, 1ull << 30) : cfg.slot_bytes)
                                              : std::min<uint64_t>(64u << 10, cfg.slot_bytes);
    const uint64_t want = round_up(part * eb / ((kind == DFX_BROADCAST ? 2 : 4) * R), 16);
    slice_cap = std::min(std::max(want, lo), hi);
  }
  // fold steps: no slots; slices of fold_slice_bytes, or (0) one slice, the whole channel share
  if (fold) slice_cap = cfg.fold_slice_bytes ? cfg.fold_slice_bytes : (1ull << 31);
  uint64_t slot_bytes = std::min<uint64_t>(slice_cap, round_up(part * eb, 16));
  const uint64_t slice_elems = slot_bytes / eb;
  const uint64_t rounds = std::max<uint64_t>(1, ceil_div(part, slice_elems));
  if (rounds > 0xfffffffeull) return DFX_ERR_INVALID_ARG;
  const uint64_t K = cfg.nslots;
  // (a direct broadcast fills no slot: its connectors are the flag lines alone)
  // (a collective in fold steps has none either: R x C lines with the published addresses and C shared lines of counters)
  *conn_bytes_out = fold ? round_up((R + 1) * C * DFX_FLAG_STRIDE, 256)
                         : round_up(R * C * DFX_FLAG_STRIDE + (bc_direct ? 0 : R * C * K * slot_bytes), 256);

  DfxStatic t;
  memset(&t, 0, sizeof(t));
  t.coll_id = (uint32_t)coll_id;
  t.count = count;
  t.conn_off = conn_off;
  t.block_elems = block;
  t.part_elems = part;
  t.slice_elems = (uint32_t)slice_elems;
  t.rounds = (uint32_t)rounds;
  t.slot_bytes = (uint32_t)slot_bytes;
  t.nslots = (uint16_t)K;
  t.nchan = (uint16_t)C;
  t.kind = (uint8_t)kind; t.dtype = (uint8_t)dtype; t.op = (uint8_t)op; t.root = (uint8_t)(rooted ? root : 0);
  t.priority = (int16_t)priority;
  if (R == 1) t.nprim = 1;
  else if (fold) {
    t.flags |= DFX_SQE_DIRECT | DFX_SQE_FOLD;   // (buffers are published as for the direct steps)
    t.nprim = fold_nprim((int)kind);            // one step with data and the last wait
  }
  else if (kind == DFX_ALLREDUCE) {
    // direct gather steps (one more step: the drain) where the message is long enough to gain from them
    const bool direct = cfg.direct && count * eb >= cfg.direct_min_bytes;
    if (direct) t.flags |= DFX_SQE_DIRECT;
    t.nprim = (uint32_t)(2 * R - 1) + (direct ? 1u : 0u);
  }
  else if (rooted) {
    t.nprim = 1;   // one primitive per slice, which one depends on the place in the chain
    // the reduce chain's direct step: the first rank only notifies, the second reads its send buffer
    const bool rd_direct = kind == DFX_REDUCE && cfg.direct && count * eb >= cfg.direct_min_bytes / 4;
    if (bc_direct || rd_direct) {
      // one round more than there are slices, which is the drain
      t.flags |= DFX_SQE_DIRECT;
      t.rounds = (uint32_t)rounds + 1u;
    }
  }
  else if (kind == DFX_ALLGATHER && cfg.direct && count * eb * R >= cfg.direct_min_bytes && (count * eb) % 16 == 0) {
    // direct gather steps need every block 16-byte aligned in the recv buffers
    t.flags |= DFX_SQE_DIRECT;
    t.nprim = (uint32_t)R + 1u;
  }
  else if (kind == DFX_REDUCESCATTER && cfg.direct && count * eb * R >= 2ull * cfg.direct_min_bytes && (count * eb) % 16 == 0) {
    // the opening send only notifies and the next rank reads the block from the send buffer, where
    // every block then has to be 16-byte aligned; one more step, the drain
    t.flags |= DFX_SQE_DIRECT;
    t.nprim = (uint32_t)R + 1u;
  }
  else t.nprim = (uint32_t)R;
  *out = t;
  return DFX_OK;
}

inline void backoff(uint32_t& spins) {
  ++spins;
  if (spins < 2000) _mm_pause();
  else std::this_thread::yield();
}

}  // namespace

extern "C" {

int dfx_config_default(dfx_config* cfg) {
  if (!cfg) return DFX_ERR_INVALID_ARG;
  memset(cfg, 0, sizeof(*cfg));
  cfg->struct_bytes = (uint32_t)sizeof(dfx_config);
  cfg->max_channels = 32;
  cfg->max_colls = 2048;
  cfg->sq_depth = 1024;
  cfg->cq_slots = 256;
  cfg->nslots = 4;
  cfg->slot_bytes = 256u << 10;
  cfg->chan_min_bytes = 16u << 10;
  cfg->spin_init = 16;
  cfg->spin_min = 1;
  cfg->spin_max = 64;
  cfg->spin_boost = 2;
  cfg->fetch_batch = 0;
  cfg->scan_min = 3;
  cfg->chan_spread = 1;
  cfg->cq_mode = 0;
  cfg->sq_eager = 1;
  cfg->window = 2;
  cfg->focus_bytes = 128u << 10;
  cfg->direct = 1;
  cfg->direct_min_bytes = 2u << 20;
  cfg->fold_max_bytes = 64u << 20;
  cfg->preempt = 1;
  cfg->watchdog_ms = 10000;
  cfg->quit_idle_us = 2000;
  cfg->sq_in_device = 2;
  cfg->wg_map = 0;
  cfg->order_policy = 0;
  cfg->trace = 0;
  cfg->pool_bytes = 4ull << 30;
  return DFX_OK;
}

int dfx_init(dfx_ctx** out, int nranks, const dfx_config* ucfg, void* hip_stream) {
  if (!out) return DFX_ERR_INVALID_ARG;
  *out = nullptr;
  dfx_config cfg;
  dfx_config_default(&cfg);
  if (ucfg) {
    if (ucfg->struct_bytes != sizeof(dfx_config)) return DFX_ERR_INVALID_ARG;
    cfg = *ucfg;
  }
  if (nranks < 1 || nranks > 64) return DFX_ERR_INVALID_ARG;
  if (cfg.max_channels < 1 || cfg.max_channels > 1024) return DFX_ERR_INVALID_ARG;
  if (cfg.max_colls < 1 || cfg.max_colls > DFX_MAX_COLLS) return DFX_ERR_INVALID_ARG;
  if (!is_pow2(cfg.sq_depth) || cfg.sq_depth < 2) return DFX_ERR_INVALID_ARG;
  if (cfg.cq_slots < 1 || cfg.cq_mode > 2) return DFX_ERR_INVALID_ARG;
  if (cfg.window != 1 && cfg.window != 2 && cfg.window != 4) return DFX_ERR_INVALID_ARG;
  // A ring of fused recv+send primitives that has sent `window` slices ahead on every edge needs one
  // more free slot to take its next step: with window >= nslots every connector fills and nobody can move.
  if (!is_pow2(cfg.nslots) || cfg.nslots < 2 || cfg.nslots > 64) return DFX_ERR_INVALID_ARG;
  while (cfg.window >= cfg.nslots) cfg.window /= 2;
  if (cfg.slot_bytes < 16 || (cfg.slot_bytes & 15u)) return DFX_ERR_INVALID_ARG;
  if ((cfg.fold_slice_bytes & 15u) || cfg.reserved0) return DFX_ERR_INVALID_ARG;
  if (cfg.chan_min_bytes < 16) return DFX_ERR_INVALID_ARG;
  if (cfg.spin_min < 1 || cfg.spin_init < 1 || cfg.spin_boost < 1 || cfg.spin_max < cfg.spin_min) return DFX_ERR_INVALID_ARG;
  if (cfg.sq_in_device > 2 || cfg.wg_map > 1 || cfg.order_policy > 1 || cfg.direct > 1) return DFX_ERR_INVALID_ARG;
  if (cfg.pool_bytes < (1u << 20)) return DFX_ERR_INVALID_ARG;

  dfx_ctx* c = new (std::nothrow) dfx_ctx();
  if (!c) return DFX_ERR_NO_RESOURCES;
  c->cfg = cfg;
  if (const char* e = getenv("DFX_FIFO_FENCED")) c->fifo_coherent = (e[0] == '1') ? 0u : 1u;   // comparison switch
  c->R = nranks;
  c->nwg = (uint32_t)nranks * cfg.max_channels;
  while ((1u << c->sq_shift) < cfg.sq_depth) c->sq_shift++;

#define INITCHK(call)                                      \
  do {                                                     \
    hipError_t e_ = (call);                                \
    if (e_ != hipSuccess) { g_init_hip_error = (int)e_; free_all(c); return DFX_ERR_HIP; } \
  } while (0)

  INITCHK(hipGetDevice(&c->device));
  // co-residency: every workgroup spins on flags written by others, so the whole grid must fit
  int occ = 0, ncu = 0, wall_khz = 0, large_bar = 0;
  INITCHK(dfx_daemon_occupancy(&occ));
  INITCHK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, c->device));
  // A workgroup whose wavefront count is not a multiple of the four SIMDs of a compute unit loads them
  // unevenly, and which SIMD gets the extra wavefront is the dispatcher's choice: two such
  // workgroups may not fit one compute unit even when the register arithmetic says they do.
  // Count one per compute unit then.
  if (((DFX_WG_THREADS / 64) & 3) != 0 && occ > 1) occ = 1;
  if (occ < 1 || (uint64_t)c->nwg > (uint64_t)occ * (uint64_t)ncu) { free_all(c); return DFX_ERR_NO_RESOURCES; }
  if (hipDeviceGetAttribute(&wall_khz, hipDeviceAttributeWallClockRate, c->device) == hipSuccess && wall_khz > 0)
    c->tick_us = 1000.0 / (double)wall_khz;
  (void)hipDeviceGetAttribute(&large_bar, hipDeviceAttributeIsLargeBar, c->device);
  c->sq_device = (cfg.sq_in_device == 1) || (cfg.sq_in_device == 2 && large_bar);
  if (cfg.sq_in_device == 1 && !large_bar) { free_all(c); return DFX_ERR_NO_RESOURCES; }

  if (hip_stream) c->stream = (hipStream_t)hip_stream;
  else { INITCHK(hipStreamCreateWithFlags(&c->stream, hipStreamNonBlocking)); c->own_stream = true; }
  INITCHK(hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking));
  INITCHK(hipEventCreate(&c->ev_start));
  INITCHK(hipEventCreate(&c->ev_stop));

  const size_t R = (size_t)nranks;
  const size_t sq_bytes = R * cfg.sq_depth * sizeof(DfxSqSlot) + HC_N * sizeof(uint32_t) + 256;
  const size_t cq_slots_bytes = round_up(R * cfg.cq_slots * sizeof(uint64_t), 64);
  const size_t cq_ctl_bytes = round_up(R * DFX_CQ_CTL_WORDS * sizeof(uint64_t), 64);
  const size_t cq_bytes = cq_slots_bytes + cq_ctl_bytes + R * cfg.sq_depth * sizeof(uint32_t);
  if (c->sq_device) {
    c->qmem_sq_bytes = sq_bytes;
    c->qmem_sq = take_parked_sq(c->device, sq_bytes);
    if (!c->qmem_sq) INITCHK(hipExtMallocWithFlags(&c->qmem_sq, sq_bytes, hipDeviceMallocFinegrained));
    INITCHK(hipMemset(c->qmem_sq, 0, sq_bytes));
  } else {
    INITCHK(hipHostMalloc(&c->qmem_sq, sq_bytes, hipHostMallocMapped | hipHostMallocCoherent));
    memset(c->qmem_sq, 0, sq_bytes);
  }
  INITCHK(hipHostMalloc(&c->qmem_cq, cq_bytes, hipHostMallocMapped | hipHostMallocCoherent));
  memset(c->qmem_cq, 0, cq_bytes);
  c->sq = (DfxSqSlot*)c->qmem_sq;
  c->host_ctl = (uint32_t*)((char*)c->qmem_sq + round_up(R * cfg.sq_depth * sizeof(DfxSqSlot), 256));
  c->cq = (uint64_t*)c->qmem_cq;
  c->cq_ctl = (uint64_t*)((char*)c->qmem_cq + cq_slots_bytes);
  c->sq_freed = (uint32_t*)((char*)c->qmem_cq + cq_slots_bytes + cq_ctl_bytes);

  auto dalloc = [&](void** p, size_t bytes) -> hipError_t {
    hipError_t e = hipMalloc(p, bytes);
    if (e != hipSuccess) return e;
    return hipMemset(*p, 0, bytes);
  };
  INITCHK(dalloc((void**)&c->sq_readers, R * cfg.sq_depth * sizeof(uint32_t)));
  INITCHK(dalloc((void**)&c->done_cnt, R * cfg.max_colls * sizeof(uint32_t)));
  INITCHK(dalloc((void**)&c->dev_ctl, DC_N * sizeof(uint32_t)));
  INITCHK(dalloc((void**)&c->pool, cfg.pool_bytes));
  INITCHK(dalloc((void**)&c->ctxbuf, (size_t)c->nwg * cfg.max_colls * sizeof(DfxCtxEntry)));
  INITCHK(dalloc((void**)&c->wgstate, (size_t)c->nwg * sizeof(DfxWgState)));
  INITCHK(dalloc((void**)&c->taskq_store, (size_t)c->nwg * cfg.max_colls * sizeof(uint16_t)));
  if (cfg.trace) INITCHK(dalloc((void**)&c->trace, (size_t)c->nwg * DFX_TRACE_N * sizeof(uint64_t)));
  c->pinned_tmp_bytes = std::max((size_t)c->nwg * sizeof(DfxWgState), (size_t)DFX_TRACE_N * sizeof(uint64_t) * 64);
  INITCHK(hipHostMalloc(&c->pinned_tmp, c->pinned_tmp_bytes, hipHostMallocDefault));
  INITCHK(hipDeviceSynchronize());
#undef INITCHK

  c->colls.resize(cfg.max_colls);
  for (int r = 0; r < nranks; ++r) {
    RankState* rs = new RankState();
    rs->sub.assign(cfg.max_colls, 0);
    rs->done.assign(cfg.max_colls, 0);
    c->ranks.push_back(rs);
  }
  *out = c;
  return DFX_OK;
}

int dfx_prepare(dfx_ctx* c, int coll_id, dfx_kind kind, size_t count, dfx_dtype dtype, dfx_op op, int root, int priority) {
  if (!c) return DFX_ERR_INVALID_ARG;
  if (coll_id < 0 || (uint32_t)coll_id >= c->cfg.max_colls) return DFX_ERR_INVALID_ARG;
  CollInfo& ci = c->colls[coll_id];
  if (ci.prepared) return DFX_ERR_INVALID_ARG;
  DfxStatic t;
  uint64_t conn_bytes = 0;
  const int rc = plan_collective(c->cfg, c->R, coll_id, kind, count, dtype, op, root, priority, c->pool_used, &t, &conn_bytes);
  if (rc != DFX_OK) return rc;
  if (c->pool_used + conn_bytes > c->cfg.pool_bytes) return DFX_ERR_NO_RESOURCES;
  c->pool_used += conn_bytes;
  ci.tmpl = t;
  ci.prepared = true;
  return DFX_OK;
}

int dfx_coll_info(dfx_ctx* c, int coll_id, uint32_t* nchan, uint32_t* slot_bytes, uint32_t* rounds, uint32_t* nprim) {
  if (!c || coll_id < 0 || (uint32_t)coll_id >= c->cfg.max_colls) return DFX_ERR_INVALID_ARG;
  const CollInfo& ci = c->colls[coll_id];
  if (!ci.prepared) return DFX_ERR_NOT_PREPARED;
  if (nchan) *nchan = ci.tmpl.nchan;
  if (slot_bytes) *slot_bytes = ci.tmpl.slot_bytes;
  if (rounds) *rounds = ci.tmpl.rounds;
  if (nprim) *nprim = ci.tmpl.nprim;
  return DFX_OK;
}

}  // extern "C"

namespace {

// The body of one invocation's SQE, `ahead` entries behind the tail (the caller holds the rank's mutex and
// publishes afterwards).  Counts the invocation as submitted, so that the same id again in one run is BUSY.
int stage_one(dfx_ctx* c, int rank, uint32_t ahead, int coll_id, const void* sendbuf, void* recvbuf) {
  if (coll_id < 0 || (uint32_t)coll_id >= c->cfg.max_colls) return DFX_ERR_INVALID_ARG;
  if (c->aborted.load()) return DFX_ERR_ABORTED;
  const CollInfo& ci = c->colls[coll_id];
  if (!ci.prepared) return DFX_ERR_NOT_PREPARED;
  if (!sendbuf || !recvbuf || ((uintptr_t)sendbuf & 15u) || ((uintptr_t)recvbuf & 15u)) return DFX_ERR_INVALID_ARG;
  RankState* rs = c->ranks[rank];
  if (rs->sub[coll_id] != rs->done[coll_id]) {
    drain_cq(c, rank);
    if (rs->sub[coll_id] != rs->done[coll_id]) return DFX_ERR_BUSY;
  }
  if (!sqe_slot_free(c, rank, ahead)) return DFX_ERR_SQ_FULL;
  DfxStatic e = ci.tmpl;
  e.seq = rs->sub[coll_id];
  e.sendbuf = (uint64_t)(uintptr_t)sendbuf;
  e.recvbuf = (uint64_t)(uintptr_t)recvbuf;
  sqe_write_body(c, rank, ahead, e);
  rs->sub[coll_id]++;
  return DFX_OK;
}

// Up to 32 invocations of one rank in a row: bodies, one fence, generation words, one fence.  Returns how many
// went in; *rc is the status of the first that did not (DFX_OK if all did).  The caller sees to it that the
// daemon runs.
int submit_run(dfx_ctx* c, int rank, int n, const int* coll_ids, const void* const* sendbufs, void* const* recvbufs, int* rc) {
  RankState* rs = c->ranks[rank];
  std::lock_guard<std::mutex> lk(rs->mu);
  int k = 0;
  *rc = DFX_OK;
  for (; k < n && k < 32; ++k) {
    *rc = stage_one(c, rank, (uint32_t)k, coll_ids[k], sendbufs[k], recvbufs[k]);
    if (*rc != DFX_OK) break;
  }
  if (k) {
    sqe_fence();
    sqe_publish(c, rank, (uint32_t)k);
    _mm_sfence();
    rs->n_sub.fetch_add((uint64_t)k, std::memory_order_relaxed);
  }
  // A caller that only retries submissions must still empty the CQ, or a workgroup blocked
  // on a full CQ stops reading SQEs and the SQ never drains.
  if (*rc == DFX_ERR_SQ_FULL) drain_cq(c, rank);
  return k;
}

// Write the SQE of one invocation; the caller sees to it that the daemon runs.
int submit_one(dfx_ctx* c, int rank, int coll_id, const void* sendbuf, void* recvbuf) {
  int rc = DFX_OK;
  (void)submit_run(c, rank, 1, &coll_id, &sendbuf, &recvbuf, &rc);
  return rc;
}

}  // namespace

extern "C" {

int dfx_submit(dfx_ctx* c, int rank, int coll_id, const void* sendbuf, void* recvbuf) {
  if (!c || rank < 0 || rank >= c->R) return DFX_ERR_INVALID_ARG;
  const int rc = submit_one(c, rank, coll_id, sendbuf, recvbuf);
  if (rc != DFX_OK && rc != DFX_ERR_SQ_FULL) return rc;
  // start the daemon on SQE insertion; also when the SQ is full (a quit daemon frees no slots)
  c->user_stopped.store(false);
  int rr = ensure_running(c);
  if (rr != DFX_OK) return rr;
  return rc;
}

int dfx_submit_all(dfx_ctx* c, int coll_id, const void* const* sendbufs, void* const* recvbufs, uint64_t timeout_ns) {
  if (!c || !sendbufs || !recvbufs) return DFX_ERR_INVALID_ARG;
  const uint64_t t0 = now_ns();
  c->user_stopped.store(false);
  uint32_t spins = 0;
  for (;;) {
    // every vrank's body, one fence, every vrank's generation word, one fence: the eight entries reach the
    // device together (rank mutexes are taken in rank order; every other path holds one at a time)
    int rc = DFX_OK, staged = 0;
    for (; staged < c->R; ++staged) {
      c->ranks[staged]->mu.lock();
      rc = stage_one(c, staged, 0u, coll_id, sendbufs[staged], recvbufs[staged]);
      if (rc != DFX_OK) { c->ranks[staged]->mu.unlock(); break; }
    }
    if (rc == DFX_OK) {
      sqe_fence();
      for (int r = 0; r < c->R; ++r) sqe_publish(c, r, 1);
      _mm_sfence();
      for (int r = 0; r < c->R; ++r) { c->ranks[r]->n_sub.fetch_add(1, std::memory_order_relaxed); c->ranks[r]->mu.unlock(); }
      break;
    }
    // one vrank could not take it: nothing has been published, the staged ones are taken back
    for (int r = 0; r < staged; ++r) { c->ranks[r]->sub[coll_id]--; c->ranks[r]->mu.unlock(); }
    if (rc != DFX_ERR_SQ_FULL) return rc;
    { std::lock_guard<std::mutex> lk(c->ranks[staged]->mu); drain_cq(c, staged); }
    const int rr = ensure_running(c);
    if (rr != DFX_OK) return rr;
    if (now_ns() - t0 > timeout_ns) return DFX_ERR_SQ_FULL;
    backoff(spins);
  }
  // every vrank's entry is in place: now see to the daemon (a launch finds them all at once)
  return ensure_running(c);
}

int dfx_submit_many_paced(dfx_ctx* c, int rank, int n, const int* coll_ids, const void* const* sendbufs,
                          void* const* recvbufs, const uint64_t* delays_ns, uint64_t timeout_ns) {
  if (!c || rank < 0 || rank >= c->R || n < 0 || (n > 0 && (!coll_ids || !sendbufs || !recvbufs))) return DFX_ERR_INVALID_ARG;
  const uint64_t t0 = now_ns();
  uint32_t spins = 0;
  int i = 0, since_check = -1;       // (-1: the daemon has not been looked after yet)
  bool paused = false;
  c->user_stopped.store(false);
  // Entries without a pause between them go in runs of up to 32 (two store fences per run, not per entry).
  // The daemon is looked after (launch state behind one lock, an event query) after the first run, then
  // every 32 entries, after every pause, whenever the SQ is full, and after the last entry -- not per entry.
  while (i < n) {
    if (delays_ns && delays_ns[i] && !paused) {
      const uint64_t until = now_ns() + delays_ns[i];
      while (now_ns() < until) _mm_pause();
      paused = true;
      since_check = -1;
    }
    int run = 1;
    while (i + run < n && run < 32 && !(delays_ns && delays_ns[i + run])) ++run;
    int rc = DFX_OK;
    const int k = submit_run(c, rank, run, coll_ids + i, sendbufs + i, recvbufs + i, &rc);
    if (k > 0) {
      i += k; spins = 0; paused = false;
      if (since_check < 0 || (since_check += k) >= 32 || i == n) {
        const int rr = ensure_running(c);
        if (rr != DFX_OK) return rr;
        since_check = 0;
      }
    }
    if (rc == DFX_OK) continue;
    if (rc != DFX_ERR_SQ_FULL) return i > 0 ? i : rc;
    const int rr = ensure_running(c);
    if (rr != DFX_OK) return i > 0 ? i : rr;
    if (now_ns() - t0 > timeout_ns) return i;
    backoff(spins);
  }
  return i;
}

int dfx_submit_many(dfx_ctx* c, int rank, int n, const int* coll_ids, const void* const* sendbufs,
                    void* const* recvbufs, uint64_t timeout_ns) {
  return dfx_submit_many_paced(c, rank, n, coll_ids, sendbufs, recvbufs, nullptr, timeout_ns);
}

int dfx_poll(dfx_ctx* c, int rank, dfx_cqe* out, int max) {
  if (!c || rank < 0 || rank >= c->R || (max > 0 && !out) || max < 0) return DFX_ERR_INVALID_ARG;
  RankState* rs = c->ranks[rank];
  int n = 0;
  {
    std::lock_guard<std::mutex> lk(rs->mu);
    drain_cq(c, rank);
    while (n < max && !rs->ready.empty()) { out[n++] = rs->ready.front(); rs->ready.pop_front(); }
  }
  if (outstanding(c)) {
    int rr = ensure_running(c);
    if (rr != DFX_OK && n == 0) return rr == DFX_ERR_ABORTED ? DFX_ERR_TIMEOUT : rr;
  }
  return n;
}

int dfx_wait(dfx_ctx* c, int rank, int coll_id, uint64_t timeout_ns) {
  if (!c || rank < 0 || rank >= c->R) return DFX_ERR_INVALID_ARG;
  if (coll_id < 0 || (uint32_t)coll_id >= c->cfg.max_colls) return DFX_ERR_INVALID_ARG;
  RankState* rs = c->ranks[rank];
  const uint64_t t0 = now_ns();
  uint32_t spins = 0;
  for (;;) {
    {
      std::lock_guard<std::mutex> lk(rs->mu);
      drain_cq(c, rank);
      if (rs->sub[coll_id] == rs->done[coll_id]) {
        if (!c->cb)   // with a callback set the completion belongs to the poller thread
          for (auto it = rs->ready.begin(); it != rs->ready.end(); ++it)
            if (it->coll_id == (uint32_t)coll_id) { rs->ready.erase(it); break; }
        return DFX_OK;
      }
    }
    if ((spins & 63u) == 0) {
      int rr = ensure_running(c);
      if (rr == DFX_ERR_ABORTED) return DFX_ERR_TIMEOUT;
      if (rr != DFX_OK) return rr;
      if (now_ns() - t0 > timeout_ns) return DFX_ERR_TIMEOUT;
    }
    backoff(spins);
  }
}

int dfx_wait_all(dfx_ctx* c, uint64_t timeout_ns) {
  if (!c) return DFX_ERR_INVALID_ARG;
  const uint64_t t0 = now_ns();
  uint32_t spins = 0;
  for (;;) {
    bool all = true;
    for (int r = 0; r < c->R; ++r) {
      RankState* rs = c->ranks[r];
      std::lock_guard<std::mutex> lk(rs->mu);
      drain_cq(c, r);
      if (rs->n_cqe.load() < rs->n_sub.load()) all = false;
      else if (!c->cb) rs->ready.clear();
    }
    if (all) return DFX_OK;
    if ((spins & 63u) == 0) {
      int rr = ensure_running(c);
      if (rr == DFX_ERR_ABORTED) return DFX_ERR_TIMEOUT;
      if (rr != DFX_OK) return rr;
      if (now_ns() - t0 > timeout_ns) return DFX_ERR_TIMEOUT;
    }
    backoff(spins);
  }
}

int dfx_start(dfx_ctx* c) {
  if (!c) return DFX_ERR_INVALID_ARG;
  c->user_stopped.store(false);
  return ensure_running(c);
}

int dfx_stop(dfx_ctx* c) {
  if (!c) return DFX_ERR_INVALID_ARG;
  c->user_stopped.store(true);
  {
    std::lock_guard<std::mutex> lk(c->launch_mu);
    bool idle = false;
    int rc = reap_locked(c, &idle);
    if (rc != DFX_OK) return rc;
    if (idle) return DFX_OK;
  }
  // exiting SQE to every rank (Sec. 4.4); a full SQ is retried while the daemon drains it
  const uint64_t t0 = now_ns();
  bool forced = false;
  for (int r = 0; r < c->R && !forced; ++r) {
    DfxStatic e;
    memset(&e, 0, sizeof(e));
    e.flags = DFX_SQE_EXIT;
    e.seq = (uint32_t)c->launches;   // the launch in flight
    e.coll_id = 0xffffffffu;
    for (;;) {
      int rc;
      { std::lock_guard<std::mutex> lk(c->ranks[r]->mu); rc = push_sqe(c, r, e); }
      if (rc == DFX_OK) break;
      if (hipEventQuery(c->ev_stop) != hipErrorNotReady) break;      // daemon already gone
      if (now_ns() - t0 > 2000000000ull) { forced = true; break; }
      std::this_thread::yield();
    }
  }
  // wait for the grid to drain; if it does not (e.g. non-preemptive waits), raise the abort word
  for (;;) {
    hipError_t q = hipEventQuery(c->ev_stop);
    if (q != hipErrorNotReady) break;
    if (!forced && now_ns() - t0 > 3000000000ull) forced = true;
    if (forced) {
      *(volatile uint32_t*)&c->host_ctl[HC_ABORT] = 1;
      _mm_sfence();
      c->aborted.store(true);
    }
    std::this_thread::yield();
  }
  std::lock_guard<std::mutex> lk(c->launch_mu);
  bool idle = false;
  int rc = reap_locked(c, &idle);
  if (rc != DFX_OK) return rc;
  return forced ? DFX_ERR_ABORTED : DFX_OK;
}

int dfx_stats(dfx_ctx* c, int rank, dfx_stats_t* out) {
  if (!c || rank < 0 || rank >= c->R || !out) return DFX_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lk(c->launch_mu);
  memset(out, 0, sizeof(*out));
  DfxWgState* h = (DfxWgState*)c->pinned_tmp;
  HIPCHK(c, hipMemcpyAsync(h, c->wgstate, (size_t)c->nwg * sizeof(DfxWgState), hipMemcpyDeviceToHost, c->side));
  HIPCHK(c, hipStreamSynchronize(c->side));
  std::vector<uint32_t> wgs;
  std::vector<uint32_t> tn;
  uint64_t stamp_ticks = 0, stamp_n = 0;
  for (uint32_t wg = 0; wg < c->nwg; ++wg) {
    uint32_t r = c->cfg.wg_map == 0 ? wg % (uint32_t)c->R : wg / c->cfg.max_channels;
    if ((int)r != rank) continue;
    const uint64_t* s = h[wg].stat;
    out->preemptions += s[ST_PREEMPT]; out->ctx_loads += s[ST_LOAD]; out->ctx_slot_hits += s[ST_HIT];
    out->ctx_saves += s[ST_SAVE]; out->lazy_skips += s[ST_LAZY]; out->polls += s[ST_POLLS]; out->prims += s[ST_PRIMS];
    out->sqe_fetched += s[ST_SQE]; out->cqe_posted += s[ST_CQE]; out->passes += s[ST_PASSES]; out->quits += s[ST_QUITS];
    out->max_taskq = std::max<uint64_t>(out->max_taskq, s[ST_MAXQ]);
    out->wait_us += (double)s[ST_T_WAIT] * c->tick_us; out->data_us += (double)s[ST_T_DATA] * c->tick_us;
    out->publish_us += (double)s[ST_T_PUB] * c->tick_us;
    out->scan_skips += s[ST_SCAN_SKIPS];
    out->cqe_us += (double)s[ST_T_CQE] * c->tick_us;
    out->sqe_us += (double)s[ST_T_SQE] * c->tick_us;
    stamp_ticks += s[ST_T_STAMP]; stamp_n += s[ST_N_STAMP];
    wgs.push_back(wg);
    tn.push_back(h[wg].trace_n);
  }
  out->launches = c->launches;
  if (stamp_n) out->clock_read_us = (double)stamp_ticks * c->tick_us / (double)stamp_n;
  if (c->trace && c->cfg.trace < 3) {
    std::vector<double> tot;
    double sv = 0, ld = 0, adv = 0, su = 0;
    uint64_t* buf = (uint64_t*)c->pinned_tmp;
    for (size_t i = 0; i < wgs.size(); ++i) {
      const uint32_t n = std::min<uint32_t>(tn[i], DFX_TRACE_N);
      if (!n) continue;
      HIPCHK(c, hipMemcpyAsync(buf, c->trace + (size_t)wgs[i] * DFX_TRACE_N, (size_t)n * 8, hipMemcpyDeviceToHost, c->side));
      HIPCHK(c, hipStreamSynchronize(c->side));
      for (uint32_t k = 0; k < n; ++k) {
        const uint64_t v = buf[k];
        tot.push_back((double)(v & 0xffffu) * c->tick_us);
        sv += (double)((v >> 16) & 0xfffu) * c->tick_us;
        adv += (double)((v >> 28) & 0xfffu) * c->tick_us;
        ld += (double)((v >> 40) & 0xfffu) * c->tick_us;
        su += (double)((v >> 52) & 0xfffu) * c->tick_us;
      }
    }
    if (!tot.empty()) {
      std::sort(tot.begin(), tot.end());
      double sum = 0;
      for (double x : tot) sum += x;
      out->switch_samples = tot.size();
      out->switch_us_p50 = tot[tot.size() / 2];
      out->switch_us_p99 = tot[std::min(tot.size() - 1, (size_t)((double)tot.size() * 0.99))];
      out->switch_us_mean = sum / (double)tot.size();
      out->save_us_mean = sv / (double)tot.size();
      out->load_us_mean = ld / (double)tot.size();
      out->advance_us_mean = adv / (double)tot.size();
      out->setup_us_mean = su / (double)tot.size();
    }
  }
  return DFX_OK;
}

int dfx_trace_read(dfx_ctx* c, uint32_t wg, uint64_t* out, uint32_t max, double* tick_us) {
  if (!c || !out || wg >= c->nwg) return DFX_ERR_INVALID_ARG;
  if (!c->trace) return 0;
  std::lock_guard<std::mutex> lk(c->launch_mu);
  DfxWgState* h = (DfxWgState*)c->pinned_tmp;
  HIPCHK(c, hipMemcpyAsync(h, c->wgstate + wg, sizeof(DfxWgState), hipMemcpyDeviceToHost, c->side));
  HIPCHK(c, hipStreamSynchronize(c->side));
  const uint32_t n = std::min<uint32_t>(std::min<uint32_t>(h->trace_n, DFX_TRACE_N), max);
  if (tick_us) *tick_us = c->tick_us;
  if (!n) return 0;
  uint64_t* buf = (uint64_t*)c->pinned_tmp;
  HIPCHK(c, hipMemcpyAsync(buf, c->trace + (size_t)wg * DFX_TRACE_N, (size_t)n * 8, hipMemcpyDeviceToHost, c->side));
  HIPCHK(c, hipStreamSynchronize(c->side));
  memcpy(out, buf, (size_t)n * 8);
  return (int)n;
}

int dfx_last_launch_ms(dfx_ctx* c, float* ms, uint64_t* launches_done) {
  if (!c) return DFX_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lk(c->launch_mu);
  bool idle = false;
  int rc = reap_locked(c, &idle);
  if (rc != DFX_OK) return rc;
  if (ms) *ms = c->last_ms;
  if (launches_done) *launches_done = c->launches_done;
  return DFX_OK;
}

int dfx_set_callback(dfx_ctx* c, dfx_callback fn, void* user) {
  if (!c) return DFX_ERR_INVALID_ARG;
  if (c->poller.joinable()) {
    c->poller_run.store(false);
    c->poller.join();
  }
  c->cb = fn;
  c->cb_user = user;
  if (!fn) return DFX_OK;
  c->poller_run.store(true);
  c->poller = std::thread([c]() {
    std::vector<dfx_cqe> got;
    uint32_t idle = 0;
    while (c->poller_run.load(std::memory_order_relaxed)) {
      bool any = false;
      for (int r = 0; r < c->R; ++r) {
        got.clear();
        {
          RankState* rs = c->ranks[r];
          std::lock_guard<std::mutex> lk(rs->mu);
          drain_cq(c, r);
          got.assign(rs->ready.begin(), rs->ready.end());
          rs->ready.clear();
        }
        for (const dfx_cqe& e : got) c->cb(c->cb_user, r, e.coll_id, e.seq);
        any = any || !got.empty();
      }
      if (any) { idle = 0; continue; }
      // event-driven start (Sec. 4.4) without the caller polling
      if ((++idle & 255u) == 0 && !c->user_stopped.load() && !c->aborted.load() && outstanding(c)) (void)ensure_running(c);
      if (idle < 4096) _mm_pause();
      else std::this_thread::sleep_for(std::chrono::microseconds(50));
    }
  });
  return DFX_OK;
}

int dfx_finalize(dfx_ctx* c) {
  if (!c) return DFX_ERR_INVALID_ARG;
  (void)dfx_set_callback(c, nullptr, nullptr);
  int rc = dfx_stop(c);
  bool pending = false;
  for (int r = 0; r < c->R; ++r) {
    std::lock_guard<std::mutex> lk(c->ranks[r]->mu);
    drain_cq(c, r);
    if (c->ranks[r]->n_cqe.load() < c->ranks[r]->n_sub.load()) pending = true;
  }
  (void)hipStreamSynchronize(c->stream);
  release_slot(c);
  free_all(c);
  if (rc == DFX_ERR_HIP) return rc;
  return (pending || rc == DFX_ERR_ABORTED) ? DFX_ERR_ABORTED : DFX_OK;
}

int dfx_last_hip_error(dfx_ctx* c) { return c ? c->last_hip : 0; }

int dfx_last_init_error(void) { return g_init_hip_error; }

#ifndef DFX_BUILD_ID_STR
#define DFX_BUILD_ID_STR "unknown"
#endif
const char* dfx_build_id(void) {
  static const char id[] = "DFX_BUILD_ID=" DFX_BUILD_ID_STR;
  return id + 13;
}

const char* dfx_strerror(int s) {
  switch (s) {
    case DFX_OK: return "ok";
    case DFX_ERR_INVALID_ARG: return "invalid argument";
    case DFX_ERR_NOT_PREPARED: return "collective not prepared";
    case DFX_ERR_BUSY: return "collective already outstanding on this rank";
    case DFX_ERR_SQ_FULL: return "submission queue full (retry)";
    case DFX_ERR_TIMEOUT: return "timeout";
    case DFX_ERR_HIP: return "HIP runtime error";
    case DFX_ERR_NO_RESOURCES: return "not enough resources";
    case DFX_ERR_ABORTED: return "daemon aborted";
    case DFX_ERR_TOO_LARGE: return "size beyond what the static scratch memory of this entry point is laid out for";
    default: return "unknown status";
  }
}

// ------------------------------------------------------------------------------------------
// Geometry self-check: the kernel's index arithmetic walked on the host, without a GPU
// ------------------------------------------------------------------------------------------
int dfx_check_geometry(int nranks, const dfx_config* ucfg, dfx_kind kind, size_t count, dfx_dtype dtype, dfx_op op, int root,
                       int coll_id, uint32_t wg_map, char* msg, size_t msg_bytes) {
  auto fail = [&](const char* fmt, auto... v) -> int {
    if (msg && msg_bytes) snprintf(msg, msg_bytes, fmt, v...);
    return DFX_ERR_INVALID_ARG;
  };
  if (msg && msg_bytes) msg[0] = 0;
  dfx_config cfg;
  dfx_config_default(&cfg);
  if (ucfg) { if (ucfg->struct_bytes != sizeof(dfx_config)) return fail("%s", "config size"); cfg = *ucfg; }
  if (nranks < 1 || nranks > 64 || coll_id < 0 || (uint32_t)coll_id >= cfg.max_colls || wg_map > 2) return fail("%s", "arguments");
  if (!is_pow2(cfg.nslots) || cfg.nslots < 2 || cfg.nslots > 64) return fail("%s", "nslots");
  while (cfg.window >= cfg.nslots) cfg.window /= 2;
  const uint32_t R = (uint32_t)nranks, cmax = cfg.max_channels, nwg = R * cmax;
  DfxStatic t;
  uint64_t conn_bytes = 0;
  const uint64_t conn_off = 4096;              // some block inside the pool
  int rc = plan_collective(cfg, nranks, coll_id, kind, count, dtype, op, root, 0, conn_off, &t, &conn_bytes);
  if (rc != DFX_OK) return fail("plan_collective: %d", rc);
  const uint32_t eb = elem_bytes(dtype);
  const uint64_t send_bytes = (kind == DFX_REDUCESCATTER ? count * R : count) * eb;
  const uint64_t recv_bytes = (kind == DFX_ALLGATHER ? count * R : count) * eb;
  // made-up addresses, far apart: the pool, and every rank's send and recv buffer
  const uint64_t pool = 0x100000000000ull;
  auto sendbase = [&](uint32_t r) { return 0x200000000000ull + (uint64_t)r * 0x010000000000ull; };
  auto recvbase = [&](uint32_t r) { return 0x300000000000ull + (uint64_t)r * 0x010000000000ull; };
  const uint64_t blk_lo = pool + conn_off, blk_hi = blk_lo + conn_bytes;
  const uint64_t flags_hi = blk_lo + (uint64_t)R * t.nchan * DFX_FLAG_STRIDE;
  const bool direct = (t.flags & DFX_SQE_DIRECT) != 0;
  const bool fold = (t.flags & DFX_SQE_FOLD) != 0;
  const bool no_slots = (direct && kind == DFX_BROADCAST) || fold;

  // (i) the map is a bijection between workgroups and (rank, channel); under the third labelling too
  // (XCD = (rank + channel) mod 8: the ranks of every channel's group of R workgroups rotated by the channel)
  std::vector<int> owner((size_t)R * cmax, -1);
  std::vector<int> serves((size_t)R * t.nchan, -1);
  std::vector<DfxCooked> cooked((size_t)R * t.nchan);
  for (uint32_t wg = 0; wg < nwg; ++wg) {
    WgPlace w = wg_place(wg_map == 2 ? 0u : wg_map, wg, R, cmax);
    if (wg_map == 2) w.rank = (w.rank + w.ch) % R;
    if (w.rank >= R || w.ch >= cmax) return fail("workgroup %u maps to rank %u channel %u", wg, w.rank, w.ch);
    int& o = owner[(size_t)w.rank * cmax + w.ch];
    if (o >= 0) return fail("workgroups %d and %u both map to rank %u channel %u", o, wg, w.rank, w.ch);
    o = (int)wg;
    const uint32_t vch = serving_channel(cfg.chan_spread != 0, w.ch, cmax, (uint32_t)coll_id, t.nchan);
    if (vch >= t.nchan) continue;
    int& sv = serves[(size_t)w.rank * t.nchan + vch];
    if (sv >= 0) return fail("rank %u channel %u of the collective is served by workgroups %d and %u", w.rank, vch, sv, wg);
    sv = (int)wg;
    DfxStatic q = t;
    q.sendbuf = sendbase(w.rank); q.recvbuf = recvbase(w.rank);
    cooked[(size_t)w.rank * t.nchan + vch] = cook_sqe(q, (uint8_t*)(uintptr_t)pool, w.rank, R, vch);
  }
  for (size_t i = 0; i < serves.size(); ++i)
    if (serves[i] < 0) return fail("rank %zu channel %zu of the collective has no workgroup", i / t.nchan, i % t.nchan);

  // (ii) both ends of every connector resolve to the same flag line and the same slots, inside the block
  const uint64_t conn_slot_bytes = (uint64_t)t.nslots * t.slot_bytes;
  for (uint32_t r = 0; r < R; ++r)
    for (uint32_t v = 0; v < t.nchan; ++v) {
      const DfxCooked& me = cooked[(size_t)r * t.nchan + v];
      const DfxCooked& nx = cooked[(size_t)((r + 1) % R) * t.nchan + v];
      if (me.flags_out != nx.flags_in) return fail("edge %u channel %u: sender's flag line %llx, receiver's %llx", r, v, (unsigned long long)me.flags_out, (unsigned long long)nx.flags_in);
      if (me.fifo_out != nx.fifo_in) return fail("edge %u channel %u: sender's slots %llx, receiver's %llx", r, v, (unsigned long long)me.fifo_out, (unsigned long long)nx.fifo_in);
      if (me.flags_out < blk_lo || me.flags_out + DFX_FLAG_STRIDE > flags_hi || (me.flags_out & (DFX_FLAG_STRIDE - 1)))
        return fail("edge %u channel %u: flag line %llx outside the block's flag lines", r, v, (unsigned long long)me.flags_out);
      if (!no_slots && (me.fifo_out < flags_hi || me.fifo_out + conn_slot_bytes > blk_hi))
        return fail("edge %u channel %u: slots %llx outside the block", r, v, (unsigned long long)me.fifo_out);
      if (no_slots && (me.fifo_out || me.fifo_in)) return fail("%s", "a collective without slots has slot addresses");
      if (fold) {
        // every rank of the channel finds the same lines: rank k's from any rank's own line, and the shared one
        const uint64_t sh_line = fold_shared_line(me.flags_out, r, R, t.nchan);
        if (sh_line < flags_hi || sh_line + DFX_FLAG_STRIDE > blk_hi) return fail("rank %u channel %u: shared line %llx outside the block", r, v, (unsigned long long)sh_line);
        if (sh_line != fold_shared_line(nx.flags_out, (r + 1) % R, R, t.nchan)) return fail("ranks %u and %u channel %u disagree on the shared line", r, (r + 1) % R, v);
        for (uint32_t k = 0; k < R; ++k)
          if (fold_line(me.flags_out, r, k, t.nchan) != cooked[(size_t)k * t.nchan + v].flags_out)
            return fail("rank %u channel %u: line of rank %u resolves to %llx", r, v, k, (unsigned long long)fold_line(me.flags_out, r, k, t.nchan));
      }
    }

  // (iii) every job of every workgroup's walk through the invocation stays inside its buffers and slots;
  // what is written to a recv buffer tiles it exactly; what one rank sends on an edge the next one receives
  struct Iv { uint64_t lo, hi; };
  std::vector<std::vector<Iv>> written(R);
  std::vector<uint64_t> n_out((size_t)R * t.nchan, 0), n_in((size_t)R * t.nchan, 0);
  for (uint32_t r = 0; r < R; ++r)
    for (uint32_t v = 0; v < t.nchan; ++v) {
      const DfxCooked& S = cooked[(size_t)r * t.nchan + v];
      const uint32_t prev = (r + R - 1) % R;
      uint32_t g = 0, p = 0, cidx = first_chunk(kind, r, R);
      uint64_t sent = 0, recvd = 0, steps = 0;
      for (;;) {
        if (fold) {
          // fold steps: the same look-ups as the scheduler makes when it posts a fold or a gather step
          const Prim fq = make_fold_prim(kind, p);
          const uint32_t rt = S.nslots;      // the root
          if (fq.fold == 1 || fq.fold == 2) {
            const uint32_t nk = fold_entries(kind, fq.fold, R);
            const uint32_t target = fq.fold == 1 ? fold_dest(kind) : 0u;
            if (nk > 64u || (target == 1u && nk > 63u)) return fail("rank %u channel %u: %u table entries for 64 lanes", r, v, nk);
            for (uint32_t k = 0; k < nk; ++k) {
              const uint32_t peer = fold_peer(kind, fq.fold, R, r, rt, k);
              if (peer >= R) return fail("rank %u channel %u fold step %u: entry %u names rank %u", r, v, p, k, peer);
              SliceGeom gk = slice_geometry(S, R, g, fold_chunk(kind, fq.fold, r, peer));
              if ((uint64_t)gk.bytes > (uint64_t)S.slice_elems * gk.eb) return fail("rank %u channel %u: a segment longer than the share", r, v);
              if (fq.fold == 2 && kind == KIND_BC) {          // entry k is the k-th piece of the share
                const uint32_t off = bc_piece_off(gk.bytes, k), len = bc_piece_len(gk.bytes, k);
                if (len > bc_piece_bytes((uint32_t)S.slice_elems * gk.eb)) return fail("rank %u channel %u: piece %u longer than the job's bound", r, v, k);
                if (off % gk.eb) return fail("rank %u channel %u: piece %u splits an element", r, v, k);
                gk.soff += off / gk.eb; gk.doff += off / gk.eb; gk.bytes = len;
              }
              if (!gk.bytes) continue;
              const uint64_t rd = gk.soff * gk.eb;            // every entry reads its rank's send buffer
              if (rd + gk.bytes > send_bytes) return fail("rank %u channel %u fold step %u: read of rank %u's buffer %llu+%u of %llu", r, v, p, peer, (unsigned long long)rd, gk.bytes, (unsigned long long)send_bytes);
              if ((kind == KIND_AG || kind == KIND_RS) && (rd & 15u)) return fail("rank %u channel %u fold step %u: a 16-byte read at offset %llu", r, v, p, (unsigned long long)rd);
              // a fold step writes its result to the own recv buffer (once, entry 0 stands for it), the root's, or
              // the recv buffer of every entry's rank; a gather step writes every segment to the own recv buffer
              if (fq.fold == 1 && target != 2u && k != 0) continue;
              const uint64_t wr = gk.doff * gk.eb;
              if (wr + gk.bytes > recv_bytes) return fail("rank %u channel %u fold step %u: recv buffer write %llu+%u of %llu", r, v, p, (unsigned long long)wr, gk.bytes, (unsigned long long)recv_bytes);
              written[target == 2u ? peer : (target == 1u ? rt : r)].push_back({wr, wr + gk.bytes});
            }
          }
          const SeqPos nx = next_fold_position(S.rounds, g, p, cidx);
          g = nx.g; p = nx.p; cidx = nx.cidx;
          if (g >= S.rounds) break;
          if (++steps > (uint64_t)S.rounds + 8) return fail("rank %u channel %u: the fold steps do not end", r, v);
          continue;
        }
        const Prim q = chain_drain_round(make_prim(kind, R, S.bc_pos & 3u, p, direct), kind, direct, g, S.rounds);
        const SliceGeom geo = slice_geometry(S, R, g, cidx);
        const uint64_t slot_b = (uint64_t)S.slice_elems * geo.eb;
        if (geo.bytes > slot_b) return fail("rank %u channel %u slice %u primitive %u: %u bytes in a slot of %llu", r, v, g, p, geo.bytes, (unsigned long long)slot_b);
        const bool moves = !(q.drain || (!q.recv && !q.from_send));
        const uint64_t nb = moves ? geo.bytes : 0;
        // (an empty slice -- a ragged message's last chunks -- is a handshake only: no address of it is used)
        if (nb && q.recv && !(q.din || q.din_send)) {
          const uint64_t a = S.fifo_in + (recvd & (S.nslots - 1)) * slot_b;
          if (a < S.fifo_in || a + nb > S.fifo_in + conn_slot_bytes) return fail("rank %u channel %u: read of slot at %llx leaves the connector", r, v, (unsigned long long)a);
        }
        if (nb && q.send) {
          const uint64_t a = S.fifo_out + (sent & (S.nslots - 1)) * slot_b;
          if (a < S.fifo_out || a + nb > S.fifo_out + conn_slot_bytes) return fail("rank %u channel %u: write of slot at %llx leaves the connector", r, v, (unsigned long long)a);
        }
        if (nb && q.from_send) {
          const uint64_t a = S.sendbuf + geo.soff * geo.eb;
          if (a < sendbase(r) || a + nb > sendbase(r) + send_bytes) return fail("rank %u channel %u slice %u primitive %u: send buffer read %llu+%llu of %llu", r, v, g, p, (unsigned long long)(a - sendbase(r)), (unsigned long long)nb, (unsigned long long)send_bytes);
        }
        if (nb && q.din_send) {
          const uint64_t a = sendbase(prev) + geo.soff * geo.eb;
          if (a + nb > sendbase(prev) + send_bytes) return fail("rank %u channel %u slice %u: read of the previous rank's send buffer %llu+%llu of %llu", r, v, g, (unsigned long long)(a - sendbase(prev)), (unsigned long long)nb, (unsigned long long)send_bytes);
        }
        if (nb && q.din) {
          const uint64_t a = recvbase(prev) + geo.doff * geo.eb;
          if (a + nb > recvbase(prev) + recv_bytes) return fail("rank %u channel %u slice %u: read of the previous rank's recv buffer %llu+%llu of %llu", r, v, g, (unsigned long long)(a - recvbase(prev)), (unsigned long long)nb, (unsigned long long)recv_bytes);
        }
        if (nb && q.to_recv) {
          const uint64_t a = S.recvbuf + geo.doff * geo.eb;
          if (a < recvbase(r) || a + nb > recvbase(r) + recv_bytes) return fail("rank %u channel %u slice %u primitive %u: recv buffer write %llu+%llu of %llu", r, v, g, p, (unsigned long long)(a - recvbase(r)), (unsigned long long)nb, (unsigned long long)recv_bytes);
          if (nb) written[r].push_back({a - recvbase(r), a - recvbase(r) + nb});
        }
        if (q.send || q.notify) { ++sent; ++n_out[(size_t)r * t.nchan + v]; }
        if (q.recv) { ++recvd; ++n_in[(size_t)r * t.nchan + v]; }
        const SeqPos nx = next_position(kind, R, r, cfg.window, S.rounds, S.nprim, g, p, cidx);
        g = nx.g; p = nx.p; cidx = nx.cidx;
        if (g >= S.rounds) break;
        if (++steps > (1ull << 26)) return fail("rank %u channel %u: the walk does not end", r, v);
      }
    }
  for (uint32_t r = 0; r < R; ++r)
    for (uint32_t v = 0; v < t.nchan; ++v)
      if (n_out[(size_t)r * t.nchan + v] != n_in[(size_t)((r + 1) % R) * t.nchan + v])
        return fail("edge %u channel %u: %llu slices sent or notified, %llu received", r, v, (unsigned long long)n_out[(size_t)r * t.nchan + v], (unsigned long long)n_in[(size_t)((r + 1) % R) * t.nchan + v]);
  for (uint32_t r = 0; r < R; ++r) {
    uint64_t want = recv_bytes;
    if (kind == DFX_REDUCE && r != (uint32_t)root) want = 0;
    std::vector<Iv>& w = written[r];
    std::sort(w.begin(), w.end(), [](const Iv& a, const Iv& b) { return a.lo < b.lo; });
    uint64_t at = 0;
    for (const Iv& iv : w) {
      if (iv.lo != at) return fail("rank %u: recv buffer bytes %llu .. %llu are written %s", r, (unsigned long long)std::min(at, iv.lo), (unsigned long long)std::max(at, iv.lo), iv.lo < at ? "twice" : "never");
      at = iv.hi;
    }
    if (at != want) return fail("rank %u: %llu of %llu recv buffer bytes written", r, (unsigned long long)at, (unsigned long long)want);
  }
  return DFX_OK;
}

// ------------------------------------------------------------------------------------------
// One collective without any allocation: the daemon kernel on a static scratch array
// ------------------------------------------------------------------------------------------
}  // extern "C"

// Everything a context allocates in dfx_init (SQ, CQ, control words, counters, saved contexts, task-queue store,
// workgroup state, connector flag lines and slots), laid out in one file-scope device array.  Each GPU the
// library runs on holds its own copy until the process ends.
#define DFX_NA_MAX_WG 256u                      // workgroups of the grid = nranks x channels per rank
#define DFX_NA_SLOT_BYTES (32u << 10)           // bytes per connector slot
#define DFX_NA_NSLOTS 4u                        // slots per connector
#define DFX_NA_SQ_DEPTH 2u
#define DFX_NA_CQ_SLOTS 2u
#define DFX_NA_MAX_RANKS 64u
#define DFX_NA_LINES (DFX_NA_MAX_WG + 64u)      // flag lines: one per connector, and a collective in fold steps has one more per channel
#define DFX_NA_CTL_BYTES (512u << 10)           // everything but the slots: must start at zero on every call
#define DFX_NA_SLOTS_BYTES ((size_t)DFX_NA_MAX_WG * DFX_NA_NSLOTS * DFX_NA_SLOT_BYTES)
#define DFX_NA_SCRATCH_BYTES ((size_t)DFX_NA_CTL_BYTES + DFX_NA_SLOTS_BYTES)
static __device__ __align__(256) unsigned char scratch[DFX_NA_SCRATCH_BYTES];

namespace {

// Offsets inside the zeroed part of the scratch.  The connector pool comes last: its flag lines are the end of
// the zeroed part and its slots follow them directly (a collective's connector block = flag lines, then slots).
struct NaLayout {
  size_t dev_ctl, host_ctl, sq, sq_freed, sq_readers, cq, cq_ctl, done_cnt, wgstate, taskq, ctxbuf, pool, end_of_zeroed;
};
constexpr size_t na_up(size_t x) { return (x + 255) & ~(size_t)255; }
constexpr NaLayout na_layout() {
  NaLayout L{};
  size_t o = 0;
  L.dev_ctl = o; o = na_up(o + DC_N * 4);
  L.host_ctl = o; o = na_up(o + HC_N * 4);
  L.sq = o; o = na_up(o + (size_t)DFX_NA_MAX_RANKS * DFX_NA_SQ_DEPTH * sizeof(DfxSqSlot));
  L.sq_freed = o; o = na_up(o + (size_t)DFX_NA_MAX_RANKS * DFX_NA_SQ_DEPTH * 4);
  L.sq_readers = o; o = na_up(o + (size_t)DFX_NA_MAX_RANKS * DFX_NA_SQ_DEPTH * 4);
  L.cq = o; o = na_up(o + (size_t)DFX_NA_MAX_RANKS * DFX_NA_CQ_SLOTS * 8);
  L.cq_ctl = o; o = na_up(o + (size_t)DFX_NA_MAX_RANKS * DFX_CQ_CTL_WORDS * 8);
  L.done_cnt = o; o = na_up(o + (size_t)DFX_NA_MAX_RANKS * 4);
  L.wgstate = o; o = na_up(o + (size_t)DFX_NA_MAX_WG * sizeof(DfxWgState));
  L.taskq = o; o = na_up(o + (size_t)DFX_NA_MAX_WG * 2);
  L.ctxbuf = o; o = na_up(o + (size_t)DFX_NA_MAX_WG * sizeof(DfxCtxEntry));
  // the pool's flag lines end exactly where the zeroed part ends
  L.pool = DFX_NA_CTL_BYTES - (size_t)DFX_NA_LINES * DFX_FLAG_STRIDE;
  L.end_of_zeroed = o;
  return L;
}
static_assert(na_layout().end_of_zeroed <= na_layout().pool, "the control structures overlap the connector pool");
static_assert(DFX_NA_CTL_BYTES % 256 == 0, "alignment of the slots");

struct NaSeed {                       // what the seeding kernel writes into the SQs: one entry per rank
  DfxStatic tmpl;
  uint64_t sendbuf[DFX_NA_MAX_RANKS], recvbuf[DFX_NA_MAX_RANKS];
  uint32_t nranks;
};

// clears the part of the scratch that must start at zero (a fill kernel, not a memset node: the call may be captured)
__global__ void __launch_bounds__(256) dfx_na_zero_kernel(uint4* p, uint32_t nvec) {
  for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += gridDim.x * blockDim.x) p[i] = uint4{0, 0, 0, 0};
}

// writes the SQEs the host would have written: entry 0 of every rank's SQ, generation word included
__global__ void __launch_bounds__(64) dfx_na_seed_kernel(DfxSqSlot* sq, NaSeed sd) {
  const uint32_t r = threadIdx.x;
  if (r >= sd.nranks) return;
  DfxStatic e = sd.tmpl;
  e.seq = 0;
  e.sendbuf = sd.sendbuf[r];
  e.recvbuf = sd.recvbuf[r];
  e.ready = 1;                        // generation of the first lap
  sq[(size_t)r * DFX_NA_SQ_DEPTH].e = e;
}

// after the daemon: 0 = every rank's completion is in its CQ and no error was raised
__global__ void dfx_na_status_kernel(const uint32_t* dev_ctl, const uint64_t* cq, uint32_t nranks, uint32_t* status) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  uint32_t st = 0;
  if (dev_ctl[DC_ERR]) st = 0x100u | dev_ctl[DC_ERR];
  else {
    uint32_t n = 0;
    for (uint32_t i = 0; i < nranks * DFX_NA_CQ_SLOTS; ++i) n += (uint32_t)(cq[i] >> 63);
    if (n != nranks) st = 0x200u;
  }
  *status = st;
}

struct NaDevice {
  unsigned char* ptr = nullptr;      // this device's copy of `scratch` (hipGetSymbolAddress), never the array's name
  double tick_us = 0.01;
  int max_wg = 0;                    // workgroups that can be resident at once
};
std::mutex g_na_mu;
NaDevice g_na_dev[kMaxDevices];

// Once per device, with that device current: the address of its copy of the scratch array and what the launch needs to know.
int na_setup(int device, NaDevice** out) {
  if (device < 0 || device >= kMaxDevices) return DFX_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lk(g_na_mu);
  NaDevice& d = g_na_dev[device];
  if (!d.ptr) {
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) { g_init_hip_error = (int)e; return DFX_ERR_HIP; }
    int occ = 0, ncu = 0, wall_khz = 0;
    e = dfx_daemon_occupancy(&occ);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, device);
    if (e != hipSuccess) { g_init_hip_error = (int)e; return DFX_ERR_HIP; }
    if (((DFX_WG_THREADS / 64) & 3) != 0 && occ > 1) occ = 1;   // as in dfx_init
    d.max_wg = occ * ncu;
    if (hipDeviceGetAttribute(&wall_khz, hipDeviceAttributeWallClockRate, device) == hipSuccess && wall_khz > 0)
      d.tick_us = 1000.0 / (double)wall_khz;
    d.ptr = (unsigned char*)p;
  }
  *out = &d;
  return DFX_OK;
}

}  // namespace

extern "C" {

int dfx_collective_noalloc(int nranks, dfx_kind kind, size_t count, dfx_dtype dtype, dfx_op op, int root,
                           const void* const* sendbufs, void* const* recvbufs, uint32_t* status_dev, void* hip_stream) {
  if (nranks < 1 || nranks > (int)DFX_NA_MAX_RANKS || !sendbufs || !recvbufs) return DFX_ERR_INVALID_ARG;
  if ((int)dtype < 0 || (int)dtype > 3 || (int)kind < 0 || (int)kind > 4) return DFX_ERR_INVALID_ARG;
  // the stated limit: no per-rank buffer beyond DFX_NOALLOC_MAX_BYTES
  const uint64_t eb = elem_bytes(dtype);
  const uint64_t largest = (kind == DFX_ALLGATHER || kind == DFX_REDUCESCATTER) ? (uint64_t)nranks : 1ull;
  if (count > DFX_NOALLOC_MAX_BYTES / (eb * largest)) return DFX_ERR_TOO_LARGE;
  for (int r = 0; r < nranks; ++r)
    if (!sendbufs[r] || !recvbufs[r] || ((uintptr_t)sendbufs[r] & 15u) || ((uintptr_t)recvbufs[r] & 15u)) return DFX_ERR_INVALID_ARG;

  int device = 0;
  if (hipGetDevice(&device) != hipSuccess) return DFX_ERR_HIP;
  NaDevice* nd = nullptr;
  int rc = na_setup(device, &nd);
  if (rc != DFX_OK) return rc;

  // the configuration of this path: library defaults under the scratch's sizes
  dfx_config cfg;
  dfx_config_default(&cfg);
  cfg.max_channels = std::min<uint32_t>(32u, DFX_NA_MAX_WG / (uint32_t)nranks);
  cfg.max_colls = 1;
  cfg.sq_depth = DFX_NA_SQ_DEPTH;
  cfg.cq_slots = DFX_NA_CQ_SLOTS;
  cfg.nslots = DFX_NA_NSLOTS;
  cfg.slot_bytes = DFX_NA_SLOT_BYTES;
  const uint32_t nwg = (uint32_t)nranks * cfg.max_channels;
  if ((int)nwg > nd->max_wg) return DFX_ERR_NO_RESOURCES;   // the grid must be co-resident
  // a grid shares the device with no other daemon grid: refuse while a context's daemon is in flight here
  {
    DeviceSlot& s = g_slot[device % kMaxDevices];
    std::lock_guard<std::mutex> lk(s.mu);
    if (s.owner && s.until && hipEventQuery(s.until) == hipErrorNotReady) return DFX_ERR_BUSY;
  }

  constexpr NaLayout L = na_layout();
  DfxStatic tmpl;
  uint64_t conn_bytes = 0;
  rc = plan_collective(cfg, nranks, 0, kind, count, dtype, op, root, 0, 0, &tmpl, &conn_bytes);
  if (rc != DFX_OK) return rc;
  // connector block = flag lines of the collective's R x C edges, then their slots; the scratch holds
  // DFX_NA_MAX_WG flag lines and as many connectors of DFX_NA_NSLOTS x DFX_NA_SLOT_BYTES
  const size_t flag_bytes = (size_t)(nranks + ((tmpl.flags & DFX_SQE_FOLD) ? 1 : 0)) * tmpl.nchan * DFX_FLAG_STRIDE;
  if (flag_bytes > (size_t)DFX_NA_LINES * DFX_FLAG_STRIDE || conn_bytes > flag_bytes + DFX_NA_SLOTS_BYTES + 256) return DFX_ERR_TOO_LARGE;
  // the flag lines end where the zeroed part ends, the slots begin right there
  tmpl.conn_off = (uint64_t)((size_t)DFX_NA_CTL_BYTES - flag_bytes - L.pool);

  unsigned char* base = nd->ptr;
  DfxDaemonArgs a;
  memset(&a, 0, sizeof(a));
  a.sq = (DfxSqSlot*)(base + L.sq); a.cq = (uint64_t*)(base + L.cq); a.cq_ctl = (uint64_t*)(base + L.cq_ctl);
  a.host_ctl = (uint32_t*)(base + L.host_ctl); a.sq_freed = (uint32_t*)(base + L.sq_freed);
  a.sq_readers = (uint32_t*)(base + L.sq_readers); a.done_cnt = (uint32_t*)(base + L.done_cnt);
  a.dev_ctl = (uint32_t*)(base + L.dev_ctl); a.pool = base + L.pool;
  a.ctxbuf = (DfxCtxEntry*)(base + L.ctxbuf); a.wgstate = (DfxWgState*)(base + L.wgstate);
  a.taskq_store = (uint16_t*)(base + L.taskq); a.trace = nullptr;
  a.nwg = nwg; a.scan_min = cfg.scan_min; a.epoch = 1;
  a.R = (uint32_t)nranks; a.cmax = cfg.max_channels; a.max_colls = 1; a.sq_depth = DFX_NA_SQ_DEPTH; a.sq_shift = 1; a.cq_slots = DFX_NA_CQ_SLOTS;
  a.spin_init = cfg.spin_init; a.spin_min = cfg.spin_min; a.spin_max = cfg.spin_max; a.spin_boost = cfg.spin_boost; a.preempt = 1;
  a.wg_map = 0; a.order_policy = 0; a.trace_on = 0; a.fetch_batch = 0xffffffffu; a.fifo_coherent = 1; a.chan_spread = 1;
  a.cq_mode = 0; a.sq_eager = 1; a.window = cfg.window; a.sq_local = 1; a.focus_bytes = cfg.focus_bytes;
  a.watchdog_ticks = (uint64_t)((double)cfg.watchdog_ms * 1000.0 / nd->tick_us);
  a.quit_ticks = 0;
  a.oneshot = 1;

  NaSeed sd;
  memset(&sd, 0, sizeof(sd));
  sd.tmpl = tmpl;
  sd.nranks = (uint32_t)nranks;
  for (int r = 0; r < nranks; ++r) { sd.sendbuf[r] = (uint64_t)(uintptr_t)sendbufs[r]; sd.recvbuf[r] = (uint64_t)(uintptr_t)recvbufs[r]; }

  hipStream_t st = (hipStream_t)hip_stream;
  hipLaunchKernelGGL(dfx_na_zero_kernel, dim3(64), dim3(256), 0, st, (uint4*)base, (uint32_t)(DFX_NA_CTL_BYTES / 16));
  hipLaunchKernelGGL(dfx_na_seed_kernel, dim3(1), dim3(64), 0, st, a.sq, sd);
  if (hipGetLastError() != hipSuccess) return DFX_ERR_HIP;
  if (dfx_daemon_launch(nwg, st, a) != hipSuccess) return DFX_ERR_HIP;
  if (status_dev) hipLaunchKernelGGL(dfx_na_status_kernel, dim3(1), dim3(64), 0, st, a.dev_ctl, a.cq, (uint32_t)nranks, status_dev);
  return hipGetLastError() == hipSuccess ? DFX_OK : DFX_ERR_HIP;
}

// Calibration helper for the profiler's HBM byte counters: copies `bytes` (multiple of 16)
// from src to dst (both device) with a plain kernel on the given stream (NULL = private
// stream) and waits for it.
int dfx_copy_calibrate(const void* src, void* dst, size_t bytes, void* hip_stream, float* ms) {
  if (!src || !dst || (bytes & 15u)) return DFX_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)hip_stream;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (ms) {
    if (hipEventCreate(&e0) != hipSuccess) return DFX_ERR_HIP;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return DFX_ERR_HIP; }
    (void)hipEventRecord(e0, s);
  }
  int rc = DFX_OK;
  if (dfx_copy_launch(src, dst, bytes, s) != hipSuccess) rc = DFX_ERR_HIP;
  if (ms) (void)hipEventRecord(e1, s);
  if (hipStreamSynchronize(s) != hipSuccess) rc = DFX_ERR_HIP;
  if (ms) {
    if (rc == DFX_OK && hipEventElapsedTime(ms, e0, e1) != hipSuccess) rc = DFX_ERR_HIP;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
  }
  return rc;
}

}  // extern "C"
