// Structures shared by the host library and the daemon kernel (not part of the public ABI).
#ifndef DFX_INTERNAL_H
#define DFX_INTERNAL_H

#include <stddef.h>
#include <stdint.h>

#ifndef DFX_WG_THREADS
#define DFX_WG_THREADS 320      // threads per daemon workgroup: one scheduler wavefront + the mover wavefronts
#endif
#define DFX_MOVERS (DFX_WG_THREADS - 64)   // threads of the mover wavefronts
#ifndef DFX_MOVER_GROUPS
#define DFX_MOVER_GROUPS 1      // groups the mover wavefronts work in (1 or 2): group k takes every GROUPS-th job
#endif
#define DFX_MAX_COLLS 4096      // upper bound for dfx_config.max_colls (LDS task queue = 8 KB)
#define DFX_CTX_SLOTS 64        // LDS active context slots, indexed by a hash of coll_id (Sec. 5)
#define DFX_TRACE_N 4096        // context-switch latency samples kept per workgroup
#define DFX_FLAG_STRIDE 128     // bytes per (edge, channel) flag pair: tail at +0, head at +64
#define DFX_DIRECT_OFF 16       // in the tail's line: the sender's recv buffer (8 bytes), invocation + 1 (4), 0 (4); then the same for its send buffer
#define DFX_NSTAT 24
#define DFX_CQ_CTL_WORDS 24      // 64-bit words of ring bookkeeping per vrank: reserve at 0, tail at 8, head at 16

#define DFX_SQE_EXIT 1u
#define DFX_SQE_DIRECT 2u      // collective with direct steps (reads the previous rank's recv / send buffer instead of slots)
#define DFX_CTX_DIRECT 0x80u   // the same, in the cooked context's bc_pos byte (bits 0-1: place in a chain)
#define DFX_SQE_FOLD 4u        // all-reduce in fold steps (always together with DFX_SQE_DIRECT: the buffers are published the same way)
#define DFX_CTX_FOLD 0x40u     // the same, in the cooked context's bc_pos byte
// A collective in fold steps has no slots.  Its connector block is R x nchan flag lines, one per (rank, channel),
// that carry the published buffer addresses (DFX_DIRECT_OFF), and behind them nchan shared lines, one per
// channel, with three counters that every rank of the channel adds to:
#define DFX_FOLD_PUB 0         //   +0  invocations published (buffer addresses written at SQE fetch)
#define DFX_FOLD_RED 8         //   +8  fold steps finished (the rank's chunk is combined and written where it belongs: every recv buffer, its own, or the root's)
#define DFX_FOLD_GAT 16        //   +16 gather steps finished (all-gather, broadcast: the rank has copied every block / its share)

// Static context of one invocation on one rank: what the host writes into the SQ and what a
// workgroup keeps in its context buffer (Sec. 4.2: buffer and connector addresses, rank count,
// composition of the primitive sequence).  96 bytes = six 16-byte vectors.
struct alignas(16) DfxStatic {
  uint32_t coll_id;
  uint32_t seq;          // invocation number of this (rank, coll_id)
  uint64_t sendbuf;
  uint64_t recvbuf;
  uint64_t count;
  uint64_t conn_off;     // byte offset of this collective's connector block in the pool
  uint64_t block_elems;  // ring chunk length (all-reduce) or count (others), in elements
  uint64_t part_elems;   // elements of a block that one channel covers (16-byte multiple)
  uint32_t slice_elems;  // elements per FIFO slot
  uint32_t rounds;       // slices per block and channel = repetitions of the primitive sequence
  uint32_t slot_bytes;
  uint16_t nslots;
  uint16_t nchan;
  uint8_t kind, dtype, op, root;
  uint16_t flags;
  int16_t priority;
  uint32_t nprim;        // primitives per round on every rank
  uint32_t reserved;
  uint32_t reserved2;
  uint32_t ready;        // SQ only, written last: generation of the entry
};
static_assert(sizeof(DfxStatic) == 96, "DfxStatic must be 96 bytes");

// Dynamic context (Sec. 4.2: current chunk id, aborted primitive id) plus the monotone
// connector counters of this (rank, channel).  32 bytes = two 16-byte vectors.
struct alignas(16) DfxDyn {
  uint32_t round;        // slice index ("current data chunk"); slices are taken in windows, see the daemon
  uint32_t prim;         // next primitive of the sequence ("aborted primitive")
  uint64_t sent;         // slices ever pushed into the send connector
  uint64_t recvd;        // slices ever taken from the recv connector
  uint32_t preempted;    // times this invocation was preempted on this workgroup
  uint32_t cidx;         // ring-chunk index of the next primitive (kept so that no division is needed)
};
static_assert(sizeof(DfxDyn) == 32, "DfxDyn must be 32 bytes");

// What a workgroup keeps of an invocation (device-private): the SQE "cooked" once at fetch time
// into ready-to-use addresses, so that a context load needs no address arithmetic.  96 bytes.
struct alignas(16) DfxCooked {
  uint64_t sendbuf, recvbuf, count, block_elems, part_elems;
  uint64_t flags_out;    // tail counter of my send connector (head at +64 bytes)
  uint64_t flags_in;     // tail counter of my recv connector (head at +64 bytes)
  uint64_t fifo_out;     // first slot of my send connector
  uint64_t fifo_in;      // first slot of my recv connector
  uint32_t slice_elems, rounds, seq;
  uint16_t nprim, nchan;
  uint8_t nslots, kind, dtype;
  uint8_t bc_pos;        // place in a chain: 0 = first, 1 = middle, 2 = last, 3 = second of a reduce chain with direct steps; | DFX_CTX_DIRECT
  int16_t priority;
  uint16_t vch;          // channel of the collective that this workgroup serves (0 .. nchan-1)
};
static_assert(sizeof(DfxCooked) == 96, "DfxCooked must be 96 bytes");
// (the scheduler reads some of it as 16-byte words: the readiness scan and the set-up of a primitive)
static_assert(offsetof(DfxCooked, part_elems) == 32 && offsetof(DfxCooked, flags_out) == 40 && offsetof(DfxCooked, flags_in) == 48 &&
              offsetof(DfxCooked, fifo_in) == 64 && offsetof(DfxCooked, slice_elems) == 72 && offsetof(DfxCooked, rounds) == 76 &&
              offsetof(DfxCooked, seq) == 80 && offsetof(DfxCooked, nprim) == 84 && offsetof(DfxCooked, nchan) == 86 &&
              offsetof(DfxCooked, nslots) == 88 && offsetof(DfxCooked, kind) == 89 && offsetof(DfxCooked, dtype) == 90 &&
              offsetof(DfxCooked, bc_pos) == 91 && offsetof(DfxCooked, priority) == 92 && offsetof(DfxCooked, vch) == 94,
              "DfxCooked layout");

struct alignas(16) DfxCtxEntry {
  DfxCooked st;
  DfxDyn dyn;
};
static_assert(sizeof(DfxCtxEntry) == 128, "context entry must be 128 bytes");

struct alignas(16) DfxSqSlot {   // one SQ ring entry, padded to two 64-byte lines
  DfxStatic e;
  uint32_t pad[8];
};
static_assert(sizeof(DfxSqSlot) == 128, "SQ slot must be 128 bytes");

// Per-workgroup state that survives daemon exit / voluntary quit (Sec. 4.5).
struct alignas(16) DfxWgState {
  uint64_t read_index;   // SQ entries consumed by this workgroup
  uint32_t qlen;         // task-queue length (entries are in taskq_store)
  uint32_t trace_n;      // trace samples written (monotone)
  uint64_t stat[DFX_NSTAT];
  uint64_t dbg[8];       // filled when the watchdog fires
  uint64_t pad[6];
};

enum { ST_PREEMPT = 0, ST_LOAD, ST_HIT, ST_SAVE, ST_LAZY, ST_POLLS, ST_PRIMS, ST_SQE, ST_CQE, ST_MAXQ, ST_PASSES, ST_QUITS,
       ST_T_WAIT, ST_T_DATA, ST_T_PUB, ST_SCAN_SKIPS,   // T_*: wall-clock ticks, only with trace on
       ST_T_CQE,                                         // ticks spent writing CQEs (always counted)
       ST_T_STAMP, ST_N_STAMP,                           // ticks of back-to-back clock reads and their number (trace 1, 2)
       ST_T_SQE };                                       // ticks spent fetching SQEs: probe seen -> entries cooked and queued (always counted)

// dev_ctl words (device memory)
// (abort and quit share one aligned 64-bit word: the scheduler reads both with one load; the host
// clears quit and votes, which are adjacent, with one memset)
enum { DC_ERR = 0, DC_ERR_WG = 1, DC_ABORT = 2, DC_QUIT = 3, DC_VOTES = 4, DC_N = 16 };
// host_ctl words (host-visible queue memory)
enum { HC_ABORT = 0, HC_N = 16 };

struct DfxDaemonArgs {
  DfxSqSlot* sq;            // [R][sq_depth]   host-visible
  uint64_t* cq;             // [R][cq_slots]   host-visible
  uint64_t* cq_ctl;         // [R][DFX_CQ_CTL_WORDS] host-visible: bookkeeping of the ring-buffer CQ variants
  uint32_t* host_ctl;       // [HC_N]          host-visible
  uint32_t* sq_freed;       // [R][sq_depth]   host memory: generation of the entry last read by every workgroup
  uint32_t* sq_readers;     // [R][sq_depth]   device
  uint32_t* done_cnt;       // [R][max_colls]  device
  uint32_t* dev_ctl;        // [DC_N]          device
  uint8_t* pool;            // connector pool  device
  DfxCtxEntry* ctxbuf;      // [nwg][max_colls] device
  DfxWgState* wgstate;      // [nwg]           device
  uint16_t* taskq_store;    // [nwg][max_colls] device
  uint64_t* trace;          // [nwg][DFX_TRACE_N] device (or null)
  uint32_t nwg;
  uint32_t scan_min;        // queue length from which a pass starts with a readiness scan (0 = never)
  uint32_t epoch;           // number of this launch (exit SQEs name the launch they end)
  uint32_t R, cmax, max_colls, sq_depth, sq_shift, cq_slots;
  uint32_t spin_init, spin_min, spin_max, spin_boost, preempt;
  uint32_t wg_map, order_policy, trace_on, fetch_batch, fifo_coherent, chan_spread, cq_mode, sq_eager, window, sq_local, focus_bytes;
  uint64_t watchdog_ticks;  // wall-clock ticks; 0 = off
  uint64_t quit_ticks;      // wall-clock ticks; 0 = off
  uint32_t oneshot;         // not 0: the SQs were filled before the launch with this many entries per rank and nobody
                            // will submit more: a workgroup that has read them all and finished its share votes to
                            // leave (and never withdraws the vote); the last vote ends the grid
};

#endif
