// The daemon kernel: one persistent grid that executes, preempts and schedules ring
// collectives for R virtual ranks on one MI355X (gfx950).
//
// Workgroup = (virtual rank, channel).  Every workgroup runs the scheduling loop of the
// paper's Alg. 1 (Sec. 4.3) on its own: fetch SQEs into an LDS task queue, walk the queue,
// load a collective's context into an LDS slot, execute its primitives in two-phase blocking
// fashion (bounded spin on the connector flags, then the slice's data movement), raise the
// spin threshold after a success, and on a timed-out wait save the dynamic context (lazily)
// and switch to the next collective.  Completion is counted per collective; the last channel
// posts the CQE.  Connectors are FIFOs of K slots in HBM guarded by monotone tail/head
// counters; a primitive touches nothing before both its conditions hold (Sec. 4.1, 4.5).
// Long collectives take direct steps, because every rank's buffers lie in the same HBM: in
// the copy steps (gather phase of an all-reduce, all-gather, broadcast) the result goes to the
// rank's recv buffer only (through the coherent path described below), the counter is raised
// all the same, and the next rank reads the chunk from that recv buffer; the opening send of
// a reduce phase (all-reduce, reduce-scatter, reduce chain) moves nothing, the next rank reads
// the chunk from this rank's send buffer; a last step waits until the neighbour has read
// everything (see Prim::notify / din / din_send / drain).
//
// Memory-model rules used here (AMDGPU, one agent with one L2 per XCD), two connector modes:
//   device-coherent accesses (fifo_coherent = 1, the default)
//     connector slots are only ever touched by sc1 (device-scope) buffer loads/stores, which
//     do not linger in the per-XCD caches; every mover wave drains its stores (vmcnt(0)) and
//     counts itself done in LDS; the wave that completes the count raises the connector
//     counter with a device-scope atomic; the consumer's scheduler wave polls the counter with
//     sc1 loads and its movers read the slot with sc1 loads.  No bulk L2 write-back or
//     invalidate per slice.  User buffers stay ordinary cached memory: the send buffer is made
//     visible by the system-scope acquire at SQE fetch, the recv buffer is flushed by the
//     system-scope release before the completion counter.
//   fenced (fifo_coherent = 0, kept for comparison)
//     connector slots are ordinary cached memory; the publishing wave issues an agent-scope
//     release fence (L2 write-back) before it raises the counter, and every mover wave an
//     agent-scope acquire fence (invalidate) before its loads of a slot.
//   SQ / CQ / host control words are host-visible and use system scope.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dfx_internal.h"
#include "dfx_geometry.h"

namespace {

typedef uint64_t u64;

constexpr int NT = DFX_WG_THREADS;
#ifndef DFX_UNROLL
#define DFX_UNROLL 8
#endif
constexpr int UNROLL = DFX_UNROLL;   // independent 16-byte vectors in flight per source and thread
constexpr int DT_COPY = -1;   // a primitive without a reducing side moves bytes, whatever the element type

enum { W_OK = 0, W_TIMEOUT = 1, W_STOP = 2 };
enum { STOP_NONE = 0, STOP_ABORT = 1, STOP_QUIT = 2, STOP_EXIT = 3 };

#define SCOPE_AGENT __HIP_MEMORY_SCOPE_AGENT
#define SCOPE_SYSTEM __HIP_MEMORY_SCOPE_SYSTEM

__device__ __forceinline__ u64 ld_agent64(const u64* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, SCOPE_AGENT); }
__device__ __forceinline__ void st_agent64(u64* p, u64 v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, SCOPE_AGENT); }
__device__ __forceinline__ uint32_t ld_agent32(const uint32_t* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, SCOPE_AGENT); }
__device__ __forceinline__ uint32_t ld_sys32(const uint32_t* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, SCOPE_SYSTEM); }

// Release fences end with an explicit wait: the L2 write-back they issue must have completed
// before the flag store that follows.  The compiler's own wait is dropped when it believes no
// memory operation is pending (the wave's own stores were drained earlier), and the write-back
// itself is not on its scoreboard.
__device__ __forceinline__ void fence_acquire_agent() { __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent"); }
__device__ __forceinline__ void fence_release_agent() { __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent"); __builtin_amdgcn_s_waitcnt(0); }
__device__ __forceinline__ void fence_acquire_system() { __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, ""); }
__device__ __forceinline__ void fence_release_system() { __builtin_amdgcn_fence(__ATOMIC_RELEASE, ""); __builtin_amdgcn_s_waitcnt(0); }

// ------------------------------------------------------------------------------------------
// reduce: one hop a (+) b in the storage dtype (one rounding per hop)
// ------------------------------------------------------------------------------------------
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

// two fp32 values -> packed bf16, round to nearest even: one conversion instruction on gfx950
__device__ __forceinline__ uint32_t pack_bf16_rne(float lo, float hi) {
  f32x2_t s;
  s[0] = lo; s[1] = hi;
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(s, bf16x2_t));
}

__device__ __forceinline__ uint32_t bf16x2_add(uint32_t a, uint32_t b) {
  // widen (exact), add in fp32, round to nearest even back to bf16
  return pack_bf16_rne(__uint_as_float(a << 16) + __uint_as_float(b << 16),
                       __uint_as_float(a & 0xffff0000u) + __uint_as_float(b & 0xffff0000u));
}

template <int DT>
__device__ __forceinline__ uint32_t add_word(uint32_t a, uint32_t b) {
  if (DT == DT_F32) return __float_as_uint(__uint_as_float(a) + __uint_as_float(b));
  if (DT == DT_I32) return a + b;
  if (DT == DT_F16) {
    half2_t x = __builtin_bit_cast(half2_t, a), y = __builtin_bit_cast(half2_t, b);
    return __builtin_bit_cast(uint32_t, x + y);
  }
  return bf16x2_add(a, b);
}

template <int DT>
__device__ __forceinline__ uint4 add_vec(uint4 a, uint4 b) {
  uint4 r;
  r.x = add_word<DT>(a.x, b.x);
  r.y = add_word<DT>(a.y, b.y);
  r.z = add_word<DT>(a.z, b.z);
  r.w = add_word<DT>(a.w, b.w);
  return r;
}

template <int DT>
__device__ __forceinline__ uint16_t add_half(uint16_t a, uint16_t b) {
  if (DT == DT_F16) {
    _Float16 x = __builtin_bit_cast(_Float16, a), y = __builtin_bit_cast(_Float16, b);
    return __builtin_bit_cast(uint16_t, (_Float16)(x + y));
  }
  return (uint16_t)(bf16x2_add(a, b) & 0xffffu);
}

// The other reducing functions (Sec. 4.1: "a specified reducing function"), evaluated as
// partial (op) own with the partial that arrived from the left first.  Product rounds once per
// hop like the sum; maximum / minimum pass one operand on unchanged: the partial if it is
// strictly greater (smaller), else the own value -- plain compare-and-select, so that equal
// values (+0 / -0 included) behave the same everywhere.
enum { OP_SUM = 0, OP_PROD = 1, OP_MAX = 2, OP_MIN = 3 };

template <int OP>
__device__ __forceinline__ uint32_t bf16x2_op(uint32_t a, uint32_t b) {
  const float al = __uint_as_float(a << 16), bl = __uint_as_float(b << 16);
  const float ah = __uint_as_float(a & 0xffff0000u), bh = __uint_as_float(b & 0xffff0000u);
  if (OP == OP_PROD) return pack_bf16_rne(al * bl, ah * bh);
  const bool tl = (OP == OP_MAX) ? (al > bl) : (al < bl);
  const bool th = (OP == OP_MAX) ? (ah > bh) : (ah < bh);
  return ((tl ? a : b) & 0xffffu) | ((th ? a : b) & 0xffff0000u);
}

// one 32-bit word (one fp32 / int32 element or two 16-bit ones), reducing function fixed at compile time
template <int DT, int OP>
__device__ __forceinline__ uint32_t op_word_t(uint32_t a, uint32_t b) {
  if (OP == OP_SUM) return add_word<DT>(a, b);
  if (DT == DT_F32) {
    const float x = __uint_as_float(a), y = __uint_as_float(b);
    if (OP == OP_PROD) return __float_as_uint(x * y);
    return ((OP == OP_MAX) ? (x > y) : (x < y)) ? a : b;
  }
  if (DT == DT_I32) {
    if (OP == OP_PROD) return a * b;
    const int x = (int)a, y = (int)b;
    return ((OP == OP_MAX) ? (x > y) : (x < y)) ? a : b;
  }
  if (DT == DT_F16) {
    const half2_t x = __builtin_bit_cast(half2_t, a), y = __builtin_bit_cast(half2_t, b);
    if (OP == OP_PROD) return __builtin_bit_cast(uint32_t, x * y);
    const bool tl = (OP == OP_MAX) ? (x[0] > y[0]) : (x[0] < y[0]);
    const bool th = (OP == OP_MAX) ? (x[1] > y[1]) : (x[1] < y[1]);
    return ((tl ? a : b) & 0xffffu) | ((th ? a : b) & 0xffff0000u);
  }
  return bf16x2_op<OP>(a, b);
}

// the same with the reducing function picked at run time (element-wise tails)
template <int DT>
__device__ __forceinline__ uint32_t op_word(uint32_t a, uint32_t b, int op) {
  switch (op) {
    case OP_PROD: return op_word_t<DT, OP_PROD>(a, b);
    case OP_MAX: return op_word_t<DT, OP_MAX>(a, b);
    case OP_MIN: return op_word_t<DT, OP_MIN>(a, b);
    default: return add_word<DT>(a, b);
  }
}

template <int DT, int OP>
__device__ __forceinline__ uint4 op_vec_t(uint4 a, uint4 b) {
  uint4 r;
  r.x = op_word_t<DT, OP>(a.x, b.x);
  r.y = op_word_t<DT, OP>(a.y, b.y);
  r.z = op_word_t<DT, OP>(a.z, b.z);
  r.w = op_word_t<DT, OP>(a.w, b.w);
  return r;
}

// A whole batch of vectors under one (wave-uniform) branch on the reducing function: the branch
// stays out of the unrolled loads and stores around it.
template <int DT, int N>
__device__ __forceinline__ void op_batch(uint4 (&v)[N], const uint4 (&w)[N], int op) {
  switch (op) {
    case OP_PROD:
#pragma unroll
      for (int u = 0; u < N; ++u) v[u] = op_vec_t<DT, OP_PROD>(v[u], w[u]);
      break;
    case OP_MAX:
#pragma unroll
      for (int u = 0; u < N; ++u) v[u] = op_vec_t<DT, OP_MAX>(v[u], w[u]);
      break;
    case OP_MIN:
#pragma unroll
      for (int u = 0; u < N; ++u) v[u] = op_vec_t<DT, OP_MIN>(v[u], w[u]);
      break;
    default:
#pragma unroll
      for (int u = 0; u < N; ++u) v[u] = add_vec<DT>(v[u], w[u]);
      break;
  }
}

template <int DT>
__device__ __forceinline__ uint16_t op_half(uint16_t a, uint16_t b, int op) {
  if (op == OP_SUM) return add_half<DT>(a, b);
  return (uint16_t)(op_word<DT>(a, b, op) & 0xffffu);   // the upper half combines zeros and is dropped
}

// ------------------------------------------------------------------------------------------
// slice mover: value = [fifo_in[i]] (+) [sendbuf[i]];  recvbuf[i] = value;  fifo_out[i] = value
// (each side present or not, as the primitive says).  128-bit coalesced accesses, four
// independent vectors in flight per source and thread.
//
// Connector slots are accessed through buffer instructions.  COH = 1 marks those accesses
// device-coherent (sc1: they bypass the non-coherent levels and write through), so that
// connector traffic needs no bulk L2 write-back / invalidate around every slice; COH = 0 uses
// ordinary cached accesses and relies on the agent-scope fences of the caller.
// User buffers are plain pointers, accessed with 16-byte vectors whatever their alignment; only
// the sub-vector tail of a slice is moved element by element.
// ------------------------------------------------------------------------------------------
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

// User-buffer accesses of the main loop are marked non-temporal: each byte is touched once, and
// keeping it out of the way leaves the memory-side cache to the connector slots (+3 % measured).
// They are 16-byte accesses through a type that promises only element alignment (2 bytes): the
// blocks of an all-gather / reduce-scatter of odd length start anywhere, and the hardware does
// under-aligned vector accesses at full width (element by element the same blocks ran ten times
// slower).
typedef v4u v4u_user __attribute__((aligned(2)));
__device__ __forceinline__ uint4 ld_user(const v4u_user* p) {
  return __builtin_bit_cast(uint4, __builtin_nontemporal_load(p));
}
__device__ __forceinline__ void st_user(v4u_user* p, uint4 v) {
  __builtin_nontemporal_store(__builtin_bit_cast(v4u, v), p);
}

// cache-policy operand of the buffer instructions (gfx940+): bit 0 = sc0, bit 4 = sc1
constexpr int AUX_CACHED = 0;    // ordinary cached access (per-CU cache, write-back in this XCD's L2)
constexpr int AUX_DEVICE = 16;   // sc1: device scope, coherent across the XCDs' L2s

template <int AUX>
struct Slot {   // one connector slot seen through a buffer resource
  __amdgpu_buffer_rsrc_t rsrc;
  __device__ __forceinline__ Slot(const void* base, uint32_t bytes) {
    rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
  }
  __device__ __forceinline__ uint4 ld16(uint32_t off) const {
    return __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)off, 0, AUX));
  }
  __device__ __forceinline__ void st16(uint32_t off, uint4 v) const {
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4u, v), rsrc, (int)off, 0, AUX);
  }
  __device__ __forceinline__ uint32_t ld4(uint32_t off) const { return __builtin_amdgcn_raw_buffer_load_b32(rsrc, (int)off, 0, AUX); }
  __device__ __forceinline__ void st4(uint32_t off, uint32_t v) const { __builtin_amdgcn_raw_buffer_store_b32(v, rsrc, (int)off, 0, AUX); }
  __device__ __forceinline__ uint16_t ld2(uint32_t off) const { return __builtin_amdgcn_raw_buffer_load_b16(rsrc, (int)off, 0, AUX); }
  __device__ __forceinline__ void st2(uint32_t off, uint16_t v) const { __builtin_amdgcn_raw_buffer_store_b16(v, rsrc, (int)off, 0, AUX); }
};

// GEN = false: the sum only (the common case keeps its own instantiation); GEN = true: `op` picks
// the reducing function at run time (a wave-uniform branch per vector).
template <int DT, bool GEN, int AIN, int AOUT, bool FIN, bool SB, bool RB, bool FOUT, int NTH>
__device__ __forceinline__ void move_slice(const void* fin_p, const char* __restrict__ sb, char* __restrict__ rb,
                                           void* fout_p, uint32_t bytes, uint32_t tid, int op) {
  constexpr int NT = NTH;   // threads that share the slice: the mover waves
  static_assert(FIN || SB, "a primitive has a source");
  static_assert(RB || FOUT, "a primitive has a destination");
  const Slot<AIN> fin(fin_p, FIN ? bytes : 0);
  const Slot<AOUT> fout(fout_p, FOUT ? bytes : 0);
  uint32_t done = 0;
  {
    const v4u_user* __restrict__ S = (const v4u_user*)sb;
    v4u_user* __restrict__ D = (v4u_user*)rb;
    const uint32_t nvec = bytes >> 4;
    uint32_t i = tid;
    for (; i + (UNROLL - 1) * NT < nvec; i += UNROLL * NT) {
      uint4 v[UNROLL];
      if (FIN) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) v[u] = fin.ld16((i + u * NT) << 4);
      }
      if (SB) {
        uint4 w[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) w[u] = ld_user(&S[i + u * NT]);
        if (FIN && GEN) op_batch<DT, UNROLL>(v, w, op);
        else {
#pragma unroll
          for (int u = 0; u < UNROLL; ++u) v[u] = FIN ? add_vec<DT>(v[u], w[u]) : w[u];
        }
      }
      if (FOUT) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) fout.st16((i + u * NT) << 4, v[u]);
      }
      if (RB) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) st_user(&D[i + u * NT], v[u]);
      }
    }
    if (i < nvec) {
      // remainder: the same unrolled shape with per-vector predicates, so that all loads of the
      // tail are in flight together (a short slice is one such block: one memory round trip)
      uint4 v[UNROLL];
      if (FIN) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) v[u] = fin.ld16((i + u * NT) << 4);   // out of range reads return 0
      }
      if (SB) {
        uint4 w[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) w[u] = (i + u * NT < nvec) ? ld_user(&S[i + u * NT]) : uint4{0, 0, 0, 0};
        if (FIN && GEN) op_batch<DT, UNROLL>(v, w, op);
        else {
#pragma unroll
          for (int u = 0; u < UNROLL; ++u) v[u] = FIN ? add_vec<DT>(v[u], w[u]) : w[u];
        }
      }
      if (FOUT) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) if (i + u * NT < nvec) fout.st16((i + u * NT) << 4, v[u]);
      }
      if (RB) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) if (i + u * NT < nvec) st_user(&D[i + u * NT], v[u]);
      }
    }
    done = nvec << 4;
  }
  // element-wise remainder: the sub-vector tail of a slice
  if (done < bytes) {
    if (DT == DT_F32 || DT == DT_I32) {
      const uint32_t* S = (const uint32_t*)sb;
      uint32_t* D = (uint32_t*)rb;
      for (uint32_t o = done + (tid << 2); o < bytes; o += NT << 2) {
        uint32_t v = 0;
        if (FIN) v = fin.ld4(o);
        if (SB) { uint32_t w = S[o >> 2]; v = FIN ? (GEN ? op_word<DT>(v, w, op) : add_word<DT>(v, w)) : w; }
        if (FOUT) fout.st4(o, v);
        if (RB) D[o >> 2] = v;
      }
    } else {   // 16-bit elements; pure copies also come here (every dtype is a multiple of 2 bytes)
      const uint16_t* S = (const uint16_t*)sb;
      uint16_t* D = (uint16_t*)rb;
      for (uint32_t o = done + (tid << 1); o < bytes; o += NT << 1) {
        uint16_t v = 0;
        if (FIN) v = fin.ld2(o);
        if (SB) { uint16_t w = S[o >> 1]; v = FIN ? (GEN ? op_half<DT>(v, w, op) : add_half<DT>(v, w)) : w; }
        if (FOUT) fout.st2(o, v);
        if (RB) D[o >> 1] = v;
      }
    }
  }
}

// `dtype` carries the element type in its low four bits and the reducing function above them.
template <int AIN, int AOUT, bool FIN, bool SB, bool RB, bool FOUT, int NTH>
__device__ __forceinline__ void move_dispatch(int dtype, const void* fin, const char* sb, char* rb, void* fout, uint32_t bytes, uint32_t tid) {
  if (!(FIN && SB)) { move_slice<DT_COPY, false, AIN, AOUT, FIN, SB, RB, FOUT, NTH>(fin, sb, rb, fout, bytes, tid, 0); return; }
  const int dt = dtype & 15, op = dtype >> 4;
  if (op == OP_SUM) {
    switch (dt) {
      case DT_F32: move_slice<DT_F32, false, AIN, AOUT, FIN, SB, RB, FOUT, NTH>(fin, sb, rb, fout, bytes, tid, 0); break;
      case DT_BF16: move_slice<DT_BF16, false, AIN, AOUT, FIN, SB, RB, FOUT, NTH>(fin, sb, rb, fout, bytes, tid, 0); break;
      case DT_F16: move_slice<DT_F16, false, AIN, AOUT, FIN, SB, RB, FOUT, NTH>(fin, sb, rb, fout, bytes, tid, 0); break;
      default: move_slice<DT_I32, false, AIN, AOUT, FIN, SB, RB, FOUT, NTH>(fin, sb, rb, fout, bytes, tid, 0); break;
    }
  } else {
    switch (dt) {
      case DT_F32: move_slice<DT_F32, true, AIN, AOUT, FIN, SB, RB, FOUT, NTH>(fin, sb, rb, fout, bytes, tid, op); break;
      case DT_BF16: move_slice<DT_BF16, true, AIN, AOUT, FIN, SB, RB, FOUT, NTH>(fin, sb, rb, fout, bytes, tid, op); break;
      case DT_F16: move_slice<DT_F16, true, AIN, AOUT, FIN, SB, RB, FOUT, NTH>(fin, sb, rb, fout, bytes, tid, op); break;
      default: move_slice<DT_I32, true, AIN, AOUT, FIN, SB, RB, FOUT, NTH>(fin, sb, rb, fout, bytes, tid, op); break;
    }
  }
}

#ifndef DFX_LDS_STAGE
#define DFX_LDS_STAGE 0
#endif
#if DFX_LDS_STAGE
// Experiment build (-DDFX_LDS_STAGE=1): the recv-reduce-send step with both inputs staged through LDS.
// Each mover wave brings the vectors of the connector slot and of the send buffer in with gfx950's
// 16-byte global -> LDS loads (no registers held while they travel), STAGE_D - 1 batches of STAGE_U
// vectors per lane and source ahead of the batch being reduced, reads them back with ds_read_b128, adds,
// and stores to the outgoing slot.  Per lane 2 x STAGE_U x (STAGE_D - 1) = 24 loads are in flight all the
// time, instead of 16 that are issued together and waited for together.
// The waits are counted by hand: the compiler would put vmcnt(0) in front of every LDS read that follows
// an LDS-writing load, which would undo the prefetch.  Vector memory operations of a wave complete in the
// order they were issued, so "at most N outstanding" means that everything older than the youngest N is
// done; that is also why both inputs go through LDS: a wait for a register load would wait for every
// LDS-writing load issued before it.
constexpr uint32_t STAGE_U = 4;                              // vectors per lane, source and batch
constexpr uint32_t STAGE_D = 4;                              // batches in LDS per wave (STAGE_D - 1 ahead of the one in use)
constexpr uint32_t STAGE_BATCH_BYTES = 2 * STAGE_U * 1024;   // two sources x U vectors x 64 lanes x 16 bytes
constexpr uint32_t STAGE_WAVE_BYTES = STAGE_D * STAGE_BATCH_BYTES;
typedef __attribute__((address_space(3))) unsigned char lds_byte;

template <int N>
__device__ __forceinline__ void stage_read(uint32_t lds_addr, v4u (&v)[8]) {
  asm volatile(
      "s_waitcnt vmcnt(%9)\n\t"
      "ds_read_b128 %0, %8\n\t"
      "ds_read_b128 %1, %8 offset:1024\n\t"
      "ds_read_b128 %2, %8 offset:2048\n\t"
      "ds_read_b128 %3, %8 offset:3072\n\t"
      "ds_read_b128 %4, %8 offset:4096\n\t"
      "ds_read_b128 %5, %8 offset:5120\n\t"
      "ds_read_b128 %6, %8 offset:6144\n\t"
      "ds_read_b128 %7, %8 offset:7168\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3]), "=&v"(v[4]), "=&v"(v[5]), "=&v"(v[6]), "=&v"(v[7])
      : "v"(lds_addr), "n"(N)
      : "memory");
}

// bytes: a multiple of STAGE_U x NTH x 16; fin_p and sb 16-byte aligned; stage: this workgroup's staging
// area (NTH / 64 waves x STAGE_WAVE_BYTES)
template <int DT, int NTH>
__device__ __forceinline__ void move_rrs_staged(const void* fin_p, const char* __restrict__ sb, void* fout_p, uint32_t bytes,
                                                uint32_t tid, lds_byte* stage) {
  static_assert(STAGE_U == 4, "stage_read reads 2 x 4 vectors");
  const Slot<AUX_DEVICE> fout(fout_p, bytes);
  const uint32_t wave = tid >> 6, lane = tid & 63u;
  lds_byte* mine = stage + wave * STAGE_WAVE_BYTES;
  const uint32_t lds0 = (uint32_t)(uintptr_t)mine + lane * 16u;
  const uint4* F = (const uint4*)fin_p;
  const uint4* S = (const uint4*)sb;
  const uint32_t nvec = bytes >> 4, per_batch = STAGE_U * NTH, nbatch = nvec / per_batch;
  auto bring = [&](uint32_t k) {       // batch k -> its place in LDS: 2 x STAGE_U instructions
    lds_byte* dst = mine + (k % STAGE_D) * STAGE_BATCH_BYTES;
    const uint32_t i = tid + k * per_batch;
#pragma unroll
    for (uint32_t u = 0; u < STAGE_U; ++u)
      __builtin_amdgcn_global_load_lds((const void*)&F[i + u * NTH], (__attribute__((address_space(3))) void*)(dst + u * 1024), 16, 0, AUX_DEVICE);
#pragma unroll
    for (uint32_t u = 0; u < STAGE_U; ++u)
      __builtin_amdgcn_global_load_lds((const void*)&S[i + u * NTH], (__attribute__((address_space(3))) void*)(dst + (STAGE_U + u) * 1024), 16, 0, 2 /* nt */);
  };
  for (uint32_t k = 0; k + 1 < STAGE_D && k < nbatch; ++k) bring(k);
  for (uint32_t b = 0; b < nbatch; ++b) {
    if (b + STAGE_D - 1 < nbatch) bring(b + STAGE_D - 1);
    asm volatile("" ::: "memory");
    // Issued after batch b's loads: the loads of the batches ahead (2U each) and, in the steady state, the
    // stores of the STAGE_D - 1 iterations in between (U each).  Towards the ends the stores are left out of
    // the count: a smaller count only waits for more.
    const uint32_t ahead = (nbatch - 1 - b) < (STAGE_D - 1) ? (nbatch - 1 - b) : (STAGE_D - 1);
    v4u v[8];
    const uint32_t at = lds0 + (b % STAGE_D) * STAGE_BATCH_BYTES;
    if (ahead == STAGE_D - 1 && b >= STAGE_D - 1) stage_read<(STAGE_D - 1) * 3 * STAGE_U>(at, v);
    else if (ahead == 3) stage_read<3 * 2 * STAGE_U>(at, v);
    else if (ahead == 2) stage_read<2 * 2 * STAGE_U>(at, v);
    else if (ahead == 1) stage_read<1 * 2 * STAGE_U>(at, v);
    else stage_read<0>(at, v);
    const uint32_t i = tid + b * per_batch;
#pragma unroll
    for (uint32_t u = 0; u < STAGE_U; ++u)
      fout.st16((i + u * NTH) << 4, add_vec<DT>(__builtin_bit_cast(uint4, v[u]), __builtin_bit_cast(uint4, v[STAGE_U + u])));
  }
}
#endif

// fin / sb / rb / fout are null when the primitive does not use that side.
// AUX: how connector slots are accessed (AUX_DEVICE, or AUX_CACHED in the fenced mode).
template <int AUX, int NTH>
__device__ __forceinline__ void run_prim(int dtype, const void* fin, const char* sb, char* rb, void* fout, uint32_t bytes, uint32_t tid) {
  if (fin) {
    if (sb) {
      if (rb) { if (fout) move_dispatch<AUX, AUX, true, true, true, true, NTH>(dtype, fin, sb, rb, fout, bytes, tid);    // recv-reduce-copy-send
                else move_dispatch<AUX, AUX, true, true, true, false, NTH>(dtype, fin, sb, rb, fout, bytes, tid); }      // recv-reduce-copy
      else move_dispatch<AUX, AUX, true, true, false, true, NTH>(dtype, fin, sb, rb, fout, bytes, tid);                  // recv-reduce-send
    } else {
      if (!rb) move_dispatch<AUX, AUX, true, false, false, true, NTH>(dtype, fin, sb, rb, fout, bytes, tid);             // direct recv-copy (coherent destination)
      else if (fout) move_dispatch<AUX, AUX, true, false, true, true, NTH>(dtype, fin, sb, rb, fout, bytes, tid);        // recv-copy-send
      else move_dispatch<AUX, AUX, true, false, true, false, NTH>(dtype, fin, sb, rb, fout, bytes, tid);                 // recv-copy
    }
  } else {
    if (rb) { if (fout) move_dispatch<AUX, AUX, false, true, true, true, NTH>(dtype, fin, sb, rb, fout, bytes, tid);     // copy-send
              else move_dispatch<AUX, AUX, false, true, true, false, NTH>(dtype, fin, sb, rb, fout, bytes, tid); }       // copy
    else move_dispatch<AUX, AUX, false, true, false, true, NTH>(dtype, fin, sb, rb, fout, bytes, tid);                   // send
  }
}

// ------------------------------------------------------------------------------------------
// Fold steps (make_fold_prim): the two data movers
// ------------------------------------------------------------------------------------------
// a buffer resource over memory whose address every lane holds alike (it came out of LDS)
__device__ __forceinline__ __amdgpu_buffer_rsrc_t uniform_rsrc(u64 addr, uint32_t bytes) {
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)addr), hi = __builtin_amdgcn_readfirstlane((uint32_t)(addr >> 32));
  return __builtin_amdgcn_make_buffer_rsrc((void*)(uintptr_t)(((u64)hi << 32) | lo), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ uint4 rs_ld16(__amdgpu_buffer_rsrc_t r, uint32_t off) {
  return __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, AUX_DEVICE));   // out of range reads return 0
}

constexpr int FOLD_SRC = 8;    // sources read together
constexpr int FOLD_U = 2;      // vectors per thread and source in flight

// dst[d][i] = src[0][i] (op) src[1][i] (op) ... (op) src[nsrc-1][i], left to right, for every destination d: the
// source table lists the ranks in the ring's order of combination.  Sources are other ranks' send buffers:
// device-coherent loads; the destinations are recv buffers of this and of other ranks, whose workgroups post the
// completion: device-coherent stores, which are in memory when the step counts itself done.
template <int DT, int NTH>
__device__ __forceinline__ void fold_slice(const u64* src_tab, uint32_t nsrc, const u64* dst_tab, uint32_t ndst, uint32_t bytes,
                                           uint32_t tid, int op) {
  const uint32_t nvec = bytes >> 4;
  for (uint32_t i = tid; i < nvec; i += FOLD_U * NTH) {
    uint4 acc[FOLD_U];
    for (uint32_t base = 0; base < nsrc; base += FOLD_SRC) {
      uint4 w[FOLD_SRC][FOLD_U];
#pragma unroll
      for (int k = 0; k < FOLD_SRC; ++k) {
        if (base + k < nsrc) {
          const __amdgpu_buffer_rsrc_t r = uniform_rsrc(src_tab[base + k], bytes);
#pragma unroll
          for (int u = 0; u < FOLD_U; ++u) w[k][u] = rs_ld16(r, (i + u * NTH) << 4);
        }
      }
#pragma unroll
      for (int k = 0; k < FOLD_SRC; ++k) {
        if (base + k < nsrc) {
          if (base + k == 0) {
#pragma unroll
            for (int u = 0; u < FOLD_U; ++u) acc[u] = w[0][u];
          } else op_batch<DT, FOLD_U>(acc, w[k], op);
        }
      }
    }
    for (uint32_t d = 0; d < ndst; ++d) {
      const __amdgpu_buffer_rsrc_t r = uniform_rsrc(dst_tab[d], bytes);
#pragma unroll
      for (int u = 0; u < FOLD_U; ++u)
        if (i + u * NTH < nvec) __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4u, acc[u]), r, (int)((i + u * NTH) << 4), 0, AUX_DEVICE);
    }
  }
  // the sub-vector tail of a message whose length is no multiple of 16 bytes
  const uint32_t done = nvec << 4;
  if (done < bytes) {
    constexpr uint32_t EB = (DT == DT_F32 || DT == DT_I32) ? 4u : 2u;
    for (uint32_t o = done + tid * EB; o < bytes; o += NTH * EB) {
      uint32_t v = 0;
      for (uint32_t k = 0; k < nsrc; ++k) {
        const Slot<AUX_DEVICE> src((const void*)(uintptr_t)src_tab[k], bytes);
        const uint32_t x = EB == 4 ? src.ld4(o) : (uint32_t)src.ld2(o);
        v = k == 0 ? x : (EB == 4 ? op_word<DT>(v, x, op) : (uint32_t)op_half<DT>((uint16_t)v, (uint16_t)x, op));
      }
      for (uint32_t d = 0; d < ndst; ++d) {
        const Slot<AUX_DEVICE> dst((void*)(uintptr_t)dst_tab[d], bytes);
        if (EB == 4) dst.st4(o, v); else dst.st2(o, (uint16_t)v);
      }
    }
  }
}

template <int NTH>
__device__ __forceinline__ void fold_dispatch(int dtype, const u64* src_tab, uint32_t nsrc, const u64* dst_tab, uint32_t ndst,
                                              uint32_t bytes, uint32_t tid) {
  const int op = dtype >> 4;
  switch (dtype & 15) {
    case DT_F32: fold_slice<DT_F32, NTH>(src_tab, nsrc, dst_tab, ndst, bytes, tid, op); break;
    case DT_BF16: fold_slice<DT_BF16, NTH>(src_tab, nsrc, dst_tab, ndst, bytes, tid, op); break;
    case DT_F16: fold_slice<DT_F16, NTH>(src_tab, nsrc, dst_tab, ndst, bytes, tid, op); break;
    default: fold_slice<DT_I32, NTH>(src_tab, nsrc, dst_tab, ndst, bytes, tid, op); break;
  }
}

// The gather step: segment s is len[s] bytes copied from src[s] (a rank's send buffer: device-coherent loads)
// to dst[s] (the own recv buffer); the loads of up to eight segments travel together.
template <int NTH>
__device__ __forceinline__ void gather_slices(const u64* src_tab, const u64* dst_tab, const uint32_t* len_tab, uint32_t nseg,
                                              uint32_t maxbytes, uint32_t tid) {
  const uint32_t maxvec = maxbytes >> 4;
  for (uint32_t base = 0; base < nseg; base += FOLD_SRC) {
    for (uint32_t i = tid; i < maxvec; i += FOLD_U * NTH) {
      uint4 w[FOLD_SRC][FOLD_U];
#pragma unroll
      for (int k = 0; k < FOLD_SRC; ++k) {
        if (base + k < nseg) {
          const __amdgpu_buffer_rsrc_t r = uniform_rsrc(src_tab[base + k], len_tab[base + k]);
#pragma unroll
          for (int u = 0; u < FOLD_U; ++u) w[k][u] = rs_ld16(r, (i + u * NTH) << 4);
        }
      }
#pragma unroll
      for (int k = 0; k < FOLD_SRC; ++k) {
        if (base + k < nseg) {
          v4u_user* D = (v4u_user*)(uintptr_t)dst_tab[base + k];
          const uint32_t nv = len_tab[base + k] >> 4;
#pragma unroll
          for (int u = 0; u < FOLD_U; ++u) if (i + u * NTH < nv) st_user(&D[i + u * NTH], w[k][u]);
        }
      }
    }
  }
  // sub-vector tails (only the message's last chunk can have one); every dtype is a multiple of 2 bytes
  for (uint32_t s2 = 0; s2 < nseg; ++s2) {
    const uint32_t len = len_tab[s2], done = (len >> 4) << 4;
    if (done < len) {
      const Slot<AUX_DEVICE> src((const void*)(uintptr_t)src_tab[s2], len);
      uint16_t* D = (uint16_t*)(uintptr_t)dst_tab[s2];
      for (uint32_t o = done + (tid << 1); o < len; o += NTH << 1) D[o >> 1] = src.ld2(o);
    }
  }
}

// ------------------------------------------------------------------------------------------
// LDS state of one workgroup
// ------------------------------------------------------------------------------------------
struct Job {                         // what the scheduler wave hands to the mover waves for one slice
  const void* fin; const char* sb; char* rb; void* fout;
  uint32_t bytes; int dtype;
  uint32_t coll, prim;               // for the timeline trace only
  uint32_t mode;                     // 0: the four pointers above; 1: fold step (sources and destinations in the job's tables);
                                     // 2: gather step (segments in the job's tables, bytes = the longest one)
  uint32_t nseg;                     // sources of a fold step, segments of a gather step
  uint32_t ndst;                     // destinations of a fold step
};

// What publishing and retiring a posted job needs.  Written by the scheduler when it posts the
// job; read by the mover wave that finishes the job last (counter updates) and by the scheduler
// when it retires the job (statistics, completion).
struct Flight {
  u64* tail_out; u64* head_in;       // counters to raise (null = that side is not used)
  u64 sent_new, recvd_new;           // their new values
  uint32_t last;                     // the primitive ends this workgroup's share of the invocation
  uint32_t coll, seq, nchan;
  u64* add_one;                      // fold steps: shared counter to add 1 to (null = none)
};

struct Shared {
  DfxDaemonArgs args;
  DfxCtxEntry slot[DFX_CTX_SLOTS];   // active context slots (Sec. 5, direct-mapped)
  uint32_t slot_tag[DFX_CTX_SLOTS];
  uint32_t slot_claim[DFX_CTX_SLOTS];  // readiness scan: which entry of the scan gets to fill a slot (scan step << 8 | lane)
  Job job[2];                        // posted jobs, indexed by job number & 1
  Flight fl[2];
  u64 tab_src[2][64];                // fold / gather steps: source addresses of the job, in order
  u64 tab_dst[2][64];                // fold steps: where the result goes; gather steps: where each segment goes
  uint32_t tab_len[2][64];           // gather steps: bytes of each segment
  uint32_t job_seq;                  // jobs posted so far (scheduler -> movers)
  uint32_t wave_done[2];             // mover waves that have finished job k, at index k & 1
  uint32_t jobs_done;                // jobs finished and published (movers -> scheduler)
  uint32_t leave;                    // scheduler -> movers: no more jobs
  uint32_t trace_n;                  // trace samples written (monotone)
  uint32_t qlen_out;                 // queue length handed to all waves when leaving
  u64 stat[DFX_NSTAT];               // counters (LDS atomics without return: one instruction, no wait)
  uint16_t rlist[DFX_MAX_COLLS];     // queue positions the readiness scan found runnable, ascending
  uint16_t taskq[DFX_MAX_COLLS];     // task queue (Sec. 4.2 (1))
#if DFX_LDS_STAGE
  __attribute__((aligned(16))) unsigned char stage[(DFX_MOVERS / 64) * STAGE_WAVE_BYTES];   // experiment build: staging area of the mover waves
#endif
};

__device__ __forceinline__ void raise_error(const DfxDaemonArgs& a, uint32_t code, uint32_t wg) {
  uint32_t expected = 0;
  if (__hip_atomic_compare_exchange_strong(&a.dev_ctl[DC_ERR], &expected, code, __ATOMIC_RELAXED, __ATOMIC_RELAXED, SCOPE_AGENT))
    __hip_atomic_store(&a.dev_ctl[DC_ERR_WG], wg, __ATOMIC_RELAXED, SCOPE_AGENT);
  __hip_atomic_store(&a.dev_ctl[DC_ABORT], 1u, __ATOMIC_RELEASE, SCOPE_AGENT);
}

__device__ __forceinline__ void bump(u64* stat, int i, u64 v) {
  (void)__hip_atomic_fetch_add(&stat[i], v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

__device__ __forceinline__ uint32_t bcast0(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }

// LDS slot of a collective's context: a multiplicative hash, because the ids that share a workgroup's
// queue are far from random (with single-channel collectives spread over the channels they are all
// congruent modulo the channel count)
static_assert(DFX_CTX_SLOTS == 64, "ctx_slot takes the top six bits");
__device__ __forceinline__ uint32_t ctx_slot(uint32_t coll) { return (coll * 2654435769u) >> 26; }

// LDS words shared between the scheduler and the mover waves
__device__ __forceinline__ uint32_t lds_ld(const uint32_t* p) { return __hip_atomic_load(p, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP); }
__device__ __forceinline__ void lds_st(uint32_t* p, uint32_t v) { __hip_atomic_store(p, v, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP); }

// Raise a connector counter.  A maximum instead of a store: the waves that publish two
// consecutive jobs are different ones, and their updates may reach memory in either order.
__device__ __forceinline__ void raise_counter(u64* p, u64 v) {
  (void)__hip_atomic_fetch_max(p, v, __ATOMIC_RELAXED, SCOPE_AGENT);
}

// one trace sample; the index comes from an LDS counter that both kinds of wave use
__device__ __forceinline__ void trace_put(u64* trace, uint32_t* trace_n, u64 v) {
  const uint32_t i = __hip_atomic_fetch_add(trace_n, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  trace[i % DFX_TRACE_N] = v;
}

__device__ __forceinline__ u64 timeline_sample(u64 t0, u64 t1, uint32_t coll, uint32_t prim) {
  u64 dur = t1 - t0;
  if (dur > 0xffffu) dur = 0xffffu;
  return (t0 & 0xffffffffull) | (dur << 32) | ((u64)(coll & 0xfffu) << 48) | ((u64)(prim & 0xfu) << 60);
}

}  // namespace

// Structure of a workgroup: wave 0 is the SCHEDULER, waves 1..4 are the MOVERS.
//
// The scheduler wave runs Alg. 1 on its own -- control checks, SQE fetch, queue walk, context
// load, bounded polling, preemption, lazy save, completion -- with its state in its registers
// and the task queue and context slots in LDS.  When a primitive's wait phase has succeeded it
// claims the connector slots (its private counters advance), posts the slice as a job in LDS and
// goes straight on to the wait phase of whatever comes next, while the movers carry the data.
// Up to two jobs are posted at a time, so the movers run from one slice into the next without
// waiting for the scheduler, and everything the scheduler does -- polling flags that live in
// HBM, scanning the queue, switching contexts -- overlaps with data movement.
//
// A mover wave takes the jobs in order; after its part of a slice it drains its stores and
// counts itself done in LDS.  The wave that completes the count raises the connector counters
// of that job (the data of all waves is then in memory) and reports the job finished; the
// scheduler retires finished jobs in order (statistics; for the last primitive of an invocation
// the completion counter and the CQE).  No workgroup barrier is used after start-up.
extern "C" __global__ void __launch_bounds__(DFX_WG_THREADS) dfx_daemon_kernel(DfxDaemonArgs kargs) {
  __shared__ Shared sh;
  // The arguments are read from an LDS copy: kept in scalar registers for the whole kernel they
  // overflow the scalar register file, and the spill reloads at every loop head cost more than
  // the LDS reads.
  if (threadIdx.x == 0) sh.args = kargs;
  __syncthreads();
  const DfxDaemonArgs& a = sh.args;
  const uint32_t tid = threadIdx.x;
  const uint32_t lane = tid & 63u;
  const bool sched = tid < 64;       // the scheduler wave
  const uint32_t wg = blockIdx.x;
  const WgPlace place = wg_place(a.wg_map, wg, a.R, a.cmax);
  const uint32_t rank = place.rank, ch = place.ch;
  const uint32_t D = a.sq_depth;
  const bool coh = a.fifo_coherent != 0;

  DfxWgState* ws = &a.wgstate[wg];
  DfxCtxEntry* myctx = a.ctxbuf + (size_t)wg * a.max_colls;
  uint16_t* qstore = a.taskq_store + (size_t)wg * a.max_colls;
  DfxSqSlot* sqbase = a.sq + (size_t)rank * D;
  u64* cqbase = a.cq + (size_t)rank * a.cq_slots;
  u64* trace = a.trace ? a.trace + (size_t)wg * DFX_TRACE_N : nullptr;

  // ---- restore the workgroup state left by the previous launch (Sec. 4.5)
  u64 ri = ws->read_index;
  uint32_t qlen = ws->qlen;
  for (uint32_t i = tid; i < qlen; i += NT) sh.taskq[i] = qstore[i];
  if (tid < DFX_CTX_SLOTS) sh.slot_tag[tid] = 0xffffffffu;
  if (tid < DFX_NSTAT) sh.stat[tid] = ws->stat[tid];
  if (tid == 0) {
    sh.job_seq = 0; sh.wave_done[0] = 0; sh.wave_done[1] = 0; sh.jobs_done = 0; sh.leave = 0;
    sh.trace_n = ws->trace_n;
  }
  __syncthreads();

  uint32_t stop = STOP_NONE;

  if (!sched) {
    // =====================================================================================
    // mover waves
    // =====================================================================================
    // The mover waves work in DFX_MOVER_GROUPS groups; group k takes the jobs k, k + GROUPS, ...: with two
    // groups the drain of one job's stores and the first loads of the next overlap in time.
    constexpr uint32_t GROUPS = DFX_MOVER_GROUPS, GTHREADS = DFX_MOVERS / GROUPS;
    const uint32_t mtid = (tid - 64) % GTHREADS;
    const uint32_t group = (tid - 64) / GTHREADS;
    const bool first_wave = mtid < 64;
    uint32_t seen = group;
    for (;;) {
      // the leave flag is looked at only when no job is waiting: every posted job is executed
      bool go = true;
      while ((int32_t)(lds_ld(&sh.job_seq) - seen) <= 0) {
        if (lds_ld(&sh.leave)) { go = false; break; }
        __builtin_amdgcn_s_sleep(1);
      }
      if (!go) break;
      const Job j = sh.job[seen & 1];
      u64 t0 = 0;
      if (a.trace_on > 1 && first_wave) t0 = wall_clock64();
      // fenced mode: every wave invalidates before its own loads of the slot (the poll was the scheduler's)
      if (!coh && j.fin && j.bytes) fence_acquire_agent();
#if DFX_LDS_STAGE
      if (coh && GROUPS == 1 && j.fin && j.sb && !j.rb && j.fout && (j.dtype >> 4) == OP_SUM && j.bytes &&
          j.bytes % (STAGE_U * GTHREADS * 16u) == 0 && (((uintptr_t)j.sb | (uintptr_t)j.fin) & 15u) == 0) {
        lds_byte* st = (lds_byte*)sh.stage;
        switch (j.dtype & 15) {
          case DT_F32: move_rrs_staged<DT_F32, GTHREADS>(j.fin, j.sb, j.fout, j.bytes, mtid, st); break;
          case DT_BF16: move_rrs_staged<DT_BF16, GTHREADS>(j.fin, j.sb, j.fout, j.bytes, mtid, st); break;
          case DT_F16: move_rrs_staged<DT_F16, GTHREADS>(j.fin, j.sb, j.fout, j.bytes, mtid, st); break;
          default: move_rrs_staged<DT_I32, GTHREADS>(j.fin, j.sb, j.fout, j.bytes, mtid, st); break;
        }
      } else
#endif
      if (j.mode == 1) fold_dispatch<GTHREADS>(j.dtype, sh.tab_src[seen & 1], j.nseg, sh.tab_dst[seen & 1], j.ndst, j.bytes, mtid);
      else if (j.mode == 2) gather_slices<GTHREADS>(sh.tab_src[seen & 1], sh.tab_dst[seen & 1], sh.tab_len[seen & 1], j.nseg, j.bytes, mtid);
      else if (coh) run_prim<AUX_DEVICE, GTHREADS>(j.dtype, j.fin, j.sb, j.rb, j.fout, j.bytes, mtid);
      else run_prim<AUX_CACHED, GTHREADS>(j.dtype, j.fin, j.sb, j.rb, j.fout, j.bytes, mtid);
      // this wave's stores (and loads) have been performed before it counts itself done
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      __builtin_amdgcn_s_waitcnt(0);
      u64 t1 = 0;
      if (a.trace_on > 1) t1 = wall_clock64();
      uint32_t last = 0;
      if (lane == 0) {
        const uint32_t old = __hip_atomic_fetch_add(&sh.wave_done[seen & 1], 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_WORKGROUP);
        last = (old + 1 == GTHREADS / 64) ? 1u : 0u;
        if (first_wave && a.trace_on > 1) {
          bump(sh.stat, ST_T_DATA, t1 - t0);
          if (a.trace_on == 3 && trace && j.prim != 0xffu) trace_put(trace, &sh.trace_n, timeline_sample(t0, t1, j.coll, j.prim));   // not the drain step
        }
      }
      if (bcast0(last)) {
        // all waves of the group have drained job `seen`: its data is in memory
        if (lane == 0) {
          const Flight f = sh.fl[seen & 1];
          // Jobs are published in order: a counter raised for job k tells the neighbour that every slice
          // up to k is there, so the job before must have been published (with one group every wave has
          // finished it by now and its publisher is a few instructions away; with two it may still run).
          while (lds_ld(&sh.jobs_done) != seen) __builtin_amdgcn_s_sleep(0);
          if (!coh) fence_release_agent();
          if (f.tail_out) raise_counter(f.tail_out, f.sent_new);
          if (f.head_in) raise_counter(f.head_in, f.recvd_new);
          if (f.add_one) (void)__hip_atomic_fetch_add(f.add_one, 1ull, __ATOMIC_RELAXED, SCOPE_AGENT);
          __hip_atomic_store(&sh.wave_done[seen & 1], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
          if (a.trace_on > 1) bump(sh.stat, ST_T_PUB, wall_clock64() - t1);
          lds_st(&sh.jobs_done, seen + 1);
        }
      }
      seen += GROUPS;
    }
  } else {
    // =====================================================================================
    // scheduler wave
    // =====================================================================================
    u64 last_act = wall_clock64();
    if (a.trace_on && a.trace_on < 3) {
      // what one clock read costs (the switch samples contain two of them, the split samples five): 16 in a row
      u64 tc = last_act;
#pragma unroll
      for (int k = 0; k < 16; ++k) tc = wall_clock64();
      if (lane == 0) { bump(sh.stat, ST_T_STAMP, tc - last_act); bump(sh.stat, ST_N_STAMP, 16); }
      last_act = tc;
    }
    bool acted = true, voted = false;
    uint32_t iter = 0, idle = 0, burst = 0;
    bool in_pass = false, pass_progress = false, scanned = false;
    uint32_t nready = 0, rk = 0, pass_bytes = 0;   // readiness list of the pass: length, cursor; bytes posted in the pass
    bool focus = false;                            // the pass visits the list furthest-along first, up to a byte budget
    uint32_t pos = 0;
    // context-switch sample in flight: t0 = abort decision, ts = after the save, lb/le = load
    u64 sw_t0 = 0, sw_ts = 0, sw_lb = 0, sw_le = 0;
    bool sw_pending = false;
    // The collective in hand.  Its static context stays in the LDS slot and is read where it is
    // needed (few values live across a wait); the dynamic part is in registers.  sent / recvd
    // count the slots this workgroup has CLAIMED (posted to the movers), which may run ahead
    // of the counters in memory by the jobs in flight.
    bool have = false;
    uint32_t coll = 0, sl = 0;
    uint32_t g = 0, p = 0, cidx = 0;
    u64 sent = 0, recvd = 0, thr = 0;
    bool progressed = false;
    u64 prev_recv = 0, prev_send = 0;   // the previous rank's recv / send buffer (direct steps), 0 = not read yet
    uint32_t posted = 0, retired = 0;   // jobs handed to the movers / jobs whose bookkeeping is done

    // ---- completion of this workgroup's share of an invocation (Sec. 5): completion counter,
    // and the last channel posts the CQE.  Lane 0 only.
    auto complete = [&](uint32_t c_coll, uint32_t c_seq, uint32_t c_nchan) {
      fence_release_system();   // results in the recv buffer are visible to host and later kernels
      uint32_t* dc = &a.done_cnt[(size_t)rank * a.max_colls + c_coll];
      // (a collective on one channel has nobody to count with: no round trip for the counter)
      const uint32_t old = c_nchan > 1 ? __hip_atomic_fetch_add(dc, 1u, __ATOMIC_ACQ_REL, SCOPE_AGENT) : 0u;
      if (old + 1 == c_nchan) {
        if (c_nchan > 1) __hip_atomic_store(dc, 0u, __ATOMIC_RELAXED, SCOPE_AGENT);
        const u64 tq0 = wall_clock64();
        if (a.cq_mode == 0) {
          // optimized CQ (Sec. 5): one CAS of the id into a writable slot, no ring semantics
          const u64 v = (1ull << 63) | ((u64)(c_seq & 0x7fffffffu) << 32) | c_coll;
          // where to try first: spread by id and invocation, no shared ticket to fetch (the CAS decides)
          const uint32_t t = c_coll * 7u + c_seq;
          uint32_t k = 0;
          for (;;) {
            u64 expected = 0;
            if (__hip_atomic_compare_exchange_strong(&cqbase[(t + k) % a.cq_slots], &expected, v, __ATOMIC_RELEASE,
                                                     __ATOMIC_RELAXED, SCOPE_SYSTEM))
              break;
            ++k;
            if ((k % a.cq_slots) == 0) {
              if (ld_agent32(&a.dev_ctl[DC_ABORT]) || ld_sys32(&a.host_ctl[HC_ABORT])) break;
              __builtin_amdgcn_s_sleep(50);
            }
          }
        } else {
          // The two ring-buffer CQs that Sec. 5 compares the optimized one with.  Both reserve a
          // position with an atomic in host memory and read the consumer's head to see whether
          // the ring has room.
          u64* ctl = a.cq_ctl + (size_t)rank * DFX_CQ_CTL_WORDS;
          const u64 t = __hip_atomic_fetch_add(&ctl[0], 1ull, __ATOMIC_RELAXED, SCOPE_SYSTEM);
          bool give_up = false;
          uint32_t k = 0;
          while (t - __hip_atomic_load(&ctl[16], __ATOMIC_RELAXED, SCOPE_SYSTEM) >= (u64)a.cq_slots) {
            if ((++k & 63u) == 0 && (ld_agent32(&a.dev_ctl[DC_ABORT]) || ld_sys32(&a.host_ctl[HC_ABORT]))) { give_up = true; break; }
            __builtin_amdgcn_s_sleep(20);
          }
          if (!give_up && a.cq_mode == 1) {
            // vanilla ring: entry, fence, then the shared tail, which moves in position order
            const u64 v = ((u64)(c_seq & 0x7fffffffu) << 32) | c_coll;
            __hip_atomic_store(&cqbase[t % a.cq_slots], v, __ATOMIC_RELAXED, SCOPE_SYSTEM);
            fence_release_system();
            while (__hip_atomic_load(&ctl[8], __ATOMIC_RELAXED, SCOPE_SYSTEM) != t) {
              if ((++k & 63u) == 0 && (ld_agent32(&a.dev_ctl[DC_ABORT]) || ld_sys32(&a.host_ctl[HC_ABORT]))) { give_up = true; break; }
              __builtin_amdgcn_s_sleep(2);
            }
            if (!give_up) __hip_atomic_store(&ctl[8], t + 1, __ATOMIC_RELEASE, SCOPE_SYSTEM);
          } else if (!give_up) {
            // optimized ring: id and position travel in one 64-bit atomic write, no tail, no fence;
            // the poller accepts the entry at its head when the position in it says head + 1
            const u64 v = (((t + 1) & 0xffffffffull) << 32) | ((u64)(c_seq & 0xffffu) << 16) | (c_coll & 0xffffu);
            __hip_atomic_store(&cqbase[t % a.cq_slots], v, __ATOMIC_RELEASE, SCOPE_SYSTEM);
          }
        }
        bump(sh.stat, ST_T_CQE, wall_clock64() - tq0);
        bump(sh.stat, ST_CQE, 1);
      }
    };

    // ---- retire the jobs the movers have finished (their counters are already raised)
    auto retire_finished = [&]() {
      while (retired != posted && lds_ld(&sh.jobs_done) != retired) {
        if (lane == 0) {
          const Flight f = sh.fl[retired & 1];
          bump(sh.stat, ST_PRIMS, 1);
          if (f.last) complete(f.coll, f.seq, f.nchan);
        }
        ++retired;
        acted = true;
      }
    };

    // The movers wait for nothing but their own memory operations, so the loops below that wait
    // for them end on their own; they still look at the abort words now and then, so that the
    // host can always get the grid back.
    uint32_t spins = 0;
    auto abort_seen = [&]() -> bool {
      uint32_t s = 0;
      if (lane == 0) s = (ld_agent32(&a.dev_ctl[DC_ABORT]) || ld_sys32(&a.host_ctl[HC_ABORT])) ? 1u : 0u;
      return bcast0(s) != 0;
    };

    for (;;) {
      retire_finished();
      if (stop != STOP_NONE) {
        // leaving: the posted jobs run to their end first (their slots are claimed in the saved contexts)
        if (retired == posted) break;
        if ((++spins & 0xffffu) == 0 && abort_seen()) break;
        __builtin_amdgcn_s_sleep(1);
        continue;
      }

      // ================= no collective in hand: control check, fetch, next queue entry =================
      if (!have) {
        if (!in_pass) {
          ++iter;
          uint32_t s = STOP_NONE, got = 0;
          // The SQ is probed before every pass.  (Sec. 4.3 has FIFO ordering fetch only when the queue
          // is empty or stuck and priority ordering before every pass.  Here the probe rides along
          // with the control words and costs nothing, new entries join the queue's tail either way,
          // and a workgroup that kept working without reading the SQ held back its rank's SQ slots
          // -- every workgroup must read every SQE -- and with them the submitter and the rest of
          // the grid.)  A fetch is followed by further fetches, up to fetch_batch in a row.
          const bool want = (a.sq_eager && burst < a.fetch_batch) || (qlen == 0) || !pass_progress || a.order_policy == 1 || (burst > 0 && burst < a.fetch_batch);
          const bool probe = want && qlen < a.max_colls;
          const bool slow = ((iter & 31u) == 0) || qlen == 0 || !pass_progress;
          const bool host_look = ((iter & 31u) == 0) || qlen == 0;
          // the three control words live in different memories; three lanes fetch them at once
          uint32_t w0 = 0, w1 = 0;
          if (lane == 0) {
            const u64 c2 = ld_agent64((const u64*)&a.dev_ctl[DC_ABORT]);   // abort | quit
            w0 = (uint32_t)c2; w1 = (uint32_t)(c2 >> 32);
          } else if (lane == 1) {
            if (probe) w0 = __hip_atomic_load(&sqbase[ri & (D - 1)].e.ready, __ATOMIC_RELAXED, SCOPE_SYSTEM);
          } else if (lane == 2) {
            if (host_look) w0 = ld_sys32(&a.host_ctl[HC_ABORT]);
          }
          const uint32_t c_abort = __builtin_amdgcn_readlane(w0, 0), c_quit = __builtin_amdgcn_readlane(w1, 0);
          const uint32_t c_ready = __builtin_amdgcn_readlane(w0, 1), c_habort = __builtin_amdgcn_readlane(w0, 2);
          if (c_abort || c_habort) s = STOP_ABORT;
          else if (c_quit) s = STOP_QUIT;
          if (lane == 0) {
            if (!s && slow) {
              const u64 now = wall_clock64();
              if (acted) { last_act = now; acted = false; }
              if (a.watchdog_ticks && qlen > 0 && now - last_act > a.watchdog_ticks) {
                ws->dbg[0] = ((u64)sh.taskq[0] << 32) | qlen; ws->dbg[1] = ri; ws->dbg[2] = now - last_act;
                raise_error(a, 1u, wg);
                s = STOP_ABORT;
              } else if (a.oneshot) {
                // A launch that brings all of its work with it: this workgroup is through when it has read every
                // entry of its rank's SQ, its queue is empty and its jobs are retired (completions posted).
                if (!voted && qlen == 0 && ri >= (u64)a.oneshot && retired == posted) {
                  voted = true;
                  if (__hip_atomic_fetch_add(&a.dev_ctl[DC_VOTES], 1u, __ATOMIC_ACQ_REL, SCOPE_AGENT) + 1 == a.nwg) {
                    __hip_atomic_store(&a.dev_ctl[DC_QUIT], 1u, __ATOMIC_RELEASE, SCOPE_AGENT);
                    s = STOP_QUIT;
                  }
                }
              } else if (a.quit_ticks) {
                // Voluntary quit (Sec. 4.4).  Every workgroup has duties towards the others (each
                // must read every SQE of its rank before the slot is reusable), so the grid leaves
                // as a whole: a workgroup that has been idle or stuck for the quit period casts a
                // vote and keeps running; it withdraws the vote when it becomes active again; the
                // vote that completes the set raises the quit flag, which everybody obeys.
                const bool tired = now - last_act > a.quit_ticks;
                if (tired && !voted) {
                  voted = true;
                  if (__hip_atomic_fetch_add(&a.dev_ctl[DC_VOTES], 1u, __ATOMIC_ACQ_REL, SCOPE_AGENT) + 1 == a.nwg) {
                    __hip_atomic_store(&a.dev_ctl[DC_QUIT], 1u, __ATOMIC_RELEASE, SCOPE_AGENT);
                    s = STOP_QUIT;
                  }
                } else if (!tired && voted) {
                  voted = false;
                  __hip_atomic_fetch_sub(&a.dev_ctl[DC_VOTES], 1u, __ATOMIC_ACQ_REL, SCOPE_AGENT);
                }
              }
            }
            if (!s && probe) {
              const uint32_t gen = (uint32_t)(ri >> a.sq_shift) + 1u;
              if (c_ready == gen) got = 1;
            }
          }
          s = bcast0(s);
          got = bcast0(got);
          if (s) { stop = s; continue; }

          // ---- FetchSQE (Alg. 1 line 2), up to 64 entries at a time: one per lane.
          // Every workgroup of a rank reads every SQE of the rank (Sec. 5), so a burst of a thousand
          // submissions is a thousand entries for each of them, most of them for other channels;
          // taken one by one (a fence, six loads, an atomic with its answer) they cost more than
          // the collectives they describe.
          if (got) {
            const u64 tf0 = wall_clock64();
            // how many consecutive entries from the read index on are there?
            uint32_t room = a.max_colls - qlen;
            if (room > 64) room = 64;
            const uint32_t left = burst < a.fetch_batch ? a.fetch_batch - burst : 1u;
            if (left < room) room = left;
            if (a.order_policy == 1) room = 1;       // the sorted insert below is written for one entry
            bool here = false;
            if (lane == 0) here = true;               // the control check has seen this one
            else if (lane < room) {
              const u64 idx = ri + lane;
              here = __hip_atomic_load(&sqbase[idx & (D - 1)].e.ready, __ATOMIC_RELAXED, SCOPE_SYSTEM) == (uint32_t)(idx >> a.sq_shift) + 1u;
            }
            const u64 here_mask = __ballot(here);
            uint32_t n = (here_mask == ~0ull) ? 64u : (uint32_t)__builtin_ctzll(~here_mask);   // length of the run that starts at lane 0
            // the submitter wrote the send buffers before the SQEs: drop what this CU / XCD cached
            fence_acquire_system();
            DfxStatic q;
            bool is_exit_sqe = false, is_exit = false;
            if (lane < n) {
              const uint4* src = (const uint4*)&sqbase[(ri + lane) & (D - 1)].e;
              uint4* qv = (uint4*)&q;
#pragma unroll
              for (int i = 0; i < 6; ++i) qv[i] = src[i];
              // an exit SQE ends the launch it was posted for; one left over from an earlier launch
              // (some workgroups had already gone when it arrived) is consumed and ignored
              is_exit_sqe = (q.flags & DFX_SQE_EXIT) != 0;
              is_exit = is_exit_sqe && q.seq == a.epoch;
            }
            const u64 exit_mask = __ballot(is_exit);
            if (exit_mask) n = (uint32_t)__builtin_ctzll(exit_mask) + 1;   // nothing behind an exit SQE is touched
            bool mine = false;
            uint32_t c_id = 0;
            if (lane < n) {
              c_id = q.coll_id;
              const uint32_t my_vch = is_exit_sqe ? ch : serving_channel(a.chan_spread != 0, ch, a.cmax, c_id, q.nchan);
              mine = !is_exit_sqe && my_vch < q.nchan && c_id < a.max_colls;
              if (mine) {
                // cook the static context of this invocation into the context buffer (addresses
                // resolved once, here); restart the sequence, keep the monotone connector counters
                const DfxCooked k = cook_sqe(q, a.pool, rank, a.R, my_vch);
                myctx[c_id].st = k;
                // direct gather steps: the next rank reads this rank's recv buffer; its address and
                // the invocation it belongs to go into the send connector's flag line (one 16-byte
                // device-coherent store, complete before any job of the invocation is posted)
                if (q.flags & DFX_SQE_DIRECT)
                {
                  const Slot<AUX_DEVICE> line((const void*)k.flags_out, DFX_FLAG_STRIDE);
                  line.st16(DFX_DIRECT_OFF, uint4{(uint32_t)q.recvbuf, (uint32_t)(q.recvbuf >> 32), q.seq + 1u, 0u});
                  line.st16(DFX_DIRECT_OFF + 16, uint4{(uint32_t)q.sendbuf, (uint32_t)(q.sendbuf >> 32), q.seq + 1u, 0u});
                }
                DfxDyn* dy = &myctx[c_id].dyn;
                dy->round = 0; dy->prim = 0; dy->preempted = 0;
                dy->cidx = first_chunk(q.kind, rank, a.R);
                if (sh.slot_tag[ctx_slot(c_id)] == c_id) sh.slot_tag[ctx_slot(c_id)] = 0xffffffffu;
              }
              // every workgroup of the rank reads every SQE; the last reader frees the slot (Sec. 5)
              // by writing the entry's generation where the submitter looks for it, in host memory
              const size_t sq_at = (size_t)rank * D + ((ri + lane) & (D - 1));
              uint32_t* rc = &a.sq_readers[sq_at];
              const uint32_t old = __hip_atomic_fetch_add(rc, 1u, __ATOMIC_ACQ_REL, SCOPE_AGENT);
              if (old + 1 == a.cmax) {
                __hip_atomic_store(rc, 0u, __ATOMIC_RELAXED, SCOPE_AGENT);
                __hip_atomic_store(&a.sq_freed[sq_at], (uint32_t)((ri + lane) >> a.sq_shift) + 1u, __ATOMIC_RELEASE, SCOPE_SYSTEM);
              }
            }
            // (contexts and published buffer addresses are in memory before anything is built on them)
            __builtin_amdgcn_s_waitcnt(0);
            // fold steps: the channel's count of published invocations (after the addresses, which it vouches for)
            if (mine && (q.flags & DFX_SQE_FOLD))
              (void)__hip_atomic_fetch_add((u64*)(fold_shared_line(myctx[c_id].st.flags_out, rank, a.R, q.nchan) + DFX_FOLD_PUB), 1ull,
                                           __ATOMIC_RELAXED, SCOPE_AGENT);
            // the entries that are this workgroup's join the task queue in SQ order
            const u64 mine_mask = __ballot(mine);
            if (mine) {
              if (a.order_policy == 1) {
                // priority ordering: keep the queue sorted (stable); one entry per fetch in this mode
                uint32_t at = qlen;
                const int16_t pr = q.priority;
                while (at > 0 && myctx[sh.taskq[at - 1]].st.priority < pr) { sh.taskq[at] = sh.taskq[at - 1]; --at; }
                sh.taskq[at] = (uint16_t)c_id;
              } else {
                sh.taskq[qlen + (uint32_t)__builtin_popcountll(mine_mask & ((1ull << lane) - 1ull))] = (uint16_t)c_id;
              }
            }
            qlen += (uint32_t)__builtin_popcountll(mine_mask);
            if (lane == 0) {
              bump(sh.stat, ST_SQE, n);
              bump(sh.stat, ST_T_SQE, wall_clock64() - tf0);
              __hip_atomic_fetch_max(&sh.stat[ST_MAXQ], (u64)qlen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
            __builtin_amdgcn_wave_barrier();
            acted = true;
            sw_pending = false;
            ri += n;
            if (exit_mask) {
              // the whole grid leaves (every workgroup has reader duties towards its rank's SQ)
              if (lane == 0) __hip_atomic_store(&a.dev_ctl[DC_QUIT], 1u, __ATOMIC_RELEASE, SCOPE_AGENT);
              stop = STOP_EXIT;
              continue;
            }
            burst += n;
            idle = 0;
            if (n == room) continue;   // the run may go on: probe the SQ again before walking the queue
            // (fewer entries than lanes looked: the SQ is empty behind them, go on to the pass)
          }
          burst = 0;
          if (qlen == 0) {
            // idle: back off the SQ probe (an SQ in host memory is probed across PCIe: back off further)
            ++idle;
            if (idle < 64) __builtin_amdgcn_s_sleep(8);
            else if (a.sq_local || idle < 4096) __builtin_amdgcn_s_sleep(32);
            else __builtin_amdgcn_s_sleep(127);
            continue;
          }
          idle = 0;
          // ---- start one pass over the task queue (Alg. 1 lines 4-19)
          in_pass = true;
          pass_progress = false;
          pos = 0;
          if (lane == 0) bump(sh.stat, ST_PASSES, 1);
          // ---- readiness scan: 64 queue entries per step, one per lane.  Each lane reads the
          // saved context of its entry, works out which connector sides its next primitive
          // needs, loads those counters and votes; the runnable positions are compacted into a
          // list (ballot + popcount) and the pass visits only those.  The conditions are
          // monotone: only this workgroup consumes its recv side and fills its send side, so
          // "ready" stays true until it acts.  A queue of a thousand stuck collectives costs
          // sixteen memory round trips instead of a thousand context loads and bounded spins.
          scanned = a.scan_min && qlen >= a.scan_min;
          if (scanned) {
            nready = 0; rk = 0; pass_bytes = 0;
            focus = a.focus_bytes != 0 && qlen <= 64u;
            if (lane < DFX_CTX_SLOTS) sh.slot_claim[lane] = 0xffffffffu;
            for (uint32_t base = 0; base < qlen; base += 64) {
              const uint32_t i = base + lane;
              bool rdy = false;
              uint32_t key = 0;     // 0 = not runnable; else (priority under priority ordering,) primitives done so far, then queue position
              uint32_t cid = 0;
              uint4 e0 = uint4{0, 0, 0, 0}, e1 = e0, e4 = e0, e2c = e0, e3c = e0, e5c = e0, e6c = e0, e7c = e0;
              if (i < qlen) {
                cid = sh.taskq[i];
                const uint4* e = (const uint4*)&myctx[cid];
                e0 = e[0]; e1 = e[1]; e4 = e[4];   // not needed for the vote, but for the deposit below
                const uint4 fl = e[2];    // bytes 32..47: part_elems | flags_out
                const uint4 fi = e[3];    // bytes 48..63: flags_in | fifo_out
                const uint4 ge = e[5];    // bytes 80..95: seq | nprim,nchan | nslots,kind,dtype,bc_pos | priority,vch
                const uint4 d0 = e[6];    // dyn: round | prim | sent
                const uint4 d1 = e[7];    // dyn: recvd | preempted | cidx
                e2c = fl; e3c = fi; e5c = ge; e6c = d0; e7c = d1;
                const bool e_fold = ((ge.z >> 24) & DFX_CTX_FOLD) != 0;
                Prim pq = e_fold ? make_fold_prim((int)((ge.z >> 8) & 0xffu), d0.y)
                                 : make_prim((int)((ge.z >> 8) & 0xffu), a.R, (ge.z >> 24) & 3u, d0.y, ((ge.z >> 24) & DFX_CTX_DIRECT) != 0);
                if (!e_fold && ((ge.z >> 24) & DFX_CTX_DIRECT))
                  pq = chain_drain_round(pq, (int)((ge.z >> 8) & 0xffu), true, d0.x, e[4].w);   // bytes 64..79: fifo_in | slice_elems | rounds
                const u64 f_out = ((u64)fl.w << 32) | fl.z, f_in = ((u64)fi.y << 32) | fi.x;
                const u64 e_sent = ((u64)d0.w << 32) | d0.z, e_recvd = ((u64)d1.y << 32) | d1.x;
                bool okr = true, oks = true;
                if (pq.fold)   // every rank of the channel has got as far as this step needs: (seq + 1) x R on the step's counter
                  okr = ld_agent64((const u64*)(fold_shared_line(f_out, rank, a.R, ge.y >> 16) + 8u * pq.fwait))
                        >= ((u64)ge.x + 1u) * a.R * (pq.fwait ? (u64)e[4].w : 1ull);   // (a data step counts once per slice: bytes 64..79 end in rounds)
                if (pq.recv) okr = ld_agent64((const u64*)f_in) > e_recvd;
                if (pq.send) oks = (e_sent - ld_agent64((const u64*)f_out + 8)) < (u64)(ge.z & 0xffu);
                else if (pq.drain) oks = e_sent == ld_agent64((const u64*)f_out + 8);
                rdy = okr && oks;
                if (rdy) {
                  u64 done = (u64)d0.x * (ge.y & 0xffffu) + d0.y;
                  if (a.order_policy == 1) {
                    // priority ordering (Sec. 4.3): the user's priority decides first, progress and
                    // queue position only among equals
                    if (done > 0xffu) done = 0xffu;
                    const uint32_t pr = (uint32_t)((int)(int16_t)(ge.w & 0xffffu) + 32768);
                    key = ((pr << 14) | ((uint32_t)done << 6) | (63u - lane)) + 1u;
                  } else {
                    if (done > 0xfffffu) done = 0xfffffu;
                    key = (((uint32_t)done << 8) | (63u - lane)) + 1u;
                  }
                }
              }
              // The contexts of the runnable entries are in registers now: they go into their LDS
              // slots (direct-mapped; of several entries of the scan that share a slot the first one
              // gets it), so that the pass finds them there instead of loading them from HBM again.
              if (rdy) (void)__hip_atomic_fetch_min(&sh.slot_claim[ctx_slot(cid)], ((base >> 6) << 8) | lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
              __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
              __builtin_amdgcn_wave_barrier();
              if (rdy && sh.slot_claim[ctx_slot(cid)] == (((base >> 6) << 8) | lane)) {
                uint4* dstc = (uint4*)&sh.slot[ctx_slot(cid)];
                dstc[0] = e0; dstc[1] = e1; dstc[2] = e2c; dstc[3] = e3c; dstc[4] = e4; dstc[5] = e5c; dstc[6] = e6c; dstc[7] = e7c;
                sh.slot_tag[ctx_slot(cid)] = cid;
              }
              const u64 mask = __ballot(rdy);
              if (focus) {
                // One step holds the whole queue.  The runnable entries are visited furthest-along
                // first (ties: queue order): every rank ranks them alike, so the ranks settle on
                // the same few collectives and carry those through, instead of moving all of
                // them forward side by side with all of their FIFO slots in use at once.
                uint32_t rank_in_pass = 0;
                const uint32_t nq = qlen < 64u ? qlen : 64u;
                for (uint32_t j = 0; j < nq; ++j)
                  rank_in_pass += ((uint32_t)__builtin_amdgcn_readlane((int)key, (int)j) > key) ? 1u : 0u;
                if (rdy) sh.rlist[rank_in_pass] = (uint16_t)i;
              } else if (rdy) sh.rlist[nready + (uint32_t)__builtin_popcountll(mask & ((1ull << lane) - 1ull))] = (uint16_t)i;
              nready += (uint32_t)__builtin_popcountll(mask);
            }
            __builtin_amdgcn_wave_barrier();
            if (lane == 0) { bump(sh.stat, ST_POLLS, (qlen + 63) / 64); bump(sh.stat, ST_SCAN_SKIPS, qlen - nready); }
            if (nready == 0) {           // nothing can run: the pass is over before it began
              in_pass = false;
              __builtin_amdgcn_s_sleep(4);
              continue;
            }
          }
        }
        if (scanned) {
          // (a pass that ends is not a switch between two collectives: the latency sample is dropped)
          // A focused pass also ends once it has handed the movers its share of bytes: the next scan
          // looks again at which collectives are furthest along.
          if (rk >= nready || (focus && pass_bytes >= a.focus_bytes)) { in_pass = false; sw_pending = false; continue; }
          pos = (uint32_t)sh.rlist[rk];
        } else if (pos >= qlen) { in_pass = false; sw_pending = false; continue; }

        // ---- LoadCollectiveContext: HBM context buffer -> LDS slot, 8 lanes x 16 bytes
        coll = sh.taskq[pos];
        sl = ctx_slot(coll);
        if (sw_pending && a.trace_on > 1) sw_lb = wall_clock64();
        if (sh.slot_tag[sl] != coll) {
          if (lane < 8) ((uint4*)&sh.slot[sl])[lane] = ((const uint4*)&myctx[coll])[lane];
          if (lane == 0) { sh.slot_tag[sl] = coll; bump(sh.stat, ST_LOAD, 1); }
          __builtin_amdgcn_wave_barrier();
        } else if (lane == 0) bump(sh.stat, ST_HIT, 1);
        if (sw_pending && a.trace_on > 1) sw_le = wall_clock64();
        {
          const DfxDyn& Y = sh.slot[sl].dyn;
          g = Y.round; p = Y.prim; sent = Y.sent; recvd = Y.recvd; cidx = Y.cidx;
        }
        // SetInitialSpinThreshold (Alg. 1 line 3): largest at the front, halving per position.
        // In a scanned pass every entry visited was seen runnable, and the rest of the list is
        // known work: waiting on one collective would only keep the movers idle, so the
        // threshold stays at its minimum there.
        thr = a.spin_init >> (pos < 31 ? pos : 31);
        if (thr < a.spin_min || scanned) thr = a.spin_min;
        progressed = false;
        prev_recv = 0;
        have = true;
      }

      // ================= next primitive of the collective in hand =================
      const DfxCooked& S = sh.slot[sl].st;
      const bool fold = (S.bc_pos & DFX_CTX_FOLD) != 0;
      const Prim q = fold ? make_fold_prim((int)S.kind, p)
                          : chain_drain_round(make_prim((int)S.kind, a.R, S.bc_pos & 3u, p, (S.bc_pos & DFX_CTX_DIRECT) != 0),
                                              (int)S.kind, (S.bc_pos & DFX_CTX_DIRECT) != 0, g, S.rounds);
      // fold steps wait for one of the channel's shared counters: every rank has published the invocation
      // ((invocation + 1) x R), or every rank has finished its data step for every slice (x slices per share)
      const u64* const fold_cnt = fold ? (const u64*)(fold_shared_line(S.flags_out, rank, a.R, S.nchan) + 8u * q.fwait) : nullptr;
      const u64 fold_target = ((u64)S.seq + 1u) * a.R * (q.fwait ? (u64)S.rounds : 1ull);
      u64* const tail_out = (u64*)S.flags_out;
      u64* const tail_in = (u64*)S.flags_in;
      const uint32_t K = S.nslots;

      if (sw_pending) {   // the first poll of the next collective ends the context switch
        const u64 t1 = wall_clock64();
        if (trace && a.trace_on < 3 && lane == 0) {
          // total | save | queue advance (save done -> context load begins) | load | set-up of the primitive (load done -> here)
          u64 tot = t1 - sw_t0, sv = sw_ts - sw_t0, adv = sw_lb - sw_ts, ldt = sw_le - sw_lb, su = t1 - sw_le;
          if (a.trace_on < 2) { sv = 0; adv = 0; ldt = 0; su = 0; }
          if (tot > 0xffffu) tot = 0xffffu;
          if (sv > 0xfffu) sv = 0xfffu;
          if (adv > 0xfffu) adv = 0xfffu;
          if (ldt > 0xfffu) ldt = 0xfffu;
          if (su > 0xfffu) su = 0xfffu;
          trace_put(trace, &sh.trace_n, tot | (sv << 16) | (adv << 28) | (ldt << 40) | (su << 52));
        }
        sw_pending = false;
      }
      u64 tm0 = 0;
      if (a.trace_on > 1) tm0 = wall_clock64();

      // ---- wait phase: lane 0 polls the recv side, lane 1 the send side (Sec. 4.2 (3)).
      // The first poll is sent off before the slice's geometry is worked out, which depends only on
      // the sequence position: the arithmetic runs while the counters travel, and a poll that
      // succeeds is followed by the job at once.
      u64 seen_cnt = 0;
      if (lane == 0 && q.recv) seen_cnt = ld_agent64(tail_in);
      if (lane == 1 && (q.send || q.drain)) seen_cnt = ld_agent64(tail_out + 8);
      if (lane == 0 && q.fold) seen_cnt = ld_agent64(fold_cnt);

      // ---- slice geometry and the job's four pointers
      const int kind = S.kind, dtype = S.dtype;   // dtype: element type | reducing function << 4
      const SliceGeom geo = slice_geometry(S, a.R, g, cidx);
      const uint32_t eb = geo.eb, bytes = geo.bytes;
      const u64 soff = geo.soff, doff = geo.doff;
      const size_t slot_bytes = (size_t)S.slice_elems * eb;
      const void* jfin = q.recv ? (const void*)((const uint8_t*)S.fifo_in + (size_t)(recvd & (K - 1)) * slot_bytes) : nullptr;
      void* jfout = q.send ? (void*)((uint8_t*)S.fifo_out + (size_t)(sent & (K - 1)) * slot_bytes) : nullptr;
      const char* jsb = q.from_send ? (const char*)S.sendbuf + soff * eb : nullptr;
      char* jrb = q.to_recv ? (char*)S.recvbuf + doff * eb : nullptr;
      // a notified result goes to the recv buffer through the coherent path of a slot
      if (q.notify) { jfout = jrb; jrb = nullptr; }

      // the position after this primitive (slices in windows, the chunk index stepping down the ring)
      const SeqPos nx = fold ? next_fold_position(S.rounds, g, p, cidx)
                             : next_position(kind, a.R, rank, a.window, S.rounds, S.nprim, g, p, cidx);
      const uint32_t g_next = nx.g, p_next = nx.p, cidx_next = nx.cidx;
      const bool last = (g_next >= S.rounds);
      const uint32_t inv_seq = S.seq, inv_nchan = S.nchan;

      // The movers may be busy with earlier slices meanwhile; finished ones are retired between polls.
      uint32_t res = W_OK;
      // While the first poll travels: which entry would the pass visit next, and is its context in its LDS slot?
      // If not, its load from the context buffer sets off now.  Should this wait be given up, the switch finds
      // the answer in registers (nothing below changes the queue, the list, another collective's slot or its
      // saved context before then).
      bool nx_ok = false, nx_hit = false;
      uint32_t nx_pos = 0, nx_coll = 0, nx_sl = 0;
      DfxDyn nx_dyn = {};
      uint4 nx_ctx = uint4{0, 0, 0, 0};
      if (q.recv || q.send || q.drain || q.fold) {
        const uint32_t ni = scanned ? rk + 1u : pos + 1u;
        if (scanned ? (ni < nready && !(focus && pass_bytes >= a.focus_bytes)) : (ni < qlen)) {
          nx_pos = scanned ? (uint32_t)sh.rlist[ni] : ni;
          nx_coll = sh.taskq[nx_pos];
          nx_sl = ctx_slot(nx_coll);
          nx_ok = true;
          nx_hit = sh.slot_tag[nx_sl] == nx_coll;
          if (nx_hit) nx_dyn = sh.slot[nx_sl].dyn;
          else if (lane < 8) nx_ctx = ((const uint4*)&myctx[nx_coll])[lane];
        }
        u64 n = 0;
        for (;;) {
          bool ok = true;
          if (lane == 0 && q.fold) ok = seen_cnt >= fold_target;
          if (lane == 0 && q.recv) ok = seen_cnt > recvd;
          if (lane == 1 && q.send) ok = (sent - seen_cnt) < (u64)K;
          if (lane == 1 && q.drain) ok = sent == seen_cnt;
          ++n;
          if (__ballot(!ok) == 0) break;
          retire_finished();
          if (a.preempt && n >= thr) { res = W_TIMEOUT; break; }
          if ((n & 255u) == 0) {
            uint32_t s = 0;
            if (lane == 0) {
              if (ld_agent32(&a.dev_ctl[DC_ABORT]) || ld_sys32(&a.host_ctl[HC_ABORT])) s = 1;
              else if (a.watchdog_ticks) {
                const u64 now = wall_clock64();
                if (acted) { last_act = now; acted = false; }
                if (now - last_act > a.watchdog_ticks) {
                  ws->dbg[0] = ((u64)coll << 32) | qlen; ws->dbg[1] = ((u64)g << 32) | p; ws->dbg[2] = sent; ws->dbg[3] = recvd;
                  ws->dbg[4] = ld_agent64(tail_in); ws->dbg[5] = ld_agent64(tail_out + 8); ws->dbg[6] = ri; ws->dbg[7] = now - last_act;
                  raise_error(a, 2u, wg);
                  s = 1;
                }
              }
            }
            if (bcast0(s)) { res = W_STOP; break; }
          }
          __builtin_amdgcn_s_sleep(1);
          if (lane == 0 && q.recv) seen_cnt = ld_agent64(tail_in);
          if (lane == 1 && (q.send || q.drain)) seen_cnt = ld_agent64(tail_out + 8);
          if (lane == 0 && q.fold) seen_cnt = ld_agent64(fold_cnt);
        }
        if (lane == 0) bump(sh.stat, ST_POLLS, n);
      }

      if (res == W_OK) {
        u64 tm1 = 0;
        if (a.trace_on > 1) { tm1 = wall_clock64(); if (lane == 0) bump(sh.stat, ST_T_WAIT, tm1 - tm0); }
        // The last wait of a collective in fold steps moves nothing, and the counter it has just seen says that every
        // rank's data step of this channel -- this workgroup's own job included -- is in memory: the completion is
        // posted here and now instead of queueing as an empty job behind the data jobs of other collectives.
        const bool done_here = q.fold == 3;
        // a flight slot: at most two jobs are posted and not yet retired (under priority ordering a step of a
        // collective in fold steps, which is one long job, waits until the movers have nothing else: what is
        // posted cannot be overtaken by a more urgent collective that arrives)
        const uint32_t depth = (a.order_policy == 1 && q.fold) ? 1u : 2u;
        bool given_up = false;
        while (!done_here && posted - retired >= depth) {
          retire_finished();
          if (posted - retired >= depth) {
            if ((++spins & 0xffffu) == 0 && abort_seen()) { given_up = true; break; }
            __builtin_amdgcn_s_sleep(1);
          }
        }
        if (given_up) { stop = STOP_ABORT; have = false; continue; }
        if (q.din || q.din_send) {
          // The previous rank published its buffers for this invocation before it notified anything
          // (the counter just seen).  Read once per stay of the collective in hand.
          if (prev_recv == 0) {
            const Slot<AUX_DEVICE> line((const void*)tail_in, DFX_FLAG_STRIDE);
            uint4 w = uint4{0, 0, 0, 0}, w2 = w;
            for (uint32_t tries = 0; tries < 1024u; ++tries) {
              w = line.ld16(DFX_DIRECT_OFF);
              w2 = line.ld16(DFX_DIRECT_OFF + 16);
              if (w.z == inv_seq + 1u && w2.z == inv_seq + 1u) break;
              __builtin_amdgcn_s_sleep(2);
            }
            if (w.z != inv_seq + 1u || w2.z != inv_seq + 1u) { raise_error(a, 3u, wg); stop = STOP_ABORT; have = false; continue; }
            prev_recv = ((u64)w.y << 32) | w.x;
            prev_send = ((u64)w2.y << 32) | w2.x;
          }
          jfin = q.din_send ? (const void*)((const char*)prev_send + soff * eb) : (const void*)((const char*)prev_recv + doff * eb);
        }
        uint32_t jmode = 0, jnseg = 0, jndst = 0, jbytes_fold = 0;
        if (q.fold == 1 || q.fold == 2) {
          // The addresses every rank published for this invocation (before it counted itself published, which a
          // wait of this invocation has seen for all of them): lane k looks up one rank.
          // fold_peer / fold_chunk say which rank and which chunk entry k is about.  Every entry reads a send buffer;
          // the result of a fold step goes to the own recv buffer (reduce-scatter), to the root's (reduce: its address
          // is looked up by the lane behind the R sources, hence at most 63 ranks) or to every entry's rank's
          // (all-reduce: each lane reads both addresses of its rank).
          const int kd = (int)S.kind;
          const uint32_t root = S.nslots;                       // (a collective in fold steps keeps its root there)
          const uint32_t nk = fold_entries(kd, q.fold, a.R);
          const uint32_t target = q.fold == 1 ? fold_dest(kd) : 0u;
          const bool want_root_recv = target == 1u;             // one more look-up, in lane nk
          const bool root_lane = want_root_recv && lane == nk;
          const uint32_t peer = root_lane ? root : fold_peer(kd, q.fold, a.R, rank, root, lane);
          bool bad = want_root_recv && nk >= 64u;
          if (lane < nk + (want_root_recv ? 1u : 0u)) {
            const Slot<AUX_DEVICE> line((const void*)fold_line(S.flags_out, rank, peer, S.nchan), DFX_FLAG_STRIDE);
            uint4 w = uint4{0, 0, 0, 0}, wr = w;
            for (uint32_t tries = 0; tries < 1024u; ++tries) {
              w = line.ld16(root_lane ? DFX_DIRECT_OFF : DFX_DIRECT_OFF + 16);
              if (target == 2u) wr = line.ld16(DFX_DIRECT_OFF);
              if (w.z == inv_seq + 1u && (target != 2u || wr.z == inv_seq + 1u)) break;
              __builtin_amdgcn_s_sleep(2);
            }
            bad = bad || w.z != inv_seq + 1u || (target == 2u && wr.z != inv_seq + 1u);
            const u64 base = ((u64)w.y << 32) | w.x;
            const u64 peer_recv = ((u64)wr.y << 32) | wr.x;
            const SliceGeom gk = slice_geometry(S, a.R, g, fold_chunk(kd, q.fold, rank, peer));
            // (a broadcast's one source goes in pieces: entry k is the k-th piece of the share)
            const bool pieces = q.fold == 2 && kd == KIND_BC;
            const uint32_t off = pieces ? bc_piece_off(gk.bytes, lane) : 0u;
            if (root_lane) sh.tab_dst[posted & 1][0] = base + gk.doff * gk.eb;
            else {
              sh.tab_src[posted & 1][lane] = base + gk.soff * gk.eb + off;
              if (!(want_root_recv && lane == 0))
                sh.tab_dst[posted & 1][lane] = (target == 2u ? peer_recv : (u64)S.recvbuf) + gk.doff * gk.eb + off;
              sh.tab_len[posted & 1][lane] = pieces ? bc_piece_len(gk.bytes, lane) : gk.bytes;
            }
          }
          if (__ballot(bad)) { if (lane == 0) raise_error(a, 3u, wg); stop = STOP_ABORT; have = false; continue; }
          __builtin_amdgcn_wave_barrier();
          jmode = q.fold; jnseg = nk; jndst = target == 2u ? nk : 1u;
          const SliceGeom own = slice_geometry(S, a.R, g, rank);
          if (q.fold == 1) jbytes_fold = own.bytes;
          else {                                                    // the longest segment: a channel's share of a full chunk
            jbytes_fold = (uint32_t)S.slice_elems * own.eb;
            if (kd == KIND_BC) jbytes_fold = bc_piece_bytes(jbytes_fold);
          }
        }
        // ---- post the slice (an empty one is only a handshake: the movers just raise the counters);
        // this claims the slots: the data follows, the counters after it
        if (q.send || q.notify) ++sent;
        if (q.recv) ++recvd;
        if (done_here) {
          if (lane == 0) { bump(sh.stat, ST_PRIMS, 1); complete(coll, inv_seq, inv_nchan); }
        } else if (lane == 0) {
          Job j;
          j.fin = jfin; j.fout = jfout; j.sb = jsb; j.rb = jrb;
          j.bytes = (q.drain || (!q.recv && !q.from_send)) ? 0u : bytes;   // drain and notify-only steps move nothing
          if (q.fold) j.bytes = jbytes_fold;                               // (the last fold step: nothing)
          j.mode = jmode; j.nseg = jnseg; j.ndst = jndst;
          j.dtype = dtype; j.coll = coll; j.prim = (q.drain || q.fold == 3) ? 0xffu : p;   // (prim: for the timeline only)
          sh.job[posted & 1] = j;
          Flight f;
          f.tail_out = (q.send || q.notify) ? tail_out : nullptr; f.head_in = q.recv ? tail_in + 8 : nullptr;
          f.sent_new = sent; f.recvd_new = recvd;
          f.last = last ? 1u : 0u; f.coll = coll; f.seq = inv_seq; f.nchan = inv_nchan;
          f.add_one = q.fadd ? (u64*)(fold_shared_line(S.flags_out, rank, a.R, S.nchan) + 8u * q.fadd) : nullptr;
          sh.fl[posted & 1] = f;
          lds_st(&sh.job_seq, posted + 1);
        }
        g = g_next; p = p_next; cidx = cidx_next;
        pass_bytes += bytes;
        progressed = true;
        pass_progress = true;
        acted = true;
        // AdaptivelyAdjustSpinThreshold (Alg. 1 line 9)
        if (!scanned) {
          thr *= a.spin_boost;
          if (thr > a.spin_max) thr = a.spin_max;
        }
        if (!done_here) ++posted;

        if (last) {
          // ---- CollectiveSuccess: the entry leaves the queue now; the completion counter and the
          // CQE follow at retirement, when the data is in memory
          if (lane == 0) {
            DfxDyn d; d.round = 0; d.prim = 0; d.sent = sent; d.recvd = recvd; d.preempted = 0; d.cidx = 0;
            sh.slot[sl].dyn = d;
            myctx[coll].dyn = d;
          }
          // later entries move up, the position stays (Sec. 4.3)
          --qlen;
          for (uint32_t base = pos; base < qlen; base += 64) {
            const uint32_t i = base + lane;
            uint16_t v = 0;
            if (i < qlen) v = sh.taskq[i + 1];
            __builtin_amdgcn_wave_barrier();
            if (i < qlen) sh.taskq[i] = v;
            __builtin_amdgcn_wave_barrier();
          }
          have = false;
          sw_pending = false;
          if (scanned) {
            // the entries behind the one that left have moved up by one: so do their positions in the list
            ++rk;
            for (uint32_t base = rk; base < nready; base += 64) {
              const uint32_t k = base + lane;
              if (k < nready && (uint32_t)sh.rlist[k] > pos) sh.rlist[k] = (uint16_t)(sh.rlist[k] - 1u);
            }
            __builtin_amdgcn_wave_barrier();
          }
        }
      } else {
        // ---- PreemptCollective + SaveCollectiveContext (lazy: only if it progressed)
        if (a.trace_on == 3 && trace && lane == 0)   // timeline sample of a wait that ended without the primitive: index 15
          trace_put(trace, &sh.trace_n, timeline_sample(tm0, wall_clock64(), coll, 15));
        const bool tr = a.trace_on && res == W_TIMEOUT && pos + 1 < qlen;
        if (tr) sw_t0 = wall_clock64();
        if (lane == 0) {
          if (res == W_TIMEOUT) bump(sh.stat, ST_PREEMPT, 1);
          if (progressed) {
            DfxDyn d; d.round = g; d.prim = p; d.sent = sent; d.recvd = recvd;
            d.preempted = sh.slot[sl].dyn.preempted + 1; d.cidx = cidx;
            sh.slot[sl].dyn = d;
            myctx[coll].dyn = d;
            bump(sh.stat, ST_SAVE, 1);
          } else if (res == W_TIMEOUT) bump(sh.stat, ST_LAZY, 1);
        }
        if (tr) { if (a.trace_on > 1) sw_ts = wall_clock64(); sw_pending = true; }
        have = false;
        if (res == W_STOP) { stop = STOP_ABORT; continue; }
        if (scanned) ++rk; else ++pos;
        if (nx_ok && res == W_TIMEOUT) {
          // LoadCollectiveContext of the entry looked up during the wait (the same steps as at the head of the
          // loop): its context is in its slot and the dynamic part in registers, or the load is under way and
          // goes into the slot now
          pos = nx_pos; coll = nx_coll; sl = nx_sl;
          if (nx_hit) {
            if (lane == 0) bump(sh.stat, ST_HIT, 1);
          } else {
            if (lane < 8) ((uint4*)&sh.slot[sl])[lane] = nx_ctx;
            if (lane == 0) { sh.slot_tag[sl] = coll; bump(sh.stat, ST_LOAD, 1); }
            __builtin_amdgcn_wave_barrier();
            nx_dyn = sh.slot[sl].dyn;
          }
          g = nx_dyn.round; p = nx_dyn.prim; sent = nx_dyn.sent; recvd = nx_dyn.recvd; cidx = nx_dyn.cidx;
          thr = a.spin_init >> (pos < 31 ? pos : 31);
          if (thr < a.spin_min || scanned) thr = a.spin_min;
          progressed = false;
          prev_recv = 0;
          have = true;
          if (sw_pending && a.trace_on > 1) { sw_lb = wall_clock64(); sw_le = sw_lb; }
        }
      }
    }

    // every posted job has been retired and no collective is in hand: the movers may go
    if (lane == 0) {
      if (stop == STOP_QUIT) bump(sh.stat, ST_QUITS, 1);
      ws->read_index = ri;
      ws->qlen = qlen;
      sh.qlen_out = qlen;
      lds_st(&sh.leave, 1u);
    }
  }

  // ================= leave: persist what the next launch needs =================
  __syncthreads();
  if (tid == 0) {
    ws->trace_n = sh.trace_n;
    for (int i = 0; i < DFX_NSTAT; ++i) ws->stat[i] = sh.stat[i];
  }
  const uint32_t qn = sh.qlen_out;
  for (uint32_t i = tid; i < qn; i += NT) qstore[i] = sh.taskq[i];
}

// Plain copy kernel of known traffic: calibrates the HBM byte counters of the profiler and shows
// what a streaming copy reaches.  Four independent 16-byte vectors in flight per thread.
extern "C" __global__ void __launch_bounds__(256) dfx_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t nvec) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (; i + 3 * stride < nvec; i += 4 * stride) {
    uint4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = ld_user((const v4u_user*)&src[i + u * stride]);
#pragma unroll
    for (int u = 0; u < 4; ++u) st_user((v4u_user*)&dst[i + u * stride], v[u]);
  }
  for (; i < nvec; i += stride) dst[i] = src[i];
}

// ------------------------------------------------------------------------------------------
// launch helpers for the host library (kept in this translation unit with the kernels)
// ------------------------------------------------------------------------------------------
hipError_t dfx_daemon_occupancy(int* blocks_per_cu) {
  return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, dfx_daemon_kernel, DFX_WG_THREADS, 0);
}

hipError_t dfx_daemon_launch(uint32_t nwg, hipStream_t stream, const DfxDaemonArgs& a) {
  hipLaunchKernelGGL(dfx_daemon_kernel, dim3(nwg), dim3(DFX_WG_THREADS), 0, stream, a);
  return hipGetLastError();
}

hipError_t dfx_copy_launch(const void* src, void* dst, size_t bytes, hipStream_t stream) {
  hipLaunchKernelGGL(dfx_copy_kernel, dim3(4096), dim3(256), 0, stream, (const uint4*)src, (uint4*)dst, bytes >> 4);
  return hipGetLastError();
}
