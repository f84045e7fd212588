// Index arithmetic of the daemon kernel: which workgroup serves which (rank, channel), the primitive
// sequence of every collective kind, the connector addresses of an invocation, where a slice lies in
// the buffers, and the order in which a workgroup walks through slices and primitives.
//
// Pure functions of their arguments, compiled for the device (the kernel) and for the host (the
// library's geometry self-check, which walks the same arithmetic without a GPU).
#ifndef DFX_GEOMETRY_H
#define DFX_GEOMETRY_H

#include <stddef.h>
#include <stdint.h>

#include "dfx_internal.h"

#if defined(__HIPCC__)
#define DFX_HD __host__ __device__ __forceinline__
#else
#define DFX_HD inline
#endif

constexpr int KIND_AR = 0, KIND_AG = 1, KIND_RS = 2, KIND_BC = 3, KIND_RD = 4;
constexpr int DT_F32 = 0, DT_BF16 = 1, DT_F16 = 2, DT_I32 = 3;

// Workgroup -> (rank, channel).  Workgroups go to the XCDs round-robin (workgroup w runs on XCD w mod 8).
//   map 0: workgroup = channel * R + rank: with R = 8 a vrank per XCD
//   map 1: workgroup = rank * cmax + channel: a channel's whole ring per XCD
struct WgPlace { uint32_t rank, ch; };
DFX_HD WgPlace wg_place(uint32_t wg_map, uint32_t wg, uint32_t R, uint32_t cmax) {
  WgPlace w;
  if (wg_map == 0) { w.rank = wg % R; w.ch = wg / R; }
  else { w.rank = wg / cmax; w.ch = wg % cmax; }
  return w;
}

// Channel of collective coll_id that the workgroup on channel `ch` of its rank serves (>= nchan: none).
// A collective with fewer channels than the grid has per rank starts at workgroup (coll_id * nchan) mod
// cmax, so that many small collectives spread over the rank's workgroups instead of queueing on the
// first ones; every rank derives the same start from the id, which keeps both ends of a connector on
// the same channel.
DFX_HD uint32_t serving_channel(bool spread, uint32_t ch, uint32_t cmax, uint32_t coll_id, uint32_t nchan) {
  if (spread && nchan < cmax) return (ch + cmax - (coll_id * nchan) % cmax) % cmax;
  return ch;
}

// primitive descriptor for (kind, position p in the sequence); the ring-chunk index travels in
// the dynamic context and is stepped by next_cidx, so nothing here divides
struct Prim {
  bool recv, send;         // uses recv / send connector (send: waits for a free slot and fills it)
  bool from_send, to_recv; // touches the send buffer / recv buffer
  // Direct gather steps of an all-reduce: every rank's buffers lie in the same HBM, so the copy
  // steps need no second copy through a FIFO slot.  notify: the result goes to the own recv buffer
  // with device-coherent stores and the send connector's counter is raised without a slot being
  // filled; din: the input is read from the previous rank's recv buffer instead of a slot;
  // drain: no data, the wait ends when the next rank has consumed everything notified so far
  // (the recv buffer is the caller's again once the completion is posted).
  bool notify, din, drain;
  bool din_send;   // the input is the previous rank's SEND buffer (first reduce step of a direct all-reduce / reduce-scatter)
  // Fold steps of a short collective (see make_fold_prim): fold = 1 a fold step, 2 a gather step, 3 a last wait
  // that moves nothing; 0 = none of them.  fwait: the channel's shared counter the wait phase looks at
  // (0 published, 1 folded, 2 gathered); fadd: the counter the step adds to when its data is in memory (0 = none).
  uint8_t fold, fwait, fadd;
};

// Short collectives in fold steps.  Every rank's buffers lie in the same HBM, so the dependent hops of a ring or
// a chain (a few microseconds each, whatever the size) can be replaced by steps that wait on all ranks at once:
//   fold step:   when every rank has published this invocation's buffers, a rank reads one chunk out of all R
//                send buffers and combines them in the ring's (the chain's) own order -- the same association as
//                the hops would give, hence the same bits -- and writes the result where it belongs: its own recv
//                buffer, the root's, or everybody's;
//   gather step: copies chunks out of other ranks' send buffers into the own recv buffer;
//   last wait:   no data; when every rank has got far enough, nobody reads this rank's buffers any more and
//                the completion may be posted.
// all-reduce:      fold (rank r: chunk r, x[r+1] (op) ... (op) x[r], into chunk r of ALL R recv buffers: every input is
//                  read once and every output written once), last wait (all folded: every chunk of the own recv
//                  buffer has arrived and nobody reads the own send buffer any more)
// reduce-scatter:  fold (rank r: block r into its recv buffer), last wait (all folded: the send buffers are free)
// reduce:          fold (rank r: chunk r of the message, x[root+1] (op) ... (op) x[root], into the ROOT's recv
//                  buffer), last wait (all folded)
// all-gather:      gather (all R blocks out of the send buffers), last wait (all gathered)
// broadcast:       gather (the channel's share of the root's send buffer), last wait (all gathered)
// Each step is a bounded wait followed by the data, like any primitive: nothing is touched before the wait has
// succeeded, so a collective stuck in any of them is preempted like any other.
DFX_HD uint32_t fold_nprim(int) { return 2u; }
DFX_HD Prim make_fold_prim(int kind, uint32_t p) {
  Prim q;
  q.recv = q.send = q.notify = q.din = q.drain = q.din_send = false;
  q.from_send = q.to_recv = false;
  const bool reduces = (kind == KIND_AR || kind == KIND_RS || kind == KIND_RD);
  if (p == 0) { q.fold = reduces ? 1 : 2; q.fwait = 0; q.fadd = reduces ? 1 : 2; q.from_send = true; q.to_recv = true; }
  else { q.fold = 3; q.fwait = reduces ? 1 : 2; q.fadd = 0; }
  return q;
}

// The tables of a fold or gather step (Prim::fold 1 or 2).  Entry k of a fold step is a source, listed in the order
// of combination, which begins behind this rank (all-reduce, reduce-scatter: the ring's order for this rank's chunk)
// or behind the root (reduce: the chain's); every entry is about the rank's own chunk.  Entry k of a gather step is
// a segment: all-gather: block k out of rank k's send buffer; broadcast: the k-th of eight pieces of the channel's
// share of the root's send buffer (one source cut up, so that as many loads travel together as in an all-gather).
constexpr uint32_t DFX_BC_PIECES = 8;
DFX_HD uint32_t fold_entries(int kind, uint32_t step, uint32_t R) { return (step == 2 && kind == KIND_BC) ? DFX_BC_PIECES : R; }
DFX_HD uint32_t bc_piece_bytes(uint32_t share_bytes) { return (((share_bytes + DFX_BC_PIECES - 1) / DFX_BC_PIECES) + 15u) & ~15u; }
// piece k of a share of share_bytes: where it begins and how long it is (0 = nothing left for it)
DFX_HD uint32_t bc_piece_off(uint32_t share_bytes, uint32_t k) { return k * bc_piece_bytes(share_bytes); }
DFX_HD uint32_t bc_piece_len(uint32_t share_bytes, uint32_t k) {
  const uint32_t pb = bc_piece_bytes(share_bytes), off = k * pb;
  return off >= share_bytes ? 0u : (share_bytes - off < pb ? share_bytes - off : pb);
}
DFX_HD uint32_t fold_peer(int kind, uint32_t step, uint32_t R, uint32_t rank, uint32_t root, uint32_t k) {
  if (step == 2) return kind == KIND_BC ? root : k % R;
  return ((kind == KIND_RD ? root : rank) + 1u + k) % R;
}
DFX_HD uint32_t fold_chunk(int kind, uint32_t step, uint32_t rank, uint32_t peer) {
  return step == 1 ? rank : (kind == KIND_BC ? 0u : peer);
}
// Where a fold step's result goes: 0 the own recv buffer (reduce-scatter), 1 the root's (reduce), 2 the recv buffer
// of every entry's rank (all-reduce).
DFX_HD uint32_t fold_dest(int kind) { return kind == KIND_AR ? 2u : (kind == KIND_RD ? 1u : 0u); }

// Where a fold collective's lines are, from a workgroup's own line: the line of rank r on the same channel,
// and the channel's shared line.
DFX_HD uint64_t fold_line(uint64_t own_line, uint32_t rank, uint32_t r, uint32_t nchan) {
  return own_line + ((uint64_t)r - (uint64_t)rank) * nchan * DFX_FLAG_STRIDE;
}
DFX_HD uint64_t fold_shared_line(uint64_t own_line, uint32_t rank, uint32_t R, uint32_t nchan) {
  return own_line + ((uint64_t)R - (uint64_t)rank) * nchan * DFX_FLAG_STRIDE;
}

DFX_HD Prim make_prim(int kind, uint32_t R, uint32_t bc_pos, uint32_t p, bool direct) {
  Prim q;
  q.notify = q.din = q.drain = q.din_send = false;
  q.fold = q.fwait = q.fadd = 0;
  if (R == 1) { q.recv = q.send = false; q.from_send = q.to_recv = true; return q; }   // copy
  if (kind == KIND_AR && direct) {
    const uint32_t last_reduce = R - 1;
    q.recv = p > 0; q.send = p < last_reduce; q.from_send = p <= last_reduce; q.to_recv = p >= last_reduce;
    // The opening send moves nothing either: the rank only notifies, and the next rank's first
    // reduce step reads the chunk out of this rank's send buffer (which the caller leaves alone
    // until the completion, and the drain keeps the completion behind that read).
    if (p == 0) { q.send = false; q.from_send = false; q.notify = true; }             // notify only
    else if (p == 1) q.din_send = true;                                               // recv-reduce-send / -copy from the neighbour's send buffer
    if (p == last_reduce) q.notify = true;                                            // recv-reduce-copy, notify
    else if (p > last_reduce && p < 2u * R - 2) { q.din = true; q.notify = true; }    // direct recv-copy, notify
    else if (p == 2u * R - 2) q.din = true;                                           // direct recv-copy
    else if (p == 2u * R - 1) { q.recv = false; q.to_recv = false; q.drain = true; }  // drain
    return q;
  }
  if (kind == KIND_RS && direct) {
    // the reduce phase of the direct all-reduce: notify only, then the first reduce step reads the
    // neighbour's send buffer; the drain keeps the completion behind that read
    q.recv = p > 0 && p < R; q.send = p > 0 && p + 1 < R; q.from_send = q.recv; q.to_recv = p == R - 1;
    if (p == 0) q.notify = true;
    else if (p == 1) q.din_send = true;
    else if (p == R) q.drain = true;
    return q;
  }
  if (kind == KIND_AR || kind == KIND_RS) {
    const uint32_t last_reduce = R - 1;
    if (p == 0) { q.recv = false; q.send = true; q.from_send = true; q.to_recv = false; }                         // send
    else if (p < last_reduce) { q.recv = true; q.send = true; q.from_send = true; q.to_recv = false; }           // recv-reduce-send
    else if (p == last_reduce) { q.recv = true; q.send = (kind == KIND_AR); q.from_send = true; q.to_recv = true; }  // recv-reduce-copy(-send)
    else if (p < 2u * R - 2) { q.recv = true; q.send = true; q.from_send = false; q.to_recv = true; }            // recv-copy-send
    else { q.recv = true; q.send = false; q.from_send = false; q.to_recv = true; }                               // recv-copy
  } else if (kind == KIND_AG && direct) {
    // every block is written once: the own one by a copy that notifies, the others by direct copies
    q.send = false;
    if (p == 0) { q.recv = false; q.from_send = true; q.to_recv = true; q.notify = true; }                        // copy, notify
    else if (p < R) { q.recv = true; q.from_send = false; q.to_recv = true; q.din = true; q.notify = p < R - 1; } // direct recv-copy (, notify)
    else { q.recv = false; q.from_send = false; q.to_recv = false; q.drain = true; }                              // drain
  } else if (kind == KIND_AG) {
    if (p == 0) { q.recv = false; q.send = true; q.from_send = true; q.to_recv = true; }                          // copy-send
    else if (p < R - 1) { q.recv = true; q.send = true; q.from_send = false; q.to_recv = true; }
    else { q.recv = true; q.send = false; q.from_send = false; q.to_recv = true; }
  } else if (kind == KIND_RD) {  // reduce chain root+1 -> root+2 -> ... -> root (bc_pos: 0 first, 1 middle, 2 the root, 3 second)
    if (bc_pos == 0) { q.recv = false; q.send = true; q.from_send = true; q.to_recv = false; }                    // send
    else if (bc_pos == 2) { q.recv = true; q.send = false; q.from_send = true; q.to_recv = true; }               // recv-reduce-copy
    else { q.recv = true; q.send = true; q.from_send = true; q.to_recv = false; }                                 // recv-reduce-send
    if (direct) {
      // the first rank only notifies and the second one reads the slice out of its send buffer
      if (bc_pos == 0) { q.send = false; q.from_send = false; q.notify = true; }
      else if (bc_pos == 3 || R == 2) q.din_send = true;
    }
  } else if (direct) {  // broadcast chain with direct steps: every rank writes its recv buffer only
    q.send = false; q.to_recv = true;
    q.recv = bc_pos != 0; q.din = bc_pos != 0; q.from_send = bc_pos == 0; q.notify = bc_pos != 2;
  } else {  // broadcast chain root -> root+1 -> ... -> root-1
    if (bc_pos == 0) { q.recv = false; q.send = true; q.from_send = true; q.to_recv = true; }
    else if (bc_pos == 2) { q.recv = true; q.send = false; q.from_send = false; q.to_recv = true; }
    else { q.recv = true; q.send = true; q.from_send = false; q.to_recv = true; }
  }
  return q;
}

// A chain (broadcast, reduce) has one primitive per slice, so its drain cannot be a step of the
// per-slice sequence: with direct steps it counts one round more than it has slices, and that
// round is the drain (nothing to move; the last rank of the chain has sent nothing and passes at once).
DFX_HD Prim chain_drain_round(Prim q, int kind, bool direct, uint32_t g, uint32_t rounds) {
  if (direct && (kind == KIND_BC || kind == KIND_RD) && g + 1 == rounds) {
    q.recv = q.send = q.from_send = q.to_recv = q.notify = q.din = false;
    q.drain = true;
  }
  return q;
}

// Ring chunk that the first primitive of a sequence works on (see DfxDyn.cidx): an all-gather
// starts with the rank's own block, the chains (broadcast, reduce) have one block, all-reduce and
// reduce-scatter start with the chunk of the rank before.
DFX_HD uint32_t first_chunk(int kind, uint32_t rank, uint32_t R) {
  if (kind == KIND_AG) return rank;
  if (kind == KIND_BC || kind == KIND_RD || R == 1) return 0u;
  return (rank + R - 1) % R;
}

// The SQE of an invocation "cooked" for one workgroup: every address a primitive needs resolved
// once, so that a context load is a plain copy (Sec. 4.2 (4)).  vch: channel of the collective
// that this workgroup serves.
DFX_HD DfxCooked cook_sqe(const DfxStatic& q, uint8_t* pool, uint32_t rank, uint32_t R, uint32_t vch) {
  DfxCooked k;
  k.sendbuf = q.sendbuf; k.recvbuf = q.recvbuf; k.count = q.count;
  k.block_elems = q.block_elems; k.part_elems = q.part_elems;
  uint8_t* conn = pool + q.conn_off;   // flags first, then slots
  const uint32_t e_out = rank, e_in = (rank + R - 1) % R;
  const size_t fo = (size_t)e_out * q.nchan + vch, fi = (size_t)e_in * q.nchan + vch;
  uint8_t* slots = conn + (size_t)R * q.nchan * DFX_FLAG_STRIDE;
  k.flags_out = (uint64_t)(conn + fo * DFX_FLAG_STRIDE);
  k.flags_in = (uint64_t)(conn + fi * DFX_FLAG_STRIDE);
  k.fifo_out = (uint64_t)(slots + fo * q.nslots * q.slot_bytes);
  k.fifo_in = (uint64_t)(slots + fi * q.nslots * q.slot_bytes);
  // a direct broadcast has no slots (no step of it fills or reads one)
  if ((q.kind == KIND_BC && (q.flags & DFX_SQE_DIRECT)) || (q.flags & DFX_SQE_FOLD)) k.fifo_out = k.fifo_in = 0;
  k.slice_elems = q.slice_elems; k.rounds = q.rounds; k.seq = q.seq;
  k.nprim = (uint16_t)q.nprim; k.nchan = q.nchan;
  k.nslots = (uint8_t)((q.flags & DFX_SQE_FOLD) ? q.root : q.nslots);   // (no slots in fold steps: the byte carries the root)
  k.kind = q.kind; k.dtype = (uint8_t)(q.dtype | (q.op << 4));
  // place in the chain: broadcast starts at the root, reduce at the rank after it
  const uint32_t bpos = (rank + 2 * R - q.root - (q.kind == KIND_RD ? 1u : 0u)) % R;
  k.bc_pos = bpos == 0 ? 0 : (bpos == R - 1 ? 2 : 1);
  if (q.kind == KIND_RD && (q.flags & DFX_SQE_DIRECT) && bpos == 1 && R > 2) k.bc_pos = 3;   // reads the first rank's send buffer
  if (q.flags & DFX_SQE_DIRECT) k.bc_pos |= DFX_CTX_DIRECT;   // a collective with direct steps
  if (q.flags & DFX_SQE_FOLD) k.bc_pos |= DFX_CTX_FOLD;       // an all-reduce in fold steps
  k.priority = q.priority; k.vch = (uint16_t)vch;
  return k;
}

// Where slice g of ring chunk cidx lies for the workgroup that holds context S: element offsets
// in the send and the recv buffer and the slice's length in bytes (clipped to the chunk's and the
// channel's true length: the last ones may be short or empty).
struct SliceGeom { uint64_t soff, doff; uint32_t bytes, eb; };
DFX_HD SliceGeom slice_geometry(const DfxCooked& S, uint32_t R, uint32_t g, uint32_t cidx) {
  const int kind = S.kind, dt = S.dtype & 15;
  SliceGeom o;
  o.eb = (dt == DT_F32 || dt == DT_I32) ? 4u : 2u;
  const uint32_t slice_elems = S.slice_elems, vch = S.vch;
  const uint64_t count = S.count, block_elems = S.block_elems, part_elems = S.part_elems;
  // (a reduce in fold steps is cut into R chunks like an all-reduce: rank r combines chunk r)
  const bool ring_chunks = R > 1 && (kind == KIND_AR || (kind == KIND_RD && (S.bc_pos & DFX_CTX_FOLD)));
  uint64_t blen = count;
  if (ring_chunks) {
    const uint64_t start = (uint64_t)cidx * block_elems;
    blen = start >= count ? 0 : (count - start < block_elems ? count - start : block_elems);
  }
  uint64_t lo = (uint64_t)vch * part_elems + (uint64_t)g * slice_elems;
  uint64_t hi = lo + slice_elems;
  const uint64_t pend = (uint64_t)(vch + 1) * part_elems;
  if (hi > pend) hi = pend;
  if (lo > pend) lo = pend;     // (the drain round of a chain lies behind the channel's last slice: empty, not negative)
  if (lo > blen) lo = blen;
  if (hi > blen) hi = blen;
  o.bytes = (uint32_t)(hi - lo) * o.eb;
  o.soff = lo; o.doff = lo;
  if (ring_chunks) { o.soff += (uint64_t)cidx * block_elems; o.doff = o.soff; }
  else if (kind == KIND_RS) o.soff += (uint64_t)cidx * count;
  else if (kind == KIND_AG) o.doff += (uint64_t)cidx * count;
  return o;
}


// The position after a primitive.  Slices are taken in windows of W: primitive p of every slice of the
// window, then primitive p+1 of every slice, ...  The neighbour does the same, so when this rank comes
// to (slice, p+1) the neighbour finished (slice, p) one job ago instead of at this very moment, and the
// hop latency hides behind the other slice's data.  The chunk index steps down the ring with p; a new
// window starts the sequence over.  g >= rounds afterwards: that was the last primitive of the share.
struct SeqPos { uint32_t g, p, cidx; };
DFX_HD SeqPos next_position(int kind, uint32_t R, uint32_t rank, uint32_t W, uint32_t rounds, uint32_t nprim,
                            uint32_t g, uint32_t p, uint32_t cidx) {
  SeqPos n;
  n.g = g; n.p = p; n.cidx = cidx;
  if (((g + 1) & (W - 1)) != 0 && g + 1 < rounds) ++n.g;
  else {
    n.g &= ~(W - 1);
    n.cidx = (cidx == 0) ? R - 1 : cidx - 1;
    if (++n.p == nprim) {
      n.p = 0; n.g += W;
      n.cidx = first_chunk(kind, rank, R);
    }
    if (kind == KIND_BC || kind == KIND_RD) n.cidx = 0;
  }
  return n;
}

// The walk of a collective in fold steps: the step with data (p = 0) for every slice of the share, then the
// last wait (p = 1) once.  g >= rounds afterwards: that was it.
DFX_HD SeqPos next_fold_position(uint32_t rounds, uint32_t g, uint32_t p, uint32_t cidx) {
  SeqPos n;
  n.cidx = cidx;
  if (p == 0) {
    if (g + 1 < rounds) { n.g = g + 1; n.p = 0; }
    else { n.g = g; n.p = 1; }
  } else { n.g = rounds; n.p = 0; }
  return n;
}

#endif
