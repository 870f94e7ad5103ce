// The integer decision of one edge in one round (steps S2a / S2b of Algorithm 1 pick the largest stamp received; a
// packet is lost or delivered), shared by the resolver kernels and by the kernel that resolves its own rounds.
#pragma once
#include "rfast_internal.h"

namespace {

// v mod d for 0 <= v < 2^31 and a divisor fixed for the launch, without the integer division (some thirty
// instructions per remainder, and a round takes about ten per edge): the quotient by the rounded-down reciprocal is at
// most one short, so one conditional subtraction finishes it.
struct FastMod {
  unsigned d, magic;
  __device__ explicit FastMod(int d_) : d((unsigned)d_), magic(0xFFFFFFFFu / (unsigned)d_) {}
  __device__ int operator()(int v) const {
    const unsigned r = (unsigned)v - __umulhi((unsigned)v, magic) * d;
    return (int)(r >= d ? r - d : r);
  }
};

// bit b (< 64) of a 64-bit word through one of its halves: 32-bit shifts run at full rate, 64-bit ones at a quarter
__device__ inline bool bit_of(unsigned long long bits, int b) {
  const unsigned half = b < 32 ? (unsigned)bits : (unsigned)(bits >> 32);
  return (half >> (b & 31)) & 1u;
}

__device__ inline bool delivered(unsigned long long bits, int v, const FastMod& modM) { return v <= 0 || bit_of(bits, modM(v)); }

__device__ inline void record_error(int32_t* err, int code, int round, int kind, int e) {
  if (atomicCAS(&err[0], 0, code) == 0) {
    err[1] = round;
    err[2] = kind;
    err[3] = e;
  }
}

// What one lane knows about its edge before it decides anything.  The loads come in two levels of
// dependency (by edge number; by the node numbers and the delay found there), and both are issued
// ahead of the node pass of the kernel, so that the whole resolver costs about two memory round
// trips instead of four or five.
struct EdgeIn {
  int i, j, d, old, tj, u;
  unsigned long long bits;
  bool act_i, act_j, dropped;
};

// What deciding an edge yields besides the new stamp and delivery bits (which go back into the EdgeIn):
struct EdgeOut {
  int slot;    // ring slot of the version the receiver reads, -1 if the receiver is idle
  int word;    // graph R: that slot, 0 if the receiver is idle; graph C: the edge's plan word (RfastDev::plan_c)
  bool spill;  // graph C: bit 18 of the word, the sender has to save the version that leaves its ring
};

// Decides edge e (of graph R: KIND 0, of graph C: KIND 1) for round r; q.old and q.bits are brought up to date.
// Written without branches on what differs from lane to lane (an active or idle receiver, a lost packet): one
// wavefront runs this for every round of a launch, and every divergent branch costs it both sides and the
// bookkeeping of the execution mask.
template <int KIND>
__device__ inline EdgeOut edge_compute(const RfastDev& s, const FastMod& modM, int e, int r, EdgeIn& q) {
  const int lo = q.tj - (s.M - 2);  // oldest version that stays readable in j's ring during this round
  if (q.act_i && (q.d < 0 || q.d > s.d_max)) record_error(s.err, RFAST_ERANGE, r, KIND, e);  // resolved with the clamped delay
  // S2a / S2b: the newest delivered version that is not newer than u: at most burst-1 steps back (a version is
  // delivered by force once the burst-1 before it were all lost; version 0 always counts as delivered)
  int u = q.u;
  for (int k = 1; k < s.burst; ++k) u -= delivered(q.bits, u, modM) ? 0 : 1;
  const int old = q.old;
  const int now = q.act_i && u > old ? u : old;
  const int now_slot = modM(now);
  q.old = now;
  EdgeOut o;
  o.slot = q.act_i ? now_slot : -1;
  o.spill = false;
  if (KIND == 0) {
    o.word = q.act_i ? now_slot : 0;
  } else {
    const bool live = now != old;  // never with an idle receiver
    // after this round the ring of an active sender no longer covers version lo
    const bool leaves = q.act_j && now == lo;
    o.spill = !live && leaves;  // the receiver does not consume, and the version its buffer holds leaves
    // bits 0-7 of a spill word: the slot of the version that leaves (now == lo then)
    // bits 30 and 31 sort the live edges for a consumer that wants one compare per case: the usual one (what was
    // consumed last time is still in the ring, what is consumed now stays there) and the rest
    const bool usual = live && !leaves && old >= lo;
    o.word = q.act_i ? now_slot | ((old >= lo ? modM(old) : 0xFF) << 8) | (live ? 1 << 16 : 0) | (live && leaves ? 1 << 17 : 0) |
                           (o.spill ? 1 << 18 : 0) | (usual ? 1 << 30 : 0) | (live && !usual ? (int)0x80000000 : 0)
                     : (o.spill ? now_slot | 1 << 18 : 0);
  }
  // the sender publishes version t_j + 1 this round (if it is active): lost only if the schedule says so and not all
  // of the burst-1 versions before it were lost too
  const int vn = q.tj + 1;
  bool all_lost = true;
  for (int k = 1; k < s.burst; ++k) all_lost = all_lost && !delivered(q.bits, vn - k, modM);
  const bool ok = !q.dropped || all_lost;
  const int b = modM(vn);
  const unsigned mask = 1u << (b & 31);
  unsigned w_lo = (unsigned)q.bits, w_hi = (unsigned)(q.bits >> 32);
  const bool in_lo = b < 32;
  const unsigned half = in_lo ? w_lo : w_hi;
  const unsigned changed = q.act_j ? (ok ? half | mask : half & ~mask) : half;
  w_lo = in_lo ? changed : w_lo;
  w_hi = in_lo ? w_hi : changed;
  q.bits = ((unsigned long long)w_hi << 32) | w_lo;
  return o;
}

}  // namespace
