// Integer schedule resolver: turns one round's masks into ring-slot indices.
//
// For an active receiver i and in-edge e = (j -> i) the stamp picked up is the
// newest one that has arrived on the edge (Algorithm 1, S2a / S2b), i.e. the
// newest version of j that (a) j had published before round r - delay_e and
// (b) was not lost on e, and never older than the stamp already held.  Losses
// are decided when a version is sent (experiments section: a node either sends
// its new packet or discards it).  After burst-1 consecutive losses on an edge
// the next version is delivered regardless, which keeps every read within D
// versions of the sender's counter (Assumption 3 ii).
//
// The same lane decides where the buffer rho~ of step S4 lives for its C edge.  rho~_ij
// equals a_ij * sigma_j[tau_ij], which the sender's ring still holds while
// tau_ij >= t_j - D; only a version about to leave the ring is copied to the rho~ array
// (by the receiver if it consumes exactly that version in this round, else by the sender).
//
// One workgroup, one lane per edge; every step is integer and deterministic.
#include "rfast_edge.h"
#include "rfast_internal.h"

namespace {

// kind 0: graph R (v packets), kind 1: graph C (rho packets); e counts within its graph
__device__ inline void edge_level1(const RfastDev& s, int kind, int e, const int32_t* delay, const uint8_t* drop, EdgeIn* q) {
  q->i = (kind ? s.c_dst : s.r_dst)[e];
  q->j = (kind ? s.c_src : s.r_src)[e];
  q->bits = (kind ? s.deliv_c : s.deliv_r)[e];
  q->d = delay[e];
  q->old = (kind ? s.tau_c : s.tau_r)[e];
  q->dropped = drop[e] != 0;
}

__device__ inline void edge_level2(const RfastDev& s, int r, const uint8_t* active, EdgeIn* q) {
  q->act_i = active[q->i] != 0;
  q->act_j = active[q->j] != 0;
  q->tj = s.t[q->j];  // the counters are advanced only after the last barrier of the kernel
  const int d = q->d < 0 ? 0 : (q->d > s.d_max ? s.d_max : q->d);
  const int at = r - d;
  // the sender's counter at the start of round `at`; round r itself is the current counter (its
  // history slot is being written by the node pass)
  q->u = at <= 0 ? 0 : (at >= r ? q->tj : s.t_hist[(size_t)q->j * s.H + (at % s.H)]);
}

// Decides edge e for round r, leaves the new stamp and delivery bits in q as well (a lane that keeps its edges
// over several rounds goes on from them) and writes the round's plan; what an idle receiver does not change is
// stored again unchanged.  KIND 0: graph R, 1: graph C.
template <int KIND>
__device__ inline void edge_decide_t(const RfastDev& s, const FastMod& modM, int e, int r, EdgeIn& q) {
  const EdgeOut o = edge_compute<KIND>(s, modM, e, r, q);
  (KIND ? s.tau_c : s.tau_r)[e] = q.old;
  (KIND ? s.slot_c : s.slot_r)[e] = o.slot;
  if (KIND == 0) {
    if (s.blk_plan) s.blk_plan[s.n + e] = o.word;
  } else {
    s.plan_c[e] = o.word;
    if (s.blk_plan) s.blk_plan[s.n + s.eR + e] = o.word;
    if (o.spill) s.node_spill[q.j] = 1;
  }
  (KIND ? s.deliv_c : s.deliv_r)[e] = q.bits;
}

__device__ inline void edge_decide(const RfastDev& s, const FastMod& modM, int kind, int e, int r, EdgeIn& q) {
  if (kind) edge_decide_t<1>(s, modM, e, r, q);
  else edge_decide_t<0>(s, modM, e, r, q);
}

// What the kernel that moves the rings of a multi-round launch needs to know about the state before
// the first round (when = 0, called ahead of the rounds) and after the last (when = 1), see
// RfastDev::blk_head.  Called by every lane of the one workgroup.
__device__ inline void block_head(const RfastDev& s, int when) {
  int32_t* H = s.blk_head;
  constexpr int K = kHeadWords;
  __syncthreads();  // when = 1: the last round's counters and stamps are written
  for (int j = threadIdx.x; j < s.n; j += blockDim.x) {
    H[K * j + when] = s.t[j];
    H[K * j + 2 + 2 * when] = 0x7fffffff;
    H[K * j + 3 + 2 * when] = 0x7fffffff;
  }
  __syncthreads();
  for (int e = threadIdx.x; e < s.eR; e += blockDim.x) atomicMin(&H[K * s.r_src[e] + 2 + 2 * when], s.tau_r[e]);
  for (int e = threadIdx.x; e < s.eC; e += blockDim.x) {
    const int j = s.c_src[e], tau = s.tau_c[e];
    atomicMin(&H[K * j + 3 + 2 * when], tau);
    const int outside = tau < s.t[j] - (s.M - 2) ? 1 : 0;  // the S4 buffer of the edge is in the rho_tilde array
    if (when == 0) H[K * s.n + e] = outside;
    else H[K * s.n + e] |= outside << 1;
  }
  __syncthreads();  // when = 0: the rounds below move the stamps and the counters
  if (when == 0) return;
  // the same facts per ring slot, so that the lanes of the launch test a bit where they would compute a version
  for (int j = threadIdx.x; j < s.n; j += blockDim.x) {
    const int M = s.M, t0 = H[K * j], te = H[K * j + 1];
    const int s0 = t0 % M, se = te % M;
    unsigned in_v = 0, in_s = 0, written = 0, out_v = 0, out_s = 0;
    for (int m = 0; m < M && m < 32; ++m) {
      // version held by slot m when the latest version t is in slot t mod M (negative: never written)
      const int v0 = t0 - (s0 - m < 0 ? s0 - m + M : s0 - m), v1 = te - (se - m < 0 ? se - m + M : se - m);
      const unsigned bit = 1u << m;
      if (v0 >= H[K * j + 2]) in_v |= bit;
      if (v0 >= H[K * j + 3]) in_s |= bit;
      if (v1 > t0) written |= bit;
      if (v1 >= H[K * j + 4]) out_v |= bit;
      if (v1 >= H[K * j + 5]) out_s |= bit;
    }
    H[K * j + 8] = s0;
    H[K * j + 9] = se;
    H[K * j + 10] = (int)in_v;
    H[K * j + 11] = (int)in_s;
    H[K * j + 12] = (int)written;
    H[K * j + 13] = (int)out_v;
    H[K * j + 14] = (int)out_s;
  }
}

constexpr int kResolveThreads = 1024;
constexpr int kAhead = 2;  // edges per lane whose loads are issued before the node pass

template <class P> __device__ inline void advance(P*& ptr, size_t bytes) {
  ptr = reinterpret_cast<P*>(reinterpret_cast<char*>(ptr) + bytes);
}

// rounds > 1: consecutive rounds in one launch, the schedule arrays of round q at offset q of each
// pointer, its plan record (multi-round kernels) behind the previous one and its per-round plan
// arrays plan_stride bytes behind those of the previous round (0: every round overwrites the same
// arrays, which then hold the last round only).  The rounds are sequential -- each reads the
// counters, stamps and delivery bits the one before wrote -- with the workgroup's barrier between
// them.
__global__ void __launch_bounds__(kResolveThreads) rfast_resolve_kernel(RfastDev s, int rounds, size_t plan_stride, const uint8_t* active,
                                                                         const int32_t* delay_R, const int32_t* delay_C,
                                                                         const uint8_t* drop_R, const uint8_t* drop_C) {
  __shared__ int wave_cnt[kResolveThreads / 64];
  __shared__ int base;
  const int r0 = *s.round_no;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int E = s.eR + s.eC;
  const FastMod modM(s.M);
  if (s.blk_head) block_head(s, 0);
  for (int rq = 0; rq < rounds; ++rq) {
    const int r = r0 + rq;
    EdgeIn ahead[kAhead];
#pragma unroll
    for (int a = 0; a < kAhead; ++a) {
      const int e = threadIdx.x + a * kResolveThreads;
      if (e < s.eR) edge_level1(s, 0, e, delay_R, drop_R, &ahead[a]);
      else if (e < E) edge_level1(s, 1, e - s.eR, delay_C, drop_C, &ahead[a]);
    }
#pragma unroll
    for (int a = 0; a < kAhead; ++a)
      if (threadIdx.x + a * kResolveThreads < E) edge_level2(s, r, active, &ahead[a]);
    if (threadIdx.x == 0) base = 0;
    if (threadIdx.x == 0 && s.blk_plan) s.blk_plan[s.n + E] = 0;  // a record ends with a word that is always zero
    // node pass: snapshot of the counters, and the ordered list of active nodes (ballot + prefix per chunk)
    for (int i0 = 0; i0 < s.n; i0 += kResolveThreads) {
      const int i = i0 + threadIdx.x;
      bool act = false;
      int ti = 0;
      if (i < s.n) {
        ti = s.t[i];
        s.plan_t[i] = ti;
        s.node_spill[i] = 0;
        s.t_hist[(size_t)i * s.H + (r % s.H)] = ti;
        act = active[i] != 0;
        if (s.blk_plan) s.blk_plan[i] = (ti & 0x3FFFFFFF) | (act ? (int)0x80000000 : 0);
      }
      const unsigned long long m = __ballot(act);
      if (lane == 0) wave_cnt[wave] = __popcll(m);
      __syncthreads();
      int off = base;
      for (int w = 0; w < wave; ++w) off += wave_cnt[w];
      if (act) s.active_plan[off + __popcll(m & ((1ull << lane) - 1ull))] = make_int2(i, ti);
      __syncthreads();
      if (threadIdx.x == 0) {
        int tot = 0;
        for (int w = 0; w < kResolveThreads / 64; ++w) tot += wave_cnt[w];
        base += tot;
      }
      __syncthreads();
    }
    if (threadIdx.x == 0) {
      s.n_active[0] = base;
      s.n_active[1] = r + 1;
    }
    for (int q = base + threadIdx.x; q < s.n + 8; q += kResolveThreads) s.active_plan[q] = make_int2(-1, 0);
    // edge pass (node_spill was cleared above, before the barriers); nothing in it depends on the node pass
#pragma unroll
    for (int a = 0; a < kAhead; ++a) {
      const int e = threadIdx.x + a * kResolveThreads;
      if (e < E) edge_decide(s, modM, e >= s.eR, e >= s.eR ? e - s.eR : e, r, ahead[a]);
    }
    for (int e = threadIdx.x + kAhead * kResolveThreads; e < E; e += kResolveThreads) {  // more than 2048 edges
      const int kind = e >= s.eR, el = kind ? e - s.eR : e;
      EdgeIn q;
      edge_level1(s, kind, el, kind ? delay_C : delay_R, kind ? drop_C : drop_R, &q);
      edge_level2(s, r, active, &q);
      edge_decide(s, modM, kind, el, r, q);
    }
    __syncthreads();  // every read of the counters is done
    for (int i = threadIdx.x; i < s.n; i += kResolveThreads)
      if (active[i] != 0) s.t[i] = s.plan_t[i] + 1;
    if (rq + 1 < rounds) {
      __syncthreads();  // the next round reads what this one wrote
      active += s.n;
      delay_R += s.eR;
      drop_R += s.eR;
      delay_C += s.eC;
      drop_C += s.eC;
      if (s.blk_plan) s.blk_plan += s.n + E + 1;
      advance(s.n_active, plan_stride);
      advance(s.active_plan, plan_stride);
      advance(s.plan_t, plan_stride);
      advance(s.slot_r, plan_stride);
      advance(s.slot_c, plan_stride);
      advance(s.plan_c, plan_stride);
      advance(s.node_spill, plan_stride);
    }
  }
  if (s.blk_head) block_head(s, 1);
  if (threadIdx.x == 0) *s.round_no = r0 + rounds;
}

// ---------------------------------------------------------------------------
// The same rounds with everything a round reads held on chip: the schedule of all rounds of the
// launch (delay and loss of every edge as 16-bit words, the activity masks) is copied to LDS first,
// the counters t and their history live in LDS, and every lane keeps the stamp and the delivery bits
// of its (at most two) edges in registers.  A round then costs LDS gathers and barriers; what it
// writes to global memory (plans, stamps, bits, counters, history) nobody waits for.  For graphs of
// up to 1024 nodes and about 2048 edges whose schedule fits into LDS; bit for bit the plans of the
// kernel above.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(kResolveThreads) rfast_resolve_cached_kernel(RfastDev s, int rounds, size_t plan_stride,
                                                                                const uint8_t* active, const int32_t* delay_R,
                                                                                const int32_t* delay_C, const uint8_t* drop_R,
                                                                                const uint8_t* drop_C, int lanes_R, int lanes_C) {
  extern __shared__ int lds_i[];
  __shared__ int wave_cnt[kResolveThreads / 64];
  const int n = s.n, E = s.eR + s.eC, H = s.H;
  const int T = blockDim.x;  // a multiple of 64, n <= T: barriers among few wavefronts are cheap
  // The first lanes_R lanes (whole wavefronts) look after the edges of R, the next lanes_C after those of C, up to
  // kAhead edges each: the kind of an edge is the same for all lanes of a wavefront, and small graphs have their
  // edges decided side by side in different wavefronts rather than one after the other in one.
  const bool kind = (int)threadIdx.x >= lanes_R;
  const int lane_k = kind ? (int)threadIdx.x - lanes_R : (int)threadIdx.x, lanes_k = kind ? lanes_C : lanes_R;
  const int edges_k = (int)threadIdx.x < lanes_R + lanes_C ? (kind ? s.eC : s.eR) : 0;
  const FastMod modM(s.M), modH(H);
  int* t_l = lds_i;                                                      // [n]
  int* hist_l = t_l + n;                                                 // [n][H]
  unsigned short* sched_l = reinterpret_cast<unsigned short*>(hist_l + n * H);  // [rounds][E]: delay | loss << 8 | out of range << 15
  uint8_t* act_l = reinterpret_cast<uint8_t*>(sched_l + (size_t)rounds * E + ((size_t)rounds * E & 1));  // [rounds][n]
  const int r0 = *s.round_no;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (s.blk_head) block_head(s, 0);
  for (int w = threadIdx.x; w < rounds * E; w += T) {
    const int q = w / E, e = w - q * E;
    const bool kind = e >= s.eR;
    const int d = kind ? delay_C[(size_t)q * s.eC + (e - s.eR)] : delay_R[(size_t)q * s.eR + e];
    const bool lost = (kind ? drop_C[(size_t)q * s.eC + (e - s.eR)] : drop_R[(size_t)q * s.eR + e]) != 0;
    const bool bad = d < 0 || d > s.d_max;
    sched_l[w] = (unsigned short)((d < 0 ? 0 : (d > s.d_max ? s.d_max : d)) | (lost ? 1 << 8 : 0) | (bad ? 1 << 15 : 0));
  }
  for (int w = threadIdx.x; w < rounds * n; w += T) act_l[w] = active[w];
  for (int i = threadIdx.x; i < n; i += T) t_l[i] = s.t[i];
  for (int w = threadIdx.x; w < n * H; w += T) hist_l[w] = s.t_hist[w];
  EdgeIn mine[kAhead];
#pragma unroll
  for (int a = 0; a < kAhead; ++a) {
    const int el = lane_k + a * lanes_k;
    if (el < edges_k) {
      mine[a].i = (kind ? s.c_dst : s.r_dst)[el];
      mine[a].j = (kind ? s.c_src : s.r_src)[el];
      mine[a].bits = (kind ? s.deliv_c : s.deliv_r)[el];
      mine[a].old = (kind ? s.tau_c : s.tau_r)[el];
    }
  }
  // The loads above must have landed before the round loop starts: the compiler puts the wait for a loaded register at
  // its first use, which is inside the loop, and a wait on the memory counter there also waits for every store of the
  // round before (a microsecond per round that nothing needs).  An empty asm that takes the registers is a use.
#pragma unroll
  for (int a = 0; a < kAhead; ++a) {
    unsigned lo = (unsigned)mine[a].bits, hi = (unsigned)(mine[a].bits >> 32);
    asm volatile("" : "+v"(mine[a].i), "+v"(mine[a].j), "+v"(mine[a].old), "+v"(lo), "+v"(hi));
    mine[a].bits = ((unsigned long long)hi << 32) | lo;
  }
  __syncthreads();
  const int i = threadIdx.x;  // the node this lane looks after (n <= T)
  for (int rq = 0; rq < rounds; ++rq) {
    const int r = r0 + rq, r_slot = modH(r);
    const uint8_t* act = act_l + (size_t)rq * n;
    // what the lane's edges see: schedule, activity and the sender's counters, all from LDS
#pragma unroll
    for (int a = 0; a < kAhead; ++a) {
      const int el = lane_k + a * lanes_k;
      const int e = kind ? s.eR + el : el;  // position in a round's schedule words: R's edges, then C's
      if (el < edges_k) {
        EdgeIn& q = mine[a];
        const unsigned sw = sched_l[(size_t)rq * E + e];
        const int d = sw & 0xFF;
        q.d = (sw >> 15) ? -1 : d;  // out of range: reported by edge_decide, resolved with the clamped value
        q.dropped = (sw >> 8) & 1;
        q.act_i = act[q.i] != 0;
        q.act_j = act[q.j] != 0;
        q.tj = t_l[q.j];
        const int at = r - d;
        q.u = at <= 0 ? 0 : (at >= r ? q.tj : hist_l[q.j * H + modH(at)]);
      }
    }
    if (threadIdx.x == 0 && s.blk_plan) s.blk_plan[n + E] = 0;  // a record ends with a word that is always zero
    // node pass: snapshot of the counters, and the ordered list of active nodes (ballot + prefix)
    bool on = false;
    int ti = 0;
    if (i < n) {
      ti = t_l[i];
      s.plan_t[i] = ti;
      s.node_spill[i] = 0;
      s.t_hist[(size_t)i * H + r_slot] = ti;
      on = act[i] != 0;
      if (s.blk_plan) s.blk_plan[i] = (ti & 0x3FFFFFFF) | (on ? (int)0x80000000 : 0);
    }
    const unsigned long long m = __ballot(on);
    if (lane == 0) wave_cnt[wave] = __popcll(m);
    __syncthreads();  // also: every lane has read the history of this round's delays
    if (i < n) hist_l[i * H + r_slot] = ti;
    int off = 0, total = 0;
    for (int w = 0; w < T / 64; ++w) {
      if (w < wave) off += wave_cnt[w];
      total += wave_cnt[w];
    }
    if (on) s.active_plan[off + __popcll(m & ((1ull << lane) - 1ull))] = make_int2(i, ti);
    if (threadIdx.x == 0) {
      s.n_active[0] = total;
      s.n_active[1] = r + 1;
    }
    for (int q = total + threadIdx.x; q < n + 8; q += T) s.active_plan[q] = make_int2(-1, 0);
#pragma unroll
    for (int a = 0; a < kAhead; ++a) {
      const int el = lane_k + a * lanes_k;
      if (el < edges_k) edge_decide(s, modM, kind, el, r, mine[a]);
    }
    __syncthreads();  // every read of the counters is done (and wave_cnt may be reused)
    if (on) {
      t_l[i] = ti + 1;
      s.t[i] = ti + 1;
    }
    __syncthreads();  // the next round reads what this one wrote
    if (s.blk_plan) s.blk_plan += n + E + 1;
    advance(s.n_active, plan_stride);
    advance(s.active_plan, plan_stride);
    advance(s.plan_t, plan_stride);
    advance(s.slot_r, plan_stride);
    advance(s.slot_c, plan_stride);
    advance(s.plan_c, plan_stride);
    advance(s.node_spill, plan_stride);
  }
  if (s.blk_head) block_head(s, 1);
  if (threadIdx.x == 0) *s.round_no = r0 + rounds;
}

size_t cached_lds_bytes(const RfastDev& d, int rounds) {
  const size_t E = (size_t)d.eR + d.eC;
  return ((size_t)d.n + (size_t)d.n * d.H) * sizeof(int) + (((size_t)rounds * E + 1) & ~(size_t)1) * sizeof(unsigned short) +
         (size_t)rounds * d.n;
}

}  // namespace

hipError_t rfast_launch_resolve(rfast_ctx* c, const uint8_t* active, const int32_t* delay_R,
                                const int32_t* delay_C, const uint8_t* drop_R, const uint8_t* drop_C, int rounds,
                                size_t plan_stride) {
  const RfastDev& d = c->d;
  const size_t lds = cached_lds_bytes(d, rounds);
  if (rounds > 1 && d.n <= kResolveThreads && (d.eR + 127) / 128 + (d.eC + 127) / 128 <= kResolveThreads / 64 && lds <= 150 * 1024) {
    static bool raised = false;
    if (!raised) {  // more than 64 KB of dynamic LDS has to be asked for once (the kernel has 64 B of static LDS too)
      const hipError_t e = hipFuncSetAttribute((const void*)rfast_resolve_cached_kernel,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, 152 * 1024);
      if (e != hipSuccess) return e;
      raised = true;
    }
    // whole wavefronts for the edges of R, then for those of C: one edge per lane if that fits 1024 lanes, else two;
    // as many lanes as the graph has nodes, at least four wavefronts for the copy of the schedule
    auto whole = [](int v) { return (v + 63) / 64 * 64; };
    int lanes_R = whole(d.eR), lanes_C = whole(d.eC);
    if (lanes_R + lanes_C > kResolveThreads) {
      lanes_R = whole((d.eR + 1) / 2);
      lanes_C = whole((d.eC + 1) / 2);
    }
    int threads = lanes_R + lanes_C > whole(d.n) ? lanes_R + lanes_C : whole(d.n);
    threads = threads < 256 ? 256 : threads;
    hipLaunchKernelGGL(rfast_resolve_cached_kernel, dim3(1), dim3(threads), lds, c->stream, c->d, rounds, plan_stride,
                       active, delay_R, delay_C, drop_R, drop_C, lanes_R, lanes_C);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(rfast_resolve_kernel, dim3(1), dim3(kResolveThreads), 0, c->stream, c->d, rounds, plan_stride, active,
                     delay_R, delay_C, drop_R, drop_C);
  return hipGetLastError();
}
