// Several activation rounds per launch with the state of a tile of coordinates resident in LDS,
// one tile per WORKGROUP: the form for graphs of 33 to 64 nodes (smaller graphs take the kernel of
// rfast_wave.hip, whose tile belongs to one wavefront and which needs no barrier).
//
// Everything in a round of Algorithm 1 is elementwise in the coordinate k: coordinate k of every
// node, ring slot and buffer depends, over any number of rounds, only on coordinate k of the
// others.  For the separable objective (whose gradient is elementwise too) a workgroup can
// therefore take a tile of coordinates of EVERY node, load the rings of v and of the running sums
// for them into LDS once, advance them through up to kBlockRounds rounds -- all neighbour reads of
// S2a / S2b and all publications of S3 are LDS traffic, with one barrier per round -- and write
// them back once.  HBM traffic per round drops from 13 words per coordinate and node-update to
// (2 M + 4 + 2 M + 2) / rounds words per coordinate and node (read everything, write everything,
// once per launch).  One launch also replaces up to kBlockRounds launches.
//
// Layout of the work: kLanes lanes per node, 4 consecutive coordinates per lane (one Philox call per
// lane and sample, as in the streaming kernel), so a workgroup has n kLanes lanes; x, z, the stored
// sample, the objective data and the edges of a node stay in the registers of its lanes for the
// whole launch.  The arithmetic is, operation for operation, that of rfast_state_kernel<FUSED>:
// the two paths give the same bits.
//
// The integer plans of the rounds (who is active, which slot each edge reads, where each S4
// buffer lives) are made by the resolver, one record per round, and copied to LDS sixteen rounds at
// a time.
#include "rfast_vec.h"

namespace {

constexpr int kMaxDeg = 4;  // most in-edges of R, in-edges of C and out-edges of C a node may have on this path
// Plan words a lane moves per refill: a record has at most (1 + 2 kMaxDeg) n + 1 words and a workgroup at
// least 16 n lanes, so kPlanChunk records are at most 16 (9 n + 1) <= 10 * 16 n words.
constexpr int kPlanPerLane = 10;

// kLanes: lanes per node, each owning 4 coordinates of a tile of 4 kLanes; TPB: upper bound of the
// workgroup size (n kLanes lanes, rounded up to whole wavefronts), which sets how many registers
// the compiler may use; kDeg: edge slots per node and kind (2 for rings and paths, else kMaxDeg).
// More than 32 nodes at 16 lanes each are more than 512 lanes, so the kernel runs with 128 registers: with two
// edge slots it fits them (four ring slots in flight while the tile moves instead of eight), with four it
// spills some 55 to scratch.  The alternative without spills, 8 lanes per node in workgroups of 512 with 186
// registers, was measured and is slower, because it halves the wavefronts per CU: 0.201 against 0.192 ms per
// round on a 6 x 6 mesh at p = 1 M, 0.149 against 0.088 ms on a ring of 36 nodes.
template <int kLanes, int TPB, int kDeg>
__global__ void __launch_bounds__(TPB) rfast_block_kernel(RfastDev s, RfastBlock blk) {
  constexpr int VEC = 4;
  constexpr int kRingBatch = TPB > 512 ? 4 : 8;  // ring slots (of both rings) in flight while the tile is moved
  extern __shared__ float4 lds4[];
  const int n = s.n, M = s.M;
  const int64_t p = s.p;
  const int PL = n + s.eR + s.eC;
  float4* v_l = lds4;                                  // [n][M][kLanes]
  float4* sg_l = v_l + (size_t)n * M * kLanes;         // [n][M][kLanes]
  int* plan_l = reinterpret_cast<int*>(sg_l + (size_t)n * M * kLanes);  // [kPlanChunk][PL + 1]
  const int i = threadIdx.x / kLanes, ln = threadIdx.x % kLanes;
  const int64_t k = (int64_t)blockIdx.x * (4 * kLanes) + ln * 4;
  const bool mine = i < n && k < p;
  // The S4 buffers stay in global memory: they are touched only when a version leaves a ring before
  // its receiver has consumed a newer one (a store by one lane; a load by another lane of this
  // workgroup in a later round, with the barrier of every round in between).
  float* const rt_g = s.rho_tilde + k;  // + e p: these coordinates of edge e

  // Plan records of kPlanChunk rounds at a time.  A record ends with a word that is always zero:
  // what the lanes of a node with fewer than kDeg edges read for the missing ones (slot 0, not live,
  // no spill), so that no read in the round loop is conditional.
  const int W1 = PL + 1;
  {
    const int words = (blk.rounds < kPlanChunk ? blk.rounds : kPlanChunk) * W1;
    for (int w = threadIdx.x; w < words; w += blockDim.x) plan_l[w] = s.blk_plan[w];
  }

  float4 x, z, g, h, c, m = make_float4(0.f, 0.f, 0.f, 0.f);
  const bool momentum = s.mom != nullptr;  // the optimizer variant's heavy-ball buffer (uniform)
  int re0 = 0, ce0 = 0, o0 = 0, dR = 0, dI = 0, dO = 0;
  float r_self = 0.f, c_self = 0.f;
  // the node's edges, in registers for the whole launch (at most kDeg of each kind, checked by the
  // host): LDS column of the sender's ring, weight, position of the edge's plan word in a record; a
  // missing edge has weight zero, the node's own column and the zero word of the record
  int r_col[kDeg], c_col[kDeg], r_pw[kDeg], c_pw[kDeg], o_pw[kDeg], o_eid[kDeg];
  float r_w[kDeg], c_w[kDeg], o_w[kDeg];
  const int own = i * M * kLanes + ln;  // this lane's column in the rings of its node (LDS offsets fit in 32 bits)
  unsigned put_v = 0, put_s = 0;        // one bit per slot of the node's rings: the slot is stored when the launch ends
  if (mine) {
    const size_t off = (size_t)i * p + k;
    x = V<VEC>::ld(s.x + off);
    z = V<VEC>::ld(s.z + off);
    h = V<VEC>::ld((const float*)s.prob.data0 + off);
    c = V<VEC>::ld((const float*)s.prob.data1 + off);
    if (momentum) m = V<VEC>::ld(s.mom + off);
    re0 = s.r_ptr[i]; dR = s.r_ptr[i + 1] - re0;
    ce0 = s.c_ptr[i]; dI = s.c_ptr[i + 1] - ce0;
    o0 = s.co_ptr[i]; dO = s.co_ptr[i + 1] - o0;
    r_self = s.r_self[i];
    c_self = s.c_self[i];
#pragma unroll
    for (int u = 0; u < kDeg; ++u) {
      const bool hr = u < dR, hc = u < dI, ho = u < dO;
      const int oe = ho ? s.co_eid[o0 + u] : 0;
      r_col[u] = (hr ? s.r_src[re0 + u] : i) * M * kLanes + ln;
      r_w[u] = hr ? s.r_w[re0 + u] : 0.f;
      r_pw[u] = hr ? n + re0 + u : PL;
      c_col[u] = (hc ? s.c_src[ce0 + u] : i) * M * kLanes + ln;
      c_w[u] = hc ? s.c_w[ce0 + u] : 0.f;
      c_pw[u] = hc ? n + s.eR + ce0 + u : PL;
      o_w[u] = ho ? s.co_w[o0 + u] : 0.f;
      o_pw[u] = ho ? n + s.eR + oe : PL;
      o_eid[u] = oe;
    }
    // rings: eight slots of both rings (sixteen loads) in flight at a time, then into LDS.  Only what can matter
    // is moved, as in the kernel with one tile per wavefront: the resolver has left one bit per slot saying whether
    // a receiver can still pick up the version it holds (RfastDev::blk_head); the other slots are zeros in LDS
    // (finite, for the multiply-adds with weight zero) and, further down, a slot goes back only if the launch wrote
    // it and its version is within reach afterwards.
    const int4 hd = *reinterpret_cast<const int4*>(s.blk_head + kHeadWords * i + 8);  // s0, se, in_v, in_s
    const int4 he = *reinterpret_cast<const int4*>(s.blk_head + kHeadWords * i + 12);  // written, out_v, out_s
    put_v = (unsigned)he.x & (unsigned)he.y;
    put_s = (unsigned)he.x & (unsigned)he.z;
    const float* vg = s.v_ring + (size_t)i * M * p + k;
    const float* sgg = s.sigma_ring + (size_t)i * M * p + k;
    for (int m0 = 0; m0 < M; m0 += kRingBatch) {
      float4 tv[kRingBatch], ts[kRingBatch];
      const unsigned get_v = (unsigned)hd.z >> m0, get_s = (unsigned)hd.w >> m0;  // bits past the last slot are clear
#pragma unroll
      for (int u = 0; u < kRingBatch; ++u) {
        tv[u] = ts[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (get_v & (1u << u)) tv[u] = V<VEC>::ld(vg + (size_t)(m0 + u) * p);
        if (get_s & (1u << u)) ts[u] = V<VEC>::ld(sgg + (size_t)(m0 + u) * p);
      }
#pragma unroll
      for (int u = 0; u < kRingBatch; ++u)
        if (m0 + u < M) {
          v_l[own + (m0 + u) * kLanes] = tv[u];
          sg_l[own + (m0 + u) * kLanes] = ts[u];
        }
    }
  }
  __syncthreads();
  // The stored sample of S2b is a function of (x_i, t_i); from here on it lives in registers, and so
  // do the ring slots of the node's current and next version (advanced without a division).
  int slot_cur = 0;
  if (mine) {
    const int t0 = plan_l[i] & 0x3FFFFFFF;
    g = diag_sample<VEC>(s, h, c, x, i, t0, k);
    slot_cur = t0 % M;
  }

  for (int q = 0; q < blk.rounds; ++q) {
    const int* P = plan_l + (q % kPlanChunk) * W1;
    // the records of the next kPlanChunk rounds are fetched during the last round of a chunk and
    // put into LDS once every lane is done with the old ones (the condition is uniform)
    const bool refill = (q + 1) % kPlanChunk == 0 && q + 1 < blk.rounds;
    int next_plan[kPlanPerLane];
    if (refill) {
      // every load unconditional (a word past the end reads word 0 instead and is not stored), so
      // that they are issued back to back and land while the round computes
      const int words = (blk.rounds - (q + 1) < kPlanChunk ? blk.rounds - (q + 1) : kPlanChunk) * W1;
      const int* src = s.blk_plan + (q + 1) * W1;
#pragma unroll
      for (int u = 0; u < kPlanPerLane; ++u) {
        const int w = threadIdx.x + u * (int)blockDim.x;
        next_plan[u] = src[w < words ? w : 0];
      }
    }
    // every plan word of the round in one batch of LDS reads, the node's own among them (an idle
    // node reads its edges' words for nothing, which is cheaper than a second round trip for the rest) ...
    int node_w = 0, r_slot[kDeg], c_pl[kDeg], o_pl[kDeg];
    if (mine) {
      node_w = P[i];
#pragma unroll
      for (int u = 0; u < kDeg; ++u) {
        r_slot[u] = P[r_pw[u]];
        c_pl[u] = P[c_pw[u]];
        o_pl[u] = P[o_pw[u]];
      }
    }
    if (node_w < 0) {  // bit 31: node i is activated in this round
      const int t_old = node_w & 0x3FFFFFFF;
      const int slot_new = slot_cur + 1 == M ? 0 : slot_cur + 1;
      const int leaving = slot_new + 1 == M ? 0 : slot_new + 1;
      // ... and every ring value of the round in a second one (what a missing or idle edge reads
      // is a valid address and is not used)
      float4 nb[kDeg], cur[kDeg], last[kDeg];
#pragma unroll
      for (int u = 0; u < kDeg; ++u) nb[u] = v_l[r_col[u] + r_slot[u] * kLanes];
      if (TPB > 512) __builtin_amdgcn_sched_barrier(0);  // registers: do not start the next batch early
#pragma unroll
      for (int u = 0; u < kDeg; ++u) {
        const int prev = (c_pl[u] >> 8) & 0xFF;
        cur[u] = sg_l[c_col[u] + (c_pl[u] & 0xFF) * kLanes];
        last[u] = sg_l[c_col[u] + (prev != 0xFF ? prev : 0) * kLanes];
      }
#pragma unroll
      for (int u = 0; u < kDeg; ++u)  // rare: the version consumed last time has left the sender's ring
        if ((c_pl[u] & (1 << 16)) && ((c_pl[u] >> 8) & 0xFF) == 0xFF) last[u] = V<VEC>::ld(rt_g + (size_t)(ce0 + u) * p);
      const float4 sig_cur = sg_l[own + slot_cur * kLanes];
      const float4 sig_leaving = sg_l[own + leaving * kLanes];
      // S1: local descent; with the optimizer variant along the heavy-ball buffer m <- beta m + z
      if (momentum) m = fma_s(s.beta, m, z);
      const float4 v = fma_s(-blk.gamma, momentum ? m : z, x);
      // S2a: pull the stamped neighbour copies and mix with row-stochastic weights
      float4 x_new = mul_s(r_self, v);
#pragma unroll
      for (int u = 0; u < kDeg; ++u)
        if (u < dR) x_new = fma_s(r_w[u], nb[u], x_new);
      const float4 g_new = diag_sample<VEC>(s, h, c, x_new, i, t_old + 1, k);
      // S2b: tracker sum over the in-edges of C; S4: buffer what was consumed
      float4 z_half = z;
#pragma unroll
      for (int u = 0; u < kDeg; ++u)
        if (c_pl[u] & (1 << 16)) {
          z_half = track_edge(z_half, c_w[u], cur[u], last[u], ((c_pl[u] >> 8) & 0xFF) != 0xFF);
          if (c_pl[u] & (1 << 17)) V<VEC>::st(rt_g + (size_t)(ce0 + u) * p, mul_s(c_w[u], cur[u]));
        }
      z_half = sub(add(z_half, g_new), g);
      // S3: publish version t+1 (slots nobody reads in this round); S2c: keep a_ii, push
      v_l[own + slot_new * kLanes] = v;
      if (dO > 0) {
        sg_l[own + slot_new * kLanes] = add(sig_cur, z_half);
        // S4 for receivers that do not do it themselves: version t - D leaves the ring; it sits two
        // slots ahead of the current one
#pragma unroll
        for (int u = 0; u < kDeg; ++u)
          if (o_pl[u] & (1 << 18)) V<VEC>::st(rt_g + (size_t)o_eid[u] * p, mul_s(o_w[u], sig_leaving));
      }
      x = x_new;
      z = mul_s(c_self, z_half);
      g = g_new;
      slot_cur = slot_new;
    }
    __syncthreads();  // S5: the round is over, its publications are visible
    if (refill) {
#pragma unroll
      for (int u = 0; u < kPlanPerLane; ++u) {
        const int w = threadIdx.x + u * (int)blockDim.x;
        if (w < kPlanChunk * W1) plan_l[w] = next_plan[u];
      }
      __syncthreads();
    }
  }

  if (mine) {
    const size_t off = (size_t)i * p + k;
    V<VEC>::st(s.x + off, x);
    V<VEC>::st(s.z + off, z);
    if (momentum) V<VEC>::st(s.mom + off, m);
    float* vg = s.v_ring + (size_t)i * M * p + k;
    float* sgg = s.sigma_ring + (size_t)i * M * p + k;
    for (int m0 = 0; m0 < M; m0 += kRingBatch) {
      float4 tv[kRingBatch], ts[kRingBatch];
      const unsigned back_v = put_v >> m0, back_s = put_s >> m0;
#pragma unroll
      for (int u = 0; u < kRingBatch; ++u) {
        if (back_v & (1u << u)) tv[u] = v_l[own + (m0 + u) * kLanes];
        if (back_s & (1u << u)) ts[u] = sg_l[own + (m0 + u) * kLanes];
      }
#pragma unroll
      for (int u = 0; u < kRingBatch; ++u) {
        if (back_v & (1u << u)) V<VEC>::st(vg + (size_t)(m0 + u) * p, tv[u]);
        if (back_s & (1u << u)) V<VEC>::st(sgg + (size_t)(m0 + u) * p, ts[u]);
      }
    }
  }
}

size_t block_lds_bytes(const RfastDev& d, int lanes) {
  return (size_t)2 * d.n * d.M * lanes * sizeof(float4) + (size_t)kPlanChunk * (d.n + d.eR + d.eC + 1) * sizeof(int);
}

// Lanes per node: the widest tile that fits LDS and 1024 lanes; a tile wider than 16 lanes per
// node must leave two tiles per CU of the chip to schedule.  (Graphs of up to 32 nodes take the
// kernel with one tile per wavefront instead, so a workgroup here has more than 512 lanes.)
constexpr int kLaneChoices[] = {28, 24, 16};
constexpr size_t kLdsBudget = 156 * 1024;

int block_lanes(const RfastDev& d) {
  for (int lanes : kLaneChoices) {
    const int threads = (d.n * lanes + 63) / 64 * 64;
    const bool fits = threads <= 1024 && block_lds_bytes(d, lanes) <= kLdsBudget &&
                      (int64_t)kPlanChunk * (d.n + d.eR + d.eC + 1) <= (int64_t)kPlanPerLane * threads;
    if (fits && (lanes == 16 || (d.p + 4 * lanes - 1) / (4 * lanes) >= 512)) return lanes;
  }
  return 0;
}

}  // namespace

// The tile of every node must fit into the LDS of one CU next to the plans, a workgroup holds at
// least 16 lanes per node, no node has more than kMaxDeg edges of a kind, and the path exists for the
// separable objective (the heavy-ball buffer of the optimizer variant is one more register set).
bool rfast_block_eligible(const rfast_ctx* c) {
  const RfastDev& d = c->d;
  return d.prob.kind == RFAST_OBJ_DIAG_QUADRATIC && (d.p % 4) == 0 && c->max_degree <= kMaxDeg && d.M <= 32 &&
         block_lanes(d) != 0;  // (rings of at most 32 slots: one bit per slot in the records of the resolver)
}

int rfast_block_lanes(const rfast_ctx* c) { return block_lanes(c->d); }

template <int kLanes, int TPB, int kDeg>
static hipError_t launch_block(rfast_ctx* c, const RfastBlock& blk, unsigned threads) {
  static bool raised = false;
  if (!raised) {  // more than 64 KB of dynamic LDS has to be asked for once per kernel
    const hipError_t e = hipFuncSetAttribute((const void*)rfast_block_kernel<kLanes, TPB, kDeg>,
                                             hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    raised = true;
  }
  const int64_t tiles = (c->d.p + 4 * kLanes - 1) / (4 * kLanes);
  if (tiles > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL((rfast_block_kernel<kLanes, TPB, kDeg>), dim3((unsigned)tiles), dim3(threads), block_lds_bytes(c->d, kLanes),
                     c->stream, c->d, blk);
  return hipGetLastError();
}

template <int kLanes>
static hipError_t launch_block_lanes(rfast_ctx* c, const RfastBlock& blk) {
  const unsigned threads = (unsigned)((c->d.n * kLanes + 63) / 64 * 64);
  if (threads <= 512) return c->max_degree <= 2 ? launch_block<kLanes, 512, 2>(c, blk, threads)
                                                : launch_block<kLanes, 512, kMaxDeg>(c, blk, threads);
  return c->max_degree <= 2 ? launch_block<kLanes, 1024, 2>(c, blk, threads)
                            : launch_block<kLanes, 1024, kMaxDeg>(c, blk, threads);
}

hipError_t rfast_launch_block(rfast_ctx* c, const RfastBlock& blk) {
  switch (block_lanes(c->d)) {
    case 28: return launch_block_lanes<28>(c, blk);
    case 24: return launch_block_lanes<24>(c, blk);
    case 16: return launch_block_lanes<16>(c, blk);
    default: return hipErrorInvalidValue;
  }
}
