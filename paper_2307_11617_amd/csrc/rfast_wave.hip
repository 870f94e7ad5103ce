// Several activation rounds per launch with the tile of one WAVEFRONT resident in LDS.
//
// Like rfast_block.hip (every step of Algorithm 1 is elementwise in the coordinate, so a tile of
// coordinates of every node can stay on chip over many rounds), with one difference that removes
// every barrier from the round loop: a tile belongs to a single wavefront.  The 64 lanes of a
// wavefront are split among ALL nodes (16 nodes: 4 lanes per node, 4 coordinates per lane, a tile of
// 16 coordinates), so every neighbour read of S2a / S2b and every publication of S3 stays within the
// wavefront, whose LDS operations execute in program order: a round needs no synchronisation with
// any other wavefront, the wavefronts of a CU drift out of step, and while one waits for its LDS
// reads another computes.  The plan words of a round are read from global memory one round ahead
// (the records of all rounds are a few KB that every wavefront of the chip reads, so they stay in the
// caches), which leaves LDS to the rings and takes the plan reads out of the critical path.  The S4
// buffers live in the registers of the receiving node's lanes: a buffer is needed only after its
// version has left the sender's ring, and in the round in which it leaves the receiver's lanes copy
// it from that ring themselves (the resolver marks the round and names the slot), whether the
// receiver is active or not.  So the round loop touches global memory for the plan words only.
//
// The arithmetic is, operation for operation, that of rfast_state_kernel<FUSED> and of
// rfast_block_kernel: the three paths give the same bits.  (One liberty: where those skip a missing
// or idle edge, this kernel runs it through the multiply-add with weight zero, which spares the round
// loop most of its branches.  Adding zero changes nothing but the sign of a sum that is exactly zero,
// as long as the ring values are finite.)
#include <algorithm>

#include "rfast_vec.h"

namespace {

constexpr int kWaveMaxDeg = 6;  // most in-edges of R, in-edges of C and out-edges of C a node may have on this path
                                // (kernels for 2, 4 and 6 edge slots per node: an exponential graph on 32 nodes has 5
                                // edges per node and kind; 8 slots would not fit the registers of two wavefronts per SIMD)
constexpr int kWaveMaxNodes = 32;  // at least 2 lanes (8 coordinates, 32 B of a row) per node
constexpr unsigned kXcds = 8;      // accelerator dies; consecutive workgroups go round them
constexpr unsigned kTileRun = 64;  // neighbouring tiles that one XCD takes in a row
constexpr unsigned kSyncTileRun = 4;  // the same for the multi-step synchronous kernel (measured: 4 is 3 % faster there than 64)

// Orders the LDS and global accesses of the lanes of one wavefront: everything before it is done
// (in program order of the wavefront) before anything after it starts.
__device__ inline void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// lw: lanes per node (64 / n, rounded down); kDeg: edge slots per node and kind; MOM: the optimizer
// variant is in use, heavy-ball buffer, weight decay or both (a template flag, so that the plain method
// carries neither the registers and the copies at the join nor the tests).
// W: wavefronts per workgroup.  Every wavefront still owns a tile of 4 lw coordinates and runs its
// rounds without looking at the others; the W tiles of a workgroup are neighbours, and the workgroup
// moves their rings between HBM and LDS together, so that a row segment is W times as wide (16 nodes,
// W = 2: 128 B, a whole cache line per row; with one wavefront per workgroup every load and store
// instruction touched 16 half lines).  The barriers this costs stand before and after the round loop,
// not in it.
// (A persistent grid, as many workgroups as the chip holds with each streaming through a region of
// its own, was measured and dropped: its workgroups run in step, so that all of them move tiles at one
// time and compute at another, and a launch of 20 rounds took 10.9 ms against 8.6 ms.  With a delay of
// its own for every workgroup at the start, up to 14 us, and what depends on the node alone set up once
// per wavefront, 10 rounds took 5.1 ms against 5.3, but 20 rounds 7.4 against 7.1 and 500 rounds 101.8
// against 93.9: the same round loop, instruction for instruction, ran 8 % slower.)
// Occupancy is pinned to two wavefronts per SIMD, which is what the LDS of a CU holds at nine ring
// slots: once the registers allowed three, the eight wavefronts of a CU were spread unevenly over
// its SIMDs and the launch took 4 % longer.
//
// Only what can matter is moved.  Stamps never go back (S2a / S2b take the largest stamp received), so
// a version older than every stamp held on its sender's out-edges will never be read again: such a
// slot is neither loaded (LDS gets zeros, which the multiply-adds with weight zero need to be finite)
// nor, if the launch wrote it and it is out of reach again by the end, stored; slots the launch did
// not write are not stored either, nor x and z of a node it never activated, and an S4 buffer is moved
// only while its version is outside its sender's ring.  With the delays of the bidirectional-ring
// workload that is 30 rows per node instead of 46.
// Multipliers for the two divisions of a lane number that the kernel starts with, by the lanes per node and by the
// lanes of a row segment: x / d = (x * ceil(2^16 / d)) >> 16 for x < 256 and d <= 256 (the error of the quotient,
// x (d ceil(2^16 / d) - 2^16) / (2^16 d), stays below 1 / d).  The division itself is some 25 instructions, which
// every wavefront of a launch would run.
struct WaveDiv {
  unsigned lanes, segment;
};
static WaveDiv wave_div(int lw, int W) {
  WaveDiv dv;
  dv.lanes = (65536u + (unsigned)lw - 1) / (unsigned)lw;
  dv.segment = (65536u + (unsigned)(lw * W) - 1) / (unsigned)(lw * W);
  return dv;
}

template <int kDeg, bool MOM, int W>
__global__ void __launch_bounds__(64 * W) __attribute__((amdgpu_waves_per_eu(2, 2))) rfast_wave_kernel(RfastDev s, RfastBlock blk, int lw, WaveDiv dv) {
  constexpr int VEC = 4;
  extern __shared__ float4 lds4[];
  const int n = s.n, M = s.M;
  const int64_t p = s.p;
  const int W1 = n + s.eR + s.eC + 1;  // words of a plan record; the last one is always zero
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i = (int)(((unsigned)lane * dv.lanes) >> 16), ln = lane - i * lw;  // lane / lw
  // Workgroup b runs on XCD b mod 8, each with an L2 of its own.  Neighbouring workgroups go to the same
  // XCD, one right after the other, in runs that cover kTileRun tiles (4 KB of every row on 16 nodes):
  // that keeps the rows an XCD moves at one time on few pages (a launch of 10 rounds, which is all moving,
  // took 8.1 ms with such runs and 9.3 ms with runs of 4 tiles), and where a row segment is less than a
  // cache line the neighbour finds the other part in that L2.
  constexpr unsigned kRun = kTileRun / W;
  const unsigned xcd = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
  const int64_t group = ((int64_t)(slot / kRun) * kXcds + xcd) * kRun + slot % kRun;
  const int64_t k_wg = group * (4 * lw * W);  // first coordinate of the workgroup
  if (k_wg >= p) return;  // a workgroup past the end (the grid is whole runs): all of its wavefronts leave
  const int64_t k = k_wg + (wave * lw + ln) * 4;
  const bool wave_has = k_wg + (int64_t)wave * lw * 4 < p;  // this wavefront has a tile (the last workgroup may be ragged)
  const bool mine = i < n && k < p;
  const size_t ring_f4 = (size_t)n * M * lw;   // float4 of one ring of one wavefront's tile
  float4* v_l = lds4 + (size_t)wave * 2 * ring_f4;  // [n][M][lw], the tile of this wavefront
  float4* sg_l = v_l + ring_f4;                     // [n][M][lw]
  // LDS addresses are byte offsets: column of the lane in a node's ring + slot * bytes per slot, one
  // 24-bit multiply-add each
  const unsigned slot_bytes = (unsigned)lw * sizeof(float4);
  auto at = [&](float4* ring, unsigned column, int slot) -> float4& {
    return *reinterpret_cast<float4*>(reinterpret_cast<char*>(ring) + (__umul24((unsigned)slot, slot_bytes) + column));
  };
  // Moving the rings: lane T of the workgroup moves column cT (of the lw W columns of a row segment) of
  // node iT, i.e. column lT of the tile of wavefront wT.  With W = 1 that is the lane's own column.
  const int seg = lw * W;
  const int iT = W == 1 ? i : (int)((threadIdx.x * dv.segment) >> 16), cT = (int)threadIdx.x - iT * seg;  // threadIdx.x / seg
  const int wT = W == 1 ? 0 : (int)(((unsigned)cT * dv.lanes) >> 16), lT = cT - wT * lw;                  // cT / lw
  const int64_t kT = k_wg + 4 * cT;
  const bool moves = iT < n && kT < p;
  float4* mv_l = lds4 + (size_t)wT * 2 * ring_f4 + (size_t)iT * M * lw + lT;  // + slot * lw (+ ring_f4 for the sums)
  // What the resolver, which has been through all rounds of the launch already, left about the moved node: the slot
  // of its latest version after the launch and, one bit per ring slot, which slots hold versions that a receiver
  // can still pick up before the launch (the others are not loaded), which the launch writes, and which hold
  // versions that can still be picked up after it (RfastDev::blk_head).
  int se_T = 0;
  unsigned in_v = 0, in_s = 0, put_v = 0, put_s = 0;
  if (moves) {
    const int4 a = *reinterpret_cast<const int4*>(s.blk_head + kHeadWords * iT + 8);   // s0, se, in_v, in_s
    const int4 b = *reinterpret_cast<const int4*>(s.blk_head + kHeadWords * iT + 12);  // written, out_v, out_s
    se_T = a.y; in_v = (unsigned)a.z; in_s = (unsigned)a.w;
    // a slot goes back if the launch wrote it and somebody can still read its version; with a rebase on the way
    // out every readable slot of the running sums is shifted, written or not
    put_v = (unsigned)b.x & (unsigned)b.y;
    put_s = blk.rebase ? (unsigned)b.z : (unsigned)b.x & (unsigned)b.z;
  }

  float4 x, z, g, h, c, m = make_float4(0.f, 0.f, 0.f, 0.f);
  const bool momentum = MOM && s.mom != nullptr;  // the heavy-ball buffer of the optimizer variant is in use
  int ce0 = 0, dR = 0, dI = 0, dO = 0;
  // The S4 buffers of the node's in-edges, in registers: a buffer matters only once its version has left
  // the sender's ring, and the receiver's own lanes copy it from that ring in the round in which it leaves
  // (active or not), so no other lane and no global memory is involved between load and store.
  float4 rt[kDeg];
  float r_self = 0.f, c_self = 0.f;
  // the node's edges, in registers for the whole launch: LDS column of the sender's ring, weight,
  // position of the edge's plan word in a record; a missing edge has weight zero, the node's own
  // column and the zero word of the record
  unsigned r_col[kDeg], c_col[kDeg];
  // positions of plan words as unsigned byte offsets: a 32-bit offset from a uniform base, no 64-bit address arithmetic
  unsigned r_pw[kDeg], c_pw[kDeg];
  float r_w[kDeg], c_w[kDeg];
  int c_from[kDeg];  // sender of each in-edge of C
  int rt_where[kDeg], end_slot[kDeg];
#pragma unroll
  for (int u = 0; u < kDeg; ++u) {
    rt_where[u] = end_slot[u] = 0;
    r_col[u] = c_col[u] = 0;
    r_pw[u] = c_pw[u] = 4u * (W1 - 1);
    r_w[u] = c_w[u] = 0.f;
    c_from[u] = 0;
    rt[u] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
  const unsigned own = (unsigned)(i * M * lw + ln) * sizeof(float4);  // this lane's column in the rings of its node
  unsigned node_pw = 4u * (W1 - 1);
  if (mine) {
    node_pw = 4u * i;
    const int re0 = s.r_ptr[i];
    dR = s.r_ptr[i + 1] - re0;
    ce0 = s.c_ptr[i];
    dI = s.c_ptr[i + 1] - ce0;
    dO = s.co_ptr[i + 1] - s.co_ptr[i];
    r_self = s.r_self[i];
    c_self = s.c_self[i];
#pragma unroll
    for (int u = 0; u < kDeg; ++u) {
      const bool hr = u < dR, hc = u < dI;
      r_col[u] = (unsigned)((hr ? s.r_src[re0 + u] : i) * M * lw + ln) * sizeof(float4);
      r_w[u] = hr ? s.r_w[re0 + u] : 0.f;
      r_pw[u] = 4u * (hr ? n + re0 + u : W1 - 1);
      c_from[u] = hc ? s.c_src[ce0 + u] : i;
      c_col[u] = (unsigned)(c_from[u] * M * lw + ln) * sizeof(float4);
      c_w[u] = hc ? s.c_w[ce0 + u] : 0.f;
      c_pw[u] = 4u * (hc ? n + s.eR + ce0 + u : W1 - 1);
    }
  }
  // Plan words are read through a buffer descriptor over the records of this launch: the address is
  // descriptor + uniform record offset + 32-bit lane offset, formed by the load itself (no 64-bit
  // address arithmetic per word), and a read past the records returns zero instead of faulting.
  // First those of round 0 (every lane: the lanes of a wavefront without a node read the zero word).
  const __amdgpu_buffer_rsrc_t plans = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<int*>(s.blk_plan), 0, blk.rounds * W1 * (int)sizeof(int), 0x00020000);
  const int rec_bytes = W1 * (int)sizeof(int);
  auto word = [&](int round, unsigned byte_offset) {
    return __builtin_amdgcn_raw_buffer_load_b32(plans, byte_offset, round * rec_bytes, 0);
  };
  struct Plan {
    int node, r[kDeg], c[kDeg];
  };
  auto fetch = [&](int round, Plan& P) {
    P.node = word(round, node_pw);
#pragma unroll
    for (int u = 0; u < kDeg; ++u) {
      P.r[u] = word(round, r_pw[u]);
      P.c[u] = word(round, c_pw[u]);
    }
  };
  Plan plan_a, plan_b;  // two register sets that take turns: one in use, one arriving
  fetch(0, plan_a);
  if (mine) {
    const size_t off = (size_t)i * p + k;
    x = V<VEC>::ld(s.x + off);
    z = V<VEC>::ld(s.z + off);
    h = V<VEC>::ld((const float*)s.prob.data0 + off);
    c = V<VEC>::ld((const float*)s.prob.data1 + off);
    if (momentum) m = V<VEC>::ld(s.mom + off);
    // an S4 buffer is in the rho_tilde array only while its version is outside its sender's ring (rare)
#pragma unroll
    for (int u = 0; u < kDeg; ++u)
      if (u < dI) {
        rt_where[u] = s.blk_head[kHeadWords * n + ce0 + u];
        end_slot[u] = s.blk_head[kHeadWords * c_from[u] + 9];  // of the sender's latest version after the launch
        if (rt_where[u] & 1) rt[u] = V<VEC>::ld(s.rho_tilde + (size_t)(ce0 + u) * p + k);
      }
  }
  // rings: kBatch slots of both rings in flight at a time (rings of up to twelve slots in one round trip to
  // memory), then into LDS; a slot whose version nobody can read any more gets zeros instead
  constexpr int kBatch = kDeg <= 2 ? 12 : (kDeg <= 4 ? 10 : 8);
  if (moves) {
    const float* vg = s.v_ring + (size_t)iT * M * p + kT;
    const float* sgg = s.sigma_ring + (size_t)iT * M * p + kT;
    for (int m0 = 0; m0 < M; m0 += kBatch) {
      float4 tv[kBatch], ts[kBatch];
      const unsigned get_v = in_v >> m0, get_s = in_s >> m0;  // bits past the last slot are clear
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        tv[u] = ts[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (get_v & (1u << u)) tv[u] = V<VEC>::ld(vg);
        if (get_s & (1u << u)) ts[u] = V<VEC>::ld(sgg);
        vg += p;
        sgg += p;
      }
#pragma unroll
      for (int u = 0; u < kBatch; ++u)
        if (m0 + u < M) {
          mv_l[(size_t)(m0 + u) * lw] = tv[u];
          mv_l[ring_f4 + (size_t)(m0 + u) * lw] = ts[u];
        }
    }
  }
  // The stored sample of S2b is a function of (x_i, t_i); from here on it lives in registers, and so
  // does the LDS address of the node's current version in its v ring (advanced by one slot per activation,
  // back to the first slot after the last: no division, no multiplication).
  // These are LDS addresses proper (32 bits, the start of the array included), so that the access needs no
  // further addition.
  typedef float Vec4 __attribute__((ext_vector_type(4)));
  typedef __attribute__((address_space(3))) Vec4 LdsVec4;
  const unsigned a_own =
      (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)lds4 + (unsigned)(wave * 2 * ring_f4 * sizeof(float4)) + own;
  unsigned a_cur = a_own;
  int ver_next = 1, ver_first = 1;  // version of the node's next activation (counted here: the plan's copy would need a mask and an add)
  const unsigned a_end = a_own + __umul24((unsigned)M, slot_bytes), sg_off = (unsigned)n * M * slot_bytes;
  auto own_ld = [&](unsigned a) {
    const Vec4 t = *(LdsVec4*)(uintptr_t)a;
    return make_float4(t.x, t.y, t.z, t.w);
  };
  auto own_st = [&](unsigned a, float4 w) {
    const Vec4 t = {w.x, w.y, w.z, w.w};
    *(LdsVec4*)(uintptr_t)a = t;
  };
  if (mine) {
    const int t0 = plan_a.node & 0x3FFFFFFF;
    g = diag_sample<VEC, MOM>(s, h, c, x, i, t0, k);
    a_cur = a_own + __umul24((unsigned)s.blk_head[kHeadWords * i + 8], slot_bytes);  // the slot of version t0
    ver_next = ver_first = t0 + 1;
  }
  if (W > 1) __syncthreads();  // the tiles of the workgroup are in LDS
  else wave_sync();

  // one round with the plan words P, while those of the round after it arrive in N
  auto round = [&](int q, const Plan& P, Plan& N) {
    const bool active = P.node < 0;  // bit 31: node i is activated in this round (never set in the zero word)
    const unsigned a_new = a_cur + slot_bytes == a_end ? a_own : a_cur + slot_bytes;
    float4 nb[kDeg], cur[kDeg], last[kDeg], sig_cur;
    // S4 for a buffer whose version leaves its sender's ring in this round without the receiver consuming
    // a newer one (bit 18; the word then names the slot of that version): copied while it is still there
    // (rare: one test for all in-edges of the node)
    int leaving = 0;
#pragma unroll
    for (int u = 0; u < kDeg; ++u) leaving |= P.c[u];
    if (leaving & (1 << 18)) {
#pragma unroll
      for (int u = 0; u < kDeg; ++u)
        if (P.c[u] & (1 << 18)) rt[u] = mul_s(c_w[u], at(sg_l, c_col[u], P.c[u] & 0xFF));
    }
    // the plan words of the next round, from global memory, used one round from now
    fetch(min(q + 1, blk.rounds - 1), N);
    if (active) {
      // every ring value of the round in one batch of LDS reads (what a missing or idle edge reads
      // is a valid address; its value is multiplied by zero)
#pragma unroll
      for (int u = 0; u < kDeg; ++u) nb[u] = at(v_l, r_col[u], P.r[u]);
#pragma unroll
      for (int u = 0; u < kDeg; ++u) {
        const int prev = (P.c[u] >> 8) & 0xFF;  // 0xFF: not in the ring (any slot will do, the value is not used)
        cur[u] = at(sg_l, c_col[u], P.c[u] & 0xFF);
        last[u] = at(sg_l, c_col[u], min(prev, M - 1));
      }
      sig_cur = own_ld(a_cur + sg_off);
      // S1: local descent; with the optimizer variant along the heavy-ball buffer m <- beta m + z
      if (momentum) m = fma_s(s.beta, m, z);
      const float4 v = fma_s(-blk.gamma, momentum ? m : z, x);
      // S2a: pull the stamped neighbour copies and mix with row-stochastic weights
      float4 x_new = mul_s(r_self, v);
      // (a missing edge has weight zero and reads the node's own ring: it adds zero, without a branch)
#pragma unroll
      for (int u = 0; u < kDeg; ++u) x_new = fma_s(r_w[u], nb[u], x_new);
      const float4 g_new = diag_sample<VEC, MOM>(s, h, c, x_new, i, ver_next, k);
      ++ver_next;
      // S2b: tracker sum over the in-edges of C; S4: buffer what was consumed
      float4 z_half = z;
#pragma unroll
      for (int u = 0; u < kDeg; ++u) {
        // The usual case — a live edge (bit 16) whose previous version is still in the ring (bits 8-15 below
        // 0xFF) and whose consumed version does not leave it (bit 17 clear) — and the idle edge run through the
        // same multiply-add, the idle edge with weight zero (it adds zero to z): no branch; the other live
        // cases are rare and branch.
        // (bits 30 and 31 of the word say which case it is: one signed compare each)
        const float a_eff = P.c[u] > 0x3FFFFFFF ? c_w[u] : 0.f;
        z_half = track_edge(z_half, a_eff, cur[u], last[u], true);
        if (P.c[u] < 0) {
          if (((P.c[u] >> 8) & 0xFF) != 0xFF) z_half = track_edge(z_half, c_w[u], cur[u], last[u], true);
          else z_half = track_edge(z_half, c_w[u], cur[u], rt[u], false);  // the version consumed last time has left the ring
          if (P.c[u] & (1 << 17)) rt[u] = mul_s(c_w[u], cur[u]);  // consumed, and leaving the ring in this round
        }
      }
      z_half = sub(add(z_half, g_new), g);
      // S3: publish version t+1 (slots nobody reads in this round); S2c: keep a_ii, push
      own_st(a_new, v);
      if (dO > 0) own_st(a_new + sg_off, add(sig_cur, z_half));
      x = x_new;
      z = mul_s(c_self, z_half);
      g = g_new;
      a_cur = a_new;
    }
    wave_sync();  // S5: the round is over, its publications are visible to the lanes of this wavefront
  };
  if (wave_has) {
    for (int q = 0; q < blk.rounds; q += 2) {
      round(q, plan_a, plan_b);
      if (q + 1 < blk.rounds) round(q + 1, plan_b, plan_a);
    }
  }
  // The last plan words asked for are not used.  They are looked at here all the same, on every path: memory
  // operations complete in order, and as long as the compiler has to assume that a load may still be under way on
  // some path, each wait it places for that load in the write-back is a wait for every store issued before it.
  auto settle = [](const Plan& P) {
    asm volatile("" ::"v"(P.node));
#pragma unroll
    for (int u = 0; u < kDeg; ++u) asm volatile("" ::"v"(P.r[u]), "v"(P.c[u]));
  };
  settle(plan_a);
  settle(plan_b);

  // Write-back.  With blk.rebase the running sums are rebased on the way (what rfast_rebase_kernel does, and with
  // its operations): sender j's latest sum leaves every slot of its ring, and a_ij times it every buffer it feeds.
  // s.t holds the counters after the launch, and t mod M is the slot of a node's latest version then.
  if (mine) {
    const size_t off = (size_t)i * p + k;
    if (ver_next != ver_first) {  // x and z of a node that was not activated are what they were
      V<VEC>::st(s.x + off, x);
      V<VEC>::st(s.z + off, z);
      if (momentum) V<VEC>::st(s.mom + off, m);
    }
#pragma unroll
    for (int u = 0; u < kDeg; ++u)
      // the buffer lives in the array only if its version is outside the sender's ring now
      if (u < dI && (rt_where[u] & 2)) {
        if (blk.rebase) rt[u] = sub(rt[u], mul_s(c_w[u], at(sg_l, c_col[u], end_slot[u])));
        V<VEC>::st(s.rho_tilde + (size_t)(ce0 + u) * p + k, rt[u]);
      }
  }
  if (W > 1) __syncthreads();  // every wavefront of the workgroup is through with its rounds
  else wave_sync();
  if (moves) {
    float4 base = make_float4(0.f, 0.f, 0.f, 0.f);
    const bool shift = blk.rebase && put_s != 0;  // nobody reads the sums of a node without out-edges
    if (shift) base = mv_l[ring_f4 + (size_t)se_T * lw];
    float* vg = s.v_ring + (size_t)iT * M * p + kT;
    float* sgg = s.sigma_ring + (size_t)iT * M * p + kT;
    for (int m0 = 0; m0 < M; m0 += kBatch) {
      float4 tv[kBatch], ts[kBatch];
      const unsigned back_v = put_v >> m0, back_s = put_s >> m0;  // bits past the last slot are clear
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        if (back_v & (1u << u)) tv[u] = mv_l[(size_t)(m0 + u) * lw];
        if (back_s & (1u << u)) {
          ts[u] = mv_l[ring_f4 + (size_t)(m0 + u) * lw];
          if (shift) ts[u] = sub(ts[u], base);
        }
      }
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        if (back_v & (1u << u)) V<VEC>::st(vg, tv[u]);
        if (back_s & (1u << u)) V<VEC>::st(sgg, ts[u]);
        vg += p;
        sgg += p;
      }
    }
  }
}

// ---------------------------------------------------------------------------
// The synchronous push-pull step of eq. (2), several steps per launch, on the same tiling: every
// node steps at once and reads its neighbours' current x - gamma z and z, which the lanes of the
// wavefront exchange through two LDS rows per node.  x, z, the stored sample and the objective data
// stay in registers; the arithmetic is that of rfast_sync_descent_kernel + rfast_sync_step_kernel
// (the stored sample of a step is the new sample of the step before: the same function of the same
// arguments that the one-step kernels recompute).  On return z is in its own array and slot 0 of
// the v ring holds the last x - gamma z, as after the one-step kernels.
// ---------------------------------------------------------------------------
template <int kDeg, bool MOM>
__global__ void __launch_bounds__(64) rfast_sync_wave_kernel(RfastDev s, float gamma, int rounds, int lw) {
  constexpr int VEC = 4;
  extern __shared__ float4 lds4[];
  const int n = s.n;
  const int64_t p = s.p;
  const int lane = threadIdx.x;
  const int i = lane / lw, ln = lane - i * lw;
  const unsigned xcd = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
  const int64_t tile = ((int64_t)(slot / kSyncTileRun) * kXcds + xcd) * kSyncTileRun + slot % kSyncTileRun;
  const int64_t k = tile * (4 * lw) + ln * 4;
  const bool mine = i < n && k < p;
  float4* v_l = lds4;                   // [n][lw]
  float4* z_l = v_l + (size_t)n * lw;   // [n][lw]
  if (!mine) return;  // no barrier below: the lanes of a wavefront without coordinates may leave
  const int own = i * lw + ln;
  const size_t off = (size_t)i * p + k;
  float4 x = V<VEC>::ld(s.x + off), z = V<VEC>::ld(s.z + off);
  const float4 h = V<VEC>::ld((const float*)s.prob.data0 + off), c = V<VEC>::ld((const float*)s.prob.data1 + off);
  float4 m = make_float4(0.f, 0.f, 0.f, 0.f);
  if (MOM) m = V<VEC>::ld(s.mom + off);
  const int re0 = s.r_ptr[i], ce0 = s.c_ptr[i];
  const int dR = s.r_ptr[i + 1] - re0, dI = s.c_ptr[i + 1] - ce0;
  const float r_self = s.r_self[i], c_self = s.c_self[i];
  int r_col[kDeg], c_col[kDeg];
  float r_w[kDeg], c_w[kDeg];
#pragma unroll
  for (int u = 0; u < kDeg; ++u) {
    r_col[u] = (u < dR ? s.r_src[re0 + u] : i) * lw + ln;
    r_w[u] = u < dR ? s.r_w[re0 + u] : 0.f;
    c_col[u] = (u < dI ? s.c_src[ce0 + u] : i) * lw + ln;
    c_w[u] = u < dI ? s.c_w[ce0 + u] : 0.f;
  }
  int t = s.t[i];
  float4 g = diag_sample<VEC>(s, h, c, x, i, t, k), v = x;
  for (int q = 0; q < rounds; ++q) {
    if (MOM) m = fma_s(s.beta, m, z);
    v = fma_s(-gamma, MOM ? m : z, x);
    v_l[own] = v;
    z_l[own] = z;
    wave_sync();  // every node's v and z of this step are out
    float4 nb[kDeg], zb[kDeg];
#pragma unroll
    for (int u = 0; u < kDeg; ++u) {
      nb[u] = v_l[r_col[u]];
      zb[u] = z_l[c_col[u]];
    }
    float4 x_new = mul_s(r_self, v);
#pragma unroll
    for (int u = 0; u < kDeg; ++u) x_new = fma_s(r_w[u], nb[u], x_new);  // a missing edge: weight zero, own row
    const float4 g_new = diag_sample<VEC>(s, h, c, x_new, i, t + 1, k);
    float4 z_new = mul_s(c_self, z);
#pragma unroll
    for (int u = 0; u < kDeg; ++u) z_new = fma_s(c_w[u], zb[u], z_new);
    z_new = sub(add(z_new, g_new), g);
    wave_sync();  // every read of this step is done before the next one overwrites the rows
    x = x_new;
    z = z_new;
    g = g_new;
    ++t;
  }
  V<VEC>::st(s.x + off, x);
  V<VEC>::st(s.z + off, z);
  if (MOM) V<VEC>::st(s.mom + off, m);
  V<VEC>::st(s.v_ring + (size_t)i * s.M * p + k, v);
}

size_t wave_lds_bytes(const RfastDev& d, int lw) { return (size_t)2 * d.n * d.M * lw * sizeof(float4); }

}  // namespace

// The separable objective, p a multiple of 4, at most 32 nodes with at most kWaveMaxDeg edges of a
// kind each, rings of at most 32 slots (one bit per slot in the records of the resolver), and the rings of one
// wavefront's tile fitting into LDS.
bool rfast_wave_eligible(const rfast_ctx* c) {
  const RfastDev& d = c->d;
  return d.prob.kind == RFAST_OBJ_DIAG_QUADRATIC && (d.p % 4) == 0 && c->max_degree <= kWaveMaxDeg &&
         d.n <= kWaveMaxNodes && d.M <= 32 && wave_lds_bytes(d, 64 / d.n) <= 156 * 1024;
}

int rfast_wave_lanes(const rfast_ctx* c) { return 64 / c->d.n; }

// Wavefronts per workgroup.  Short launches, which are mostly tile movement, gain from row segments of a
// whole cache line of 128 B (as many wavefronts, 2 or 4, as that takes, unless LDS then holds fewer
// wavefronts per CU); long ones lose more to the workgroup's barriers and to its wavefronts leaving together
// than the wider segments save.  Measured on 16 nodes x 11.2 M coordinates, nine ring slots, ms per launch
// with 1 / 2 / 4 wavefronts: 10 rounds 5.60 / 5.29 / 5.35, 20 rounds 7.15 / 7.17 / 7.27, 100 rounds
// 22.5 / 23.4 / 23.1.
static int wave_group(const rfast_ctx* c, int rounds) {
  const RfastDev& d = c->d;
  const int lw = 64 / d.n;
  const size_t one = wave_lds_bytes(d, lw), cu = 160 * 1024;
  if (c->wave_group == 1 || c->wave_group == 2 || c->wave_group == 4) return (size_t)c->wave_group * one <= cu ? c->wave_group : 1;
  if (rounds >= 16) return 1;
  const size_t resident = std::min<size_t>(cu / one, 8);  // wavefronts of this kernel a CU holds (two per SIMD at most)
  int w = 1;
  while (w < 4 && (size_t)(w * lw) * sizeof(float4) < 128 && std::min<size_t>(cu / (2 * w * one) * (2 * w), 8) >= resident) w *= 2;
  return w;
}

template <int kDeg, bool MOM, int W>
static hipError_t launch_wave(rfast_ctx* c, const RfastBlock& blk) {
  static bool raised = false;
  if (!raised) {  // more than 64 KB of dynamic LDS has to be asked for once per kernel
    const hipError_t e = hipFuncSetAttribute((const void*)rfast_wave_kernel<kDeg, MOM, W>,
                                             hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    raised = true;
  }
  const RfastDev& d = c->d;
  if (!d.blk_plan || !d.blk_head) return hipErrorInvalidValue;
  const int lw = 64 / d.n;
  const int64_t run = (int64_t)kXcds * (kTileRun / W), per = (int64_t)4 * lw * W;
  const int64_t groups = ((d.p + per - 1) / per + run - 1) / run * run;  // whole runs: a workgroup past the end leaves at once
  if (groups > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL((rfast_wave_kernel<kDeg, MOM, W>), dim3((unsigned)groups), dim3(64 * W), (size_t)W * wave_lds_bytes(d, lw),
                     c->stream, c->d, blk, lw, wave_div(lw, W));
  return hipGetLastError();
}

// A launch that does nothing (one workgroup that finds no coordinates and leaves): the first launch of a kernel
// pays for loading its code, about 0.7 ms, which belongs to setting a context up and not to its first run.
template <int kDeg, bool MOM, int W>
static hipError_t prime_wave(rfast_ctx* c) {
  const hipError_t e = hipFuncSetAttribute((const void*)rfast_wave_kernel<kDeg, MOM, W>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  if (e != hipSuccess) return e;
  RfastDev none = c->d;
  none.p = 0;
  RfastBlock blk;
  blk.gamma = 0.f;
  blk.rounds = 0;
  blk.rebase = 0;
  hipLaunchKernelGGL((rfast_wave_kernel<kDeg, MOM, W>), dim3(1), dim3(64 * W), 0, c->stream, none, blk, 64 / c->d.n, wave_div(64 / c->d.n, W));
  return hipGetLastError();
}

template <int kDeg, bool MOM>
static hipError_t prime_wave_w(rfast_ctx* c) {
  const size_t one = wave_lds_bytes(c->d, 64 / c->d.n), cu = 160 * 1024;
  hipError_t e = prime_wave<kDeg, MOM, 1>(c);
  if (e == hipSuccess && 2 * one <= cu) e = prime_wave<kDeg, MOM, 2>(c);
  if (e == hipSuccess && 4 * one <= cu) e = prime_wave<kDeg, MOM, 4>(c);
  return e;
}

// Loads the instantiations of the multi-round kernel that this context can launch (rfast_create,
// rfast_set_optimizer).
hipError_t rfast_wave_prime(rfast_ctx* c) {
  if (!rfast_wave_eligible(c)) return hipSuccess;
  const int deg = c->max_degree;
  if (c->d.mom || c->d.wd != 0.f)
    return deg <= 2 ? prime_wave_w<2, true>(c) : (deg <= 4 ? prime_wave_w<4, true>(c) : prime_wave_w<kWaveMaxDeg, true>(c));
  return deg <= 2 ? prime_wave_w<2, false>(c) : (deg <= 4 ? prime_wave_w<4, false>(c) : prime_wave_w<kWaveMaxDeg, false>(c));
}

template <int kDeg, bool MOM>
static hipError_t launch_wave_w(rfast_ctx* c, const RfastBlock& blk) {
  switch (wave_group(c, blk.rounds)) {
    case 4: return launch_wave<kDeg, MOM, 4>(c, blk);
    case 2: return launch_wave<kDeg, MOM, 2>(c, blk);
    default: return launch_wave<kDeg, MOM, 1>(c, blk);
  }
}

hipError_t rfast_launch_wave(rfast_ctx* c, const RfastBlock& blk) {
  const int deg = c->max_degree;
  if (c->d.mom || c->d.wd != 0.f)
    return deg <= 2 ? launch_wave_w<2, true>(c, blk) : (deg <= 4 ? launch_wave_w<4, true>(c, blk) : launch_wave_w<kWaveMaxDeg, true>(c, blk));
  return deg <= 2 ? launch_wave_w<2, false>(c, blk) : (deg <= 4 ? launch_wave_w<4, false>(c, blk) : launch_wave_w<kWaveMaxDeg, false>(c, blk));
}

// The synchronous mode through the multi-step kernel: the separable objective, p a multiple of 4,
// at most 32 nodes with at most kWaveMaxDeg in-edges of a kind each.
bool rfast_sync_wave_eligible(const rfast_ctx* c) {
  const RfastDev& d = c->d;
  return d.prob.kind == RFAST_OBJ_DIAG_QUADRATIC && (d.p % 4) == 0 && c->max_degree <= kWaveMaxDeg && d.n <= kWaveMaxNodes;
}

template <int kDeg, bool MOM>
static hipError_t launch_sync_wave(rfast_ctx* c, float gamma, int rounds) {
  const RfastDev& d = c->d;
  const int lw = 64 / d.n;
  const int64_t run = (int64_t)kXcds * kSyncTileRun;
  const int64_t tiles = ((d.p + 4 * lw - 1) / (4 * lw) + run - 1) / run * run;
  if (tiles > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL((rfast_sync_wave_kernel<kDeg, MOM>), dim3((unsigned)tiles), dim3(64),
                     (size_t)2 * d.n * lw * sizeof(float4), c->stream, c->d, gamma, rounds, lw);
  return hipGetLastError();
}

hipError_t rfast_launch_sync_wave(rfast_ctx* c, float gamma, int rounds) {
  const int deg = c->max_degree;
  if (c->d.mom)
    return deg <= 2 ? launch_sync_wave<2, true>(c, gamma, rounds)
                    : (deg <= 4 ? launch_sync_wave<4, true>(c, gamma, rounds) : launch_sync_wave<kWaveMaxDeg, true>(c, gamma, rounds));
  return deg <= 2 ? launch_sync_wave<2, false>(c, gamma, rounds)
                  : (deg <= 4 ? launch_sync_wave<4, false>(c, gamma, rounds) : launch_sync_wave<kWaveMaxDeg, false>(c, gamma, rounds));
}
