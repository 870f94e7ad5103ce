// Several activation rounds per launch for problems small enough to live in the LDS of ONE compute
// unit: the least-squares and logistic objectives (whose gradient couples the coordinates of a node,
// so that the coordinate tiles of rfast_wave.hip do not apply) when x, z, the stored samples, both
// rings and the S4 buffers of every node fit into LDS together.  Such a round is otherwise a chain of
// four kernels of 3-7 us each (mix, rows, columns, track) that move a few kilobytes; here one
// workgroup keeps the whole state on chip over up to kBlockRounds rounds, with two barriers per round:
//   S1, S2a, S3 (v)         one lane per coordinate of an active node: v = x - gamma z, x' = w_ii v + sum w_ij v_j
//   ---- barrier
//   gradient, rows          four lanes per sampled row: r_s = phi(a_s . x') - y_s
//   ---- barrier
//   gradient, columns; S2b, S2c, S3 (rho), S4
//                           four lanes per four coordinates, one for every fourth row: g' = (1/B) sum_s r_s a_s
//                           (+ lambda x'); then one lane per coordinate: the tracker update with it
// The lane that mixes a coordinate is the lane that tracks it, so the tracker half of one round and the
// mixing half of the next need no barrier between them.
//
// A single compute unit issues one instruction per SIMD every four cycles whatever the number of lanes
// in it: the round is bound by instruction issue and LDS latency, not by arithmetic, and the layout
// follows from that (few, full wavefront instructions; the sums across lanes with DPP moves inside
// quads, which are ALU instructions, instead of LDS permutes; shifts and a multiply-high for the
// divisions; nothing read from global memory inside a round except the plan record and the row
// numbers of the round after next, which travel in registers for a whole round before they are parked).
//
// The arithmetic is, operation for operation and in the same order, that of rfast_state_kernel<MIX>,
// rfast_rows_kernel, rfast_cols_kernel<4> and rfast_state_kernel<TRACK>: the two paths give the same
// bits.  The rows kernel has lane c of a wavefront sum the products of coordinates 4c .. 4c+3 (+ 256 m)
// and adds the 64 lanes' sums as a butterfly from distance 32 down to 1; here lane j of a quad holds
// the sixteen sums c = j, j+4, ..., adds them in that butterfly's order (distances 32 .. 4 stay inside
// the lane) and ends with the two quad steps.  The columns kernel sums the rows in four interleaved
// groups and adds the groups in order; the four lanes of a quad are those groups.
// The integer plans of the rounds are the records the resolver writes for the multi-round kernels, or, on
// small graphs, records of the same form that two more wavefronts of this workgroup write (RES below).
#include "rfast_edge.h"
#include "rfast_vec.h"

namespace {

constexpr int kTinyThreads = 1024;
constexpr int kTinyResWaves = 2;      // resolver wavefronts: one for the edges of R, one for those of C
constexpr int kTinyResThreads = 576 + 64 * kTinyResWaves;  // nine wavefronts of workers and the resolvers (170 registers each)
constexpr size_t kTinyLds = 150 * 1024;
constexpr int kTinyMaxItems = 4;  // sampled rows per lane in flight from global memory: n B <= kTinyMaxItems * kTinyThreads

// value of lane (lane ^ 1) and (lane ^ 2): quad permutes [1,0,3,2] and [2,3,0,1]
__device__ inline float quad_xor1(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, false));
}
__device__ inline float quad_xor2(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, false));
}
// value of lane J of the quad in all four
template <int J> __device__ inline float quad_lane(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), J * 0x55, 0xF, 0xF, false));
}

// x / d for small non-negative x, with sh = log2 d when d is a power of two, else -1
__device__ inline int div_small(int x, int d, int sh) { return sh >= 0 ? x >> sh : x / d; }

struct TinyShape {
  int ps;            // floats from one stored row to the next in LDS: p plus padding that spreads rows over the banks
  size_t state_f;    // x, z, g: 3 n p; rings: 2 n M p; S4 buffers: eC p
  size_t data_f;     // floats of the objective data when they are kept in LDS, else 0
  size_t ints;       // graph, active list, residuals, row numbers and plan words
  size_t bytes;
};

__host__ __device__ inline TinyShape tiny_shape(const RfastDev& d, bool data_in_lds, bool resolver = false) {
  TinyShape t;
  const size_t n = d.n, M = d.M, p = (size_t)d.p;
  const size_t B = d.prob.batch > 0 ? d.prob.batch : d.prob.samples;
  // consecutive rows 16 banks apart: eight lanes reading four floats each of two rows then cover all 32 banks
  t.ps = data_in_lds ? (int)(p + (48 - p % 32) % 32) : (int)p;
  t.state_f = (3 + 2 * M) * n * p + (size_t)d.eC * p;
  t.data_f = data_in_lds ? n * (size_t)d.prob.samples * ((size_t)t.ps + 1) : 0;
  // graph: three pointer arrays, two self weights, R: src, w; C: src, w, out eid, out w; the active list and its
  // length; residuals of a round; row numbers of two rounds (sampled batches only); two plan records
  t.ints = 3 * (n + 1) + 2 * n + 2 * (size_t)d.eR + 4 * (size_t)d.eC + n + 1 + n * B + (d.prob.batch > 0 ? 2 * n * B : 0) +
           2 * (n + d.eR + d.eC + 1) + (resolver ? kTinyResWaves * n * (2 + (size_t)d.H) : 0);  // resolvers: counters, activity flags, history, one set each
  t.bytes = t.state_f * 4 + ((t.data_f + 3) / 4 * 4) * 4 + t.ints * 4;
  return t;
}

// The caller's schedule of the rounds of a launch (the arguments of rfast_run), for the kernel that resolves them itself
struct TinySched {
  const uint8_t* active;     // [rounds][n]
  const int32_t* delay_R;    // [rounds][eR]
  const int32_t* delay_C;    // [rounds][eC]
  const uint8_t* drop_R;     // [rounds][eR]
  const uint8_t* drop_C;     // [rounds][eC]
};

__device__ inline void tiny_wave_sync() {  // orders the LDS accesses of the lanes of one wavefront
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// DATA: the objective data (rows and targets) are copied into LDS at the start.
// RES: graphs of up to 64 nodes and 64 edges of a kind: the last two wavefronts of the workgroup are resolvers, one
// for the edges of R, one for those of C.  Lane L of either looks after node L and edge L of its graph, keeps the
// counters and their history in LDS (each wavefront its own copy, so that the two never wait for each other) and its
// edge's stamp and delivery bits in registers, reads the caller's schedule a round ahead, and forms its part of the
// plan record of round q+2 while the other wavefronts finish round q (the decisions are those of the resolver
// kernels: edge_compute).  Nothing integer goes to global memory before the end of the launch, and no resolver kernel
// runs ahead of this one: on one compute unit next to another that idles, the resolver's 1.6 us per round is more
// than half of this kernel's.
template <bool DATA, bool RES>
__global__ void __launch_bounds__(RES ? kTinyResThreads : kTinyThreads)
    rfast_tiny_kernel(RfastDev s, RfastBlock blk, const int32_t* batch_idx, int round0, TinySched sched) {
  constexpr int T = RES ? kTinyResThreads : kTinyThreads;  // lanes of the workgroup
  constexpr int WORK = RES ? T - 64 * kTinyResWaves : T;    // ... that do the floating-point work
  extern __shared__ float4 lds4[];
  const int n = s.n, M = s.M, eR = s.eR, eC = s.eC;
  const int p = (int)s.p, P4 = p >> 2;
  const int np = n * p;
  const int S = s.prob.samples;
  const bool sampled = s.prob.batch > 0;
  const int B = sampled ? s.prob.batch : S;
  const int nB = n * B;
  const int W1 = n + eR + eC + 1;
  const int tid = threadIdx.x, lane = tid & 63, j = tid & 3;
  const bool worker = tid < WORK, res_wave = RES && tid >= WORK;
  const int res_kind = res_wave ? (tid - WORK) >> 6 : 0;  // 0: the resolver of graph R (and of the node words), 1: of graph C
  const TinyShape shape = tiny_shape(s, DATA, RES);
  const int ps = shape.ps;
  float* x_l = reinterpret_cast<float*>(lds4);  // [n][p]
  float* z_l = x_l + np;                        // [n][p]
  float* g_l = z_l + np;                        // [n][p]  the stored sample of every node
  float* v_l = g_l + np;                        // [n][M][p]
  float* sg_l = v_l + (size_t)np * M;           // [n][M][p]
  float* rt_l = sg_l + (size_t)np * M;          // [eC][p]  S4 buffers that have left their sender's ring
  float* data_l = rt_l + (size_t)eC * p;        // DATA: [n][S] rows of ps floats, then [n][S] targets
  int* ip = reinterpret_cast<int*>(data_l + (shape.data_f + 3) / 4 * 4);
  int* r_ptr = ip;              ip += n + 1;
  int* c_ptr = ip;              ip += n + 1;
  int* co_ptr = ip;             ip += n + 1;
  float* r_self = reinterpret_cast<float*>(ip);  ip += n;
  float* c_self = reinterpret_cast<float*>(ip);  ip += n;
  int* r_src = ip;              ip += eR;
  float* r_w = reinterpret_cast<float*>(ip);     ip += eR;
  int* c_src = ip;              ip += eC;
  float* c_w = reinterpret_cast<float*>(ip);     ip += eC;
  int* co_eid = ip;             ip += eC;
  float* co_w = reinterpret_cast<float*>(ip);    ip += eC;
  int* act_l = ip;              ip += n;          // the round's active nodes, in order
  int* nact_l = ip;             ip += 1;
  float* resid_l = reinterpret_cast<float*>(ip); ip += nB;   // [n][B] residuals of the round
  int* row_l = ip;              ip += sampled ? 2 * nB : 0;  // [2][n][B] sampled rows of this round and the next
  int* plan_l = ip;             ip += 2 * W1;                // [2][W1]
  // resolvers, a set each: the counters, the activity flags of the round being resolved, [n][H] counters at the
  // start of the last H rounds
  int* t_l = ip + res_kind * n * (2 + s.H);
  int* act2_l = t_l + n;
  int* hist_l = act2_l + n;
  const int* t_first = ip;  // the counters of the first resolver

  // ---- everything on chip: graph, state, first plan record, objective data
  for (int q = tid; q <= n; q += T) {
    r_ptr[q] = s.r_ptr[q];
    c_ptr[q] = s.c_ptr[q];
    co_ptr[q] = s.co_ptr[q];
  }
  for (int q = tid; q < n; q += T) {
    r_self[q] = s.r_self[q];
    c_self[q] = s.c_self[q];
  }
  for (int q = tid; q < eR; q += T) {
    r_src[q] = s.r_src[q];
    r_w[q] = s.r_w[q];
  }
  for (int q = tid; q < eC; q += T) {
    c_src[q] = s.c_src[q];
    c_w[q] = s.c_w[q];
    co_eid[q] = s.co_eid[q];
    co_w[q] = s.co_w[q];
  }
  if (!RES && tid < W1) plan_l[tid] = s.blk_plan[tid];
  for (int q = tid; q < np / 4; q += T) {
    const int i = q / P4, k4 = q - i * P4;
    const int t0 = RES ? s.t[i] : s.blk_plan[i] & 0x3FFFFFFF;  // the node's counter before the first round
    reinterpret_cast<float4*>(x_l)[q] = reinterpret_cast<const float4*>(s.x)[q];
    reinterpret_cast<float4*>(z_l)[q] = reinterpret_cast<const float4*>(s.z)[q];
    reinterpret_cast<float4*>(g_l)[q] = reinterpret_cast<const float4*>(s.g + (size_t)(t0 & 1) * np)[(size_t)i * P4 + k4];
  }
  for (int q = tid; q < np * M / 4; q += T) {
    reinterpret_cast<float4*>(v_l)[q] = reinterpret_cast<const float4*>(s.v_ring)[q];
    reinterpret_cast<float4*>(sg_l)[q] = reinterpret_cast<const float4*>(s.sigma_ring)[q];
  }
  for (int q = tid; q < eC * P4; q += T) reinterpret_cast<float4*>(rt_l)[q] = reinterpret_cast<const float4*>(s.rho_tilde)[q];
  if (DATA) {
    const int rows = n * S;
    for (int q = tid; q < rows * P4; q += T) {
      const int r = q / P4, k4 = q - r * P4;
      *reinterpret_cast<float4*>(data_l + (size_t)r * ps + 4 * k4) = reinterpret_cast<const float4*>(s.prob.data0)[q];
    }
    for (int q = tid; q < rows; q += T) data_l[(size_t)rows * ps + q] = ((const float*)s.prob.data1)[q];
  }
  if (sampled)
    for (int q = tid; q < nB; q += T) row_l[q] = batch_idx[q];

  const unsigned m_magic = 0xFFFFFFFFu / (unsigned)M;
  const int b_sh = (B & (B - 1)) == 0 ? __ffs(B) - 1 : -1;
  const int p_sh = (p & (p - 1)) == 0 ? __ffs(p) - 1 : -1;
  // ---- the resolver wavefront: its state, the record of round 0 into LDS, that of round 1 into registers
  const FastMod modM(M), modH(s.H);
  const int H = s.H, r0 = RES ? *s.round_no : 0;
  const int edges = res_kind ? eC : eR;    // of this resolver's graph
  EdgeIn ed;                               // the lane's edge
  int last_slot = -1;                      // its slot in the last round resolved (what reads of the slot fields return)
  int sc_act = 0, sc_d = 0, sc_x = 0;      // the schedule of the next round to resolve, fetched a round ahead
  int pend_node = 0, pend_edge = 0;        // its record, formed a round before it is parked in LDS
  // schedule of round rel (counted from the first round of the launch) into the registers above
  auto fetch_schedule = [&](int rel) {
    if (rel >= blk.rounds) return;
    if (lane < n) sc_act = sched.active[(size_t)rel * n + lane];
    if (lane < edges) {
      sc_d = (res_kind ? sched.delay_C : sched.delay_R)[(size_t)rel * edges + lane];
      sc_x = (res_kind ? sched.drop_C : sched.drop_R)[(size_t)rel * edges + lane];
    }
  };
  // resolves round rel from the schedule in the registers: the record into pend_*, the state one round on
  auto resolve = [&](int rel) {
    const int r = r0 + rel;
    if (lane < n) act2_l[lane] = sc_act != 0;
    tiny_wave_sync();
    if (lane < edges) {
      ed.d = sc_d;
      ed.dropped = sc_x != 0;
      ed.act_i = act2_l[ed.i] != 0;
      ed.act_j = act2_l[ed.j] != 0;
      ed.tj = t_l[ed.j];
      const int d = sc_d < 0 ? 0 : (sc_d > s.d_max ? s.d_max : sc_d);
      const int at = r - d;
      // the sender's counter at the start of round `at`; round r itself is the current counter
      ed.u = at <= 0 ? 0 : (at >= r ? ed.tj : hist_l[ed.j * H + modH(at)]);
    }
    tiny_wave_sync();  // every lane has read the history of this round's delays
    int ti = 0;
    bool on = false;
    if (lane < n) {
      ti = t_l[lane];
      on = sc_act != 0;
      hist_l[lane * H + modH(r)] = ti;
    }
    pend_node = (ti & 0x3FFFFFFF) | (on ? (int)0x80000000 : 0);
    if (lane < edges) {
      const EdgeOut o = res_kind ? edge_compute<1>(s, modM, lane, r, ed) : edge_compute<0>(s, modM, lane, r, ed);
      pend_edge = o.word;
      last_slot = o.slot;
    }
    tiny_wave_sync();  // every read of the counters is done
    if (on) t_l[lane] = ti + 1;
    tiny_wave_sync();
  };
  // parks the record in pend_* as that of a round with the given parity
  auto park = [&](int parity) {
    int* rec = plan_l + parity * W1;
    if (res_kind == 0) {
      if (lane < n) rec[lane] = pend_node;
      if (lane < eR) rec[n + lane] = pend_edge;
      if (lane == 0) rec[W1 - 1] = 0;  // a record ends with a word that is always zero
    } else if (lane < eC) {
      rec[n + eR + lane] = pend_edge;
    }
  };
  if (res_wave) {
    if (lane < n) t_l[lane] = s.t[lane];
    for (int q = lane; q < n * H; q += 64) hist_l[q] = s.t_hist[q];
    if (lane < edges) {
      ed.i = (res_kind ? s.c_dst : s.r_dst)[lane];
      ed.j = (res_kind ? s.c_src : s.r_src)[lane];
      ed.bits = (res_kind ? s.deliv_c : s.deliv_r)[lane];
      ed.old = (res_kind ? s.tau_c : s.tau_r)[lane];
    }
    fetch_schedule(0);
    tiny_wave_sync();
    resolve(0);
    park(0);
    fetch_schedule(1);
    if (blk.rounds > 1) {
      resolve(1);
      fetch_schedule(2);
    }
  }
  // the plan record and the row numbers of the round after next travel in registers for one round
  int pend_plan = 0, pend_row[kTinyMaxItems] = {0, 0, 0, 0};
  if (blk.rounds > 1) {
    if (!RES && tid < W1) pend_plan = s.blk_plan[(size_t)W1 + tid];
    if (sampled) {
#pragma unroll
      for (int u = 0; u < kTinyMaxItems; ++u)
        if (tid + u * T < nB) pend_row[u] = batch_idx[(size_t)nB + tid + u * T];
    }
  }
  __syncthreads();
  const float* rows_base = DATA ? data_l : (const float*)s.prob.data0;                      // [n][S] rows of ps floats
  const float* targets = DATA ? data_l + (size_t)n * S * ps : (const float*)s.prob.data1;   // [n][S]
  const float inv = 1.0f / (float)B;
  // l2 term of the logistic objective plus the weight decay of the optimizer variant
  const float lam = (s.prob.kind == RFAST_OBJ_LOGISTIC ? s.prob.lambda : 0.f) + s.wd;
  const bool logistic = s.prob.kind == RFAST_OBJ_LOGISTIC;

  for (int q = 0; q < blk.rounds; ++q) {
    const int* P = plan_l + (q & 1) * W1;  // [n] node words, [eR] slots of R edges, [eC] plan words of C edges
    const int* rows_q = row_l + (q & 1) * nB;

    // ---- S1, S2a, S3 (v half): as rfast_state_kernel<MIX>; lane t, t + 1024, ... of the flattened [n][p]
#pragma unroll 1
    for (int t = worker ? tid : np; t < np; t += WORK) {
      const int i = div_small(t, p, p_sh), k = t - i * p;
      const int word = P[i];
      if (word < 0) {  // bit 31: active
        const unsigned t_old = (unsigned)(word & 0x3FFFFFFF);
        unsigned sl = t_old - __umulhi(t_old, m_magic) * (unsigned)M;  // t_old mod M: the quotient is at most one short
        if (sl >= (unsigned)M) sl -= M;
        const int slot_new = (int)sl + 1 == M ? 0 : (int)sl + 1;
        const float v = fmaf(-blk.gamma, z_l[t], x_l[t]);
        float x_new = r_self[i] * v;
        for (int e = r_ptr[i]; e < r_ptr[i + 1]; ++e) x_new = fmaf(r_w[e], v_l[(r_src[e] * M + P[n + e]) * p + k], x_new);
        v_l[(i * M + slot_new) * p + k] = v;  // the slot nobody reads in this round
        x_l[t] = x_new;
      }
    }
    // the round's active nodes in order, by the last wavefront
    if (tid >= T - 64) {
      int cnt = 0;
      for (int base = 0; base < n; base += 64) {
        const bool a = base + lane < n && P[base + lane] < 0;
        const unsigned long long mask = __ballot(a);
        if (a) act_l[cnt + __popcll(mask & ((1ull << lane) - 1))] = base + lane;
        cnt += __popcll(mask);
      }
      if (lane == 0) *nact_l = cnt;
    }
    __syncthreads();

    // the next round's record and rows: fetched a round ago, parked now (their buffers were last read before this
    // barrier), and the fetch for the round after that goes out
    if (q + 1 < blk.rounds) {
      if (RES) {
        if (res_wave) park((q + 1) & 1);
      } else if (tid < W1) {
        plan_l[((q + 1) & 1) * W1 + tid] = pend_plan;
      }
      if (sampled) {
#pragma unroll
        for (int u = 0; u < kTinyMaxItems; ++u)
          if (tid + u * T < nB) row_l[((q + 1) & 1) * nB + tid + u * T] = pend_row[u];
      }
      if (q + 2 < blk.rounds) {
        if (!RES && tid < W1) pend_plan = s.blk_plan[(size_t)(q + 2) * W1 + tid];
        if (sampled) {
#pragma unroll
          for (int u = 0; u < kTinyMaxItems; ++u)
            if (tid + u * T < nB) pend_row[u] = batch_idx[(size_t)(q + 2) * nB + tid + u * T];
        }
      }
    }

    // ---- gradient, rows: as rfast_rows_kernel; a quad per (active node, sampled row)
    const int tasks = *nact_l * B;
    for (int f = worker ? tid >> 2 : tasks; f < tasks; f += WORK / 4) {
      const int a = div_small(f, B, b_sh);
      const int i = act_l[a], b = f - a * B;
      int row = b;
      if (sampled) {
        row = rows_q[i * B + b];
        if (row < 0 || row >= S) {
          if (atomicCAS(&s.err[0], 0, RFAST_ERANGE) == 0) {
            s.err[1] = round0 + q;
            s.err[2] = 2;
            s.err[3] = i;
          }
          row = row < 0 ? 0 : S - 1;
        }
      }
      const float* ar = rows_base + ((size_t)i * S + row) * ps;
      const float* xr = x_l + i * p;
      float acc[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) acc[u] = 0.f;
      for (int k0 = 0; k0 < P4; k0 += 64) {  // float4 number k0 + c belongs to lane c of the wavefront form
#pragma unroll
        for (int ug = 0; ug < 4; ++ug) {
          if (k0 + 16 * ug < P4) {
            float4 av[4], xv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              const int k4 = k0 + 16 * ug + 4 * u + j;
              const int kc = k4 < P4 ? k4 : 0;
              av[u] = *reinterpret_cast<const float4*>(ar + 4 * kc);
              xv[u] = *reinterpret_cast<const float4*>(xr + 4 * kc);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
              if (k0 + 16 * ug + 4 * u + j < P4) {
                float c = acc[4 * ug + u];
                c = fmaf(av[u].x, xv[u].x, c);
                c = fmaf(av[u].y, xv[u].y, c);
                c = fmaf(av[u].z, xv[u].z, c);
                c = fmaf(av[u].w, xv[u].w, c);
                acc[4 * ug + u] = c;
              }
          }
        }
      }
      // lane c = j + 4u of the wavefront form: distance 32 pairs u with u ^ 8, 16 with u ^ 4, 8 with u ^ 2, 4 with u ^ 1
#pragma unroll
      for (int h = 8; h > 0; h >>= 1) {
#pragma unroll
        for (int u = 0; u < h; ++u) acc[u] += acc[u + h];
      }
      float sum = acc[0];
      sum += quad_xor2(sum);
      sum += quad_xor1(sum);
      if (j == 0) {
        const float y = targets[(size_t)i * S + row];
        resid_l[i * B + b] = logistic ? 1.0f / (1.0f + expf(-sum)) - y : sum - y;
      }
    }
    __syncthreads();

    // ---- gradient, columns (as rfast_cols_kernel<4>): lane j of a quad sums rows j, j + 4, ... for the quad's four
    // coordinates; every lane then adds the four sums of its own coordinate in order;
    // then S2b, S2c, S3 (rho half), S4 (as rfast_state_kernel<TRACK>)
    // the resolver goes on to the round after next while the others finish this one
    if (res_wave && q + 2 < blk.rounds) {
      resolve(q + 2);
      fetch_schedule(q + 3);
    }
#pragma unroll 1
    for (int t = worker ? tid : np; t < np; t += WORK) {
      const int i = div_small(t, p, p_sh), k = t - i * p;
      const int word = P[i];
      if (word < 0) {
        const float* base = rows_base + (size_t)i * S * ps + (k & ~3);
        const float* r_sh = resid_l + i * B;
        const int* row_sh = rows_q + i * B;
        float4 part = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int b0 = j; b0 < B; b0 += 16) {
          float4 av[4];
          float r[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int b = b0 + 4 * u < B ? b0 + 4 * u : j;
            r[u] = r_sh[b];
            int row = b;
            if (sampled) {
              row = row_sh[b];
              row = row < 0 ? 0 : row >= S ? S - 1 : row;  // reported by the rows pass
            }
            av[u] = *reinterpret_cast<const float4*>(base + (size_t)row * ps);
          }
#pragma unroll
          for (int u = 0; u < 4; ++u)
            if (b0 + 4 * u < B) {
              part.x = fmaf(r[u], av[u].x, part.x);
              part.y = fmaf(r[u], av[u].y, part.y);
              part.z = fmaf(r[u], av[u].z, part.z);
              part.w = fmaf(r[u], av[u].w, part.w);
            }
        }
        // the sum of group J sits in lane J; this lane's coordinate is component j of it
        float mine[4];
#define RFAST_TINY_PICK(J)                                                                                                   \
  {                                                                                                                          \
    const float a0 = quad_lane<J>(part.x), a1 = quad_lane<J>(part.y), a2 = quad_lane<J>(part.z), a3 = quad_lane<J>(part.w);  \
    mine[J] = j == 0 ? a0 : j == 1 ? a1 : j == 2 ? a2 : a3;                                                                  \
  }
        RFAST_TINY_PICK(0) RFAST_TINY_PICK(1) RFAST_TINY_PICK(2) RFAST_TINY_PICK(3)
#undef RFAST_TINY_PICK
        const float acc = ((mine[0] + mine[1]) + mine[2]) + mine[3];
        const float g_new = fmaf(lam, x_l[t], acc * inv);
        const float g_old = g_l[t];
        const unsigned t_old = (unsigned)(word & 0x3FFFFFFF);
        unsigned sl = t_old - __umulhi(t_old, m_magic) * (unsigned)M;
        if (sl >= (unsigned)M) sl -= M;
        const int sl_old = (int)sl;
        const int sl_new = sl_old + 1 == M ? 0 : sl_old + 1;
        // S2b: tracker sum over the in-edges of C; an edge whose stamp did not move contributes exactly zero
        float z_half = z_l[t];
        for (int e = c_ptr[i]; e < c_ptr[i + 1]; ++e) {
          const int pl = P[n + eR + e];
          if (!(pl & (1 << 16))) continue;
          const float* ring = sg_l + c_src[e] * M * p + k;
          const int prev = (pl >> 8) & 0xFF;
          const float cur = ring[(pl & 0xFF) * p];
          float* rt = rt_l + e * p + k;
          const float last = prev != 0xFF ? ring[prev * p] : *rt;
          z_half = track_edge(z_half, c_w[e], cur, last, prev != 0xFF);
          if (pl & (1 << 17)) *rt = c_w[e] * cur;  // S4: consumed, and leaving the ring
        }
        z_half = (z_half + g_new) - g_old;
        z_l[t] = c_self[i] * z_half;
        g_l[t] = g_new;
        if (co_ptr[i + 1] > co_ptr[i]) {
          float* own = sg_l + i * M * p + k;
          own[sl_new * p] = own[sl_old * p] + z_half;
          // S4 for receivers that do not do it themselves: the version that leaves this node's ring with this
          // activation, M - 2 versions back, which sits two slots ahead
          for (int o = co_ptr[i]; o < co_ptr[i + 1]; ++o)
            if (P[n + eR + co_eid[o]] & (1 << 18)) {
              const int sl_leave = sl_old + 2 >= M ? sl_old + 2 - M : sl_old + 2;
              rt_l[co_eid[o] * p + k] = co_w[o] * own[sl_leave * p];
            }
        }
      }
    }
    // S5: the round is over.  No barrier here: the next round's mixing reads and writes what this lane wrote itself,
    // and slots of v that were written before the last barrier but one.
  }
  __syncthreads();

  // ---- write-back; the counters after the launch are the resolver's: those of the resolver kernel that ran ahead
  // of this one (s.t), or those of the resolver wavefront, which stores its integer state now
  if (res_wave) {
    if (res_kind == 0) {
      if (lane < n) s.t[lane] = t_l[lane];
      for (int q = lane; q < n * H; q += 64) s.t_hist[q] = hist_l[q];
      if (lane == 0) *s.round_no = r0 + blk.rounds;
    }
    if (lane < edges) {
      (res_kind ? s.tau_c : s.tau_r)[lane] = ed.old;
      (res_kind ? s.deliv_c : s.deliv_r)[lane] = ed.bits;
      (res_kind ? s.slot_c : s.slot_r)[lane] = last_slot;
    }
  }
  for (int q = tid; q < np / 4; q += T) {
    const int i = q / P4, k4 = q - i * P4;
    reinterpret_cast<float4*>(s.x)[q] = reinterpret_cast<const float4*>(x_l)[q];
    reinterpret_cast<float4*>(s.z)[q] = reinterpret_cast<const float4*>(z_l)[q];
    const int t_end = RES ? t_first[i] : s.t[i];
    reinterpret_cast<float4*>(s.g + (size_t)(t_end & 1) * np)[(size_t)i * P4 + k4] = reinterpret_cast<const float4*>(g_l)[q];
  }
  for (int q = tid; q < np * M / 4; q += T) {
    reinterpret_cast<float4*>(s.v_ring)[q] = reinterpret_cast<const float4*>(v_l)[q];
    reinterpret_cast<float4*>(s.sigma_ring)[q] = reinterpret_cast<const float4*>(sg_l)[q];
  }
  for (int q = tid; q < eC * P4; q += T) reinterpret_cast<float4*>(s.rho_tilde)[q] = reinterpret_cast<const float4*>(rt_l)[q];
}

bool tiny_data_fits(const RfastDev& d) { return tiny_shape(d, true).bytes <= kTinyLds; }

// whether the graph is small enough for the resolver wavefront: a lane per node, per edge of R and per edge of C
bool tiny_resolves(const RfastDev& d) {
  const int64_t B = d.prob.batch > 0 ? d.prob.batch : d.prob.samples;
  return d.n <= 64 && d.eR <= 64 && d.eC <= 64 && (int64_t)d.n * d.p <= 4 * (kTinyResThreads - 64) &&
         (int64_t)d.n * B <= (int64_t)kTinyMaxItems * kTinyResThreads && tiny_shape(d, false, true).bytes <= kTinyLds;
}

template <bool DATA, bool RES>
hipError_t launch_tiny(rfast_ctx* c, const RfastBlock& blk, const int32_t* bi, int round0, const TinySched& sched) {
  static bool raised = false;
  if (!raised) {  // more than 64 KB of dynamic LDS has to be asked for once per kernel
    const hipError_t e =
        hipFuncSetAttribute((const void*)rfast_tiny_kernel<DATA, RES>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    raised = true;
  }
  hipLaunchKernelGGL((rfast_tiny_kernel<DATA, RES>), dim3(1), dim3(RES ? kTinyResThreads : kTinyThreads),
                     tiny_shape(c->d, DATA, RES).bytes, c->stream, c->d, blk, bi, round0, sched);
  return hipGetLastError();
}

}  // namespace

// Least squares or logistic regression without the heavy-ball buffer, p a multiple of 4, at most kTinyMaxItems
// sampled rows per lane, a plan record of at most one word per lane, and the whole state of the
// problem (x, z, samples, both rings and the S4 buffers of every node) within the LDS of one compute unit.
bool rfast_tiny_eligible(const rfast_ctx* c) {
  const RfastDev& d = c->d;
  if (d.prob.kind != RFAST_OBJ_LEAST_SQUARES && d.prob.kind != RFAST_OBJ_LOGISTIC) return false;
  if ((d.p % 4) != 0 || d.mom != nullptr || d.M > 255) return false;
  const int64_t B = d.prob.batch > 0 ? d.prob.batch : d.prob.samples;
  if ((int64_t)d.n * B > kTinyMaxItems * kTinyThreads) return false;
  if ((int64_t)d.n + d.eR + d.eC + 1 > kTinyThreads) return false;
  return tiny_shape(d, false).bytes <= kTinyLds;
}

// ... and a graph small enough for the kernel to resolve its rounds itself: no resolver launch ahead of it, and the
// caller's schedule goes to rfast_launch_tiny instead
bool rfast_tiny_resolves(const rfast_ctx* c) { return rfast_tiny_eligible(c) && tiny_resolves(c->d); }

// The schedule pointers are those of rfast_run for the first round of the launch; they are read only if
// rfast_tiny_resolves(c), otherwise the plan records of the resolver kernel (c->d.blk_plan) are.
hipError_t rfast_launch_tiny(rfast_ctx* c, const RfastBlock& blk, const int32_t* d_batch_idx, int round0, const uint8_t* d_active,
                             const int32_t* d_delay_R, const int32_t* d_delay_C, const uint8_t* d_drop_R, const uint8_t* d_drop_C) {
  const RfastDev& d = c->d;
  if (!rfast_tiny_eligible(c)) return hipErrorInvalidValue;
  const bool res = tiny_resolves(d);
  if (!res && !d.blk_plan) return hipErrorInvalidValue;
  const int32_t* bi = d.prob.batch > 0 ? d_batch_idx : nullptr;
  if (d.prob.batch > 0 && !bi) return hipErrorInvalidValue;
  const TinySched sched = {d_active, d_delay_R, d_delay_C, d_drop_R, d_drop_C};
  if (res) {
    if (!d_active || (d.eR && (!d_delay_R || !d_drop_R)) || (d.eC && (!d_delay_C || !d_drop_C))) return hipErrorInvalidValue;
    return tiny_shape(d, true, true).bytes <= kTinyLds ? launch_tiny<true, true>(c, blk, bi, round0, sched)
                                                       : launch_tiny<false, true>(c, blk, bi, round0, sched);
  }
  return tiny_data_fits(d) ? launch_tiny<true, false>(c, blk, bi, round0, sched) : launch_tiny<false, false>(c, blk, bi, round0, sched);
}
