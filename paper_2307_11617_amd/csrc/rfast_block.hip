// Several activation rounds per launch with the state of a tile of coordinates resident in LDS.
//
// Everything in a round of Algorithm 1 is elementwise in the coordinate k: coordinate k of every
// node, ring slot and buffer depends, over any number of rounds, only on coordinate k of the
// others.  For the separable objective (whose gradient is elementwise too) a workgroup can
// therefore take 64 coordinates of EVERY node, load the rings of v and of the running sums for
// them into LDS once, advance them through up to kBlockRounds rounds -- all neighbour reads of
// S2a / S2b and all publications of S3 are LDS traffic -- and write them back once.  HBM traffic
// per round drops from 13 words per coordinate and node-update to (2 M + 4 + 2 M + 2) / rounds
// words per coordinate and node (read everything, write everything, once per launch); the 160 KB
// of LDS per CU are what makes the tile fit (config 2: 16 nodes x 2 rings x 9 slots x 256 B = 72 KB).
// One launch also replaces up to kBlockRounds launches, which is where the path pays: see
// rfast_block_eligible below for what was measured.
//
// Layout of the work: 16 lanes per node, 4 consecutive coordinates per lane (one Philox call per
// lane and sample, as in the streaming kernel), so a workgroup has 16 n lanes; x, z, the stored
// sample and the objective data of a node stay in the registers of its 16 lanes for the whole
// launch.  The arithmetic is, operation for operation, that of rfast_state_kernel<FUSED>: the two
// paths give the same bits.
//
// The integer plans of the rounds (who is active, which slot each edge reads, where each S4
// buffer lives) are made by the resolver, one record per round, and copied to LDS first.
#include "rfast_vec.h"

namespace {

constexpr int kLanes = 16;  // lanes per node; each owns 4 coordinates of the 64-coordinate tile

// VEC: 4 or -4 (non-temporal global accesses); TPB: upper bound of the workgroup size (16 lanes per
// node; with 256 the compiler may use twice the registers of 1024)
template <int VEC, int TPB>
__global__ void __launch_bounds__(TPB) rfast_block_kernel(RfastDev s, RfastBlock blk) {
  extern __shared__ float4 lds4[];
  const int n = s.n, M = s.M;
  const int64_t p = s.p;
  const int PL = n + s.eR + s.eC;
  float4* v_l = lds4;                                  // [n][M][16]
  float4* sg_l = v_l + (size_t)n * M * kLanes;         // [n][M][16]
  float4* rt_l = sg_l + (size_t)n * M * kLanes;        // [eC][16]
  int* plan_l = reinterpret_cast<int*>(rt_l + (size_t)s.eC * kLanes);  // [kBlockRounds][PL]
  // the graph, so that no round has to wait for global memory: sender and weight per in-edge of R and
  // of C, edge id and weight per out-edge of C
  int* r_src_l = plan_l + kBlockRounds * PL;                   // [eR]
  float* r_w_l = reinterpret_cast<float*>(r_src_l + s.eR);     // [eR]
  int* c_src_l = reinterpret_cast<int*>(r_w_l + s.eR);         // [eC]
  float* c_w_l = reinterpret_cast<float*>(c_src_l + s.eC);     // [eC]
  int* co_eid_l = reinterpret_cast<int*>(c_w_l + s.eC);        // [eC]
  float* co_w_l = reinterpret_cast<float*>(co_eid_l + s.eC);   // [eC]
  const int i = threadIdx.x / kLanes, ln = threadIdx.x % kLanes;
  const int64_t k = (int64_t)blockIdx.x * (4 * kLanes) + ln * 4;
  const bool mine = i < n && k < p;

  for (int q = threadIdx.x; q < blk.rounds * PL; q += blockDim.x) plan_l[q] = s.blk_plan[q];
  for (int e = threadIdx.x; e < s.eR; e += blockDim.x) {
    r_src_l[e] = s.r_src[e];
    r_w_l[e] = s.r_w[e];
  }
  for (int e = threadIdx.x; e < s.eC; e += blockDim.x) {
    c_src_l[e] = s.c_src[e];
    c_w_l[e] = s.c_w[e];
    co_eid_l[e] = s.co_eid[e];
    co_w_l[e] = s.co_w[e];
  }

  float4 x, z, g, h, c;
  int re0 = 0, re1 = 0, ce0 = 0, ce1 = 0, o0 = 0, o1 = 0;
  float r_self = 0.f, c_self = 0.f;
  const int own = i * M * kLanes + ln;  // this lane's column in the rings of its node (LDS offsets fit in 32 bits)
  if (mine) {
    const size_t off = (size_t)i * p + k;
    x = V<VEC>::ld(s.x + off);
    z = V<VEC>::ld(s.z + off);
    h = V<VEC>::ld((const float*)s.prob.data0 + off);
    c = V<VEC>::ld((const float*)s.prob.data1 + off);
    re0 = s.r_ptr[i]; re1 = s.r_ptr[i + 1];
    ce0 = s.c_ptr[i]; ce1 = s.c_ptr[i + 1];
    o0 = s.co_ptr[i]; o1 = s.co_ptr[i + 1];
    r_self = s.r_self[i];
    c_self = s.c_self[i];
    // rings: eight slots of both rings (sixteen loads) in flight at a time, then into LDS
    const float* vg = s.v_ring + (size_t)i * M * p + k;
    const float* sgg = s.sigma_ring + (size_t)i * M * p + k;
    for (int m0 = 0; m0 < M; m0 += 8) {
      float4 tv[8], ts[8];
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (m0 + u < M) {
          tv[u] = V<VEC>::ld(vg + (size_t)(m0 + u) * p);
          ts[u] = V<VEC>::ld(sgg + (size_t)(m0 + u) * p);
        }
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (m0 + u < M) {
          v_l[own + (m0 + u) * kLanes] = tv[u];
          sg_l[own + (m0 + u) * kLanes] = ts[u];
        }
    }
    for (int e = ce0; e < ce1; ++e) rt_l[e * kLanes + ln] = V<VEC>::ld(s.rho_tilde + (size_t)e * p + k);
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
    const int* P = plan_l + q * PL;
    if (mine && P[i] < 0) {  // bit 31: node i is activated in this round
      const int t_old = P[i] & 0x3FFFFFFF;
      const int slot_new = slot_cur + 1 == M ? 0 : slot_cur + 1;
      // S1: local descent
      const float4 v = fma_s(-blk.gamma[q], z, x);
      // S2a: pull the stamped neighbour copies and mix with row-stochastic weights (LDS reads of up
      // to four edges are issued together)
      float4 x_new = mul_s(r_self, v);
      for (int e0 = re0; e0 < re1; e0 += 4) {
        float4 nb[4];
        float w[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (e0 + u < re1) {
            nb[u] = v_l[(r_src_l[e0 + u] * M + P[n + e0 + u]) * kLanes + ln];
            w[u] = r_w_l[e0 + u];
          }
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (e0 + u < re1) x_new = fma_s(w[u], nb[u], x_new);
      }
      const float4 g_new = diag_sample<VEC>(s, h, c, x_new, i, t_old + 1, k);
      // S2b: tracker sum over the in-edges of C; S4: buffer what was consumed
      float4 z_half = z;
      for (int e0 = ce0; e0 < ce1; e0 += 4) {
        float4 cur[4], last[4];
        float ca[4];
        int pl[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          pl[u] = e0 + u < ce1 ? P[n + s.eR + e0 + u] : 0;
          if (pl[u] & (1 << 16)) {
            const int ring = c_src_l[e0 + u] * M * kLanes + ln;
            const int prev = (pl[u] >> 8) & 0xFF;
            cur[u] = sg_l[ring + (pl[u] & 0xFF) * kLanes];
            last[u] = prev != 0xFF ? sg_l[ring + prev * kLanes] : rt_l[(e0 + u) * kLanes + ln];
            ca[u] = c_w_l[e0 + u];
          }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (pl[u] & (1 << 16)) {
            const float4 rho = mul_s(ca[u], cur[u]);
            z_half = add(z_half, sub(rho, ((pl[u] >> 8) & 0xFF) != 0xFF ? mul_s(ca[u], last[u]) : last[u]));
            if (pl[u] & (1 << 17)) rt_l[(e0 + u) * kLanes + ln] = rho;
          }
      }
      z_half = sub(add(z_half, g_new), g);
      // S3: publish version t+1 (slots nobody reads in this round); S2c: keep a_ii, push
      v_l[own + slot_new * kLanes] = v;
      if (o1 > o0) {
        sg_l[own + slot_new * kLanes] = add(sg_l[own + slot_cur * kLanes], z_half);
        // S4 for receivers that do not do it themselves: version t - D leaves the ring; it sits two
        // slots ahead of the current one
        for (int o = o0; o < o1; ++o) {
          const int eid = co_eid_l[o];
          if (P[n + s.eR + eid] & (1 << 18)) {
            const int leaving = slot_cur + 2 >= M ? slot_cur + 2 - M : slot_cur + 2;
            rt_l[eid * kLanes + ln] = mul_s(co_w_l[o], sg_l[own + leaving * kLanes]);
          }
        }
      }
      x = x_new;
      z = mul_s(c_self, z_half);
      g = g_new;
      slot_cur = slot_new;
    }
    __syncthreads();  // S5: the round is over, its publications are visible
  }

  if (mine) {
    const size_t off = (size_t)i * p + k;
    V<VEC>::st(s.x + off, x);
    V<VEC>::st(s.z + off, z);
    float* vg = s.v_ring + (size_t)i * M * p + k;
    float* sgg = s.sigma_ring + (size_t)i * M * p + k;
    for (int m0 = 0; m0 < M; m0 += 8) {
      float4 tv[8], ts[8];
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (m0 + u < M) {
          tv[u] = v_l[own + (m0 + u) * kLanes];
          ts[u] = sg_l[own + (m0 + u) * kLanes];
        }
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (m0 + u < M) {
          V<VEC>::st(vg + (size_t)(m0 + u) * p, tv[u]);
          V<VEC>::st(sgg + (size_t)(m0 + u) * p, ts[u]);
        }
    }
    for (int e = ce0; e < ce1; ++e) V<VEC>::st(s.rho_tilde + (size_t)e * p + k, rt_l[e * kLanes + ln]);
  }
}

size_t block_lds_bytes(const RfastDev& d) {
  return ((size_t)2 * d.n * d.M + d.eC) * kLanes * sizeof(float4) + (size_t)kBlockRounds * (d.n + d.eR + d.eC) * sizeof(int) +
         ((size_t)2 * d.eR + 4 * d.eC) * sizeof(int);
}

}  // namespace

// The tile of every node must fit into the LDS of one CU next to the plans, a workgroup holds 16
// lanes per node, and the path exists for the separable objective without the momentum variant.
// It is taken where rounds are bound by kernel launches, not by HBM: one workgroup of 16 n lanes per
// CU issues about 780 instructions per round and tile, which is slower than streaming once the
// state is large (measured on 16 nodes, ms per round, this path / one pass per round: p = 4096
// 0.0072 / 0.0115, 16 384 0.0074 / 0.0121, 65 536 0.0155 / 0.0188, 262 144 0.048 / 0.045,
// 1 048 576 0.186 / 0.156, 11.2 M 1.90 / 1.53), so it stops at 8 MB of x.
bool rfast_block_eligible(const rfast_ctx* c) {
  const RfastDev& d = c->d;
  return d.prob.kind == RFAST_OBJ_DIAG_QUADRATIC && d.mom == nullptr && (d.p % 4) == 0 && d.n * kLanes <= 1024 &&
         block_lds_bytes(d) <= 156 * 1024 && (double)d.n * (double)d.p * 4.0 <= 8.0e6;
}

template <int VEC, int TPB>
static hipError_t launch_block(rfast_ctx* c, const RfastBlock& blk, unsigned threads, unsigned tiles, size_t lds) {
  static bool raised = false;
  if (!raised) {  // more than 64 KB of dynamic LDS has to be asked for once per kernel
    const hipError_t e = hipFuncSetAttribute((const void*)rfast_block_kernel<VEC, TPB>,
                                             hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    raised = true;
  }
  hipLaunchKernelGGL((rfast_block_kernel<VEC, TPB>), dim3(tiles), dim3(threads), lds, c->stream, c->d, blk);
  return hipGetLastError();
}

hipError_t rfast_launch_block(rfast_ctx* c, const RfastBlock& blk) {
  const RfastDev& d = c->d;
  const size_t lds = block_lds_bytes(d);
  const bool streaming = (double)d.n * (double)d.p * 4.0 >= 32.0e6;
  const unsigned threads = (unsigned)((d.n * kLanes + 63) / 64 * 64);
  const int64_t tiles = (d.p + 4 * kLanes - 1) / (4 * kLanes);
  if (tiles > 0x7fffffffLL) return hipErrorInvalidValue;
  if (threads <= 256)
    return streaming ? launch_block<-4, 256>(c, blk, threads, (unsigned)tiles, lds)
                     : launch_block<4, 256>(c, blk, threads, (unsigned)tiles, lds);
  return streaming ? launch_block<-4, 1024>(c, blk, threads, (unsigned)tiles, lds)
                   : launch_block<4, 1024>(c, blk, threads, (unsigned)tiles, lds);
}
