// Local stochastic gradients grad f_i(x_i; zeta) for the objectives that are
// not separable per coordinate (step S2b of Algorithm 1 needs the sample at the
// freshly mixed x_i), plus the initial gradients z^0 = g^0 of every objective.
//
// Least squares / logistic regression: a GEMV pair on the sampled rows,
//   r_s = phi(a_s . x) - y_s,   g = (1/B) sum_s r_s a_s (+ lambda x),
// phi = identity (least squares, y = b) or the logistic function.  The rows
// kernel gives one wavefront per sampled row (float4 loads, 64-lane reduction);
// the columns kernel gives one float4 of g per lane of a wavefront and streams the
// same rows again, coalesced along k, its four wavefronts sharing the rows.
// In a run of consecutive rounds the column sums share a kernel with the tracker
// update of their round and the mixing of the next (rfast_cols_track_mix_kernel,
// further down): two kernels per round instead of four.
#include "rfast_internal.h"
#include "rfast_vec.h"

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// a sampled row number as read from the caller's array: clamped into the node's samples, and reported, if outside
__device__ inline int checked_row(const RfastDev& s, int i, int row) {
  if (row < 0 || row >= s.prob.samples) {
    if (atomicCAS(&s.err[0], 0, RFAST_ERANGE) == 0) {
      s.err[1] = s.n_active[1] - 1;  // the number of this round (its plan recorded the count of rounds including it)
      s.err[2] = 2;
      s.err[3] = i;
    }
    row = row < 0 ? 0 : s.prob.samples - 1;
  }
  return row;
}

__device__ inline int sample_row(const RfastDev& s, const int32_t* batch_idx, int i, int b, int B) {
  if (batch_idx == nullptr) return b;
  int row = batch_idx[(size_t)i * B + b];
  if (row < 0 || row >= s.prob.samples) {
    if (atomicCAS(&s.err[0], 0, RFAST_ERANGE) == 0) {
      s.err[1] = s.n_active[1] - 1;  // the number of this round (its plan recorded the count of rounds including it)
      s.err[2] = 2;
      s.err[3] = i;
    }
    row = row < 0 ? 0 : s.prob.samples - 1;
  }
  return row;
}

// node handled by blockIdx.y and the stamp of its stored sample (-1: the initial gradient is being
// formed): all nodes at initialisation, the round's work slots otherwise
__device__ inline int pick_node(const RfastDev& s, bool init, int* t_old) {
  if (init) {
    *t_old = -1;
    return blockIdx.y;
  }
  const int2 slot = s.active_plan[blockIdx.y];
  *t_old = slot.y;
  return slot.x;
}

// active != NULL: blockIdx.y is the node itself and active[node] says whether the round activates it (the caller's
// schedule): the row number is then fetched at the same time as the flag, not after a look at the list of work slots.
__global__ void __launch_bounds__(kThreads) rfast_rows_kernel(RfastDev s, const int32_t* batch_idx, int B, bool init,
                                                              const uint8_t* active) {
  const int b = blockIdx.x * kWaves + (threadIdx.x >> 6);
  int i, row;
  if (active) {
    i = blockIdx.y;
    const uint8_t flag = active[i];
    const int raw = batch_idx && b < B ? batch_idx[(size_t)i * B + b] : b;
    asm volatile("" ::: "memory");  // both loads go out before the branch on the first
    if (!flag || b >= B) return;
    row = checked_row(s, i, raw);
  } else {
    int t_unused;
    i = pick_node(s, init, &t_unused);
    if (i < 0 || b >= B) return;
    row = sample_row(s, batch_idx, i, b, B);
  }
  const int lane = threadIdx.x & 63;
  const int64_t p = s.p;
  const float* a = (const float*)s.prob.data0 + ((size_t)i * s.prob.samples + row) * p;
  const float* x = s.x + (size_t)i * p;
  // the target goes out with the row, not after the dot product (one round trip to memory less at the end)
  const float y = ((const float*)s.prob.data1)[(size_t)i * s.prob.samples + row];
  float acc = 0.f;
  if ((p & 3) == 0) {
    // sixteen 1 KiB pieces of the row (4096 coordinates) per step, all thirty-two loads issued before the first
    // use: one wavefront per row has nothing else to hide the memory latency with, and a step costs a round trip
    constexpr int kPieces = 16;
    for (int64_t k0 = (int64_t)lane * 4; k0 < p; k0 += 256 * kPieces) {
      float4 av[kPieces], xv[kPieces];
#pragma unroll
      for (int u = 0; u < kPieces; ++u)
        if (k0 + 256 * u < p) {
          av[u] = *reinterpret_cast<const float4*>(a + k0 + 256 * u);
          xv[u] = *reinterpret_cast<const float4*>(x + k0 + 256 * u);
        }
#pragma unroll
      for (int u = 0; u < kPieces; ++u)
        if (k0 + 256 * u < p) {
          acc = fmaf(av[u].x, xv[u].x, acc);
          acc = fmaf(av[u].y, xv[u].y, acc);
          acc = fmaf(av[u].z, xv[u].z, acc);
          acc = fmaf(av[u].w, xv[u].w, acc);
        }
    }
  } else {
    for (int64_t k = lane; k < p; k += 64) acc = fmaf(a[k], x[k], acc);
  }
  acc = wave_sum(acc);
  if (lane == 0) {
    const float r = s.prob.kind == RFAST_OBJ_LOGISTIC ? 1.0f / (1.0f + expf(-acc)) - y : acc - y;
    s.resid[(size_t)i * B + b] = r;
  }
}

// VEC = 4: a workgroup owns 256 coordinates (one float4 per lane); its four wavefronts each take
// every fourth sampled row (a row is then one coalesced 1 KiB read per wavefront and the row
// number is wavefront-uniform) and the four partial sums meet in LDS.  That gives p/256
// workgroups per node instead of p/1024 and a quarter of the loop per lane: with a few dozen
// rows per node there is not enough work to hide the latency otherwise.  VEC = 1: one coordinate
// per lane, every lane walks over all rows.
template <int VEC>
__global__ void __launch_bounds__(kThreads) rfast_cols_kernel(RfastDev s, const int32_t* batch_idx, int B, bool init) {
  extern __shared__ float sh[];  // [B] residuals, [B] row numbers, then (VEC = 4) [4][64] float4 partial sums
  int t_old;
  const int i = pick_node(s, init, &t_old);
  if (i < 0) return;
  float* r_sh = sh;
  int* row_sh = reinterpret_cast<int*>(sh + B);
  for (int b = threadIdx.x; b < B; b += kThreads) {
    r_sh[b] = s.resid[(size_t)i * B + b];
    row_sh[b] = sample_row(s, batch_idx, i, b, B);
  }
  __syncthreads();
  const int64_t p = s.p;
  float* g_new = s.g + (size_t)((t_old + 1) & 1) * s.n * p + (size_t)i * p;
  const float inv = 1.0f / (float)B;
  // l2 term of the logistic objective plus the weight decay of the optimizer variant
  const float lam = (s.prob.kind == RFAST_OBJ_LOGISTIC ? s.prob.lambda : 0.f) + s.wd;
  if (VEC == 4) {
    const int lane = threadIdx.x & 63, rg = threadIdx.x >> 6;
    const int64_t k = ((int64_t)blockIdx.x * 64 + lane) * 4;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (k < p) {
      const float* base = (const float*)s.prob.data0 + (size_t)i * s.prob.samples * p + k;
#pragma unroll 4
      for (int b = rg; b < B; b += kWaves) {
        const float4 av = *reinterpret_cast<const float4*>(base + (size_t)row_sh[b] * p);
        const float r = r_sh[b];
        acc.x = fmaf(r, av.x, acc.x);
        acc.y = fmaf(r, av.y, acc.y);
        acc.z = fmaf(r, av.z, acc.z);
        acc.w = fmaf(r, av.w, acc.w);
      }
    }
    float4* part = reinterpret_cast<float4*>(sh + ((2 * B + 3) & ~3));
    part[rg * 64 + lane] = acc;
    __syncthreads();
    if (rg == 0 && k < p) {
#pragma unroll
      for (int q = 1; q < kWaves; ++q) {
        const float4 o = part[q * 64 + lane];
        acc.x += o.x; acc.y += o.y; acc.z += o.z; acc.w += o.w;
      }
      const float4 xv = *reinterpret_cast<const float4*>(s.x + (size_t)i * p + k);
      *reinterpret_cast<float4*>(g_new + k) = make_float4(fmaf(lam, xv.x, acc.x * inv), fmaf(lam, xv.y, acc.y * inv),
                                                          fmaf(lam, xv.z, acc.z * inv), fmaf(lam, xv.w, acc.w * inv));
    }
  } else {
    const int64_t k = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (k >= p) return;
    const float* base = (const float*)s.prob.data0 + (size_t)i * s.prob.samples * p + k;
    float acc = 0.f;
    for (int b = 0; b < B; ++b) acc = fmaf(r_sh[b], base[(size_t)row_sh[b] * p], acc);
    g_new[k] = fmaf(lam, s.x[(size_t)i * p + k], acc * inv);
  }
}

// ---------------------------------------------------------------------------
// Consecutive rounds of these objectives as TWO kernels per round instead of four.  A kernel that moves a few
// kilobytes per workgroup lasts 4-7 us whatever it does (launch, then three or four dependent round trips to
// memory), and at p of a few thousand a round is four such kernels in a row.  Mixing (S1, S2a, S3) of round r+1
// needs nothing of round r's tracker update (S2b, S2c, S3, S4) but the node's own new z, so the lane that
// tracks four coordinates of a node in round r mixes them for round r+1 right away:
//   rfast_rows_kernel              r_s of round r, from the mixed x of round r
//   rfast_cols_track_mix_kernel    g' of round r from the residuals, the tracker update with it, and then x', v
//                                  of round r+1 for the nodes that round activates
// (a node active in round r+1 but not in round r is mixed by the same workgroups, from z in memory).  Every
// step computes what rfast_cols_kernel<4>, rfast_state_kernel<TRACK> and rfast_state_kernel<MIX> compute, in the
// same order: same bits.  What a round reads of other nodes was written by an earlier launch: the versions of v
// that round r+1 mixes were published by round r's mixing at the latest, the running sums that round r tracks by
// round r-1's tracking at the latest.  The loads of the tracker update and of the mixing go out before the
// column sums, so that they are back when those are done.
// ---------------------------------------------------------------------------
constexpr int kChainKB = 8;     // in-edge loads in flight per batch
constexpr int kChainRows = 16;  // sampled rows in flight per wavefront of the column sums

// S1, S2a of one float4 of node i for the round whose R slots are slot_r: v and x' from z and x (the v of the
// in-neighbours in vb, loaded by chain_mix_loads)
__device__ inline void chain_mix_loads(const RfastDev& s, const int32_t* slot_r, int i, int64_t k, float4* vb, float* vw) {
  const int re0 = s.r_ptr[i], re1 = s.r_ptr[i + 1];
#pragma unroll
  for (int q = 0; q < kChainKB; ++q)
    if (re0 + q < re1) {
      vb[q] = *reinterpret_cast<const float4*>(s.v_ring + ((size_t)s.r_src[re0 + q] * s.M + slot_r[re0 + q]) * s.p + k);
      vw[q] = s.r_w[re0 + q];
    }
}
__device__ inline void chain_mix(const RfastDev& s, const int32_t* slot_r, int i, int64_t k, float gamma, float4 z, float4 x,
                                 float4* vb, float* vw, float4* v, float4* x_new) {
  const int re0 = s.r_ptr[i], re1 = s.r_ptr[i + 1];
  *v = fma_s(-gamma, z, x);
  float4 acc = mul_s(s.r_self[i], *v);
#pragma unroll
  for (int q = 0; q < kChainKB; ++q)
    if (re0 + q < re1) acc = fma_s(vw[q], vb[q], acc);
  for (int eb = re0 + kChainKB; eb < re1; eb += kChainKB) {  // in-degree above one batch
#pragma unroll
    for (int q = 0; q < kChainKB; ++q)
      if (eb + q < re1) {
        vb[q] = *reinterpret_cast<const float4*>(s.v_ring + ((size_t)s.r_src[eb + q] * s.M + slot_r[eb + q]) * s.p + k);
        vw[q] = s.r_w[eb + q];
      }
#pragma unroll
    for (int q = 0; q < kChainKB; ++q)
      if (eb + q < re1) acc = fma_s(vw[q], vb[q], acc);
  }
  *x_new = acc;
}

// s points at the plan arrays of round r and active at its activity flags (the caller's schedule: one byte per node);
// active_next (NULL: there is no next round to mix for) and next_slot_r are those of round r+1, gamma_next its step
// size.  Grid (ceil(p / 256), n): a workgroup per node and 256 coordinates.  It finds everything it needs about its
// node by the node's number, in one round trip to memory, instead of looking its node up in the list of work slots first.
__global__ void __launch_bounds__(kThreads) rfast_cols_track_mix_kernel(RfastDev s, const int32_t* batch_idx, int B,
                                                                        const uint8_t* active, const uint8_t* active_next,
                                                                        const int32_t* next_slot_r, float gamma_next) {
  extern __shared__ float sh[];  // [B] residuals, [B] row numbers, then [4][64] float4 partial sums
  const int64_t p = s.p;
  const int M = s.M;
  const int i = blockIdx.y;
  const int lane = threadIdx.x & 63, rg = threadIdx.x >> 6;
  const int64_t k = ((int64_t)blockIdx.x * 64 + lane) * 4;
  const bool mine = rg == 0 && k < p;  // the lane that owns coordinates k .. k+3 of the node
  float4 vb[kChainKB];
  float vw[kChainKB];
  // Whatever can be fetched by the node's number alone goes out together with the activity flags, before anything
  // branches on them (the addresses are valid for every node): one round trip to memory instead of two.
  const uint8_t flag = active[i], flag_next = active_next != nullptr ? active_next[i] : (uint8_t)0;
  const int t_old = s.plan_t[i];  // the node's counter at the start of round r
  const int ce0 = s.c_ptr[i], ce1 = s.c_ptr[i + 1];
  const bool pushes = s.co_ptr[i + 1] > s.co_ptr[i];
  // the first 256 residuals and row numbers: loaded here, parked in LDS once the owner's loads below are out too
  const int b_first = threadIdx.x;
  float r_first = 0.f;
  int row_first = b_first;
  if (b_first < B) {
    r_first = s.resid[(size_t)i * B + b_first];
    if (batch_idx) row_first = batch_idx[(size_t)i * B + b_first];
  }
  asm volatile("" ::: "memory");  // the loads above stay above the branches below
  const bool on = flag != 0, on_next = flag_next != 0;
  const int t_next = on_next ? t_old + (on ? 1 : 0) : -1;  // ... of round r+1, if that round activates the node
  if (!on) {
    // ---- a node that round r+1 activates and round r did not: S1, S2a, S3 (v half) from memory
    if (!mine || !on_next) return;
    const size_t node_off = (size_t)i * p + k;
    const float4 z = *reinterpret_cast<const float4*>(s.z + node_off);
    const float4 x = *reinterpret_cast<const float4*>(s.x + node_off);
    chain_mix_loads(s, next_slot_r, i, k, vb, vw);
    float4 v, x_new;
    chain_mix(s, next_slot_r, i, k, gamma_next, z, x, vb, vw, &v, &x_new);
    *reinterpret_cast<float4*>(s.v_ring + ((size_t)i * M + (t_next + 1) % M) * p + k) = v;
    *reinterpret_cast<float4*>(s.x + node_off) = x_new;
    return;
  }
  float* r_sh = sh;
  int* row_sh = reinterpret_cast<int*>(sh + B);
  const size_t node_off = (size_t)i * p + k;
  const int slot_new = (t_old + 1) % M, slot_cur = t_old % M;
  // ---- the owner's operands of the tracker update and of the next mixing go out before the column sums
  float4 x_i, z_i, g_old, sig_cur, sg[kChainKB], rt[kChainKB];
  float ca[kChainKB];
  int pl[kChainKB];
  if (mine) {
    x_i = *reinterpret_cast<const float4*>(s.x + node_off);
    z_i = *reinterpret_cast<const float4*>(s.z + node_off);
    g_old = *reinterpret_cast<const float4*>(s.g + (size_t)(t_old & 1) * s.n * p + node_off);
    if (pushes) sig_cur = *reinterpret_cast<const float4*>(s.sigma_ring + ((size_t)i * M + slot_cur) * p + k);
#pragma unroll
    for (int q = 0; q < kChainKB; ++q) {
      const int e = ce0 + q;
      pl[q] = e < ce1 ? s.plan_c[e] : 0;
      if (pl[q] & (1 << 16)) {
        const float* ring = s.sigma_ring + (size_t)s.c_src[e] * M * p + k;
        const int prev = (pl[q] >> 8) & 0xFF;
        sg[q] = *reinterpret_cast<const float4*>(ring + (size_t)(pl[q] & 0xFF) * p);
        rt[q] = *reinterpret_cast<const float4*>(prev != 0xFF ? ring + (size_t)prev * p : s.rho_tilde + (size_t)e * p + k);
        ca[q] = s.c_w[e];
      }
    }
  }
  if (b_first < B) {
    r_sh[b_first] = r_first;
    row_sh[b_first] = checked_row(s, i, row_first);
  }
  for (int b = threadIdx.x + kThreads; b < B; b += kThreads) {
    r_sh[b] = s.resid[(size_t)i * B + b];
    row_sh[b] = sample_row(s, batch_idx, i, b, B);
  }
  if (mine && t_next >= 0) chain_mix_loads(s, next_slot_r, i, k, vb, vw);
  __syncthreads();  // residuals and row numbers are in LDS

  // ---- as rfast_cols_kernel<4>: wavefront rg sums rows rg, rg + 4, ...; sixteen rows in flight
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  if (k < p) {
    const float* base = (const float*)s.prob.data0 + (size_t)i * s.prob.samples * p + k;
    for (int b0 = rg; b0 < B; b0 += kWaves * kChainRows) {
      float4 av[kChainRows];
#pragma unroll
      for (int u = 0; u < kChainRows; ++u) {
        const int b = b0 + kWaves * u;
        if (b < B) av[u] = *reinterpret_cast<const float4*>(base + (size_t)row_sh[b] * p);
      }
#pragma unroll
      for (int u = 0; u < kChainRows; ++u) {
        const int b = b0 + kWaves * u;
        if (b < B) {
          const float r = r_sh[b];
          acc.x = fmaf(r, av[u].x, acc.x);
          acc.y = fmaf(r, av[u].y, acc.y);
          acc.z = fmaf(r, av[u].z, acc.z);
          acc.w = fmaf(r, av[u].w, acc.w);
        }
      }
    }
  }
  float4* part = reinterpret_cast<float4*>(sh + ((2 * B + 3) & ~3));
  part[rg * 64 + lane] = acc;
  __syncthreads();
  if (!mine) return;
#pragma unroll
  for (int q = 1; q < kWaves; ++q) {
    const float4 o = part[q * 64 + lane];
    acc.x += o.x; acc.y += o.y; acc.z += o.z; acc.w += o.w;
  }
  const float inv = 1.0f / (float)B;
  // l2 term of the logistic objective plus the weight decay of the optimizer variant
  const float lam = (s.prob.kind == RFAST_OBJ_LOGISTIC ? s.prob.lambda : 0.f) + s.wd;
  const float4 g_new = make_float4(fmaf(lam, x_i.x, acc.x * inv), fmaf(lam, x_i.y, acc.y * inv), fmaf(lam, x_i.z, acc.z * inv),
                                   fmaf(lam, x_i.w, acc.w * inv));
  *reinterpret_cast<float4*>(s.g + (size_t)((t_old + 1) & 1) * s.n * p + node_off) = g_new;
  // S2b, S4: as rfast_state_kernel<TRACK>
  float4 z_half = z_i;
#pragma unroll
  for (int q = 0; q < kChainKB; ++q)
    if (pl[q] & (1 << 16)) {
      z_half = track_edge(z_half, ca[q], sg[q], rt[q], ((pl[q] >> 8) & 0xFF) != 0xFF);
      if (pl[q] & (1 << 17)) *reinterpret_cast<float4*>(s.rho_tilde + (size_t)(ce0 + q) * p + k) = mul_s(ca[q], sg[q]);
    }
  for (int eb = ce0 + kChainKB; eb < ce1; eb += kChainKB) {  // in-degree above one batch
#pragma unroll
    for (int q = 0; q < kChainKB; ++q) {
      const int e = eb + q;
      pl[q] = e < ce1 ? s.plan_c[e] : 0;
      if (pl[q] & (1 << 16)) {
        const float* ring = s.sigma_ring + (size_t)s.c_src[e] * M * p + k;
        const int prev = (pl[q] >> 8) & 0xFF;
        sg[q] = *reinterpret_cast<const float4*>(ring + (size_t)(pl[q] & 0xFF) * p);
        rt[q] = *reinterpret_cast<const float4*>(prev != 0xFF ? ring + (size_t)prev * p : s.rho_tilde + (size_t)e * p + k);
        ca[q] = s.c_w[e];
      }
    }
#pragma unroll
    for (int q = 0; q < kChainKB; ++q)
      if (pl[q] & (1 << 16)) {
        z_half = track_edge(z_half, ca[q], sg[q], rt[q], ((pl[q] >> 8) & 0xFF) != 0xFF);
        if (pl[q] & (1 << 17)) *reinterpret_cast<float4*>(s.rho_tilde + (size_t)(eb + q) * p + k) = mul_s(ca[q], sg[q]);
      }
  }
  z_half = sub(add(z_half, g_new), g_old);
  // S2c, S3 (rho half)
  const float4 z_new = mul_s(s.c_self[i], z_half);
  *reinterpret_cast<float4*>(s.z + node_off) = z_new;
  if (pushes) {
    *reinterpret_cast<float4*>(s.sigma_ring + ((size_t)i * M + slot_new) * p + k) = add(sig_cur, z_half);
    if (s.node_spill[i] != 0) {  // S4 for receivers that do not do it themselves in this round
      const float4 leaving = *reinterpret_cast<const float4*>(s.sigma_ring + ((size_t)i * M + (t_old - (M - 2)) % M) * p + k);
      for (int o = s.co_ptr[i]; o < s.co_ptr[i + 1]; ++o)
        if (s.plan_c[s.co_eid[o]] & (1 << 18))
          *reinterpret_cast<float4*>(s.rho_tilde + (size_t)s.co_eid[o] * p + k) = mul_s(s.co_w[o], leaving);
    }
  }
  // ---- round r+1 for this node: S1, S2a, S3 (v half), as rfast_state_kernel<MIX>, on the z just formed
  if (t_next >= 0) {
    float4 v, x_new;
    chain_mix(s, next_slot_r, i, k, gamma_next, z_new, x_i, vb, vw, &v, &x_new);
    *reinterpret_cast<float4*>(s.v_ring + ((size_t)i * M + (t_next + 1) % M) * p + k) = v;
    *reinterpret_cast<float4*>(s.x + node_off) = x_new;
  }
}

// initial gradient of the diagonal quadratic (sample version 0) and z^0 = g^0
__global__ void __launch_bounds__(kThreads) rfast_copy_z_kernel(RfastDev s) {
  const size_t tot = (size_t)s.n * s.p;
  for (size_t q = (size_t)blockIdx.x * kThreads + threadIdx.x; q < tot; q += (size_t)gridDim.x * kThreads) s.z[q] = s.g[q];
}

hipError_t gemv_pair(rfast_ctx* c, const int32_t* batch_idx, bool init) {
  const RfastDev& d = c->d;
  const int B = d.prob.batch > 0 ? d.prob.batch : d.prob.samples;
  const int32_t* bi = d.prob.batch > 0 ? batch_idx : nullptr;
  hipLaunchKernelGGL(rfast_rows_kernel, dim3((B + kWaves - 1) / kWaves, d.n), dim3(kThreads), 0, c->stream, d, bi, B, init, nullptr);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const bool vec4 = (d.p % 4) == 0;
  const int64_t per_block = vec4 ? 256 : kThreads;  // coordinates per workgroup
  const unsigned gx = (unsigned)((d.p + per_block - 1) / per_block);
  const size_t shm = (size_t)((2 * B + 3) & ~3) * 4 + (vec4 ? (size_t)kWaves * 64 * 16 : 0);
  if (vec4)
    hipLaunchKernelGGL(rfast_cols_kernel<4>, dim3(gx, d.n), dim3(kThreads), shm, c->stream, d, bi, B, init);
  else
    hipLaunchKernelGGL(rfast_cols_kernel<1>, dim3(gx, d.n), dim3(kThreads), shm, c->stream, d, bi, B, init);
  return hipGetLastError();
}

}  // namespace

// Consecutive rounds as two kernels each: least squares or logistic regression, p a multiple of 4, no heavy-ball
// buffer (its update belongs to the mixing pass).
bool rfast_chain_eligible(const rfast_ctx* c) {
  const RfastDev& d = c->d;
  if (d.prob.kind != RFAST_OBJ_LEAST_SQUARES && d.prob.kind != RFAST_OBJ_LOGISTIC) return false;
  const int B = d.prob.batch > 0 ? d.prob.batch : d.prob.samples;
  return (d.p % 4) == 0 && d.mom == nullptr && (size_t)((2 * B + 3) & ~3) * 4 + (size_t)kWaves * 64 * 16 <= 60 * 1024;
}

// r_s of the round whose activity flags are d_active
hipError_t rfast_launch_rows(rfast_ctx* c, const int32_t* batch_idx, const uint8_t* d_active) {
  const RfastDev& d = c->d;
  const int B = d.prob.batch > 0 ? d.prob.batch : d.prob.samples;
  hipLaunchKernelGGL(rfast_rows_kernel, dim3((B + kWaves - 1) / kWaves, d.n), dim3(kThreads), 0, c->stream, d,
                     d.prob.batch > 0 ? batch_idx : nullptr, B, false, d_active);
  return hipGetLastError();
}

// g' and the tracker update of the round whose plan arrays c->d points at and whose activity flags are d_active, and
// (d_active_next != NULL) the mixing of the round after it, whose plan arrays lie next_set_bytes further on
hipError_t rfast_launch_cols_track_mix(rfast_ctx* c, const int32_t* batch_idx, const uint8_t* d_active, const uint8_t* d_active_next,
                                       size_t next_set_bytes, float gamma_next) {
  const RfastDev& d = c->d;
  const int B = d.prob.batch > 0 ? d.prob.batch : d.prob.samples;
  const size_t shm = (size_t)((2 * B + 3) & ~3) * 4 + (size_t)kWaves * 64 * 16;
  const int64_t tiles = (d.p + 255) / 256;
  if (tiles > 0x7fffffffLL || d.n > 65535) return hipErrorInvalidValue;
  const int32_t* next_slot_r = reinterpret_cast<const int32_t*>(reinterpret_cast<const char*>(d.slot_r) + next_set_bytes);
  hipLaunchKernelGGL(rfast_cols_track_mix_kernel, dim3((unsigned)tiles, d.n), dim3(kThreads), shm, c->stream, d,
                     d.prob.batch > 0 ? batch_idx : nullptr, B, d_active, d_active_next, next_slot_r, gamma_next);
  return hipGetLastError();
}

hipError_t rfast_softmax_gradient(rfast_ctx* c, const int32_t* batch_idx, bool init);  // rfast_softmax.hip
hipError_t rfast_diag_init_gradient(rfast_ctx* c);                                       // rfast_round.hip

size_t rfast_gemv_scratch_floats(int32_t n, const rfast_problem* prob) {
  if (prob->kind != RFAST_OBJ_LEAST_SQUARES && prob->kind != RFAST_OBJ_LOGISTIC) return 0;
  const int B = prob->batch > 0 ? prob->batch : prob->samples;
  return (size_t)n * (size_t)B;
}

hipError_t rfast_launch_gradient(rfast_ctx* c, const int32_t* batch_idx) {
  switch (c->d.prob.kind) {
    case RFAST_OBJ_LEAST_SQUARES:
    case RFAST_OBJ_LOGISTIC: return gemv_pair(c, batch_idx, false);
    case RFAST_OBJ_SOFTMAX_BF16: return rfast_softmax_gradient(c, batch_idx, false);
    default: return hipErrorInvalidValue;
  }
}

hipError_t rfast_launch_init_grad(rfast_ctx* c, const int32_t* batch_idx0) {
  hipError_t e;
  switch (c->d.prob.kind) {
    case RFAST_OBJ_DIAG_QUADRATIC: e = rfast_diag_init_gradient(c); break;
    case RFAST_OBJ_LEAST_SQUARES:
    case RFAST_OBJ_LOGISTIC: e = gemv_pair(c, batch_idx0, true); break;
    case RFAST_OBJ_SOFTMAX_BF16: e = rfast_softmax_gradient(c, batch_idx0, true); break;
    default: return hipErrorInvalidValue;
  }
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(rfast_copy_z_kernel, dim3(1024), dim3(kThreads), 0, c->stream, c->d);
  return hipGetLastError();
}
