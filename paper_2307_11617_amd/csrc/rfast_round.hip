// State-update kernels of one activation round (Algorithm 1, steps S1-S5).
//
// One work item = (active node, tile of coordinates).  Everything is
// elementwise in the coordinate k, has no reuse and moves 4 bytes per ~1 flop,
// so the kernels are pure HBM streams: every access is a float4 per lane
// (1 KiB per wavefront instruction), loads of one phase are issued back to back
// before their first use, and inactive nodes cost nothing.
//
//   FUSED  separable objective (diagonal quadratic): S1, S2a, gradient, S2b,
//          S2c, S3, S4 in one pass.
//   MIX    S1, S2a and the v half of S3; the gradient kernels run next.
//   TRACK  S2b, S2c, the rho half of S3, S4.
//
// The per-edge running sums rho_li of S2c are kept as ONE running sum per sender,
// sigma_i = sum of z_half, with rho_li = a_li * sigma_i formed by the receiver:
// algebraically identical to the per-edge recursion, bit-identical when a_li is
// a power of two, and it replaces dO reads + dO writes per coordinate by 1 + 1.
#include "rfast_internal.h"
#include "rfast_vec.h"

namespace {

constexpr int kThreads = 256;

// ------------------------------------------------------------------- kernel
// Loads of one live in-edge of C (plan word pl): the running sum being consumed and the one
// consumed last time (rho~ of S4), which is read from the sender's ring while it is still there.
template <int VEC>
__device__ inline void load_edge(const RfastDev& s, int e, int pl, int M, int64_t p, int64_t k, typename V<VEC>::T* sg,
                                 typename V<VEC>::T* rt) {
  const float* ring = s.sigma_ring + (size_t)s.c_src[e] * M * p + k;
  const int prev = (pl >> 8) & 0xFF;
  const float* last = prev != 0xFF ? ring + (size_t)prev * p : s.rho_tilde + (size_t)e * p + k;
  *sg = V<VEC>::ld(ring + (size_t)(pl & 0xFF) * p);
  *rt = V<VEC>::ld(last);
}

// Softmax objective: the GEMMs read the weights as bf16, 8 consecutive features of one class per
// 16-byte unit (layout [d/8][K][8]).  The 1024 coordinates of one tile are 1024/K whole features
// x K classes, i.e. exactly the elements [1024*tile, 1024*tile + 1024) of that layout in another
// order: permute through LDS and write them out coalesced, instead of a pass that re-reads x.
template <int VEC>
__device__ inline void emit_bf16_blocked(const RfastDev& s, int i, int tile, typename V<VEC>::T x_new) {
  __shared__ unsigned short perm[kThreads * 4];
  const int K = s.prob.K;
  const int l = threadIdx.x * 4, f = l / K, k0 = l % K;
  unsigned short* dst = perm + (f >> 3) * (8 * K) + k0 * 8 + (f & 7);
  const float4 w = *reinterpret_cast<const float4*>(&x_new);
  dst[0] = rfast_f32_to_bf16(w.x);
  dst[8] = rfast_f32_to_bf16(w.y);
  dst[16] = rfast_f32_to_bf16(w.z);
  dst[24] = rfast_f32_to_bf16(w.w);
  __syncthreads();
  unsigned short* wt = (unsigned short*)s.gscratch + (size_t)i * s.p + (size_t)tile * (kThreads * 4);
  *reinterpret_cast<uint2*>(wt + l) = *reinterpret_cast<const uint2*>(perm + l);
}

// MOM: the optimizer variant's heavy-ball buffer is in use (a template flag so that the
// plain method carries neither the branch nor the registers).
// KB: in-edge loads kept in flight per phase.  8 costs 139 registers (3 wavefronts per SIMD), 4 costs
// 91 (5 wavefronts): graphs with many in-edges per node want the deeper batch, graphs with few want
// the wavefronts (measured: bidirectional ring 1.53 vs 1.59 ms with 8 vs 4, tree/star 0.293 vs 0.274).
template <int MODE, int VEC, bool MOM, int KB>
__global__ void __launch_bounds__(kThreads) rfast_state_kernel(RfastDev s, float gamma, int tiles_per_node) {
  using T = typename V<VEC>::T;
  const int a = blockIdx.x / tiles_per_node;
  const int2 slot = s.active_plan[a];  // {node, its counter at the start of the round}, node < 0: no work
  if (slot.x < 0) return;
  const int tile = blockIdx.x - a * tiles_per_node;
  const int64_t k = ((int64_t)tile * kThreads + threadIdx.x) * V<VEC>::W;
  if (k >= s.p) return;

  constexpr bool kMix = MODE != RFAST_MODE_TRACK, kTrack = MODE != RFAST_MODE_MIX;
  const int i = slot.x;
  const int64_t p = s.p;
  const int M = s.M;
  const int t_old = slot.y;
  const int slot_new = (t_old + 1) % M;
  const int slot_cur = t_old % M;
  const size_t node_off = (size_t)i * p + k;
  float* g_old_p = s.g + (size_t)(t_old & 1) * s.n * p + node_off;
  float* g_new_p = s.g + (size_t)((t_old + 1) & 1) * s.n * p + node_off;
  const int re0 = s.r_ptr[i], re1 = s.r_ptr[i + 1];
  const int ce0 = s.c_ptr[i], ce1 = s.c_ptr[i + 1];
  // The running sums of S2c share one factor per sender: rho_li = a_li * sigma_i with
  // sigma_i = sum of every z_half node i produced (1 read + 1 write instead of dO + dO).
  const bool pushes = s.co_ptr[i + 1] > s.co_ptr[i];

  // ---- every load of the first batch of each phase is issued before its first use:
  //      with few wavefronts per CU this is what keeps enough bytes in flight
  T x_i, z_i, g_old, g_new, h, c, sig_cur, m_i;
  T vb[KB], sg[KB], rt[KB];
  float vw[KB], ca[KB];
  int pl[KB];  // plan words of the C in-edges of the current batch (0: nothing to do)
  const bool spills = pushes && s.node_spill[i] != 0;
  z_i = V<VEC>::ld(s.z + node_off);
  if (kMix) {
    x_i = V<VEC>::ld(s.x + node_off);
    if (MOM) m_i = V<VEC>::ld(s.mom + node_off);
#pragma unroll
    for (int q = 0; q < KB; ++q)
      if (re0 + q < re1) {
        vb[q] = V<VEC>::ld(s.v_ring + ((size_t)s.r_src[re0 + q] * M + s.slot_r[re0 + q]) * p + k);
        vw[q] = s.r_w[re0 + q];
      }
  }
  if (kTrack) {
    if (MODE == RFAST_MODE_FUSED) {
      h = V<VEC>::ld((const float*)s.prob.data0 + node_off);
      c = V<VEC>::ld((const float*)s.prob.data1 + node_off);
    } else {
      g_old = V<VEC>::ld(g_old_p);
      g_new = V<VEC>::ld(g_new_p);
    }
    if (pushes) sig_cur = V<VEC>::ld(s.sigma_ring + ((size_t)i * M + slot_cur) * p + k);
#pragma unroll
    for (int q = 0; q < KB; ++q) {
      const int e = ce0 + q;
      pl[q] = e < ce1 ? s.plan_c[e] : 0;
      if (pl[q] & (1 << 16)) {
        load_edge<VEC>(s, e, pl[q], M, p, k, &sg[q], &rt[q]);
        ca[q] = s.c_w[e];
      }
    }
  }

  T x_new;
  if (kMix) {
    // S1: local descent; with the optimizer variant along the heavy-ball buffer m <- beta m + z
    T dir = z_i;
    if (MOM) {
      dir = fma_s(s.beta, m_i, z_i);
      V<VEC>::st(s.mom + node_off, dir);
    }
    const T v = fma_s(-gamma, dir, x_i);
    // S2a: pull the stamped neighbour copies and mix with row-stochastic weights
    x_new = mul_s(s.r_self[i], v);
#pragma unroll
    for (int q = 0; q < KB; ++q)
      if (re0 + q < re1) x_new = fma_s(vw[q], vb[q], x_new);
    for (int eb = re0 + KB; eb < re1; eb += KB) {  // in-degree above one batch
#pragma unroll
      for (int q = 0; q < KB; ++q)
        if (eb + q < re1) {
          vb[q] = V<VEC>::ld(s.v_ring + ((size_t)s.r_src[eb + q] * M + s.slot_r[eb + q]) * p + k);
          vw[q] = s.r_w[eb + q];
        }
#pragma unroll
      for (int q = 0; q < KB; ++q)
        if (eb + q < re1) x_new = fma_s(vw[q], vb[q], x_new);
    }
    // S3 (v half): publish version t+1
    V<VEC>::st(s.v_ring + ((size_t)i * M + slot_new) * p + k, v);
    V<VEC>::st(s.x + node_off, x_new);
    if (MODE == RFAST_MODE_MIX) {
      if constexpr (VEC != 1) {  // p is a multiple of 2048 for this objective: every tile is full
        if (s.prob.kind == RFAST_OBJ_SOFTMAX_BF16 && (1024 % s.prob.K) == 0) emit_bf16_blocked<VEC>(s, i, tile, x_new);
      }
      return;
    }
  }

  if (MODE == RFAST_MODE_FUSED) {
    // New sample at the new point; the old sample is the same function of the old x and the
    // old counter, so it is recomputed rather than kept in memory (2 words per coordinate less).
    g_new = diag_sample<VEC>(s, h, c, x_new, i, t_old + 1, k);
    g_old = diag_sample<VEC>(s, h, c, x_i, i, t_old, k);
  }

  // S2b: tracker sum over the in-edges of C; S4: buffer what was consumed.
  // An edge whose stamp did not move holds rho == rho~ exactly and is skipped.
  T z_half = z_i;
#pragma unroll
  for (int q = 0; q < KB; ++q)
    if (pl[q] & (1 << 16)) {
      z_half = track_edge(z_half, ca[q], sg[q], rt[q], ((pl[q] >> 8) & 0xFF) != 0xFF);
      if (pl[q] & (1 << 17)) V<VEC>::st(s.rho_tilde + (size_t)(ce0 + q) * p + k, mul_s(ca[q], sg[q]));
    }
  for (int eb = ce0 + KB; eb < ce1; eb += KB) {  // in-degree above one batch
#pragma unroll
    for (int q = 0; q < KB; ++q) {
      const int e = eb + q;
      pl[q] = e < ce1 ? s.plan_c[e] : 0;
      if (pl[q] & (1 << 16)) {
        load_edge<VEC>(s, e, pl[q], M, p, k, &sg[q], &rt[q]);
        ca[q] = s.c_w[e];
      }
    }
#pragma unroll
    for (int q = 0; q < KB; ++q)
      if (pl[q] & (1 << 16)) {
        z_half = track_edge(z_half, ca[q], sg[q], rt[q], ((pl[q] >> 8) & 0xFF) != 0xFF);
        if (pl[q] & (1 << 17)) V<VEC>::st(s.rho_tilde + (size_t)(eb + q) * p + k, mul_s(ca[q], sg[q]));
      }
  }
  z_half = sub(add(z_half, g_new), g_old);

  // S2c: keep a_ii; push: sigma_i grows by z_half.  S3 (rho half): new version t+1
  V<VEC>::st(s.z + node_off, mul_s(s.c_self[i], z_half));
  if (pushes) {
    V<VEC>::st(s.sigma_ring + ((size_t)i * M + slot_new) * p + k, add(sig_cur, z_half));
    // S4 for receivers that do not do it themselves in this round: version t - D of this node's
    // running sum leaves the ring with this activation; a receiver whose buffer rho~ is that
    // version gets it copied to the rho~ array now (the slot read here is not the one written above).
    if (spills) {
      const T leaving = V<VEC>::ld(s.sigma_ring + ((size_t)i * M + (t_old - (M - 2)) % M) * p + k);
      for (int o = s.co_ptr[i]; o < s.co_ptr[i + 1]; ++o)
        if (s.plan_c[s.co_eid[o]] & (1 << 18)) V<VEC>::st(s.rho_tilde + (size_t)s.co_eid[o] * p + k, mul_s(s.co_w[o], leaving));
    }
  }
}

// Writes the current sample of every node, g_i = sample(x_i, t_i), into g[t_i & 1][i]: the
// initial gradient g^0 (t = 0, initialisation of Algorithm 1) and the copy that reads of
// the G field return.
template <int VEC>
__global__ void __launch_bounds__(kThreads) rfast_diag_sample_kernel(RfastDev s) {
  const int i = blockIdx.y;
  const int64_t k = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * VEC;
  if (k >= s.p) return;
  const size_t off = (size_t)i * s.p + k;
  using T = typename V<VEC>::T;
  const int t = s.t[i];
  const T h = V<VEC>::ld((const float*)s.prob.data0 + off);
  const T c = V<VEC>::ld((const float*)s.prob.data1 + off);
  V<VEC>::st(s.g + (size_t)(t & 1) * s.n * s.p + off, diag_sample<VEC>(s, h, c, V<VEC>::ld(s.x + off), i, t, k));
}

// Rebase of the running sums.  sigma_j only ever enters as a_ij*sigma_j - rho~_ij, so
// subtracting c_j = sigma_j(latest) from every ring slot of sender j and a_ij*c_j from
// every buffer rho~_ij fed by j changes nothing in exact arithmetic; in fp32 it
// removes the ever-growing common offset that the difference otherwise has to cancel.
template <int VEC>
__global__ void __launch_bounds__(kThreads) rfast_rebase_kernel(RfastDev s) {
  using T = typename V<VEC>::T;
  const int j = blockIdx.y;
  const int64_t k = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * V<VEC>::W;
  if (k >= s.p) return;
  const int o0 = s.co_ptr[j], o1 = s.co_ptr[j + 1];
  if (o0 == o1) return;  // nobody reads this sender's sums
  float* ring = s.sigma_ring + (size_t)j * s.M * s.p + k;
  const T c = V<VEC>::ld(ring + (size_t)(s.t[j] % s.M) * s.p);
  for (int m = 0; m < s.M; ++m) V<VEC>::st(ring + (size_t)m * s.p, sub(V<VEC>::ld(ring + (size_t)m * s.p), c));
  for (int o = o0; o < o1; ++o) {
    float* rt = s.rho_tilde + (size_t)s.co_eid[o] * s.p + k;
    V<VEC>::st(rt, sub(V<VEC>::ld(rt), mul_s(s.co_w[o], c)));
  }
}

// ---------------------------------------------------------------------------
// Synchronous push-pull step, eq. (2) of the paper (the recursion R-FAST is built on):
//   x_i' = sum_j w_ij (x_j - gamma z_j),   z_i' = sum_j a_ij z_j + grad f_i(x_i') - grad f_i(x_i)
// Every node steps at once, so the v_j = x_j - gamma z_j of all nodes are formed
// first (slot 0 of the v ring serves as the buffer) and z is double-buffered
// (parity 0: the z array, parity 1: slot 1 of the v ring).
// ---------------------------------------------------------------------------
__device__ inline float* sync_z(const RfastDev& s, int parity, int i) {
  return parity == 0 ? s.z + (size_t)i * s.p : s.v_ring + ((size_t)i * s.M + 1) * s.p;
}

// rounds: steps taken at once (the plan arrays are left as the last of them leaves them)
__global__ void __launch_bounds__(256) rfast_sync_plan_kernel(RfastDev s, int rounds) {
  for (int i = threadIdx.x; i < s.n; i += blockDim.x) {
    const int ti = s.t[i] + rounds - 1;
    s.plan_t[i] = ti;
    s.active_plan[i] = make_int2(i, ti);
    s.t[i] = ti + 1;
  }
  if (threadIdx.x == 0) {
    *s.n_active = s.n;
    for (int q = 0; q < 8; ++q) s.active_plan[s.n + q] = make_int2(-1, 0);
    *s.round_no = *s.round_no + rounds;
    s.n_active[1] = *s.round_no;
  }
}

template <int VEC>
__global__ void __launch_bounds__(kThreads) rfast_sync_descent_kernel(RfastDev s, float gamma, int parity) {
  const int i = blockIdx.y;
  const int64_t k = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * V<VEC>::W;
  if (k >= s.p) return;
  const auto x = V<VEC>::ld(s.x + (size_t)i * s.p + k);
  auto dir = V<VEC>::ld(sync_z(s, parity, i) + k);
  if (s.mom) {
    dir = fma_s(s.beta, V<VEC>::ld(s.mom + (size_t)i * s.p + k), dir);
    V<VEC>::st(s.mom + (size_t)i * s.p + k, dir);
  }
  V<VEC>::st(s.v_ring + (size_t)i * s.M * s.p + k, fma_s(-gamma, dir, x));
}

// PHASE 0: mix only (x').  PHASE 1: tracker only (reads g' written by the gradient
// kernels).  PHASE 2: mix + diagonal-quadratic gradient + tracker in one pass.
template <int VEC, int PHASE>
__global__ void __launch_bounds__(kThreads) rfast_sync_step_kernel(RfastDev s, int parity) {
  using T = typename V<VEC>::T;
  const int i = blockIdx.y;
  const int64_t k = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * V<VEC>::W;
  if (k >= s.p) return;
  const int64_t p = s.p;
  const int t_old = s.plan_t[i];
  const size_t off = (size_t)i * p + k;
  float* g_old_p = s.g + (size_t)(t_old & 1) * s.n * p + off;
  float* g_new_p = s.g + (size_t)((t_old + 1) & 1) * s.n * p + off;
  T x_new, g_new, g_old;
  if (PHASE != 1) {
    const T x_old = V<VEC>::ld(s.x + off);
    x_new = mul_s(s.r_self[i], V<VEC>::ld(s.v_ring + (size_t)i * s.M * p + k));
    for (int e = s.r_ptr[i]; e < s.r_ptr[i + 1]; ++e)
      x_new = fma_s(s.r_w[e], V<VEC>::ld(s.v_ring + (size_t)s.r_src[e] * s.M * p + k), x_new);
    V<VEC>::st(s.x + off, x_new);
    if (PHASE == 0) return;
    const T h = V<VEC>::ld((const float*)s.prob.data0 + off);
    const T c = V<VEC>::ld((const float*)s.prob.data1 + off);
    g_new = diag_sample<VEC>(s, h, c, x_new, i, t_old + 1, k);
    g_old = diag_sample<VEC>(s, h, c, x_old, i, t_old, k);
  } else {
    g_new = V<VEC>::ld(g_new_p);
    g_old = V<VEC>::ld(g_old_p);
  }
  T z_new = mul_s(s.c_self[i], V<VEC>::ld(sync_z(s, parity, i) + k));
  for (int e = s.c_ptr[i]; e < s.c_ptr[i + 1]; ++e)
    z_new = fma_s(s.c_w[e], V<VEC>::ld(sync_z(s, parity, s.c_src[e]) + k), z_new);
  z_new = sub(add(z_new, g_new), g_old);
  V<VEC>::st(sync_z(s, parity ^ 1, i) + k, z_new);
}

template <int VEC>
__global__ void __launch_bounds__(kThreads) rfast_sync_fold_kernel(RfastDev s) {
  const int i = blockIdx.y;
  const int64_t k = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * V<VEC>::W;
  if (k >= s.p) return;
  V<VEC>::st(s.z + (size_t)i * s.p + k, V<VEC>::ld(sync_z(s, 1, i) + k));
}

template <int MODE, bool MOM, int KB>
hipError_t launch(rfast_ctx* c, float gamma) {
  const RfastDev& d = c->d;
  const bool vec4 = (d.p % 4) == 0;
  const int64_t per_block = (int64_t)kThreads * (vec4 ? 4 : 1);
  const int64_t tiles = (d.p + per_block - 1) / per_block;
  const int64_t blocks = tiles * d.n;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  // Stream past the caches once the state dwarfs them (256 MB of last-level cache).  Wavefronts per
  // SIMD matter: the bidirectional ring (about 15 streams per node-update) is fastest at 3, slower at
  // 2 (capped through reserved LDS: +11 %) and at 4 or 5 (+2 %, +4 %); the register count of KB sets it.
  const bool streaming = (double)d.n * (double)d.p * 4.0 >= 32.0e6;
  if (vec4 && streaming)
    hipLaunchKernelGGL((rfast_state_kernel<MODE, -4, MOM, KB>), dim3((unsigned)blocks), dim3(kThreads), 0, c->stream, d, gamma, (int)tiles);
  else if (vec4)
    hipLaunchKernelGGL((rfast_state_kernel<MODE, 4, MOM, KB>), dim3((unsigned)blocks), dim3(kThreads), 0, c->stream, d, gamma, (int)tiles);
  else
    hipLaunchKernelGGL((rfast_state_kernel<MODE, 1, MOM, KB>), dim3((unsigned)blocks), dim3(kThreads), 0, c->stream, d, gamma, (int)tiles);
  return hipGetLastError();
}

}  // namespace

hipError_t rfast_diag_init_gradient(rfast_ctx* c) {
  const RfastDev& d = c->d;
  const bool vec4 = (d.p % 4) == 0;
  const int64_t per_block = (int64_t)kThreads * (vec4 ? 4 : 1);
  const unsigned gx = (unsigned)((d.p + per_block - 1) / per_block);
  if (vec4)
    hipLaunchKernelGGL(rfast_diag_sample_kernel<4>, dim3(gx, d.n), dim3(kThreads), 0, c->stream, d);
  else
    hipLaunchKernelGGL(rfast_diag_sample_kernel<1>, dim3(gx, d.n), dim3(kThreads), 0, c->stream, d);
  return hipGetLastError();
}

// phase: 0 plan + descent + mix, 1 tracker, 2 plan + descent + fused step, 3 fold z back into its array
hipError_t rfast_launch_sync(rfast_ctx* c, int phase, float gamma, int parity) {
  const RfastDev& d = c->d;
  const bool vec4 = (d.p % 4) == 0;
  const int64_t per_block = (int64_t)kThreads * (vec4 ? 4 : 1);
  const dim3 grid((unsigned)((d.p + per_block - 1) / per_block), d.n), blk(kThreads);
  const bool streaming = vec4 && (double)d.n * (double)d.p * 4.0 >= 32.0e6;
  if (phase == 0 || phase == 2) {
    hipLaunchKernelGGL(rfast_sync_plan_kernel, dim3(1), dim3(256), 0, c->stream, d, 1);
    if (streaming) hipLaunchKernelGGL(rfast_sync_descent_kernel<-4>, grid, blk, 0, c->stream, d, gamma, parity);
    else if (vec4) hipLaunchKernelGGL(rfast_sync_descent_kernel<4>, grid, blk, 0, c->stream, d, gamma, parity);
    else hipLaunchKernelGGL(rfast_sync_descent_kernel<1>, grid, blk, 0, c->stream, d, gamma, parity);
  }
  if (streaming) {
    if (phase == 0) hipLaunchKernelGGL((rfast_sync_step_kernel<-4, 0>), grid, blk, 0, c->stream, d, parity);
    if (phase == 1) hipLaunchKernelGGL((rfast_sync_step_kernel<-4, 1>), grid, blk, 0, c->stream, d, parity);
    if (phase == 2) hipLaunchKernelGGL((rfast_sync_step_kernel<-4, 2>), grid, blk, 0, c->stream, d, parity);
    if (phase == 3) hipLaunchKernelGGL(rfast_sync_fold_kernel<-4>, grid, blk, 0, c->stream, d);
  } else if (vec4) {
    if (phase == 0) hipLaunchKernelGGL((rfast_sync_step_kernel<4, 0>), grid, blk, 0, c->stream, d, parity);
    if (phase == 1) hipLaunchKernelGGL((rfast_sync_step_kernel<4, 1>), grid, blk, 0, c->stream, d, parity);
    if (phase == 2) hipLaunchKernelGGL((rfast_sync_step_kernel<4, 2>), grid, blk, 0, c->stream, d, parity);
    if (phase == 3) hipLaunchKernelGGL(rfast_sync_fold_kernel<4>, grid, blk, 0, c->stream, d);
  } else {
    if (phase == 0) hipLaunchKernelGGL((rfast_sync_step_kernel<1, 0>), grid, blk, 0, c->stream, d, parity);
    if (phase == 1) hipLaunchKernelGGL((rfast_sync_step_kernel<1, 1>), grid, blk, 0, c->stream, d, parity);
    if (phase == 2) hipLaunchKernelGGL((rfast_sync_step_kernel<1, 2>), grid, blk, 0, c->stream, d, parity);
    if (phase == 3) hipLaunchKernelGGL(rfast_sync_fold_kernel<1>, grid, blk, 0, c->stream, d);
  }
  return hipGetLastError();
}

// the integer side of `rounds` synchronous steps taken by one launch of the multi-step kernel
hipError_t rfast_launch_sync_plan(rfast_ctx* c, int rounds) {
  hipLaunchKernelGGL(rfast_sync_plan_kernel, dim3(1), dim3(256), 0, c->stream, c->d, rounds);
  return hipGetLastError();
}

hipError_t rfast_launch_rebase(rfast_ctx* c) {
  const RfastDev& d = c->d;
  const bool vec4 = (d.p % 4) == 0;
  const int64_t per_block = (int64_t)kThreads * (vec4 ? 4 : 1);
  const unsigned gx = (unsigned)((d.p + per_block - 1) / per_block);
  if (vec4)
    hipLaunchKernelGGL(rfast_rebase_kernel<4>, dim3(gx, d.n), dim3(kThreads), 0, c->stream, d);
  else
    hipLaunchKernelGGL(rfast_rebase_kernel<1>, dim3(gx, d.n), dim3(kThreads), 0, c->stream, d);
  return hipGetLastError();
}

hipError_t rfast_launch_state(rfast_ctx* c, int mode, float gamma) {
  const bool mom = c->d.mom != nullptr;
  // three or more in-edges per node on average (both graphs together): the deeper load batch
  const bool deep = (int64_t)c->d.eR + c->d.eC >= 3 * (int64_t)c->d.n;
  switch (mode) {
    case RFAST_MODE_FUSED:
      if (deep) return mom ? launch<RFAST_MODE_FUSED, true, 8>(c, gamma) : launch<RFAST_MODE_FUSED, false, 8>(c, gamma);
      return mom ? launch<RFAST_MODE_FUSED, true, 4>(c, gamma) : launch<RFAST_MODE_FUSED, false, 4>(c, gamma);
    case RFAST_MODE_MIX:
      if (deep) return mom ? launch<RFAST_MODE_MIX, true, 8>(c, gamma) : launch<RFAST_MODE_MIX, false, 8>(c, gamma);
      return mom ? launch<RFAST_MODE_MIX, true, 4>(c, gamma) : launch<RFAST_MODE_MIX, false, 4>(c, gamma);
    default:  // S1 is not part of this pass
      return deep ? launch<RFAST_MODE_TRACK, false, 8>(c, gamma) : launch<RFAST_MODE_TRACK, false, 4>(c, gamma);
  }
}
