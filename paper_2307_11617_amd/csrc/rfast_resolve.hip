// Integer schedule resolver: turns one round's masks into ring-slot indices.
//
// For an active receiver i and in-edge e = (j -> i) the stamp picked up is
// "the largest local iteration stamp received" (Algorithm 1, S2a / S2b): the
// newest version of j that (a) j had published before round r - delay_e and
// (b) was not lost on e, and never older than the stamp already held.  Losses
// are decided when a version is sent (experiments section: a node either sends
// its new packet or discards it).  After burst-1 consecutive losses on an edge
// the next version is delivered regardless, which keeps every read within D
// versions of the sender's counter (Assumption 3 ii).
//
// One workgroup; every step is integer and deterministic.
#include "rfast_internal.h"

namespace {

__device__ inline bool delivered(unsigned long long bits, int v, int M) {
  return v <= 0 || ((bits >> (v % M)) & 1ull);
}

__device__ inline void record_error(int32_t* err, int code, int round, int kind, int e) {
  if (atomicCAS(&err[0], 0, code) == 0) {
    err[1] = round;
    err[2] = kind;
    err[3] = e;
  }
}

// kind 0: graph R (v packets), kind 1: graph C (rho packets)
__device__ void resolve_edges(const RfastDev& s, int kind, int r, const uint8_t* active,
                              const int32_t* delay, const uint8_t* drop) {
  const int32_t* ptr = kind ? s.c_ptr : s.r_ptr;
  const int32_t* src = kind ? s.c_src : s.r_src;
  int32_t* tau = kind ? s.tau_c : s.tau_r;
  int32_t* slot = kind ? s.slot_c : s.slot_r;
  unsigned long long* deliv = kind ? s.deliv_c : s.deliv_r;
  for (int i = threadIdx.x; i < s.n; i += blockDim.x) {
    const bool recv_active = active[i] != 0;
    for (int e = ptr[i]; e < ptr[i + 1]; ++e) {
      const int j = src[e];
      unsigned long long bits = deliv[e];
      if (recv_active) {
        int d = delay[e];
        if (d < 0 || d > s.d_max) {
          record_error(s.err, RFAST_ERANGE, r, kind, e);
          d = d < 0 ? 0 : s.d_max;
        }
        const int at = r - d;
        int u = at <= 0 ? 0 : s.t_hist[(size_t)j * s.H + (at % s.H)];
        while (!delivered(bits, u, s.M)) --u;  // at most burst-1 steps
        const int old = tau[e];
        const int now = u > old ? u : old;
        tau[e] = now;
        slot[e] = now % s.M;
        if (kind) s.skip_c[e] = (now == old);
      } else {
        slot[e] = -1;
        if (kind) s.skip_c[e] = 1;
      }
      if (active[j] != 0) {  // the sender publishes version t_j + 1 this round
        const int vn = s.plan_t[j] + 1;
        bool ok = drop[e] == 0;
        if (!ok) {
          bool all_lost = true;
          for (int k = 1; k < s.burst; ++k) all_lost = all_lost && !delivered(bits, vn - k, s.M);
          ok = all_lost;
        }
        const unsigned long long bit = 1ull << (vn % s.M);
        deliv[e] = ok ? (bits | bit) : (bits & ~bit);
      }
    }
  }
}

__global__ void __launch_bounds__(256) rfast_resolve_kernel(RfastDev s, const uint8_t* active,
                                                            const int32_t* delay_R, const int32_t* delay_C,
                                                            const uint8_t* drop_R, const uint8_t* drop_C) {
  __shared__ int cnt;
  const int r = *s.round_no;
  if (threadIdx.x == 0) cnt = 0;
  __syncthreads();
  for (int i = threadIdx.x; i < s.n; i += blockDim.x) {
    const int ti = s.t[i];
    s.plan_t[i] = ti;
    s.t_hist[(size_t)i * s.H + (r % s.H)] = ti;
  }
  __syncthreads();
  // ordered list of active nodes (thread 0; n is at most a few thousand)
  if (threadIdx.x == 0) {
    int c = 0;
    for (int i = 0; i < s.n; ++i)
      if (active[i] != 0) s.active_list[c++] = i;
    *s.n_active = c;
  }
  resolve_edges(s, 0, r, active, delay_R, drop_R);
  resolve_edges(s, 1, r, active, delay_C, drop_C);
  __syncthreads();
  for (int i = threadIdx.x; i < s.n; i += blockDim.x)
    if (active[i] != 0) s.t[i] = s.plan_t[i] + 1;
  if (threadIdx.x == 0) *s.round_no = r + 1;
}

}  // namespace

hipError_t rfast_launch_resolve(rfast_ctx* c, const uint8_t* active, const int32_t* delay_R,
                                const int32_t* delay_C, const uint8_t* drop_R, const uint8_t* drop_C) {
  hipLaunchKernelGGL(rfast_resolve_kernel, dim3(1), dim3(256), 0, c->stream, c->d, active, delay_R, delay_C,
                     drop_R, drop_C);
  return hipGetLastError();
}
