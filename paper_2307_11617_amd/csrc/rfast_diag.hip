// Diagnostics of the current state as wavefront reductions:
//   consensus error ||x - 1 xbar^T||^2 and optimality gap ||xbar - x*||^2 (the
//   quantities of Theorem 1 and the merit function of Theorem 2), ||z||^2, and
//   the residual of the tracking-conservation identity of Lemma 3,
//   sum_i z_i + sum_e (rho_e latest - rho~_e) - sum_i g_i  (zero in exact arithmetic).
// One lane owns four consecutive coordinates (one when p is not a multiple of four)
// and walks over the nodes once, then over the edges of C (coalesced along k, the arrays of the nodes read once);
// partial sums are kept in fp64, reduced across the 64 lanes with shuffles
// then across the workgroup through LDS, and added to the result with one fp64 atomic per workgroup.
#include "rfast_vec.h"

namespace {

constexpr int kThreads = 256;

__device__ inline double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

__global__ void rfast_diag_zero(double* out) {
  if (threadIdx.x < 8) out[threadIdx.x] = 0.0;
}

template <int VEC>
__device__ inline float comp(const typename V<VEC>::T& v, int u) { return reinterpret_cast<const float*>(&v)[u]; }

// VEC = 4: four coordinates per lane (float4 loads, one Philox call per node for the four);
// VEC = 1: p not a multiple of four.
template <int VEC>
__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(4))) rfast_diag_kernel(RfastDev s, const float* xstar, double* out) {
  using T = typename V<VEC>::T;
  constexpr int W = V<VEC>::W;
  const int64_t p = s.p;
  const bool separable = s.prob.kind == RFAST_OBJ_DIAG_QUADRATIC;
  const float* hp = (const float*)s.prob.data0;
  const float* cp = (const float*)s.prob.data1;
  double acc[7] = {0, 0, 0, 0, 0, 0, 0};
  for (int64_t k = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * W; k < p; k += (int64_t)gridDim.x * kThreads * W) {
    // One walk over the nodes, their arrays read once.  What needs the average xbar, which is known only after
    // the walk, is accumulated about a reference that is known from the start, node 0's own value:
    //   sum_i (x_i - xbar)^2 = sum_i d_i^2 - 2 dx sum_i d_i + n dx^2,       d_i = x_i - x_0, dx = xbar - x_0
    //   sum_i h_i (xbar - c_i)^2 = dc^2 sum_i h_i - 2 dc sum_i h_i f_i + sum_i h_i f_i^2,  f_i = c_i - c_0, dc = xbar - c_0
    // (differences of fp32 values, exact in fp64; whatever cancels in these sums is of the size of the spread of
    // the x_i, or of the c_i, not of the values themselves).
    double gs[W], flight[W], sd[W], sd2[W], sh[W], shf[W], shf2[W];  // flight: sum of the z_i, then what is on the edges too
    float x0[W], c0[W];
#pragma unroll
    for (int u = 0; u < W; ++u) {
      gs[u] = flight[u] = sd[u] = sd2[u] = sh[u] = shf[u] = shf2[u] = 0.0;
      x0[u] = c0[u] = 0.f;
    }
#pragma unroll 1
    for (int i = 0; i < s.n; ++i) {
      const size_t off = (size_t)i * p + k;
      const int ti = s.t[i];
      const T x = V<VEC>::ld(s.x + off), z = V<VEC>::ld(s.z + off);
      T h, c, g;
      if (separable) {
        // the separable objective keeps no sample in memory: it is a function of (x_i, t_i)
        h = V<VEC>::ld(hp + off);
        c = V<VEC>::ld(cp + off);
        g = diag_sample<VEC>(s, h, c, x, i, ti, k);
      } else {
        g = V<VEC>::ld(s.g + (size_t)(ti & 1) * s.n * p + off);
      }
#pragma unroll
      for (int u = 0; u < W; ++u) {
        const double zi = comp<VEC>(z, u);
        if (i == 0) x0[u] = comp<VEC>(x, u);
        const double d = (double)comp<VEC>(x, u) - (double)x0[u];
        sd[u] += d;
        sd2[u] += d * d;
        flight[u] += zi;
        acc[1] += zi * zi;
        gs[u] += comp<VEC>(g, u);
        if (separable) {
          const double hi = comp<VEC>(h, u);
          if (i == 0) c0[u] = comp<VEC>(c, u);
          const double f = (double)comp<VEC>(c, u) - (double)c0[u];
          sh[u] += hi;
          shf[u] += hi * f;
          shf2[u] += hi * f * f;
        }
      }
    }
#pragma unroll 2
    for (int e = 0; e < s.eC; ++e) {
      const int j = s.c_src[e];
      const int tj = s.t[j], tau = s.tau_c[e];
      const float a = s.c_w[e];
      const float* ring = s.sigma_ring + (size_t)j * s.M * p + k;
      const T latest = V<VEC>::ld(ring + (size_t)(tj % s.M) * p);
      // rho~ is read from the sender's ring while its version is still there (tau >= t_j - D)
      const bool in_ring = tau >= tj - (s.M - 2);
      const T last = V<VEC>::ld(in_ring ? ring + (size_t)(tau % s.M) * p : s.rho_tilde + (size_t)e * p + k);
#pragma unroll
      for (int u = 0; u < W; ++u) {
        const float rt = in_ring ? a * comp<VEC>(last, u) : comp<VEC>(last, u);
        flight[u] += (double)(a * comp<VEC>(latest, u)) - (double)rt;
      }
    }
    T xbar_f, xs_f;
    if (xstar) xs_f = V<VEC>::ld(xstar + k);
#pragma unroll
    for (int u = 0; u < W; ++u) {
      const double dx = sd[u] / s.n, xbar = (double)x0[u] + dx;
      reinterpret_cast<float*>(&xbar_f)[u] = (float)xbar;
      acc[6] += xbar * xbar;
      acc[0] += sd2[u] - 2.0 * dx * sd[u] + s.n * dx * dx;
      if (separable) {
        const double dc = xbar - (double)c0[u];
        acc[5] += 0.5 * (dc * dc * sh[u] - 2.0 * dc * shf[u] + shf2[u]);
      }
      const double res = flight[u] - gs[u];
      acc[2] += res * res;
      acc[3] += gs[u] * gs[u];
      if (xstar) acc[4] += (xbar - comp<VEC>(xs_f, u)) * (xbar - comp<VEC>(xs_f, u));
    }
    if (s.xbar) V<VEC>::st(s.xbar + k, xbar_f);  // staged for the loss kernels of the objectives that need it
  }
  // one fp64 atomic per quantity and workgroup: the seven results are single addresses, and
  // tens of thousands of atomics on them would serialise
  __shared__ double part[kThreads / 64][7];
#pragma unroll
  for (int q = 0; q < 7; ++q) {
    const double w = wave_sum(acc[q]);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6][q] = w;
  }
  __syncthreads();
  if (threadIdx.x < 7) {
    double w = 0.0;
    for (int v = 0; v < kThreads / 64; ++v) w += part[v][threadIdx.x];
    atomicAdd(&out[threadIdx.x], w);
  }
}

// sum_i f_i(xbar) for least squares and logistic regression over each node's FULL
// local data: one wavefront per row, a . xbar reduced across the 64 lanes.
__global__ void __launch_bounds__(kThreads) rfast_loss_rows_kernel(RfastDev s, double* out) {
  const int i = blockIdx.y;
  const int row = blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
  if (row >= s.prob.samples) return;
  const int lane = threadIdx.x & 63;
  const int64_t p = s.p;
  const float* a = (const float*)s.prob.data0 + ((size_t)i * s.prob.samples + row) * p;
  double acc = 0.0;
  for (int64_t k = lane; k < p; k += 64) acc += (double)a[k] * (double)s.xbar[k];
  acc = wave_sum(acc);
  if (lane == 0) {
    const double y = ((const float*)s.prob.data1)[(size_t)i * s.prob.samples + row];
    double l;
    if (s.prob.kind == RFAST_OBJ_LOGISTIC) l = (acc > 0 ? acc + log1p(exp(-acc)) : log1p(exp(acc))) - y * acc;
    else l = 0.5 * (acc - y) * (acc - y);
    atomicAdd(&out[5], l / s.prob.samples);
  }
}

// The six results in the order of rfast_diag, from the accumulators (what rfast_diagnostics does on the host).
__global__ void rfast_diag_finish(const double* acc, double l2_half_n, int has_xstar, double* out) {
  if (threadIdx.x == 0) {
    out[0] = acc[0];
    out[1] = acc[1];
    out[2] = acc[2];
    out[3] = acc[3];
    out[4] = has_xstar ? acc[4] : -1.0;
    out[5] = acc[5] + l2_half_n * acc[6];
  }
}

// Scratch of rfast_diagnostics_static, the entry point that allocates nothing: the fp64 accumulators of the
// reductions, then the node average xbar that the loss kernels of the non-separable objectives read.  One copy per
// GPU, held until the process ends; every call on a GPU shares it.
constexpr size_t kStaticAccBytes = 256;
constexpr int64_t kStaticMaxCoords = 1 << 20;
__device__ __align__(256) unsigned char scratch[kStaticAccBytes + kStaticMaxCoords * sizeof(float)];
constexpr int kMaxDevices = 64;
void* g_scratch[kMaxDevices] = {};  // device address of `scratch` on each GPU (the array's name is no device address in host code)

}  // namespace

// Looks up the address of the static scratch array on the current device, once per device.
hipError_t rfast_static_scratch_init() {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  if (g_scratch[dev]) return hipSuccess;
  void* ptr = nullptr;
  e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
  if (e != hipSuccess) return e;
  if (!ptr) return hipErrorInvalidSymbol;
  g_scratch[dev] = ptr;
  return hipSuccess;
}

int64_t rfast_static_max_coords() { return kStaticMaxCoords; }

// rfast_launch_diag with the accumulators and xbar in the static scratch of the current device, and the six
// results written to d_out (device) by a last small kernel.  The caller has checked the size.
hipError_t rfast_launch_diag_static(rfast_ctx* c, const float* d_xstar, double* d_out, double l2_half_n) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices || !g_scratch[dev]) return hipErrorNotInitialized;
  unsigned char* base = static_cast<unsigned char*>(g_scratch[dev]);
  double* acc = reinterpret_cast<double*>(base);
  float* keep = c->d.xbar;
  c->d.xbar = c->d.prob.kind == RFAST_OBJ_DIAG_QUADRATIC ? nullptr : reinterpret_cast<float*>(base + kStaticAccBytes);
  e = rfast_launch_diag(c, d_xstar, acc);  // clears the accumulators with a kernel first
  c->d.xbar = keep;
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(rfast_diag_finish, dim3(1), dim3(64), 0, c->stream, acc, l2_half_n, d_xstar ? 1 : 0, d_out);
  return hipGetLastError();
}

hipError_t rfast_launch_diag(rfast_ctx* c, const float* d_xstar, double* d_out) {
  hipLaunchKernelGGL(rfast_diag_zero, dim3(1), dim3(64), 0, c->stream, d_out);
  const bool vec4 = (c->d.p % 4) == 0 && ((uintptr_t)d_xstar % 16) == 0;
  const int64_t per_block = (int64_t)kThreads * (vec4 ? 4 : 1);
  int64_t blocks = (c->d.p + per_block - 1) / per_block;
  if (blocks > 2048) blocks = 2048;  // grid-stride beyond that: 8 workgroups per CU
  const bool streaming = (double)c->d.n * (double)c->d.p * 4.0 >= 32.0e6;  // far beyond the caches: non-temporal loads
  if (vec4 && streaming)
    hipLaunchKernelGGL(rfast_diag_kernel<-4>, dim3((unsigned)blocks), dim3(kThreads), 0, c->stream, c->d, d_xstar, d_out);
  else if (vec4)
    hipLaunchKernelGGL(rfast_diag_kernel<4>, dim3((unsigned)blocks), dim3(kThreads), 0, c->stream, c->d, d_xstar, d_out);
  else
    hipLaunchKernelGGL(rfast_diag_kernel<1>, dim3((unsigned)blocks), dim3(kThreads), 0, c->stream, c->d, d_xstar, d_out);
  const int kind = c->d.prob.kind;
  if (kind == RFAST_OBJ_LEAST_SQUARES || kind == RFAST_OBJ_LOGISTIC)
    hipLaunchKernelGGL(rfast_loss_rows_kernel, dim3((c->d.prob.samples + 3) / 4, c->d.n), dim3(kThreads), 0, c->stream, c->d,
                       d_out);
  if (kind == RFAST_OBJ_SOFTMAX_BF16) {
    const hipError_t e = rfast_softmax_loss(c, d_out + 5);
    if (e != hipSuccess) return e;
  }
  return hipGetLastError();
}
