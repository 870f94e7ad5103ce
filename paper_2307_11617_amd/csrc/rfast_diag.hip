// Diagnostics of the current state as wavefront reductions:
//   consensus error ||x - 1 xbar^T||^2 and optimality gap ||xbar - x*||^2 (the
//   quantities of Theorem 1 and the merit function of Theorem 2), ||z||^2, and
//   the residual of the tracking-conservation identity of Lemma 3,
//   sum_i z_i + sum_e (rho_e latest - rho~_e) - sum_i g_i  (zero in exact arithmetic).
// One lane owns one coordinate and walks over nodes and edges (coalesced along
// k); partial sums are kept in fp64, reduced across the 64 lanes with shuffles
// and added to the result with one fp64 atomic per wavefront.
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

__global__ void __launch_bounds__(kThreads) rfast_diag_kernel(RfastDev s, const float* xstar, double* out) {
  const int64_t p = s.p;
  double acc[7] = {0, 0, 0, 0, 0, 0, 0};
  for (int64_t k = (int64_t)blockIdx.x * kThreads + threadIdx.x; k < p; k += (int64_t)gridDim.x * kThreads) {
    double xs = 0.0, zs = 0.0, gs = 0.0;
    for (int i = 0; i < s.n; ++i) {
      const size_t off = (size_t)i * p + k;
      const double zi = s.z[off];
      xs += s.x[off];
      zs += zi;
      acc[1] += zi * zi;
      if (s.prob.kind == RFAST_OBJ_DIAG_QUADRATIC)  // the sample is a function of (x_i, t_i), not kept in memory
        gs += diag_sample<1>(s, ((const float*)s.prob.data0)[off], ((const float*)s.prob.data1)[off], s.x[off], i, s.t[i], k);
      else
        gs += s.g[(size_t)(s.t[i] & 1) * s.n * p + off];
    }
    const double xbar = xs / s.n;
    s.xbar[k] = (float)xbar;
    acc[6] += xbar * xbar;
    double loss = 0.0;
    for (int i = 0; i < s.n; ++i) {
      const size_t off = (size_t)i * p + k;
      const double dx = (double)s.x[off] - xbar;
      acc[0] += dx * dx;
      if (s.prob.kind == RFAST_OBJ_DIAG_QUADRATIC) {
        const double h = ((const float*)s.prob.data0)[off], c = ((const float*)s.prob.data1)[off];
        loss += 0.5 * h * (xbar - c) * (xbar - c);
      }
    }
    double flight = 0.0;
    for (int e = 0; e < s.eC; ++e) {
      const int j = s.c_src[e];
      // rho~ is read from the sender's ring while its version is still there (tau >= t_j - D)
      const int tau = s.tau_c[e];
      const float rt = tau >= s.t[j] - (s.M - 2) ? s.c_w[e] * s.sigma_ring[((size_t)j * s.M + (tau % s.M)) * p + k]
                                                 : s.rho_tilde[(size_t)e * p + k];
      flight += (double)(s.c_w[e] * s.sigma_ring[((size_t)j * s.M + (s.t[j] % s.M)) * p + k]) - (double)rt;
    }
    const double res = zs + flight - gs;
    acc[2] += res * res;
    acc[3] += gs * gs;
    if (xstar) acc[4] += (xbar - xstar[k]) * (xbar - xstar[k]);
    acc[5] += loss;
  }
#pragma unroll
  for (int q = 0; q < 7; ++q) {
    const double w = wave_sum(acc[q]);
    if ((threadIdx.x & 63) == 0) atomicAdd(&out[q], w);
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

}  // namespace

hipError_t rfast_launch_diag(rfast_ctx* c, const float* d_xstar, double* d_out) {
  hipLaunchKernelGGL(rfast_diag_zero, dim3(1), dim3(64), 0, c->stream, d_out);
  int64_t blocks = (c->d.p + kThreads - 1) / kThreads;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(rfast_diag_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, c->stream, c->d, d_xstar, d_out);
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
