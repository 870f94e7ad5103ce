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
#include "rfast_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

__device__ inline int sample_row(const RfastDev& s, const int32_t* batch_idx, int i, int b, int B) {
  if (batch_idx == nullptr) return b;
  int row = batch_idx[(size_t)i * B + b];
  if (row < 0 || row >= s.prob.samples) {
    if (atomicCAS(&s.err[0], 0, RFAST_ERANGE) == 0) {
      s.err[1] = s.n_active[1];  // the round counter as this round's plan recorded it
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

__global__ void __launch_bounds__(kThreads) rfast_rows_kernel(RfastDev s, const int32_t* batch_idx, int B, bool init) {
  int t_unused;
  const int i = pick_node(s, init, &t_unused);
  if (i < 0) return;
  const int b = blockIdx.x * kWaves + (threadIdx.x >> 6);
  if (b >= B) return;
  const int lane = threadIdx.x & 63;
  const int64_t p = s.p;
  const int row = sample_row(s, batch_idx, i, b, B);
  const float* a = (const float*)s.prob.data0 + ((size_t)i * s.prob.samples + row) * p;
  const float* x = s.x + (size_t)i * p;
  float acc = 0.f;
  if ((p & 3) == 0) {
    // four 1 KiB pieces of the row per step, all eight loads issued before the first use:
    // one wavefront per row has nothing else to hide the memory latency with
    int64_t k = (int64_t)lane * 4;
    for (; k + 768 < p; k += 1024) {
      float4 av[4], xv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        av[u] = *reinterpret_cast<const float4*>(a + k + 256 * u);
        xv[u] = *reinterpret_cast<const float4*>(x + k + 256 * u);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        acc = fmaf(av[u].x, xv[u].x, acc);
        acc = fmaf(av[u].y, xv[u].y, acc);
        acc = fmaf(av[u].z, xv[u].z, acc);
        acc = fmaf(av[u].w, xv[u].w, acc);
      }
    }
    for (; k < p; k += 256) {
      const float4 av = *reinterpret_cast<const float4*>(a + k);
      const float4 xv = *reinterpret_cast<const float4*>(x + k);
      acc = fmaf(av.x, xv.x, acc);
      acc = fmaf(av.y, xv.y, acc);
      acc = fmaf(av.z, xv.z, acc);
      acc = fmaf(av.w, xv.w, acc);
    }
  } else {
    for (int64_t k = lane; k < p; k += 64) acc = fmaf(a[k], x[k], acc);
  }
  acc = wave_sum(acc);
  if (lane == 0) {
    const float y = ((const float*)s.prob.data1)[(size_t)i * s.prob.samples + row];
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

// initial gradient of the diagonal quadratic (sample version 0) and z^0 = g^0
__global__ void __launch_bounds__(kThreads) rfast_copy_z_kernel(RfastDev s) {
  const size_t tot = (size_t)s.n * s.p;
  for (size_t q = (size_t)blockIdx.x * kThreads + threadIdx.x; q < tot; q += (size_t)gridDim.x * kThreads) s.z[q] = s.g[q];
}

hipError_t gemv_pair(rfast_ctx* c, const int32_t* batch_idx, bool init) {
  const RfastDev& d = c->d;
  const int B = d.prob.batch > 0 ? d.prob.batch : d.prob.samples;
  const int32_t* bi = d.prob.batch > 0 ? batch_idx : nullptr;
  hipLaunchKernelGGL(rfast_rows_kernel, dim3((B + kWaves - 1) / kWaves, d.n), dim3(kThreads), 0, c->stream, d, bi, B, init);
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
