// Vector access helpers and the counter-based Gaussian noise of the separable
// objective, shared by the state-update and the diagnostics kernels (gfx950 only).
#pragma once
#include "rfast_internal.h"
#include "rfast_philox.h"

// ------------------------------------------------------------ vector helpers
// VEC = 4: float4 per lane.  VEC = -4: the same with non-temporal (streaming)
// loads and stores, used when the state is far larger than the caches, so
// that lines with no reuse do not displace anything.  VEC = 1: scalar, p % 4 != 0.
typedef float nt_f4 __attribute__((ext_vector_type(4)));
template <int VEC> struct V;
template <> struct V<4> {
  using T = float4;
  static constexpr int W = 4;
  static __device__ inline T ld(const float* p) { return *reinterpret_cast<const float4*>(p); }
  static __device__ inline void st(float* p, T v) { *reinterpret_cast<float4*>(p) = v; }
};
template <> struct V<-4> {
  using T = float4;
  static constexpr int W = 4;
  static __device__ inline T ld(const float* p) {
    const nt_f4 t = __builtin_nontemporal_load(reinterpret_cast<const nt_f4*>(p));
    return make_float4(t.x, t.y, t.z, t.w);
  }
  static __device__ inline void st(float* p, T v) {
    const nt_f4 t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, reinterpret_cast<nt_f4*>(p));
  }
};
template <> struct V<1> {
  using T = float;
  static constexpr int W = 1;
  static __device__ inline T ld(const float* p) { return *p; }
  static __device__ inline void st(float* p, T v) { *p = v; }
};
__device__ inline float4 fma_s(float a, float4 b, float4 c) {
  return make_float4(fmaf(a, b.x, c.x), fmaf(a, b.y, c.y), fmaf(a, b.z, c.z), fmaf(a, b.w, c.w));
}
__device__ inline float fma_s(float a, float b, float c) { return fmaf(a, b, c); }
__device__ inline float4 mul_s(float a, float4 b) { return make_float4(a * b.x, a * b.y, a * b.z, a * b.w); }
__device__ inline float mul_s(float a, float b) { return a * b; }
__device__ inline float4 add(float4 a, float4 b) { return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w); }
__device__ inline float add(float a, float b) { return a + b; }
__device__ inline float4 sub(float4 a, float4 b) { return make_float4(a.x - b.x, a.y - b.y, a.z - b.z, a.w - b.w); }
__device__ inline float sub(float a, float b) { return a - b; }
__device__ inline float4 mul(float4 a, float4 b) { return make_float4(a.x * b.x, a.y * b.y, a.z * b.z, a.w * b.w); }
__device__ inline float mul(float a, float b) { return a * b; }

// S2b for one in-edge of C: z + rho - rho~ with rho = a sigma_j[tau].  While the buffer is still the
// sender's running sum of the version consumed last time (from_ring), rho - rho~ equals
// a (sigma_j[tau] - sigma_j[tau_prev]): the difference is taken first, so that its rounding error
// does not grow with the running sum; a buffer from the rho~ array is already the product.
template <class T> __device__ inline T track_edge(T z, float a, T cur, T last, bool from_ring) {
  if (from_ring) return fma_s(a, sub(cur, last), z);
  return add(z, sub(mul_s(a, cur), last));
}

// ------------------------------------------------- counter-based Gaussian noise
// sin and cos of 2*pi*w/2^32 with the hardware instructions, which take their argument in turns:
// w is read as a signed fraction of a turn in [-1/2, 1/2).  Measured over 2^24 angles against
// double precision the absolute error of either is below 1.9e-7 (most of it the rounding of w to
// a float), two units in the last place of a value near one.
__device__ inline void sincos_turns(uint32_t w, float* s, float* c) {
  const float t = (float)(int32_t)w * (1.0f / 4294967296.0f);
  *s = __builtin_amdgcn_sinf(t);
  *c = __builtin_amdgcn_cosf(t);
}

// Box-Muller on two Philox words, in polar form: radius scale * sqrt(-2 ln u) and the sine and cosine of the
// angle, so that the caller adds radius * cos and radius * sin to its sums with one multiply-add each.
// scale2 = scale * sqrt(2 ln 2): -2 ln u = (2 ln 2)(-log2 u), and the negation is the square root's source
// modifier.
__device__ inline void box_muller_polar(uint32_t ou, uint32_t oa, float scale2, float* r, float* s, float* c) {
  // (m + 1) 2^-24 for the 24-bit m, as one exact multiply-add (no rounding: the result has 25 bits at most
  // only for m + 1 = 2^24, a power of two)
  const float u = fmaf((float)(ou >> 8), 1.0f / 16777216.0f, 1.0f / 16777216.0f);
  // u lies in [2^-24, 1]: no denormal, zero or negative argument, so the hardware log2 and square
  // root (1 ulp each) serve without the range fix-ups of the library routines
  *r = scale2 * __builtin_amdgcn_sqrtf(-__builtin_amdgcn_logf(u));
  sincos_turns(oa, s, c);
}

// g + scale * (four normals of coordinate group q)
__device__ inline float4 add_noise4(float4 g, float scale, uint64_t seed, uint32_t node, uint32_t version, uint64_t q) {
  uint32_t o[4];
  rfast_philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), node, version, (uint32_t)seed, (uint32_t)(seed >> 32), o);
  const float scale2 = scale * 1.17741002251547469f;  // sqrt(2 ln 2)
  float r0, s0, c0, r1, s1, c1;
  box_muller_polar(o[0], o[1], scale2, &r0, &s0, &c0);
  box_muller_polar(o[2], o[3], scale2, &r1, &s1, &c1);
  return make_float4(fmaf(r0, c0, g.x), fmaf(r0, s0, g.y), fmaf(r1, c1, g.z), fmaf(r1, s1, g.w));
}
template <int VEC>
__device__ inline typename V<VEC>::T add_noise(typename V<VEC>::T g, float scale, uint64_t seed, uint32_t node, uint32_t ver, int64_t k);
template <> __device__ inline float4 add_noise<4>(float4 g, float scale, uint64_t seed, uint32_t node, uint32_t ver, int64_t k) {
  return add_noise4(g, scale, seed, node, ver, (uint64_t)k >> 2);
}
template <> __device__ inline float4 add_noise<-4>(float4 g, float scale, uint64_t seed, uint32_t node, uint32_t ver, int64_t k) {
  return add_noise4(g, scale, seed, node, ver, (uint64_t)k >> 2);
}
// one coordinate: the same instructions on its group of four, so that it gets the very bits the vector form gives it
template <> __device__ inline float add_noise<1>(float g, float scale, uint64_t seed, uint32_t node, uint32_t ver, int64_t k) {
  const int l = (int)(k & 3);
  const float4 g4 = make_float4(g, g, g, g);
  const float4 z = add_noise4(g4, scale, seed, node, ver, (uint64_t)k >> 2);
  return l == 0 ? z.x : l == 1 ? z.y : l == 2 ? z.z : z.w;
}


// fp32 -> bf16 bits, round to nearest even (the rounding both softmax GEMM operands get)
__device__ inline unsigned short rfast_f32_to_bf16(float f) {
  const uint32_t u = __float_as_uint(f);
  return (unsigned short)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

// ------------------------------------------- sample of the diagonal quadratic
// grad f_i(x; zeta^version) = h (x - c) + noise_std * N(0, I)[node, version] (+ weight decay * x).
// A pure function of (x, node, version): the "stored" sample of step S2b is recomputed
// from the node's own x and counter wherever it is needed, with these very
// instructions, instead of being written to and read back from memory.
// (WD = false: the caller knows that there is no weight decay, and the test goes away)
template <int VEC, bool WD = true>
__device__ inline typename V<VEC>::T diag_sample(const RfastDev& s, typename V<VEC>::T h, typename V<VEC>::T c,
                                                 typename V<VEC>::T x, int node, int version, int64_t k) {
  typename V<VEC>::T g = mul(h, sub(x, c));
  if (s.prob.noise_std != 0.0f)
    g = add_noise<VEC>(g, s.prob.noise_std, s.prob.noise_seed, (uint32_t)node, (uint32_t)version, k);
  if (WD && s.wd != 0.0f) g = fma_s(s.wd, x, g);  // weight decay is part of the sampled gradient
  return g;
}
