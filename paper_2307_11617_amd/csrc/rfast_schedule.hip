// On-device schedule generation: the asynchrony of one round (Assumption 3 of the
// paper: which nodes are active, how stale each edge is, which packets are lost,
// which rows are sampled) as a pure function of (seed, round), so that long runs
// need no schedule upload.
//
//   word(stream, r, e) = Philox4x32-10(counter = (e div 4, stream, r, 0), key = seed)[e mod 4]
//   active[i]  = word(0, r, i) < floor(p_active[i] * 2^32)
//                event-driven mode (Algorithm 2: one agent i^k per global iteration k = r):
//                u = word(6, r, 0); active[i] = cdf[i-1] <= u < cdf[i]  (cdf[-1] = 0, the last
//                threshold closed at 2^32 - 1), cdf = 32-bit cumulative selection thresholds
//   delay_R[e] = word(1, r, e) mod (d_max + 1)          delay_C[e]: stream 2
//   drop_R[e]  = word(3, r, e) < floor(p_drop * 2^32)     drop_C[e]: stream 4
//   rows of node i: perm(b), b = 0..B-1; perm = 4-round balanced Feistel network on
//   2h bits (h = ceil(bits/2), bits = bit length of samples-1, at least 1) with
//   cycle walking back into [0, samples), round keys = Philox(counter = (i, 5, r, 0)).
//   Round function on the h-bit half R with key K:
//     t = R * 0x9E3779B1 + K;  t ^= t >> 15;  t *= 0x85EBCA77;  F = t >> (32 - h)   (mod 2^32)
#include "rfast_internal.h"
#include "rfast_philox.h"

namespace {

__device__ inline uint32_t word(uint64_t seed, uint32_t stream, uint32_t r, uint32_t e) {
  uint32_t o[4];
  rfast_philox4x32_10(e >> 2, stream, r, 0u, (uint32_t)seed, (uint32_t)(seed >> 32), o);
  return o[e & 3u];
}

__device__ inline unsigned long long threshold(float prob) {
  return (unsigned long long)floor((double)prob * 4294967296.0);
}

// blockIdx.y: the round, counted from the current one; its arrays follow those of the round before
// (the layout rfast_run takes uploaded schedules in)
__global__ void __launch_bounds__(256) rfast_generate_kernel(RfastDev s, uint64_t seed, const float* p_active, int d_max,
                                                             float p_drop, int B, bool events) {
  const uint32_t r = (uint32_t)*s.round_no + blockIdx.y;
  const size_t y = blockIdx.y;
  s.gen_active += y * s.n;
  s.gen_delay_r += y * s.eR;
  s.gen_delay_c += y * s.eC;
  s.gen_drop_r += y * s.eR;
  s.gen_drop_c += y * s.eC;
  s.gen_batch += y * s.n * B;
  int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (q < s.n) {
    if (events) {
      const uint32_t u = word(seed, 6u, r, 0u);
      const uint32_t lo = q ? s.gen_cdf[q - 1] : 0u, hi = s.gen_cdf[q];
      s.gen_active[q] = u >= lo && (u < hi || (q == s.n - 1 && hi > lo));
    } else {
      s.gen_active[q] = (unsigned long long)word(seed, 0u, r, (uint32_t)q) < threshold(p_active[q]);
    }
    return;
  }
  q -= s.n;
  if (q < s.eR) { s.gen_delay_r[q] = (int32_t)(word(seed, 1u, r, (uint32_t)q) % (uint32_t)(d_max + 1)); return; }
  q -= s.eR;
  if (q < s.eC) { s.gen_delay_c[q] = (int32_t)(word(seed, 2u, r, (uint32_t)q) % (uint32_t)(d_max + 1)); return; }
  q -= s.eC;
  if (q < s.eR) { s.gen_drop_r[q] = (unsigned long long)word(seed, 3u, r, (uint32_t)q) < threshold(p_drop); return; }
  q -= s.eR;
  if (q < s.eC) { s.gen_drop_c[q] = (unsigned long long)word(seed, 4u, r, (uint32_t)q) < threshold(p_drop); return; }
  q -= s.eC;
  if (q < (int64_t)s.n * B) {
    const uint32_t node = (uint32_t)(q / B), b = (uint32_t)(q % B);
    const uint32_t samples = (uint32_t)s.prob.samples;
    uint32_t key[4];
    rfast_philox4x32_10(node, 5u, r, 0u, (uint32_t)seed, (uint32_t)(seed >> 32), key);
    int bits = 32 - __clz((int)(samples - 1));
    if (bits < 1) bits = 1;
    const int h = (bits + 1) / 2;
    const uint32_t mask = (1u << h) - 1u;
    uint32_t x = b;
    do {  // cycle walking: b < samples lies on a cycle that re-enters [0, samples)
      uint32_t L = (x >> h) & mask, R = x & mask;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        uint32_t t = R * 0x9E3779B1u + key[j];
        t ^= t >> 15;
        t *= 0x85EBCA77u;
        const uint32_t F = t >> (32 - h);
        const uint32_t nl = R;
        R = L ^ F;
        L = nl;
      }
      x = (L << h) | R;
    } while (x >= samples);
    s.gen_batch[q] = (int32_t)x;
  }
}

}  // namespace

hipError_t rfast_launch_generate(rfast_ctx* c, uint64_t seed, const float* d_p_active, int d_max, float p_drop, bool events,
                                 int rounds) {
  const RfastDev& d = c->d;
  const int B = d.prob.kind == RFAST_OBJ_DIAG_QUADRATIC ? 0 : d.prob.batch;
  const int64_t total = (int64_t)d.n + 2 * (int64_t)d.eR + 2 * (int64_t)d.eC + (int64_t)d.n * B;
  if (rounds < 1 || rounds > c->gen_depth || rounds > 65535) return hipErrorInvalidValue;
  hipLaunchKernelGGL(rfast_generate_kernel, dim3((unsigned)((total + 255) / 256), (unsigned)rounds), dim3(256), 0, c->stream, d,
                     seed, d_p_active, d_max, p_drop, B, events);
  return hipGetLastError();
}
