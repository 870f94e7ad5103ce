// Softmax-regression minibatch gradient on the matrix cores (step S2b of
// Algorithm 1 needs grad f_i at the freshly mixed x_i; this is the only dense
// contraction on the path, so it is the only place MFMA is used).
//
// x_i is W (d x K, row-major).  With Xb the B sampled rows of the node's bf16
// pool:   logits = Xb * bf16(W)            (B x K, contraction over d)
//         E      = bf16((softmax(logits) - onehot) / B)
//         G      = Xb^T * E                (d x K, contraction over B)
// bf16 x bf16 products accumulate in fp32 (v_mfma_f32_32x32x16_bf16).  Both
// MFMA operands want 8 consecutive elements of the contraction index per lane,
// so three small kernels keep every operand contiguous along it:
//   prep      Wt[f/8][k][f%8] = bf16(W[f][k])      (transpose through LDS; blocks of 8
//             features so that a stage of 64 features is one contiguous 16 KiB run)
//   forward   tile of 64 sampled rows x all K classes: X rows and Wt blocks are
//             both contiguous in f; row softmax in the same block; E is written
//             class-major, Et[k][b]
//   backward  tile of 64 features x all K classes: Et rows are contiguous in b;
//             the X tile is transposed while it is staged into LDS
// Operand layout of the 32x32x16 instruction (lane l of 64):
//   A: row l%32, contraction indices 8*(l/32) .. +7      (8 bf16)
//   B: column l%32, contraction indices 8*(l/32) .. +7   (8 bf16)
//   C/D: column l%32, rows 8*(v/4) + 4*(l/32) + v%4 for v = 0..15
#include "rfast_vec.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned short u16;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));  // plain vector type: stays in registers

constexpr int kTile = 64;       // rows (forward) / features (backward) per block, and staging depth
constexpr int kPad = 8;         // LDS row padding in bf16 elements (16 bytes)
constexpr int kLd = kTile + kPad;

__device__ inline u16 f32_to_bf16(float f) { return rfast_f32_to_bf16(f); }

// node handled by work slot `slot` and the stamp of its stored sample (-1 while the initial gradient
// is formed): all nodes at initialisation, the round's work slots otherwise (slot < n + 8: the
// XCD-aware ids pad the slot count to a multiple of 8, and the slot array carries 8 spare entries)
__device__ inline int pick_node(const RfastDev& s, bool init, int slot, int* t_old) {
  *t_old = -1;
  if (init) return slot < s.n ? slot : -1;
  const int2 ap = s.active_plan[slot];
  *t_old = ap.y;
  return ap.x;
}

// Workgroups are dealt to the 8 XCDs round-robin by linear id.  The `per_node`
// workgroups of one node share that node's W (forward) or E (backward), so they
// are decoded onto one XCD and hit in its L2: id -> (node slot, part).
__device__ inline void xcd_decode(int per_node, int* slot, int* part) {
  const int L = blockIdx.x;
  const int xcd = L & 7, q = L >> 3;
  *slot = (q / per_node) * 8 + xcd;
  *part = q % per_node;
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

struct Scratch {
  u16* wt;  // [n][K][d]
  u16* et;  // [n][K][B]
};
__device__ __host__ inline Scratch scratch_of(const RfastDev& s, int B) {
  Scratch r;
  r.wt = (u16*)s.gscratch;
  r.et = r.wt + (size_t)s.n * s.prob.K * s.prob.d;
  return r;
}

// ---------------------------------------------------------------- prep: Wt = bf16(W), blocked transpose
// grid (d/64, nodes).  LDS tile T[f][k] (row stride K+4: the transposed reads of
// phase 2 then fall on distinct banks); phase 2 gathers 8 features of one class
// and writes them as one 16-byte unit, lanes along k, fully coalesced.
// wsrc != NULL: convert that matrix (the node average, for the loss) into node slot 0.
__global__ void __launch_bounds__(256) rfast_softmax_prep(RfastDev s, int B, bool init, const float* wsrc) {
  extern __shared__ u16 lds[];  // [64][K+4]
  int t_unused;
  const int i = pick_node(s, init, blockIdx.y, &t_unused);
  if (i < 0) return;
  const int d = s.prob.d, K = s.prob.K, TS = K + 4;
  const int f0 = blockIdx.x * kTile;
  const float* W = wsrc ? wsrc : s.x + (size_t)i * s.p;
  for (int q = threadIdx.x; q < kTile * K / 4; q += blockDim.x) {
    const int f = q / (K / 4), k4 = (q % (K / 4)) * 4;
    const float4 w = *reinterpret_cast<const float4*>(W + (size_t)(f0 + f) * K + k4);
    uint2 pk;
    pk.x = f32_to_bf16(w.x) | ((uint32_t)f32_to_bf16(w.y) << 16);
    pk.y = f32_to_bf16(w.z) | ((uint32_t)f32_to_bf16(w.w) << 16);
    *reinterpret_cast<uint2*>(&lds[f * TS + k4]) = pk;
  }
  __syncthreads();
  u16* wt = scratch_of(s, B).wt + (size_t)i * K * d + (size_t)(f0 / 8) * K * 8;
  for (int q = threadIdx.x; q < K * 8; q += blockDim.x) {
    const int k = q % K, c = q / K;
    u16 h[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) h[j] = lds[(c * 8 + j) * TS + k];
    uint4 pk;
    pk.x = h[0] | ((uint32_t)h[1] << 16);
    pk.y = h[2] | ((uint32_t)h[3] << 16);
    pk.z = h[4] | ((uint32_t)h[5] << 16);
    pk.w = h[6] | ((uint32_t)h[7] << 16);
    *reinterpret_cast<uint4*>(wt + ((size_t)c * K + k) * 8) = pk;
  }
}

// ------------------------------------------------------------------------- forward
// one workgroup per (node, 64-row block), XCD-aware ids; NW = K/32 wavefronts: wave w owns classes 32w .. 32w+31.
// The contraction over d runs in stages of 64 features through two LDS buffers;
// the global loads of the next two stages are already in flight (in registers)
// while the current one is multiplied, because with one or two workgroups per
// CU a single outstanding stage cannot cover the memory latency.
template <int NW>
struct FwdShape {
  static constexpr int kThreads = 64 * NW;
  static constexpr int kXc = (kTile * kTile / 8 + kThreads - 1) / kThreads;  // 16-byte chunks of the X tile per lane
  static constexpr int kWc = 4;                                              // ... of the Wt tile per lane
  static constexpr int kGs = 32 * NW * 8 + 8;  // LDS stride of one 8-feature block of Wt (K*8 + 16 bytes of pad)
  static constexpr int kBuf = kTile * kLd + 8 * kGs;  // one staging buffer: X tile, then 8 blocks of Wt
};

template <int NW>
__device__ __forceinline__ void fwd_load(u32x4 (&x)[FwdShape<NW>::kXc], u32x4 (&w)[4], const u16* pool, const int* rows,
                                         const u16* wt, int d, int f0, int tid) {
  constexpr int T = FwdShape<NW>::kThreads;
#pragma unroll
  for (int c = 0; c < FwdShape<NW>::kXc; ++c) {
    const int q = tid + c * T;
    if ((kTile * kTile / 8) % T == 0 || q < kTile * kTile / 8)
      x[c] = *reinterpret_cast<const u32x4*>(pool + (size_t)rows[q / (kTile / 8)] * d + f0 + (q % (kTile / 8)) * 8);
  }
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const int q = tid + c * T;
    w[c] = *reinterpret_cast<const u32x4*>(wt + (size_t)(f0 / 8) * (32 * NW * 8) + (size_t)q * 8);  // contiguous run
  }
}

template <int NW>
__device__ __forceinline__ void fwd_store(const u32x4 (&x)[FwdShape<NW>::kXc], const u32x4 (&w)[4], u16* Xs, u16* Ws,
                                          int tid) {
  constexpr int T = FwdShape<NW>::kThreads;
#pragma unroll
  for (int c = 0; c < FwdShape<NW>::kXc; ++c) {
    const int q = tid + c * T;
    if ((kTile * kTile / 8) % T == 0 || q < kTile * kTile / 8)
      *reinterpret_cast<u32x4*>(&Xs[(q / (kTile / 8)) * kLd + (q % (kTile / 8)) * 8]) = x[c];
  }
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const int q = tid + c * T;
    *reinterpret_cast<u32x4*>(&Ws[(q / (32 * NW)) * FwdShape<NW>::kGs + (q % (32 * NW)) * 8]) = w[c];
  }
}

template <int NW>
__device__ __forceinline__ void fwd_multiply(f32x16 (&acc)[2], const u16* Xs, int wave, int lane) {
  const u16* Ws = Xs + kTile * kLd;
#pragma unroll
  for (int kk = 0; kk < kTile; kk += 16) {
    const int off = kk + 8 * (lane >> 5);
    const bf16x8 bfrag =
        *reinterpret_cast<const bf16x8*>(&Ws[(kk / 8 + (lane >> 5)) * FwdShape<NW>::kGs + (wave * 32 + (lane & 31)) * 8]);
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
      const bf16x8 afrag = *reinterpret_cast<const bf16x8*>(&Xs[(rt * 32 + (lane & 31)) * kLd + off]);
      acc[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag, bfrag, acc[rt], 0, 0, 0);
    }
  }
}

// LOSS: instead of E, accumulate the mean cross-entropy of rows b0.. of EVERY node's
// pool under the W held in node slot 0 (the node average) into *loss_out (B = samples).
// SC > 0: the number of 64-feature stages is this compile-time constant and the stage loop is
// unrolled completely.  The compiler's wait-count bookkeeping only tells "the oldest stage has
// arrived, two younger ones may still be in flight" apart in straight-line code: with a loop (or
// conditional prefetches) it waits for every outstanding load at each stage, which exposes the
// memory latency once per stage pair (0.84 us per stage measured) whatever the prefetch depth.
template <int NW, bool LOSS, int SC = 0>
__global__ void __launch_bounds__(64 * NW) rfast_softmax_forward(RfastDev s, const int32_t* batch_idx, int B, bool init,
                                                                 double* loss_out) {
  extern __shared__ u16 lds[];
  int slot, rb;
  xcd_decode(B / kTile, &slot, &rb);
  int t_unused;
  const int i = pick_node(s, init, slot, &t_unused);
  if (i < 0) return;
  constexpr int K = 32 * NW;
  constexpr int kBuf = FwdShape<NW>::kBuf;
  const int d = s.prob.d;
  __shared__ int rows[kTile];
  __shared__ int labs[kTile];
  const int b0 = rb * kTile;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const u16* pool = (const u16*)s.prob.data0 + (size_t)i * s.prob.samples * d;
  const int32_t* labels = (const int32_t*)s.prob.data1 + (size_t)i * s.prob.samples;
  const Scratch sc = scratch_of(s, B);
  const u16* wt = sc.wt + (LOSS ? (size_t)0 : (size_t)i * K * d);
  // The label of a row is not needed before the softmax: its load (which depends on the row number,
  // itself a load) is issued here and only parked in LDS after the contraction.
  int my_label = 0;
  if (tid < kTile) {
    const int row = sample_row(s, batch_idx, i, b0 + tid, B);
    rows[tid] = row;
    my_label = labels[row];
    // a label outside [0, K) would index the logits in LDS out of bounds: clamped and reported, like a sample row
    if (my_label < 0 || my_label >= K) {
      if (atomicCAS(&s.err[0], 0, RFAST_ERANGE) == 0) {
        s.err[1] = s.n_active[1] - 1;
        s.err[2] = 3;
        s.err[3] = i;
      }
      my_label = my_label < 0 ? 0 : K - 1;
    }
  }
  __syncthreads();

  f32x16 acc[2];
#pragma unroll
  for (int v = 0; v < 16; ++v) { acc[0][v] = 0.f; acc[1][v] = 0.f; }

  const int S = SC > 0 ? SC : d / kTile;
  if constexpr (SC > 0) {
    // three register sets in rotation: while stage st is multiplied out of LDS, the loads of
    // stages st+1 .. st+3 are in flight and only the oldest of them is waited for
    u32x4 rx[3][FwdShape<NW>::kXc], rw[3][4];
    u16* bufs[2] = {lds, lds + kBuf};
    fwd_load<NW>(rx[0], rw[0], pool, rows, wt, d, 0, tid);
    fwd_store<NW>(rx[0], rw[0], bufs[0], bufs[0] + kTile * kLd, tid);
    if (1 < SC) fwd_load<NW>(rx[1], rw[1], pool, rows, wt, d, 1 * kTile, tid);
    if (2 < SC) fwd_load<NW>(rx[2], rw[2], pool, rows, wt, d, 2 * kTile, tid);
    if (3 < SC) fwd_load<NW>(rx[0], rw[0], pool, rows, wt, d, 3 * kTile, tid);
#pragma unroll
    for (int st = 0; st < SC; ++st) {
      __syncthreads();  // bufs[st & 1] holds stage st; everyone is done reading the other buffer
      fwd_multiply<NW>(acc, bufs[st & 1], wave, lane);
      if (st + 1 < SC) {
        fwd_store<NW>(rx[(st + 1) % 3], rw[(st + 1) % 3], bufs[(st + 1) & 1], bufs[(st + 1) & 1] + kTile * kLd, tid);
        if (st + 4 < SC) fwd_load<NW>(rx[(st + 1) % 3], rw[(st + 1) % 3], pool, rows, wt, d, (st + 4) * kTile, tid);
      }
    }
    __syncthreads();
  } else {
  // (ax, aw) carry the odd stages, (bx, bw) the even ones; neither pair is ever
  // copied, so a wait for one never implies a wait for the other (loads retire in order).
  u32x4 ax[FwdShape<NW>::kXc], aw[4], bx[FwdShape<NW>::kXc], bw[4];
  u16* buf0 = lds;
  u16* buf1 = lds + kBuf;
  fwd_load<NW>(bx, bw, pool, rows, wt, d, 0, tid);
  fwd_store<NW>(bx, bw, buf0, buf0 + kTile * kLd, tid);
  if (S > 1) fwd_load<NW>(ax, aw, pool, rows, wt, d, kTile, tid);
  if (S > 2) fwd_load<NW>(bx, bw, pool, rows, wt, d, 2 * kTile, tid);
  for (int st = 0; st < S; st += 2) {
    __syncthreads();  // buf0 holds stage st; everyone is done reading buf1
    fwd_multiply<NW>(acc, buf0, wave, lane);
    if (st + 1 < S) {
      fwd_store<NW>(ax, aw, buf1, buf1 + kTile * kLd, tid);  // stage st+1
      if (st + 3 < S) fwd_load<NW>(ax, aw, pool, rows, wt, d, (st + 3) * kTile, tid);
      __syncthreads();  // buf1 holds stage st+1; everyone is done reading buf0
      fwd_multiply<NW>(acc, buf1, wave, lane);
      if (st + 2 < S) {
        fwd_store<NW>(bx, bw, buf0, buf0 + kTile * kLd, tid);  // stage st+2
        if (st + 4 < S) fwd_load<NW>(bx, bw, pool, rows, wt, d, (st + 4) * kTile, tid);
      }
    }
  }
  __syncthreads();
  }

  if (tid < kTile) labs[tid] = my_label;
  // logits -> LDS [64][K+1] fp32 (reuses the staging space)
  float* L = reinterpret_cast<float*>(lds);
  constexpr int ldl = K + 1;
#pragma unroll
  for (int rt = 0; rt < 2; ++rt)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = rt * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
      L[row * ldl + wave * 32 + (lane & 31)] = acc[rt][v];
    }
  __syncthreads();
  // Row softmax, all 64 rows at once: lane = row, wave w = classes 32w .. 32w+31 (the
  // odd row stride K+1 keeps the 64 lanes on distinct LDS banks).  The per-row maximum
  // and sum cross the NW waves through a few words of LDS instead of 12 dependent
  // wavefront shuffles per row, which cost more than the whole contraction.
  __shared__ float red[2][4][kTile];
  const float invB = 1.0f / (float)B;
  float* Lr = L + lane * ldl + wave * 32;
  const float logit_label = L[lane * ldl + labs[lane]];
  float m = -INFINITY;
#pragma unroll 8
  for (int j = 0; j < 32; ++j) m = fmaxf(m, Lr[j]);
  red[0][wave][lane] = m;
  __syncthreads();  // every logit_label is read before any logit is overwritten below
#pragma unroll
  for (int w2 = 0; w2 < NW; ++w2) m = fmaxf(m, red[0][w2][lane]);
  float sum = 0.f;
#pragma unroll 8
  for (int j = 0; j < 32; ++j) {
    const float e = __expf(Lr[j] - m);
    Lr[j] = e;
    sum += e;
  }
  red[1][wave][lane] = sum;
  __syncthreads();
  sum = 0.f;
#pragma unroll
  for (int w2 = 0; w2 < NW; ++w2) sum += red[1][w2][lane];
  if (LOSS) {
    if (wave == 0) {
      double row_loss = (double)logf(sum) + (double)m - (double)logit_label;  // -log softmax[label]
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) row_loss += __shfl_xor(row_loss, o, 64);
      if (lane == 0) atomicAdd(loss_out, row_loss / (double)B);
    }
    return;
  }
  {
    const float inv = 1.0f / sum;
    const int lab = labs[lane] - wave * 32;
#pragma unroll 8
    for (int j = 0; j < 32; ++j) Lr[j] = (Lr[j] * inv - (j == lab ? 1.0f : 0.0f)) * invB;
  }
  __syncthreads();
  // Et[k][b0 .. b0+64): 8 consecutive rows per 16-byte store
  u16* et = sc.et + (size_t)i * K * B;
  for (int q = tid; q < K * kTile / 8; q += 64 * NW) {
    const int k = q / (kTile / 8), c = (q % (kTile / 8)) * 8;
    u16 h[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) h[j] = f32_to_bf16(L[(c + j) * ldl + k]);
    uint4 pk;
    pk.x = h[0] | ((uint32_t)h[1] << 16);
    pk.y = h[2] | ((uint32_t)h[3] << 16);
    pk.z = h[4] | ((uint32_t)h[5] << 16);
    pk.w = h[6] | ((uint32_t)h[7] << 16);
    *reinterpret_cast<uint4*>(et + (size_t)k * B + b0 + c) = pk;
  }
}

// ------------------------------------------------------------------------ backward
// one workgroup per (node, 64-feature block), XCD-aware ids; wave w owns classes
// 32w .. 32w+31 and both 32-feature tiles.  The contraction over the B sampled
// rows runs in stages of 64 rows through two LDS buffers; the next stage's global
// loads are issued before the current stage is multiplied.  The X tile is
// transposed on its way into LDS (Xt[f][b]) so that both operands are contiguous in b.
// X tile of the backward pass: 64 sampled rows x 64 features = 512 chunks of 16 bytes.
// Chunk q belongs to row q % 64 (so the lanes of a wavefront hold 64 different rows of
// the same 8 features) and feature group q / 64.
template <int NW>
__device__ __forceinline__ void bwd_load(u32x4 (&x)[FwdShape<NW>::kXc], u32x4 (&e)[4], const u16* pool, const int* rows,
                                         const u16* et, int d, int B, int f0, int b0, int tid) {
  constexpr int T = FwdShape<NW>::kThreads;
#pragma unroll
  for (int c = 0; c < FwdShape<NW>::kXc; ++c) {
    const int q = tid + c * T;
    if ((kTile * kTile / 8) % T == 0 || q < kTile * kTile / 8)
      x[c] = *reinterpret_cast<const u32x4*>(pool + (size_t)rows[q & 63] * d + f0 + (q >> 6) * 8);
  }
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const int q = tid + c * T;
    e[c] = *reinterpret_cast<const u32x4*>(et + (size_t)(q / (kTile / 8)) * B + b0 + (q % (kTile / 8)) * 8);
  }
}

// Transposed store Xt[f][b].  Neighbouring lanes hold neighbouring rows b, so an even lane
// and its odd partner swap halves: the even lane then owns features 0-3 of both rows, the
// odd lane features 4-7, and each writes four 32-bit words (two rows of one feature) that
// fall on consecutive LDS banks across the wavefront.
template <int NW>
__device__ __forceinline__ void bwd_store(const u32x4 (&x)[FwdShape<NW>::kXc], const u32x4 (&e)[4], u16* Xt, u16* Es,
                                          int tid) {
  constexpr int T = FwdShape<NW>::kThreads;
  const bool odd = tid & 1;
#pragma unroll
  for (int c = 0; c < FwdShape<NW>::kXc; ++c) {
    const int q = tid + c * T;
    // every lane of the wavefront takes part in the exchange (q < 512 is wave-uniform: 512 % 64 == 0)
    if ((kTile * kTile / 8) % T == 0 || q < kTile * kTile / 8) {
      const int r = q & 63, f = (q >> 6) * 8;
      const uint32_t mine0 = odd ? x[c][2] : x[c][0], mine1 = odd ? x[c][3] : x[c][1];
      const uint32_t send0 = odd ? x[c][0] : x[c][2], send1 = odd ? x[c][1] : x[c][3];
      const uint32_t got0 = __shfl_xor(send0, 1, 64), got1 = __shfl_xor(send1, 1, 64);
      // rows (r & ~1, r | 1): the even row goes to the low half of the word
      const uint32_t lo0 = odd ? got0 : mine0, hi0 = odd ? mine0 : got0;
      const uint32_t lo1 = odd ? got1 : mine1, hi1 = odd ? mine1 : got1;
      const int fb = f + (odd ? 4 : 0), rb = r & ~1;
      *reinterpret_cast<uint32_t*>(&Xt[(fb + 0) * kLd + rb]) = (lo0 & 0xFFFFu) | (hi0 << 16);
      *reinterpret_cast<uint32_t*>(&Xt[(fb + 1) * kLd + rb]) = (lo0 >> 16) | (hi0 & 0xFFFF0000u);
      *reinterpret_cast<uint32_t*>(&Xt[(fb + 2) * kLd + rb]) = (lo1 & 0xFFFFu) | (hi1 << 16);
      *reinterpret_cast<uint32_t*>(&Xt[(fb + 3) * kLd + rb]) = (lo1 >> 16) | (hi1 & 0xFFFF0000u);
    }
  }
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const int q = tid + c * T;
    *reinterpret_cast<u32x4*>(&Es[(q / (kTile / 8)) * kLd + (q % (kTile / 8)) * 8]) = e[c];
  }
}

// SC > 0: B = 64 * SC rows at compile time: every row number is fetched once up front (not one
// dependent load per stage on the critical path), the stage loop is unrolled completely and three
// stages of loads stay in flight with exact wait counts (see the forward pass).
template <int NW, int SC = 0>
__global__ void __launch_bounds__(64 * NW) rfast_softmax_backward(RfastDev s, const int32_t* batch_idx, int B, bool init) {
  extern __shared__ u16 lds[];
  int slot, fb;
  const int d = s.prob.d;
  xcd_decode(d / kTile, &slot, &fb);
  int t_old;
  const int i = pick_node(s, init, slot, &t_old);
  if (i < 0) return;
  constexpr int K = 32 * NW;
  constexpr int kBuf = (kTile + K) * kLd;  // Xt tile [64 features][kLd], then Es [K][kLd]
  __shared__ int rows[2][kTile];
  const int f0 = fb * kTile;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const u16* pool = (const u16*)s.prob.data0 + (size_t)i * s.prob.samples * d;
  const u16* et = scratch_of(s, B).et + (size_t)i * K * B;

  f32x16 acc[2];
#pragma unroll
  for (int v = 0; v < 16; ++v) { acc[0][v] = 0.f; acc[1][v] = 0.f; }

  if constexpr (SC > 0) {
    __shared__ int rows_all[(SC > 0 ? SC : 1) * kTile];
    for (int r = tid; r < SC * kTile; r += 64 * NW) rows_all[r] = sample_row(s, batch_idx, i, r, B);
    __syncthreads();
    u32x4 rx[3][FwdShape<NW>::kXc], re[3][4];
    bwd_load<NW>(rx[0], re[0], pool, rows_all, et, d, B, f0, 0, tid);
    if (1 < SC) bwd_load<NW>(rx[1], re[1], pool, rows_all + kTile, et, d, B, f0, kTile, tid);
    if (2 < SC) bwd_load<NW>(rx[2], re[2], pool, rows_all + 2 * kTile, et, d, B, f0, 2 * kTile, tid);
#pragma unroll
    for (int st = 0; st < SC; ++st) {
      u16* Xt = lds + (st & 1) * kBuf;
      u16* Es = Xt + kTile * kLd;
      bwd_store<NW>(rx[st % 3], re[st % 3], Xt, Es, tid);  // stage st (its buffer was last read two stages ago)
      if (st + 3 < SC)
        bwd_load<NW>(rx[st % 3], re[st % 3], pool, rows_all + (st + 3) * kTile, et, d, B, f0, (st + 3) * kTile, tid);
      __syncthreads();
#pragma unroll
      for (int kk = 0; kk < kTile; kk += 16) {
        const int off = kk + 8 * (lane >> 5);
        const bf16x8 bfrag = *reinterpret_cast<const bf16x8*>(&Es[(wave * 32 + (lane & 31)) * kLd + off]);
#pragma unroll
        for (int ft = 0; ft < 2; ++ft) {
          const bf16x8 afrag = *reinterpret_cast<const bf16x8*>(&Xt[(ft * 32 + (lane & 31)) * kLd + off]);
          acc[ft] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag, bfrag, acc[ft], 0, 0, 0);
        }
      }
    }
  } else {
  const int S = B / kTile;
  for (int r = tid; r < kTile; r += 64 * NW) rows[0][r] = sample_row(s, batch_idx, i, r, B);
  __syncthreads();
  u32x4 x[FwdShape<NW>::kXc], e[4];
  bwd_load<NW>(x, e, pool, rows[0], et, d, B, f0, 0, tid);
  for (int st = 0; st < S; ++st) {
    u16* Xt = lds + (st & 1) * kBuf;
    u16* Es = Xt + kTile * kLd;
    bwd_store<NW>(x, e, Xt, Es, tid);  // stage st (its buffer was last read two stages ago)
    if (st + 1 < S)
      for (int r = tid; r < kTile; r += 64 * NW) rows[(st + 1) & 1][r] = sample_row(s, batch_idx, i, (st + 1) * kTile + r, B);
    __syncthreads();
    if (st + 1 < S) bwd_load<NW>(x, e, pool, rows[(st + 1) & 1], et, d, B, f0, (st + 1) * kTile, tid);
#pragma unroll
    for (int kk = 0; kk < kTile; kk += 16) {
      const int off = kk + 8 * (lane >> 5);
      const bf16x8 bfrag = *reinterpret_cast<const bf16x8*>(&Es[(wave * 32 + (lane & 31)) * kLd + off]);
#pragma unroll
      for (int ft = 0; ft < 2; ++ft) {
        const bf16x8 afrag = *reinterpret_cast<const bf16x8*>(&Xt[(ft * 32 + (lane & 31)) * kLd + off]);
        acc[ft] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag, bfrag, acc[ft], 0, 0, 0);
      }
    }
  }
  }
  float* G = s.g + (size_t)((t_old + 1) & 1) * s.n * s.p + (size_t)i * s.p;
  const float* Wi = s.x + (size_t)i * s.p;  // weight decay of the optimizer variant acts on the fp32 weights
  const float wd = s.wd;
#pragma unroll
  for (int ft = 0; ft < 2; ++ft)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int f = f0 + ft * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
      const size_t o = (size_t)f * K + wave * 32 + (lane & 31);
      G[o] = wd != 0.0f ? fmaf(wd, Wi[o], acc[ft][v]) : acc[ft][v];
    }
}

}  // namespace

// The state kernel that mixes x (S2a) can emit the blocked bf16 copy of the new weights itself when
// its 1024-coordinate tile covers whole 8-feature blocks: K divides 1024.
bool rfast_softmax_prep_is_fused(const rfast_problem* prob) {
  return prob->kind == RFAST_OBJ_SOFTMAX_BF16 && (prob->K == 32 || prob->K == 64 || prob->K == 128);
}

// Shapes the kernels assume; checked once at context creation.
bool rfast_softmax_shape_ok(const rfast_problem* prob) {
  const int B = prob->batch > 0 ? prob->batch : prob->samples;
  return prob->d % kTile == 0 && prob->K % 32 == 0 && prob->K >= 32 && prob->K <= 128 && B % kTile == 0;
}

size_t rfast_softmax_scratch_bytes(int32_t n, const rfast_problem* prob) {
  if (prob->kind != RFAST_OBJ_SOFTMAX_BF16) return 0;
  const int B = prob->batch > 0 ? prob->batch : prob->samples;
  return ((size_t)n * prob->K * prob->d + (size_t)n * prob->K * B) * sizeof(u16);
}

hipError_t rfast_softmax_gradient(rfast_ctx* c, const int32_t* batch_idx, bool init) {
  const RfastDev& d = c->d;
  if (!rfast_softmax_shape_ok(&d.prob)) return hipErrorInvalidValue;
  const int B = d.prob.batch > 0 ? d.prob.batch : d.prob.samples;
  const int32_t* bi = d.prob.batch > 0 ? batch_idx : nullptr;
  const int K = d.prob.K, NW = K / 32;
  const unsigned threads = 64u * (unsigned)NW;
  const size_t lds_prep = (size_t)kTile * (K + 4) * sizeof(u16);
  const size_t lds_fwd_stage = 2 * (size_t)(kTile * kLd + 8 * (K * 8 + 8)) * sizeof(u16);
  const size_t lds_logits = (size_t)kTile * (K + 1) * sizeof(float);
  const size_t lds_fwd = lds_fwd_stage > lds_logits ? lds_fwd_stage : lds_logits;
  const size_t lds_bwd = 2 * (size_t)(kTile + K) * kLd * sizeof(u16);
  const unsigned n8 = (unsigned)((d.n + 7) / 8 * 8);  // node slots, padded so that ids decode per XCD
  // during rounds the mixing pass has already written the bf16 copy of the weights it produced
  if (init || !rfast_softmax_prep_is_fused(&d.prob))
    hipLaunchKernelGGL(rfast_softmax_prep, dim3(d.prob.d / kTile, d.n), dim3(256), lds_prep, c->stream, d, B, init, (const float*)nullptr);
  const dim3 fgrid(n8 * (unsigned)(B / kTile)), bgrid(n8 * (unsigned)(d.prob.d / kTile));
  switch (NW) {
    case 1:
      hipLaunchKernelGGL((rfast_softmax_forward<1, false>), fgrid, dim3(threads), lds_fwd, c->stream, d, bi, B, init, (double*)nullptr);
      hipLaunchKernelGGL(rfast_softmax_backward<1>, bgrid, dim3(threads), lds_bwd, c->stream, d, bi, B, init);
      break;
    case 2:
      hipLaunchKernelGGL((rfast_softmax_forward<2, false>), fgrid, dim3(threads), lds_fwd, c->stream, d, bi, B, init, (double*)nullptr);
      hipLaunchKernelGGL(rfast_softmax_backward<2>, bgrid, dim3(threads), lds_bwd, c->stream, d, bi, B, init);
      break;
    case 3:
      hipLaunchKernelGGL((rfast_softmax_forward<3, false>), fgrid, dim3(threads), lds_fwd, c->stream, d, bi, B, init, (double*)nullptr);
      hipLaunchKernelGGL(rfast_softmax_backward<3>, bgrid, dim3(threads), lds_bwd, c->stream, d, bi, B, init);
      break;
    default:
      if (d.prob.d == 16 * kTile)
        hipLaunchKernelGGL((rfast_softmax_forward<4, false, 16>), fgrid, dim3(threads), lds_fwd, c->stream, d, bi, B, init, (double*)nullptr);
      else
        hipLaunchKernelGGL((rfast_softmax_forward<4, false>), fgrid, dim3(threads), lds_fwd, c->stream, d, bi, B, init, (double*)nullptr);
      if (B == 4 * kTile)
        hipLaunchKernelGGL((rfast_softmax_backward<4, 4>), bgrid, dim3(threads), lds_bwd, c->stream, d, bi, B, init);
      else
        hipLaunchKernelGGL(rfast_softmax_backward<4>, bgrid, dim3(threads), lds_bwd, c->stream, d, bi, B, init);
      break;
  }
  return hipGetLastError();
}

// sum_i f_i(xbar): mean cross-entropy of every node's whole pool under W = bf16(xbar).
// Needs the pool size to be a multiple of the 64-row tile; otherwise the loss is left at NaN.
hipError_t rfast_softmax_loss(rfast_ctx* c, double* d_out) {
  const RfastDev& d = c->d;
  const int K = d.prob.K, NW = K / 32, S = d.prob.samples;
  if (!rfast_softmax_shape_ok(&d.prob) || S % kTile != 0) {
    static const double kNan = __builtin_nan("");
    return hipMemcpyAsync(d_out, &kNan, sizeof(double), hipMemcpyHostToDevice, c->stream);
  }
  const unsigned threads = 64u * (unsigned)NW;
  const size_t lds_prep = (size_t)kTile * (K + 4) * sizeof(u16);
  const size_t lds_stage = 2 * (size_t)(kTile * kLd + 8 * (K * 8 + 8)) * sizeof(u16);
  const size_t lds_logits = (size_t)kTile * (K + 1) * sizeof(float);
  const size_t lds_fwd = lds_stage > lds_logits ? lds_stage : lds_logits;
  hipLaunchKernelGGL(rfast_softmax_prep, dim3(d.prob.d / kTile, 1), dim3(256), lds_prep, c->stream, d, S, true,
                     (const float*)d.xbar);
  const unsigned n8 = (unsigned)((d.n + 7) / 8 * 8);
  const dim3 grid(n8 * (unsigned)(S / kTile));
  switch (NW) {
    case 1: hipLaunchKernelGGL((rfast_softmax_forward<1, true>), grid, dim3(threads), lds_fwd, c->stream, d, (const int32_t*)nullptr, S, true, d_out); break;
    case 2: hipLaunchKernelGGL((rfast_softmax_forward<2, true>), grid, dim3(threads), lds_fwd, c->stream, d, (const int32_t*)nullptr, S, true, d_out); break;
    case 3: hipLaunchKernelGGL((rfast_softmax_forward<3, true>), grid, dim3(threads), lds_fwd, c->stream, d, (const int32_t*)nullptr, S, true, d_out); break;
    default: hipLaunchKernelGGL((rfast_softmax_forward<4, true>), grid, dim3(threads), lds_fwd, c->stream, d, (const int32_t*)nullptr, S, true, d_out); break;
  }
  return hipGetLastError();
}
