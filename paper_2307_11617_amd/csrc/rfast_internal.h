// Internal layout shared by the translation units of librfast (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "rfast.h"

// ---------------------------------------------------------------------------
// Device-side view of one context.  Passed to kernels by value.
//
// State is node-major structure-of-arrays: every logical vector is contiguous
// in the coordinate k, so one wavefront reads 64 consecutive float4 (1 KiB).
//   x, z        [n][p]
//   g           [2][n][p]   the sample of version t lives in g[t & 1]
//   v_ring      [n][M][p]   M = D + 2 slots, version t in slot t mod M
//   sigma_ring  [n][M][p]   sender-side running sum sigma_j = sum of every z_half node j
//                           produced; the running sum rho_ij of Algorithm 1 (S2c) is
//                           a_ij * sigma_j for every out-neighbour i, so one ring per
//                           sender replaces one ring per edge
//   rho_tilde   [eC][p]     receiver side.  The buffer of S4 holds a_ij * sigma_j[tau_ij], a value
//                           that also sits in the sender's ring while tau_ij >= t_j - D.  It is
//                           therefore read from the ring ("implicit") and only written out
//                           ("explicit") in the round in which that version is about to leave
//                           the ring: by the receiver if it consumes exactly that version then,
//                           by the sender otherwise.  Invariant: tau_ij < t_j - D  =>  the array
//                           holds a_ij * sigma_j[tau_ij].
// ---------------------------------------------------------------------------
struct RfastDev {
  int32_t n, M, H, eR, eC, d_max, burst;
  int64_t p;
  float* x;
  float* z;
  float* g;
  float* v_ring;
  float* sigma_ring;
  float* rho_tilde;
  // graph, off-diagonal entries only (row = receiver)
  const int32_t* r_ptr;   // [n+1] into R off-diagonal entries
  const int32_t* r_src;   // [eR] sender j
  const int32_t* r_dst;   // [eR] receiver i
  const float* r_w;       // [eR] w_ij
  const float* r_self;    // [n]  w_ii
  const int32_t* c_ptr;   // [n+1] into C off-diagonal entries (in-edges of i are consecutive ids)
  const int32_t* c_src;   // [eC] sender j
  const int32_t* c_dst;   // [eC] receiver i
  const float* c_w;       // [eC] a_ij
  const float* c_self;    // [n]  a_ii
  const int32_t* co_ptr;  // [n+1] out-edges of sender j over C
  const int32_t* co_eid;  // [eC] edge id
  const float* co_w;      // [eC] a_lj
  const int32_t* ro_ptr;  // [n+1] out-edges of sender j over R
  const int32_t* ro_eid;  // [eR]
  // integer state
  int32_t* t;             // [n]
  int32_t* t_hist;        // [n][H]   t_hist[j][s mod H] = t_j at the start of round s
  int32_t* tau_r;         // [eR]
  int32_t* tau_c;         // [eC]
  unsigned long long* deliv_r;  // [eR] bit s set: the version in slot s was delivered on this edge
  unsigned long long* deliv_c;  // [eC]
  int32_t* round_no;      // [1]
  int32_t* err;           // [4] code, round, kind, edge (first error wins)
  // per-round plan written by the resolver, read by the state kernels
  int32_t* n_active;      // [2]: active nodes of the round, round counter after it
  // [n + 8] work slots of the round: {node, t_node at the start of the round}, the active nodes in
  // increasing order first, then {-1, 0}.  One 8-byte load tells a workgroup whether it has work, for
  // which node and at which counter (instead of a chain of three dependent loads).
  int2* active_plan;
  int32_t* plan_t;        // [n]   t_i at the start of the round
  int32_t* slot_r;        // [eR]  resolved slot, -1 if receiver inactive
  int32_t* slot_c;        // [eC]
  // everything the state kernels need to know about a C edge in this round, in one word:
  //   bits 0-7   ring slot of the version consumed (valid when live)
  //   bits 8-15  ring slot of the version consumed last time, 0xFF = it is in the rho_tilde array
  //   bit 16     live: the receiver is active and its stamp moved (otherwise the edge contributes exactly zero)
  //   bit 17     the receiver writes what it consumes to the rho_tilde array
  //   bit 18     the sender copies a_ij * sigma_j[t_j - D] to the rho_tilde array
  //   bit 30     live, bits 8-15 are a slot and bit 17 is clear (the usual live edge)
  //   bit 31     live otherwise
  int32_t* plan_c;        // [eC]
  uint8_t* node_spill;    // [n]   some out-edge of this node has bit 18 set
  // The plan of one round once more, as one record for the kernel that keeps a tile of coordinates
  // in LDS over several rounds (NULL: not wanted): [n] node words (bit 31 active, low 30 bits the
  // counter at the start of the round), [eR] ring slot per R edge, [eC] plan word per C edge.
  int32_t* blk_plan;
  // What a multi-round launch needs to know about the state before its first round and after its last,
  // written by the resolver around the rounds it resolves (NULL: not wanted).  [n][kHeadWords] per node j:
  //   0, 1    its counter before and after
  //   2, 3    the oldest version of its v ring that a receiver could still pick up before (the smallest stamp held
  //           on j's out-edges over R; INT_MAX if j has none), the same for its ring of running sums (out-edges over C)
  //   4, 5    both once more for after
  //   8, 9    the ring slot of its latest version before and after (the counter mod M)
  //   10, 11  one bit per slot of its v ring / its ring of sums: the slot holds a version that can still be picked
  //           up before the launch (such slots are loaded, the others are zeros in LDS)
  //   12      one bit per slot: the launch writes the slot
  //   13, 14  as 10, 11, for after the launch (what is stored is a slot of 12 that is also one of 13 or 14; with a
  //           rebase on the way out, every slot of 14)
  // (rings of up to 32 slots).  Then [eC] per C edge: bit 0 set if its S4 buffer was in the rho_tilde array before
  // (its version outside the sender's ring), bit 1 if it is after.
  int32_t* blk_head;
  // schedule of the current round when it is generated on the device
  uint8_t* gen_active;    // [n]
  int32_t* gen_delay_r;   // [eR]
  int32_t* gen_delay_c;   // [eC]
  uint8_t* gen_drop_r;    // [eR]
  uint8_t* gen_drop_c;    // [eC]
  int32_t* gen_batch;     // [n][batch]
  uint32_t* gen_cdf;      // [n] selection thresholds of the event-driven mode (one node per iteration)
  float* xbar;            // [p] node average, written by the diagnostics kernel
  // optimizer variant: heavy-ball buffers m_i [n][p] (caller's memory, NULL when beta == 0)
  float* mom;
  float beta, wd;
  // gradient scratch
  float* resid;           // [n][rows] residuals of the GEMV pair / unused
  void* gscratch;         // softmax: bf16 W copy and E matrix
  rfast_problem prob;
};

struct rfast_ctx {
  RfastDev d;
  hipStream_t stream;
  int32_t nnzR, nnzC;
  std::string err;
  bool profiling = false;
  std::vector<hipEvent_t> ev[3][2];
  size_t ev_used[3] = {0, 0, 0};
  double* d_diag = nullptr;  // carved from the workspace
  int32_t rebase_interval = 512;  // rounds between automatic rebases of the running sums (0 = never)
  // replayable HIP graph of kGraphRounds generated rounds (rfast_run_generated), and what it was built for
  bool use_graphs = false;
  hipGraphExec_t graph_exec = nullptr;
  hipStream_t capture_stream = nullptr;
  uint64_t graph_seed = 0;
  const float* graph_p_active = nullptr;
  int32_t graph_max_delay = 0;
  float graph_p_drop = 0.f, graph_gamma = 0.f;
  int32_t sync_parity = 0;  // 1: the current z of the synchronous mode lives in slot 1 of the v ring
  int64_t host_round = 0;       // mirror of the device round counter, for the step-size schedule
  int32_t gamma_step = 0;       // rounds per decay step, 0 = constant step size
  float gamma_factor = 1.f;
  bool needs_init = false;      // rfast_set_optimizer was called and rfast_init has not followed yet
  int32_t use_blocks = 1;       // 1: where it pays, 2: wherever possible; rfast_run / rfast_run_generated may advance several rounds per launch
  int32_t wave_group = 0;       // wavefronts per workgroup of the wavefront-tile kernel (0: chosen by the launcher)
  int32_t* blk_plan_base = nullptr;  // kBlockRounds plan records
  int32_t* blk_head_base = nullptr;  // kHeadWords n + eC words, see RfastDev::blk_head
  int32_t max_degree = 0;       // most in-edges of R, in-edges of C or out-edges of C at any node
  // the per-round plan arrays of RfastDev exist kResolveAhead times; `plan_set` is the set d points at
  char* plan_set0 = nullptr;
  size_t plan_set_bytes = 0;
  int32_t plan_set = 0;
  int32_t gen_depth = 1;        // rounds the generator's arrays hold
  int32_t gen_last = 0;         // which of them the last round executed used (reads of the SCHED fields)
};

enum { RFAST_MODE_FUSED = 0, RFAST_MODE_MIX = 1, RFAST_MODE_TRACK = 2 };

// rounds that one launch of the LDS-resident kernel can advance, rounds whose plan records it holds
// in LDS at a time, and the shortest launch that pays where the state is large (the launch moves
// every ring slot in and out once: measured on 16 nodes x 11.2 M coordinates, about 7 ms per launch
// plus 0.33 ms per round against 1.53 ms per round of the streaming kernel: even from 6 rounds on)
constexpr int kHeadWords = 16;  // words per node in RfastDev::blk_head
constexpr int kBlockRounds = 512;
constexpr int kPlanChunk = 16;
constexpr int kBlockMinRoundsLarge = 8;
// rounds the resolver may run ahead of the kernels that read its plans (rfast_run, one pass per round)
constexpr int kResolveAhead = 32;
struct RfastBlock {
  float gamma;                // step size of its rounds (a launch does not straddle a decay step)
  int32_t rounds;             // 1 .. kBlockRounds
  int32_t rebase;             // wavefront-tile kernel: the running sums are rebased as the tiles are written back
};

// launchers (each enqueues on ctx->stream and returns a hipError_t)
hipError_t rfast_launch_resolve(rfast_ctx* c, const uint8_t* active, const int32_t* delay_R,
                                const int32_t* delay_C, const uint8_t* drop_R, const uint8_t* drop_C, int rounds = 1,
                                size_t plan_stride = 0);
hipError_t rfast_launch_state(rfast_ctx* c, int mode, float gamma);
hipError_t rfast_launch_rebase(rfast_ctx* c);
// several rounds of the separable objective on LDS-resident tiles; the rounds' plans are in blk_plan
bool rfast_wave_eligible(const rfast_ctx* c);   // the multi-round kernel with one tile per wavefront
int rfast_wave_lanes(const rfast_ctx* c);       // its lanes per node
hipError_t rfast_launch_wave(rfast_ctx* c, const RfastBlock& blk);
hipError_t rfast_wave_prime(rfast_ctx* c);      // loads the kernels this context can launch, with launches that do nothing
bool rfast_block_eligible(const rfast_ctx* c);  // the multi-round kernel with one tile per workgroup
int rfast_block_lanes(const rfast_ctx* c);  // lanes per node of the multi-round kernel, 0 if no tile fits
hipError_t rfast_launch_block(rfast_ctx* c, const RfastBlock& blk);
// least squares / logistic regression: consecutive rounds as two kernels each (rows; columns + track + the next mixing)
bool rfast_chain_eligible(const rfast_ctx* c);
hipError_t rfast_launch_rows(rfast_ctx* c, const int32_t* d_batch_idx, const uint8_t* d_active);
hipError_t rfast_launch_cols_track_mix(rfast_ctx* c, const int32_t* d_batch_idx, const uint8_t* d_active, const uint8_t* d_active_next,
                                       size_t next_set_bytes, float gamma_next);
bool rfast_tiny_eligible(const rfast_ctx* c);   // the multi-round kernel for least squares / logistic problems that fit one CU's LDS
bool rfast_tiny_resolves(const rfast_ctx* c);   // ... and it resolves its rounds itself (no resolver launch ahead of it)
hipError_t rfast_launch_tiny(rfast_ctx* c, const RfastBlock& blk, const int32_t* d_batch_idx, int round0, const uint8_t* d_active,
                             const int32_t* d_delay_R, const int32_t* d_delay_C, const uint8_t* d_drop_R, const uint8_t* d_drop_C);
hipError_t rfast_launch_generate(rfast_ctx* c, uint64_t seed, const float* d_p_active, int d_max, float p_drop, bool events,
                                 int rounds = 1);
hipError_t rfast_launch_sync(rfast_ctx* c, int phase, float gamma, int parity);
hipError_t rfast_launch_sync_plan(rfast_ctx* c, int rounds);
bool rfast_sync_wave_eligible(const rfast_ctx* c);  // several synchronous steps per launch
hipError_t rfast_launch_sync_wave(rfast_ctx* c, float gamma, int rounds);
hipError_t rfast_launch_init_grad(rfast_ctx* c, const int32_t* batch_idx0);
hipError_t rfast_diag_init_gradient(rfast_ctx* c);  // separable objective: g[t_i & 1][i] = sample(x_i, t_i) for every node
hipError_t rfast_launch_gradient(rfast_ctx* c, const int32_t* batch_idx);
hipError_t rfast_launch_diag(rfast_ctx* c, const float* d_xstar, double* d_out);
hipError_t rfast_static_scratch_init();  // address of the static scratch array on the current device (once per device)
int64_t rfast_static_max_coords();
hipError_t rfast_launch_diag_static(rfast_ctx* c, const float* d_xstar, double* d_out, double l2_half_n);
hipError_t rfast_softmax_loss(rfast_ctx* c, double* d_out);  // adds sum_i f_i(xbar) to *d_out
bool rfast_softmax_prep_is_fused(const rfast_problem* prob);
size_t rfast_grad_scratch_bytes(int32_t n, int64_t p, const rfast_problem* prob);
