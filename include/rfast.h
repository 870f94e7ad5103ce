/*
 * rfast.h — C ABI of the MI355X (gfx950) library that advances a batch of
 * simulated R-FAST workers by one asynchronous activation round.
 *
 * The method is "R-FAST: Robust Fully-Asynchronous Stochastic Gradient
 * Tracking over General Topology" (arXiv 2307.11617).  One round lets every
 * node flagged active perform the node update of Algorithm 1 (steps S1-S5;
 * global view: Algorithm 2) once, all of them reading the state as of the
 * start of the round:
 *   S1   v_i   = x_i - gamma z_i
 *   S2a  x_i'  = w_ii v_i + sum_{j in N_in(W), j != i} w_ij v_j^(tau_v,ij)
 *   S2b  z_i^½ = z_i + sum_{j in N_in(A), j != i} (rho_ij^(tau_rho,ij) - rho~_ij)
 *                + grad f_i(x_i'; zeta') - grad f_i(x_i; zeta)      (stored sample)
 *   S2c  z_i'  = a_ii z_i^½ ;  rho_li += a_li z_i^½  for every out-neighbour l
 *   S3   publish (t_i+1, v_i) and (t_i+1, rho_li)
 *   S4   rho~_ij = the rho_ij just consumed
 *   S5   t_i += 1
 * W is the row-stochastic pull matrix, A the column-stochastic push matrix
 * (Assumption 1).  Here W is called R and A is called C.
 *
 * Conventions
 *  - Every graph is CSR with ROW = RECEIVER: row i lists node i's in-neighbours
 *    j (ascending, unique), the self-loop (j == i) included and mandatory.
 *    Rows of R sum to 1; for every j the entries (.,j) of C sum to 1.
 *  - "Off-diagonal entry e" = the e-th entry of the CSR with j != i, counted in
 *    CSR order.  All per-edge arrays (delays, drops, stamps, rho rings) use
 *    this numbering; e of graph R and e of graph C are separate numberings.
 *  - Version t of node j is what j published at its t-th activation; version 0
 *    is the zero vector (initialisation of Algorithm 1).  Version t lives in
 *    ring slot t mod (D+2): D+1 readable versions plus the slot being written.
 *  - "device" pointers are HIP device memory of the current device; "host"
 *    pointers are ordinary host memory.  The library never frees or keeps a
 *    host pointer past the call.  Device memory passed in stays owned by the
 *    caller and must outlive the context.
 *  - All calls return RFAST_OK (0) or a negative rfast_status; none throws or
 *    aborts.  rfast_last_error() gives a text for the last failure.
 *  - A context is bound to one HIP stream; calls on one context must be
 *    serialised by the caller.  Work is enqueued asynchronously unless stated.
 */
#ifndef RFAST_H
#define RFAST_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rfast_ctx rfast_ctx;

typedef enum rfast_status {
  RFAST_OK = 0,
  RFAST_EINVAL = -1, /* null pointer, bad size, bad enum, misaligned buffer        */
  RFAST_ESTOCH = -2, /* weights negative, diagonal missing, R rows / C columns != 1 */
  RFAST_EGRAPH = -3, /* malformed CSR, or G(R), G(C^T) share no spanning-tree root  */
  RFAST_ERANGE = -4, /* delay outside [0, D-burst+1], D or sample index out of range */
  RFAST_ENOMEM = -5, /* workspace too small                                        */
  RFAST_EHIP = -6    /* a HIP runtime call failed                                  */
} rfast_status;

/* Local objectives f_i (problem (1): F = sum_i f_i; each node samples an
 * unbiased stochastic gradient of its own f_i, Assumption 5). */
typedef enum rfast_objective {
  RFAST_OBJ_DIAG_QUADRATIC = 0, /* f_i = 1/2 sum_k h_ik (x_k - c_ik)^2, gradient + noise_std*N(0,I) */
  RFAST_OBJ_LEAST_SQUARES = 1,  /* f_i = 1/(2m) ||A_i x - b_i||^2                                   */
  RFAST_OBJ_LOGISTIC = 2,       /* f_i = mean_s [log(1+exp(a_s.x)) - y_s a_s.x] + lambda/2 ||x||^2  */
  RFAST_OBJ_SOFTMAX_BF16 = 3    /* softmax regression, W = x as d x K row-major, bf16 MFMA GEMMs;
                                   needs d % 64 == 0, K in {32,64,96,128}, rows per gradient % 64 == 0 */
} rfast_objective;

typedef struct rfast_problem {
  int32_t kind;        /* rfast_objective */
  int32_t samples;     /* rows held per node (LS: m; logistic/softmax: pool size); 0 for diag quadratic */
  int32_t batch;       /* rows per sampled gradient; 0 = all `samples` rows (full local gradient)       */
  int32_t d, K;        /* softmax only: features, classes; p must equal d*K                             */
  float lambda;        /* logistic only: l2 coefficient                                                 */
  float noise_std;     /* diag quadratic only: std of the additive gradient noise                       */
  uint64_t noise_seed; /* diag quadratic only: key of the counter-based generator (see below)           */
  const void* data0;   /* device. diag: h  fp32 [n][p]. LS/logistic: rows fp32 [n][samples][p].
                          softmax: pool bf16 [n][samples][d]                                            */
  const void* data1;   /* device. diag: c  fp32 [n][p]. LS: b fp32 [n][samples]. logistic: y fp32 (0/1)
                          [n][samples]. softmax: labels int32 [n][samples]                              */
} rfast_problem;
/* Gradient noise of the diagonal quadratic: coordinates are taken in groups of
 * four; group q of (node i, sample version t) is Philox4x32-10 (Salmon et al.,
 * SC'11) of counter (q mod 2^32, q div 2^32, i, t) under key (seed mod 2^32,
 * seed div 2^32), giving words o0..o3.  u = ((o >> 8) + 1) / 2^24,
 * angle = 2 pi o' / 2^32; (o0, o1) yields coordinates 4q, 4q+1 as r cos, r sin
 * with r = sqrt(-2 ln u); (o2, o3) yields 4q+2, 4q+3.  The sample version of
 * the initial gradient is 0, that of the t-th activation is t. */

typedef enum rfast_field {
  RFAST_X = 0,         /* fp32 [n][p]                                             */
  RFAST_Z = 1,         /* fp32 [n][p]                                             */
  RFAST_G = 2,         /* fp32 [n][p]  stored gradient sample of each node.  For the diagonal quadratic the
                          sample is a pure function of (x_i, t_i): it is recomputed where needed and on
                          read; writing it is accepted and has no effect                              */
  RFAST_V_RING = 3,    /* fp32 [n][D+2][p]  slot s of node j = version t, t mod (D+2) == s.  In the three ring
                          fields a slot whose version no receiver can pick up any more (stamps never go
                          back, S2a / S2b: it is older than every stamp held on its sender's out-edges of
                          that graph) reads as zeros; the library does not keep such slots up to date */
  RFAST_RHO_RING = 4,  /* fp32 [nnzC_off][D+2][p]  sender-side running sums rho_ij = a_ij * sigma_j (expanded on read) */
  RFAST_RHO_TILDE = 5, /* fp32 [nnzC_off][p]  receiver-side buffers (assembled on read: a buffer whose version
                          is still in its sender's ring is taken from there, cf. RFAST_SIGMA_RING)   */
  RFAST_T_NODE = 6,    /* int32 [n]  local iteration counters t_i                  */
  RFAST_TAU_R = 7,     /* int32 [nnzR_off]  largest stamp picked up per R edge     */
  RFAST_TAU_C = 8,     /* int32 [nnzC_off]                                         */
  RFAST_SLOT_R = 9,    /* int32 [nnzR_off]  ring slot resolved in the last round (receiver active), else -1 */
  RFAST_SLOT_C = 10,   /* int32 [nnzC_off]                                         */
  RFAST_ROUND = 11,    /* int32 [1]  rounds executed                               */
  RFAST_SIGMA_RING = 12, /* fp32 [n][D+2][p]  per-sender running sum of z_half, as stored */
  RFAST_DELIV_R = 13,    /* uint64 [nnzR_off]  bit s set: the version in ring slot s was delivered on this edge */
  RFAST_DELIV_C = 14,    /* uint64 [nnzC_off]                                                                */
  RFAST_T_HIST = 15,     /* int32 [n][D+1]  t_j at the start of round s, stored at s mod (D+1)              */
  /* schedule of the last round generated on the device (rfast_run_generated), read-only: */
  RFAST_SCHED_ACTIVE = 16,  /* uint8 [n] */
  RFAST_SCHED_DELAY_R = 17, /* int32 [nnzR_off] */
  RFAST_SCHED_DELAY_C = 18, /* int32 [nnzC_off] */
  RFAST_SCHED_DROP_R = 19,  /* uint8 [nnzR_off] */
  RFAST_SCHED_DROP_C = 20,  /* uint8 [nnzC_off] */
  RFAST_SCHED_BATCH = 21,   /* int32 [n][batch] */
  RFAST_MOMENTUM = 22       /* fp32 [n][p]  heavy-ball buffers m_i (only after rfast_set_optimizer gave one) */
} rfast_field;

typedef struct rfast_diag {
  double consensus_sq;    /* || x - 1 xbar^T ||_F^2, xbar = (1/n) sum_i x_i (merit function of Theorem 2) */
  double z_sq;            /* || z ||_F^2                                                                   */
  double conservation_sq; /* || sum_i z_i + sum_e (rho_e latest - rho~_e) - sum_i g_i ||^2 (Lemma 3: 0)    */
  double gsum_sq;         /* || sum_i g_i ||^2 (scale for the line above)                                  */
  double xbar_gap_sq;     /* || xbar - x* ||^2, or -1 if no x* was given (optimality gap of Theorem 1)     */
  double loss_at_xbar;    /* sum_i f_i(xbar): the training loss at the network average (full local data),
                             plus n * weight_decay/2 ||xbar||^2 under rfast_set_optimizer                   */
} rfast_diag;

/* Bytes of device workspace rfast_create needs for these sizes (pure function;
 * returns 0 if an argument is out of range).  nnzR / nnzC count the diagonal. */
size_t rfast_workspace_bytes(int32_t n, int64_t p, int32_t nnzR, int32_t nnzC, int32_t D,
                             const rfast_problem* prob);

/* Assumption 2 as a host-only check: host_is_root[i] (nullable) = 1 iff node i is the
 * root of a spanning tree of G(R) (reaches every node along sender -> receiver edges)
 * AND of G(C^T) (is reached by every node along C's sender -> receiver edges).  Returns
 * the number of common roots (0 = the pair of graphs violates the assumption) or a
 * negative rfast_status.  CSR as for rfast_create (row = receiver); weights are not needed. */
int rfast_common_roots(int32_t n, const int32_t* R_rowptr, const int32_t* R_col, const int32_t* C_rowptr,
                       const int32_t* C_col, uint8_t* host_is_root);

/* Builds a context.  R_*, C_*: host CSR (row = receiver) with fp32 weights.
 * D: largest staleness in sender versions any read may have (Assumption 3 ii),
 *    1 <= D+2 <= 64.  burst >= 1: a version whose burst-1 predecessors on the
 *    same edge were all lost is delivered even if flagged lost, so per-round
 *    delays may range over [0, D-burst+1].
 * prob: objective and device pointers to its data (copied by value).
 * d_workspace: device, >= rfast_workspace_bytes(...), 256-byte aligned.
 * hip_stream: a hipStream_t (NULL = the null stream).
 * Checks Assumption 1 (RFAST_ESTOCH), CSR shape and Assumption 2 (RFAST_EGRAPH).
 * On failure *out is NULL and rfast_last_error(NULL) describes the cause. */
int rfast_create(rfast_ctx** out, int32_t n, int64_t p,
                 const int32_t* R_rowptr, const int32_t* R_col, const float* R_w,
                 const int32_t* C_rowptr, const int32_t* C_col, const float* C_w,
                 int32_t D, int32_t burst, const rfast_problem* prob,
                 void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* Initialisation of Algorithm 1: x = x0 (device fp32 [n][p], NULL = zeros),
 * g = z = grad f_i(x0; zeta^0), every ring, buffer and stamp zero, round 0.
 * d_batch_idx0: device int32 [n][batch] rows of the initial sample (objectives
 * with batch > 0), else NULL. */
int rfast_init(rfast_ctx* ctx, const float* d_x0, const int32_t* d_batch_idx0);

/* One activation round (asynchronous on the context's stream).  All pointers
 * are DEVICE memory and must stay valid until the round has executed:
 *  d_active  uint8 [n]          node i performs S1-S5 iff non-zero
 *  d_delay_R int32 [nnzR_off]   receiver sees the sender as of the start of round r-delay
 *  d_delay_C int32 [nnzC_off]
 *  d_drop_R  uint8 [nnzR_off]   the packet the edge's sender publishes THIS round is lost
 *  d_drop_C  uint8 [nnzC_off]
 *  gamma     step size of S1
 *  d_batch_idx int32 [n][batch] sample rows per node (used for active nodes), NULL if batch == 0
 * Stamps resolve as: newest non-lost version the sender had published before
 * round r-delay, never older than the stamp already held.  A delay or row index
 * out of range is clamped on the device and recorded; rfast_check() reports it. */
int rfast_round(rfast_ctx* ctx, const uint8_t* d_active, const int32_t* d_delay_R,
                const int32_t* d_delay_C, const uint8_t* d_drop_R, const uint8_t* d_drop_C,
                float gamma, const int32_t* d_batch_idx);

/* `rounds` consecutive rounds from schedule arrays stacked along a leading
 * round axis ([rounds][n], [rounds][nnzR_off], ..., [rounds][n][batch]). */
int rfast_run(rfast_ctx* ctx, int32_t rounds, const uint8_t* d_active, const int32_t* d_delay_R,
              const int32_t* d_delay_C, const uint8_t* d_drop_R, const uint8_t* d_drop_C,
              float gamma, const int32_t* d_batch_idx);

/* `rounds` rounds whose schedule is generated on the device as a pure function
 * of (seed, round number), so that nothing is uploaded per round (Assumption 3:
 * who is active, how stale each edge is, which packets are lost, which rows are
 * sampled).  With word(stream, r, e) = Philox4x32-10(counter (e div 4, stream,
 * r, 0), key seed)[e mod 4]:
 *   active[i]  = word(0, r, i) < floor(p_active[i] * 2^32)
 *   delay_R[e] = word(1, r, e) mod (max_delay + 1);   delay_C[e]: stream 2
 *   drop_R[e]  = word(3, r, e) < floor(p_drop * 2^32);  drop_C[e]: stream 4
 *   rows of node i = perm(0..batch-1), perm a keyed bijection of [0, samples):
 *   4-round balanced Feistel network on 2h bits (h = ceil(bits/2), bits = bit
 *   length of samples-1, at least 1), cycle-walked into range, round keys
 *   Philox(counter (i, 5, r, 0)); round function on half R with key K:
 *   t = R*0x9E3779B1 + K; t ^= t >> 15; t *= 0x85EBCA77; F = t >> (32-h) (mod 2^32).
 * The schedule of a stretch of rounds is drawn by one launch and then runs as rfast_run runs an
 * uploaded one.  d_p_active: DEVICE fp32 [n].  max_delay in [0, D-burst+1] (RFAST_ERANGE). */
int rfast_run_generated(rfast_ctx* ctx, int32_t rounds, uint64_t seed, const float* d_p_active,
                        int32_t max_delay, float p_drop, float gamma);

/* Event-driven form, the global view of Algorithm 2 taken literally: `iterations`
 * global iterations k (k = RFAST_ROUND, counted from rfast_init), each activating
 * exactly one agent i^k, with delays counted in global iterations.  i^k is drawn on
 * the device: u = word(6, k, 0) (the generator of rfast_run_generated), and agent i
 * is taken when cdf[i-1] <= u < cdf[i], where cdf[i] = min(floor(2^32 * (w_0 + .. +
 * w_i) / (w_0 + .. + w_{n-1})), 2^32 - 1) in double precision and cdf[-1] = 0; u =
 * 2^32 - 1 goes to the last agent if its weight is positive (to nobody otherwise: an
 * empty iteration).  Delays, losses and sample rows are those of rfast_run_generated.
 * Slow agents (stragglers) are agents with a small weight.
 * host_weights: HOST fp32 [n], finite, >= 0, not all zero (RFAST_ERANGE), or NULL for
 * uniform selection; consumed before return. */
int rfast_run_events(rfast_ctx* ctx, int32_t iterations, uint64_t seed, const float* host_weights,
                     int32_t max_delay, float p_drop, float gamma);

/* on != 0: rfast_run_generated replays a HIP graph of 16 generated rounds (one
 * launch per 16 rounds instead of 4-7 per round) whenever at least 16 rounds are
 * asked for, profiling is off and no rebase interval is set; the remaining rounds
 * run as ordinary launches.  Results are identical either way.  Off by default. */
int rfast_use_graphs(rfast_ctx* ctx, int32_t on);

/* on != 0 (the default): rfast_run and rfast_run_generated advance up to 512 rounds with one
 * launch where that is possible and pays -- the separable objective (diagonal quadratic, with or
 * without the optimizer variant), p a multiple of 4, at most 64 nodes, no node with more than 6
 * (33 to 64 nodes: 4) in-edges of R, in-edges of C or out-edges of C, a tile of coordinates of every node's two rings
 * fitting into the 160 KB of LDS of a CU (up to 32 nodes: 64 / n lanes of one wavefront per node, 4
 * coordinates per lane, n * (D+2) * (64 / n) * 32 B; beyond: at least 16 lanes of one workgroup per
 * node, n * (D+2) * 512 B + plans), and at least 2 rounds to run before the next multiple of the
 * rebase interval and the next decay step of the step-size schedule (8 where n * p * 4 > 8 MB: a launch
 * moves every ring slot that can still be read in and out once, which a large state earns back only
 * over that many rounds), rings of at most 32 slots (D <= 30); rounds that do not qualify run one pass
 * each.  Every step of a round is elementwise in the coordinate, so a tile of coordinates can stay
 * in LDS over several rounds; the results are the same bits as round-by-round execution.
 * Least squares and logistic regression (whose gradient couples the coordinates of a node, so that
 * there are no tiles) take the same stretches of rounds with one launch of a single workgroup when the
 * whole problem fits the LDS of one CU: p a multiple of 4, no heavy-ball buffer, (3 + 2 (D+2)) n p +
 * eC p floats of state plus the graph, n (batch, or samples) residuals and row numbers and two plan
 * records within 150 KB (the samples themselves too if they still fit, else they are read from global
 * memory), at most 4096 sampled rows per round and n + eR + eC < 1024; same bits as the chain of
 * four kernels per round.  With at most 64 nodes and 64 edges of a kind that workgroup also resolves
 * the stamps of its rounds itself (no resolver kernel runs ahead of it).
 * Where these objectives do not fit one workgroup (and p is a multiple of 4, no heavy-ball buffer), rfast_run and
 * rfast_run_generated run a round as two kernels instead of four: the sampled rows' residuals, then one kernel
 * that forms the gradient, does the tracker update and mixes the same coordinates for the next round; same bits.
 * on == 0: always one kernel pass per round (four kernels for these objectives).  on == 2: as the default, but
 * 2 rounds are enough at any size (for measurements). */
int rfast_use_blocks(rfast_ctx* ctx, int32_t on);
/* *lanes_per_node = 0 if a call of rfast_run for several rounds would now run one pass per round,
 * else the number of lanes per node of the multi-round kernel (its tile is 4 * lanes coordinates;
 * 1024 / n, at least 1, for the single workgroup of the non-separable objectives);
 * *tile_per_wavefront (may be NULL) = 1 if a tile belongs to one wavefront, 0 if to a workgroup. */
int rfast_block_info(rfast_ctx* ctx, int32_t* lanes_per_node, int32_t* tile_per_wavefront);
/* Tuning knob of the wavefront-tile kernel of rfast_use_blocks: wavefronts per workgroup (1, 2 or 4; 0 = chosen by
 * the library).  The wavefronts of a workgroup own neighbouring tiles and move their rings between HBM and LDS
 * together, so a row segment of a load or store is that many times as wide; the rounds themselves are unaffected
 * and the results are the same bits.  A value whose tiles do not fit the LDS of a CU falls back to 1. */
int rfast_set_tile_group(rfast_ctx* ctx, int32_t wavefronts);

/* One step of the synchronous push-pull recursion the method is developed from
 * (eq. (2) of the paper), on the same x, z and stored gradient samples:
 *   x_i' = sum_j w_ij (x_j - gamma z_j),  z_i' = sum_j a_ij z_j + grad f_i(x_i'; zeta') - grad f_i(x_i; zeta)
 * with every node stepping at once (both sums include j = i; no delays, no losses).
 * Every t_i advances by one and the sample stamp is t_i + 1, as in rfast_round.
 * The step uses slots 0 and 1 of the v rings as buffers: do not interleave it with
 * rfast_round on the same context without an rfast_init in between.
 * d_batch_idx: device int32 [n][batch] (objectives with batch > 0), else NULL.
 * rfast_sync_run: `rounds` steps from sample rows stacked [rounds][n][batch].  Where rfast_use_blocks
 * allows it (separable objective, p a multiple of 4, at most 32 nodes with at most 6 edges of a kind)
 * the steps between two decay steps of the step-size schedule are taken by one launch that keeps
 * x, z and the samples in registers and exchanges x - gamma z and z through LDS: same bits. */
int rfast_sync_round(rfast_ctx* ctx, float gamma, const int32_t* d_batch_idx);
int rfast_sync_run(rfast_ctx* ctx, int32_t rounds, float gamma, const int32_t* d_batch_idx);

/* Between rounds (asynchronous): subtracts from every sender's running sums, and
 * from the buffers rho~ they feed, the sender's latest running sum.  Algorithm 1
 * only uses the differences rho_ij - rho~_ij (S2b), which this leaves unchanged in
 * exact arithmetic; in fp32 it stops the growth of the cancellation error of that
 * difference with the number of rounds.  Call it every few hundred rounds of a
 * long run; state read back afterwards shows the shifted rho and rho~. */
int rfast_rebase(rfast_ctx* ctx);
/* rounds > 0: every asynchronous round entry enqueues rfast_rebase whenever the round
 * counter (RFAST_ROUND, counted from rfast_init) reaches a multiple of `rounds`;
 * 0 never does.  The default is 512: without it the fp32 error of x grows
 * quadratically with the number of rounds where the objective does not damp it
 * (logistic regression at p = 4096: 1e-4 relative after about 3500 rounds), with
 * it linearly and about a hundred times more slowly.  One rebase costs about one
 * and a half rounds of a sparse graph (2(D+2) + 2 dO + 1 words per coordinate
 * per sender), i.e. 0.3 % of a run at the default; where the wavefront-tile kernel
 * of rfast_use_blocks ends a launch at such a round it rebases while it writes its
 * tiles back, at no cost. */
int rfast_set_rebase_interval(rfast_ctx* ctx, int32_t rounds);

/* Optimizer variant.  The large-scale experiment of the paper (Section
 * "Large-scale image classification", hyper-parameters ii-iv) trains with
 * momentum 0.9, weight decay 1e-4 and a learning rate divided by 10 every 30
 * epochs, without saying where these enter Algorithm 1.  The reading built here:
 *   weight decay   g = grad f_i(x; zeta) + weight_decay * x wherever a gradient is
 *                  sampled (initialisation and S2b), so it is tracked like the rest
 *                  of the gradient; the objective becomes f_i + weight_decay/2 ||x||^2;
 *   momentum       S1 becomes m_i <- momentum * m_i + z_i, v = x_i - gamma * m_i
 *                  (m_i = 0 at rfast_init; only an activated node touches its
 *                  buffer); momentum = 0 is S1 as printed.  Costs 2 more words per
 *                  coordinate and update.  The same holds for rfast_sync_round.
 * With one node this is SGD with momentum and weight decay as in the textbooks.
 * d_momentum: device fp32 [n][p], 16-byte aligned, owned by the caller, must
 * outlive the context; required iff momentum != 0.  momentum in [0, 1),
 * weight_decay >= 0 (RFAST_ERANGE otherwise).  Because the stored gradients and
 * the buffers change meaning, rfast_init must follow before the next round
 * (rounds return RFAST_EINVAL until it has). */
int rfast_set_optimizer(rfast_ctx* ctx, float momentum, float weight_decay, float* d_momentum);
/* Step-decayed learning rate (same experiment, hyper-parameter ii): round number r
 * (RFAST_ROUND, counted from rfast_init) runs with gamma * factor^(r div step_rounds),
 * where gamma is what the round call passes.  step_rounds = 0 (default) switches it off.
 * factor must be finite and > 0. */
int rfast_set_gamma_schedule(rfast_ctx* ctx, int32_t step_rounds, float factor);

/* Waits for the stream, then returns RFAST_OK or the first error a round
 * recorded on the device (RFAST_ERANGE) with its round and edge in the text. */
int rfast_check(rfast_ctx* ctx);

/* Waits for the stream and copies one field to HOST memory.  `bytes` must be
 * exactly the field's size (RFAST_EINVAL otherwise). */
int rfast_read_state(rfast_ctx* ctx, int32_t field, void* host_dst, size_t bytes);

/* Waits for the stream and overwrites one field from HOST memory: the inverse
 * of rfast_read_state, for checkpoint / resume.  Restoring X, Z, G, V_RING,
 * SIGMA_RING, RHO_TILDE, T_NODE, TAU_R, TAU_C, DELIV_R, DELIV_C, T_HIST,
 * ROUND (and MOMENTUM when used) into a context created with the same arguments reproduces the run bit
 * for bit.  RHO_RING (derived), SLOT_R and SLOT_C (per-round plan) cannot be
 * written (RFAST_EINVAL). */
int rfast_write_state(rfast_ctx* ctx, int32_t field, const void* host_src, size_t bytes);

/* Reductions over the current state (synchronous).  d_xstar: device fp32 [p] or NULL. */
int rfast_diagnostics(rfast_ctx* ctx, const float* d_xstar, rfast_diag* host_out);

/* rfast_diagnostics for callers that cannot allocate or wait: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same reductions and kernels, but their scratch (the fp64 accumulators
 * and, for the objectives whose loss needs it, the node average xbar) lives in a static device array of the
 * library instead of the workspace, nothing is allocated, freed or copied to the host, and the call does not
 * wait: the six results are written, in the order of rfast_diag, to d_out (DEVICE, 6 doubles, 8-byte aligned)
 * by the last kernel enqueued on the context's stream.  xbar_gap_sq is -1 without d_xstar.
 * Limit: least squares, logistic and softmax objectives need p <= 1 048 576 (the xbar part of the scratch,
 * 4 MiB + 256 B per GPU for the life of the process); larger p returns RFAST_ERANGE.  The diagonal quadratic
 * has no limit.  All contexts on one GPU share the array: calls that overlap on one GPU (different streams)
 * race; calls on one stream, or otherwise ordered, do not.  (rfast_sync_round's pending z is folded back
 * first, as in rfast_diagnostics.) */
int rfast_diagnostics_static(rfast_ctx* ctx, const float* d_xstar, double* d_out);

/* Kernel timing: when enabled, HIP events bracket the state-update kernels and
 * the gradient kernels of each round (at most 4096 rounds are kept since the
 * last enable).  rfast_kernel_time waits for the stream and returns the summed
 * milliseconds and the number of timed launches of `which`
 * (0 = fused/mix+track state kernels, 1 = gradient kernels, 2 = resolver). */
int rfast_profile_enable(rfast_ctx* ctx, int32_t on);
int rfast_kernel_time(rfast_ctx* ctx, int32_t which, double* ms_sum, int64_t* launches);

const char* rfast_last_error(const rfast_ctx* ctx);
void rfast_destroy(rfast_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* RFAST_H */
