// C-ABI entry points of librfast: argument checks, workspace layout, launch order.
#include <math.h>
#include <string.h>

#include <algorithm>
#include <string>
#include <type_traits>
#include <vector>

#include "rfast_internal.h"

size_t rfast_gemv_scratch_floats(int32_t n, const rfast_problem* prob);
size_t rfast_softmax_scratch_bytes(int32_t n, const rfast_problem* prob);
bool rfast_softmax_shape_ok(const rfast_problem* prob);

namespace {

std::string g_create_error;

constexpr size_t kAlign = 256;
inline size_t up(size_t b) { return (b + kAlign - 1) / kAlign * kAlign; }

// Sizes of every carve-out, in the order they are laid out.
struct Layout {
  size_t total = 0;
  size_t take(size_t bytes) {
    const size_t off = total;
    total += up(bytes);
    return off;
  }
};

struct Offsets {
  size_t x, z, g, v_ring, sigma_ring, rho_tilde;
  size_t r_ptr, r_src, r_dst, r_w, r_self, c_ptr, c_src, c_dst, c_w, c_self, co_ptr, co_eid, co_w, ro_ptr, ro_eid;
  size_t t, t_hist, tau_r, tau_c, deliv_r, deliv_c, round_no, err;
  size_t n_active, active_plan, plan_t, slot_r, slot_c, plan_c, node_spill, plan_set_bytes, blk_plan, blk_head;
  size_t gen_active, gen_delay_r, gen_delay_c, gen_drop_r, gen_drop_c, gen_batch, gen_cdf;
  int32_t gen_depth;
  size_t xbar, resid, gscratch, diag;
  size_t total;
};

bool sizes_ok(int32_t n, int64_t p, int32_t nnzR, int32_t nnzC, int32_t D, const rfast_problem* prob) {
  if (n < 1 || n > 65535 || p < 1 || nnzR < n || nnzC < n || D < 0 || D + 2 > 64 || prob == nullptr) return false;  // n rides in gridDim.y
  if (prob->kind < 0 || prob->kind > RFAST_OBJ_SOFTMAX_BF16) return false;
  if (prob->kind != RFAST_OBJ_DIAG_QUADRATIC && (prob->samples < 1 || prob->batch < 0 || prob->batch > prob->samples))
    return false;
  if ((prob->kind == RFAST_OBJ_LEAST_SQUARES || prob->kind == RFAST_OBJ_LOGISTIC) &&
      (prob->batch > 0 ? prob->batch : prob->samples) > 4096)
    return false;  // the sampled residuals of one node are staged in LDS
  if (prob->kind == RFAST_OBJ_SOFTMAX_BF16 &&
      (prob->d < 1 || prob->K < 1 || (int64_t)prob->d * prob->K != p || !rfast_softmax_shape_ok(prob)))
    return false;  // MFMA tiling: d % 64 == 0, K in {32, 64, 96, 128}, rows per gradient % 64 == 0
  return true;
}

Offsets layout(int32_t n, int64_t p, int32_t nnzR, int32_t nnzC, int32_t D, const rfast_problem* prob) {
  const size_t eR = (size_t)(nnzR - n), eC = (size_t)(nnzC - n), M = (size_t)D + 2, H = (size_t)D + 1;
  const size_t vec = (size_t)p * sizeof(float);
  Layout L;
  Offsets o;
  o.x = L.take(n * vec);
  o.z = L.take(n * vec);
  o.g = L.take(2 * n * vec);
  o.v_ring = L.take(n * M * vec);
  o.sigma_ring = L.take(n * M * vec);
  o.rho_tilde = L.take(eC * vec);
  o.r_ptr = L.take((n + 1) * 4);
  o.r_src = L.take(eR * 4);
  o.r_dst = L.take(eR * 4);
  o.r_w = L.take(eR * 4);
  o.r_self = L.take(n * 4);
  o.c_ptr = L.take((n + 1) * 4);
  o.c_src = L.take(eC * 4);
  o.c_dst = L.take(eC * 4);
  o.c_w = L.take(eC * 4);
  o.c_self = L.take(n * 4);
  o.co_ptr = L.take((n + 1) * 4);
  o.co_eid = L.take(eC * 4);
  o.co_w = L.take(eC * 4);
  o.ro_ptr = L.take((n + 1) * 4);
  o.ro_eid = L.take(eR * 4);
  o.t = L.take(n * 4);
  o.t_hist = L.take(n * H * 4);
  o.tau_r = L.take(eR * 4);
  o.tau_c = L.take(eC * 4);
  o.deliv_r = L.take(eR * 8);
  o.deliv_c = L.take(eC * 8);
  o.round_no = L.take(4);
  o.err = L.take(16);
  o.n_active = L.take(8);
  o.active_plan = L.take(((size_t)n + 8) * 8);
  o.plan_t = L.take(n * 4);
  o.slot_r = L.take(eR * 4);
  o.slot_c = L.take(eC * 4);
  o.plan_c = L.take(eC * 4);
  o.node_spill = L.take(n);
  // the seven arrays above are the plan of one round; kResolveAhead - 1 more such sets follow, so that the
  // resolver can run that many rounds ahead of the kernels that read the plans
  o.plan_set_bytes = L.total - o.n_active;
  (void)L.take((size_t)(kResolveAhead - 1) * o.plan_set_bytes);
  o.blk_plan = L.take((size_t)kBlockRounds * ((size_t)n + eR + eC + 1) * 4);
  o.blk_head = L.take((kHeadWords * (size_t)n + eC) * 4);
  // the generator draws the schedule of up to gen_depth rounds per launch (as many as fit 64 MB, at most kBlockRounds)
  const size_t gen_rows = (size_t)n * (size_t)(prob->kind == RFAST_OBJ_DIAG_QUADRATIC ? 0 : prob->batch);
  const size_t gen_round = (size_t)n + 5 * (eR + eC) + 4 * gen_rows;
  const size_t G = std::max<size_t>(1, std::min<size_t>(kBlockRounds, ((size_t)64 << 20) / gen_round));
  o.gen_depth = (int32_t)G;
  o.gen_active = L.take(G * n);
  o.gen_delay_r = L.take(G * eR * 4);
  o.gen_delay_c = L.take(G * eC * 4);
  o.gen_drop_r = L.take(G * eR);
  o.gen_drop_c = L.take(G * eC);
  o.gen_batch = L.take(G * gen_rows * 4);
  o.gen_cdf = L.take(n * 4);
  o.xbar = L.take(vec);
  o.resid = L.take(rfast_gemv_scratch_floats(n, prob) * 4);
  o.gscratch = L.take(rfast_softmax_scratch_bytes(n, prob));
  o.diag = L.take(64 * sizeof(double));
  o.total = L.total;
  return o;
}

struct HostGraph {
  std::vector<int32_t> ptr, src, dst, out_ptr, out_eid;
  std::vector<float> w, self, out_w;
};

// Splits a CSR (row = receiver, diagonal included) into off-diagonal in-edge and
// out-edge lists and checks Assumption 1: positive diagonal, non-negative
// weights, rows (row_stochastic) or columns summing to one.
int split_graph(const char* name, int32_t n, const int32_t* rowptr, const int32_t* col, const float* w,
                bool row_stochastic, HostGraph* g, std::string* err) {
  if (rowptr[0] != 0) { *err = std::string(name) + ": rowptr[0] != 0"; return RFAST_EGRAPH; }
  g->ptr.assign(n + 1, 0);
  g->self.assign(n, 0.f);
  std::vector<double> colsum(n, 0.0);
  for (int i = 0; i < n; ++i) {
    if (rowptr[i + 1] < rowptr[i]) { *err = std::string(name) + ": rowptr not monotone"; return RFAST_EGRAPH; }
    double rowsum = 0.0;
    int prev = -1;
    bool diag = false;
    for (int k = rowptr[i]; k < rowptr[i + 1]; ++k) {
      const int j = col[k];
      if (j < 0 || j >= n || j <= prev) {
        *err = std::string(name) + ": column indices must be in range, ascending and unique (row " + std::to_string(i) + ")";
        return RFAST_EGRAPH;
      }
      prev = j;
      if (!(w[k] > 0.f) || !std::isfinite(w[k])) {
        *err = std::string(name) + ": stored weights must be positive (row " + std::to_string(i) + ")";
        return RFAST_ESTOCH;
      }
      rowsum += w[k];
      colsum[j] += w[k];
      if (j == i) {
        diag = true;
        g->self[i] = w[k];
      } else {
        g->src.push_back(j);
        g->dst.push_back(i);
        g->w.push_back(w[k]);
      }
    }
    if (!diag) { *err = std::string(name) + ": missing self-loop at node " + std::to_string(i); return RFAST_ESTOCH; }
    if (row_stochastic && fabs(rowsum - 1.0) > 1e-6) {
      *err = std::string(name) + ": row " + std::to_string(i) + " does not sum to 1";
      return RFAST_ESTOCH;
    }
    g->ptr[i + 1] = (int32_t)g->src.size();
  }
  if (!row_stochastic)
    for (int j = 0; j < n; ++j)
      if (fabs(colsum[j] - 1.0) > 1e-6) {
        *err = std::string(name) + ": column " + std::to_string(j) + " does not sum to 1";
        return RFAST_ESTOCH;
      }
  // out-edge lists (sender-major)
  const size_t E = g->src.size();
  g->out_ptr.assign(n + 1, 0);
  for (size_t e = 0; e < E; ++e) g->out_ptr[g->src[e] + 1]++;
  for (int j = 0; j < n; ++j) g->out_ptr[j + 1] += g->out_ptr[j];
  g->out_eid.assign(E, 0);
  g->out_w.assign(E, 0.f);
  std::vector<int32_t> fill(g->out_ptr.begin(), g->out_ptr.end() - 1);
  for (size_t e = 0; e < E; ++e) {
    const int pos = fill[g->src[e]]++;
    g->out_eid[pos] = (int32_t)e;
    g->out_w[pos] = g->w[e];
  }
  return RFAST_OK;
}

// Nodes from which every node can be reached along `forward` edges sender->receiver
// (forward = true) or receiver->sender (forward = false).
std::vector<char> roots_of(int32_t n, const HostGraph& g, bool forward) {
  std::vector<std::vector<int>> adj(n);
  for (int i = 0; i < n; ++i)
    for (int e = g.ptr[i]; e < g.ptr[i + 1]; ++e) {
      if (forward) adj[g.src[e]].push_back(i);
      else adj[i].push_back(g.src[e]);
    }
  std::vector<char> is_root(n, 0);
  std::vector<int> stack;
  std::vector<char> seen;
  for (int r = 0; r < n; ++r) {
    seen.assign(n, 0);
    stack.assign(1, r);
    seen[r] = 1;
    int cnt = 1;
    while (!stack.empty()) {
      const int u = stack.back();
      stack.pop_back();
      for (int v : adj[u])
        if (!seen[v]) { seen[v] = 1; ++cnt; stack.push_back(v); }
    }
    is_root[r] = cnt == n;
  }
  return is_root;
}

template <class T>
hipError_t upload(rfast_ctx* c, char* base, size_t off, const std::vector<T>& v) {
  if (v.empty()) return hipSuccess;
  return hipMemcpyAsync(base + off, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice, c->stream);
}

int fail(rfast_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg; else g_create_error = msg;
  return code;
}
int hipfail(rfast_ctx* c, hipError_t e, const char* what) {
  return fail(c, RFAST_EHIP, std::string(what) + ": " + hipGetErrorString(e));
}

size_t field_bytes(const rfast_ctx* c, int32_t field) {
  const RfastDev& d = c->d;
  const size_t vec = (size_t)d.p * 4;
  switch (field) {
    case RFAST_X: case RFAST_Z: case RFAST_G: return d.n * vec;
    case RFAST_V_RING: return (size_t)d.n * d.M * vec;
    case RFAST_RHO_RING: return (size_t)d.eC * d.M * vec;
    case RFAST_SIGMA_RING: return (size_t)d.n * d.M * vec;
    case RFAST_RHO_TILDE: return (size_t)d.eC * vec;
    case RFAST_T_NODE: return (size_t)d.n * 4;
    case RFAST_TAU_R: case RFAST_SLOT_R: return (size_t)d.eR * 4;
    case RFAST_TAU_C: case RFAST_SLOT_C: return (size_t)d.eC * 4;
    case RFAST_ROUND: return 4;
    case RFAST_DELIV_R: return (size_t)d.eR * 8;
    case RFAST_DELIV_C: return (size_t)d.eC * 8;
    case RFAST_T_HIST: return (size_t)d.n * d.H * 4;
    case RFAST_SCHED_ACTIVE: return (size_t)d.n;
    case RFAST_SCHED_DELAY_R: return (size_t)d.eR * 4;
    case RFAST_SCHED_DELAY_C: return (size_t)d.eC * 4;
    case RFAST_SCHED_DROP_R: return (size_t)d.eR;
    case RFAST_SCHED_DROP_C: return (size_t)d.eC;
    case RFAST_SCHED_BATCH: return (size_t)d.n * (d.prob.kind == RFAST_OBJ_DIAG_QUADRATIC ? 0 : d.prob.batch) * 4;
    case RFAST_MOMENTUM: return d.mom ? d.n * vec : (size_t)-1;
    default: return (size_t)-1;
  }
}

// Ring slots whose version no receiver can pick up any more: stamps never go back, so a version older
// than every stamp held on its sender's out-edges (all versions, if the sender has none) is dead.  The
// kernels are free not to keep such slots up to date; reads of the ring fields return them as zeros.
// `ring` is a host copy of `rings` rings of [M][p] floats, ring q belonging to sender sender_of[q].
hipError_t zero_dead_slots(const rfast_ctx* c, bool sums, float* ring, int rings, const int32_t* sender_of) {
  const RfastDev& d = c->d;
  const int E = sums ? d.eC : d.eR;
  std::vector<int32_t> t(d.n), src(E), tau(E), lo(d.n, 0x7fffffff);
  hipError_t e = hipMemcpy(t.data(), d.t, (size_t)d.n * 4, hipMemcpyDeviceToHost);
  if (e == hipSuccess && E) e = hipMemcpy(src.data(), sums ? d.c_src : d.r_src, (size_t)E * 4, hipMemcpyDeviceToHost);
  if (e == hipSuccess && E) e = hipMemcpy(tau.data(), sums ? d.tau_c : d.tau_r, (size_t)E * 4, hipMemcpyDeviceToHost);
  if (e != hipSuccess) return e;
  for (int q = 0; q < E; ++q) lo[src[q]] = std::min(lo[src[q]], tau[q]);
  for (int q = 0; q < rings; ++q) {
    const int j = sender_of ? sender_of[q] : q;
    for (int m = 0; m < d.M; ++m) {
      const int back = ((t[j] - m) % d.M + d.M) % d.M, ver = t[j] - back;  // version held by slot m
      if (ver < lo[j]) memset(ring + ((size_t)q * d.M + m) * d.p, 0, (size_t)d.p * 4);
    }
  }
  return hipSuccess;
}

void time_begin(rfast_ctx* c, int which) {
  if (!c->profiling || c->ev_used[which] >= c->ev[which][0].size()) return;
  (void)hipEventRecord(c->ev[which][0][c->ev_used[which]], c->stream);
}
void time_end(rfast_ctx* c, int which) {
  if (!c->profiling || c->ev_used[which] >= c->ev[which][0].size()) return;
  (void)hipEventRecord(c->ev[which][1][c->ev_used[which]], c->stream);
  c->ev_used[which]++;
}

// the synchronous mode double-buffers z; bring it back into its own array before anything else looks at it
int fold_sync(rfast_ctx* c) {
  if (c->sync_parity == 0) return RFAST_OK;
  const hipError_t e = rfast_launch_sync(c, 3, 0.f, 1);
  if (e != hipSuccess) return hipfail(c, e, "fold launch");
  c->sync_parity = 0;
  return RFAST_OK;
}

constexpr int32_t kGraphRounds = 16;

// step size of round `round`: gamma * factor^(round div step_rounds)
float gamma_at(const rfast_ctx* c, float gamma, int64_t round) {
  if (c->gamma_step <= 0) return gamma;
  return gamma * powf(c->gamma_factor, (float)(round / c->gamma_step));
}
// ... of the round about to run
float gamma_now(const rfast_ctx* c, float gamma) { return gamma_at(c, gamma, c->host_round); }

void drop_graph(rfast_ctx* c) {
  if (c->graph_exec) (void)hipGraphExecDestroy(c->graph_exec);
  c->graph_exec = nullptr;
}

// automatic rebase of the running sums whenever the round counter reaches a multiple of
// `rebase_interval` (0 = never): a function of the round number, so a restored run repeats it
int after_round(rfast_ctx* c) {
  c->host_round++;
  if (c->rebase_interval > 0 && c->host_round % c->rebase_interval == 0) {
    const hipError_t e = rfast_launch_rebase(c);
    if (e != hipSuccess) return hipfail(c, e, "rebase launch");
  }
  return RFAST_OK;
}

}  // namespace

extern "C" int rfast_round(rfast_ctx* c, const uint8_t* d_active, const int32_t* d_delay_R, const int32_t* d_delay_C,
                           const uint8_t* d_drop_R, const uint8_t* d_drop_C, float gamma, const int32_t* d_batch_idx);

namespace {

// Captures kGraphRounds generated rounds on a private stream (capture is not allowed on
// the legacy default stream, which is what callers usually hand over) and instantiates them.
int build_graph(rfast_ctx* c, uint64_t seed, const float* d_p_active, int32_t max_delay, float p_drop, float gamma) {
  drop_graph(c);
  if (!c->capture_stream) {
    const hipError_t e = hipStreamCreateWithFlags(&c->capture_stream, hipStreamNonBlocking);
    if (e != hipSuccess) return hipfail(c, e, "hipStreamCreateWithFlags");
  }
  const RfastDev& d = c->d;
  hipStream_t user = c->stream;
  hipError_t e = hipStreamBeginCapture(c->capture_stream, hipStreamCaptureModeThreadLocal);
  if (e != hipSuccess) return hipfail(c, e, "hipStreamBeginCapture");
  c->stream = c->capture_stream;
  const int64_t round_before = c->host_round;  // capture enqueues nothing: the counter moves when the graph is launched
  int rc = RFAST_OK;
  for (int32_t r = 0; r < kGraphRounds && rc == RFAST_OK; ++r) {
    const hipError_t g = rfast_launch_generate(c, seed, d_p_active, max_delay, p_drop, false);
    if (g != hipSuccess) rc = hipfail(c, g, "schedule generator launch");
    else rc = rfast_round(c, d.gen_active, d.gen_delay_r, d.gen_delay_c, d.gen_drop_r, d.gen_drop_c, gamma, d.gen_batch);
  }
  c->stream = user;
  c->host_round = round_before;
  hipGraph_t graph = nullptr;
  e = hipStreamEndCapture(c->capture_stream, &graph);
  if (rc != RFAST_OK) {
    if (graph) (void)hipGraphDestroy(graph);
    return rc;
  }
  if (e != hipSuccess) return hipfail(c, e, "hipStreamEndCapture");
  e = hipGraphInstantiate(&c->graph_exec, graph, nullptr, nullptr, 0);
  (void)hipGraphDestroy(graph);
  if (e != hipSuccess) {
    c->graph_exec = nullptr;
    return hipfail(c, e, "hipGraphInstantiate");
  }
  c->graph_seed = seed;
  c->graph_p_active = d_p_active;
  c->graph_max_delay = max_delay;
  c->graph_p_drop = p_drop;
  c->graph_gamma = gamma_now(c, gamma);
  return RFAST_OK;
}

}  // namespace

extern "C" {

int rfast_common_roots(int32_t n, const int32_t* R_rowptr, const int32_t* R_col, const int32_t* C_rowptr,
                       const int32_t* C_col, uint8_t* host_is_root) {
  if (n < 1 || !R_rowptr || !R_col || !C_rowptr || !C_col) return fail(nullptr, RFAST_EINVAL, "NULL argument or n < 1");
  HostGraph g[2];
  const int32_t* ptrs[2] = {R_rowptr, C_rowptr};
  const int32_t* cols[2] = {R_col, C_col};
  for (int q = 0; q < 2; ++q) {
    if (ptrs[q][0] != 0) return fail(nullptr, RFAST_EGRAPH, "rowptr[0] != 0");
    g[q].ptr.assign(n + 1, 0);
    for (int i = 0; i < n; ++i) {
      if (ptrs[q][i + 1] < ptrs[q][i]) return fail(nullptr, RFAST_EGRAPH, "rowptr not monotone");
      for (int k = ptrs[q][i]; k < ptrs[q][i + 1]; ++k) {
        const int j = cols[q][k];
        if (j < 0 || j >= n) return fail(nullptr, RFAST_EGRAPH, "column index out of range");
        if (j != i) g[q].src.push_back(j);
      }
      g[q].ptr[i + 1] = (int32_t)g[q].src.size();
    }
  }
  const std::vector<char> rr = roots_of(n, g[0], true), rc = roots_of(n, g[1], false);
  int count = 0;
  for (int i = 0; i < n; ++i) {
    const bool both = rr[i] && rc[i];
    if (host_is_root) host_is_root[i] = both ? 1 : 0;
    count += both;
  }
  return count;
}

size_t rfast_workspace_bytes(int32_t n, int64_t p, int32_t nnzR, int32_t nnzC, int32_t D, const rfast_problem* prob) {
  if (!sizes_ok(n, p, nnzR, nnzC, D, prob)) return 0;
  return layout(n, p, nnzR, nnzC, D, prob).total;
}

int rfast_create(rfast_ctx** out, int32_t n, int64_t p, const int32_t* R_rowptr, const int32_t* R_col, const float* R_w,
                 const int32_t* C_rowptr, const int32_t* C_col, const float* C_w, int32_t D, int32_t burst,
                 const rfast_problem* prob, void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  if (out == nullptr) return fail(nullptr, RFAST_EINVAL, "out is NULL");
  *out = nullptr;
  if (!R_rowptr || !R_col || !R_w || !C_rowptr || !C_col || !C_w || !prob || !d_workspace)
    return fail(nullptr, RFAST_EINVAL, "NULL argument");
  if (n < 1 || n > 65535 || p < 1) return fail(nullptr, RFAST_EINVAL, "need 1 <= n <= 65535 and p >= 1");
  if (D < 0 || D + 2 > 64) return fail(nullptr, RFAST_ERANGE, "D + 2 must be in [2, 64]");
  if (burst < 1 || burst - 1 > D) return fail(nullptr, RFAST_ERANGE, "burst must be in [1, D+1]");
  const int32_t nnzR = R_rowptr[n], nnzC = C_rowptr[n];
  if (!sizes_ok(n, p, nnzR, nnzC, D, prob)) return fail(nullptr, RFAST_EINVAL, "sizes or problem description out of range");
  if (!prob->data0 || !prob->data1) return fail(nullptr, RFAST_EINVAL, "problem data pointers are NULL");
  if (((uintptr_t)d_workspace % kAlign) != 0) return fail(nullptr, RFAST_EINVAL, "workspace must be 256-byte aligned");
  if ((p % 4) == 0 && ((((uintptr_t)prob->data0) | ((uintptr_t)prob->data1)) % 16) != 0)
    return fail(nullptr, RFAST_EINVAL, "problem data must be 16-byte aligned");

  HostGraph gr, gc;
  std::string msg;
  int rc = split_graph("R", n, R_rowptr, R_col, R_w, true, &gr, &msg);
  if (rc != RFAST_OK) return fail(nullptr, rc, msg);
  rc = split_graph("C", n, C_rowptr, C_col, C_w, false, &gc, &msg);
  if (rc != RFAST_OK) return fail(nullptr, rc, msg);
  {
    // Assumption 2: G(R) and G(C^T) each contain a spanning tree and share a root.
    // In G(R) information flows sender -> receiver; in G(C^T) the edges of C are reversed.
    const std::vector<char> rr = roots_of(n, gr, true), rc2 = roots_of(n, gc, false);
    bool common = false;
    for (int i = 0; i < n; ++i) common = common || (rr[i] && rc2[i]);
    if (!common) return fail(nullptr, RFAST_EGRAPH, "G(R) and G(C^T) share no spanning-tree root (Assumption 2)");
  }
  const Offsets o = layout(n, p, nnzR, nnzC, D, prob);
  if (workspace_bytes < o.total)
    return fail(nullptr, RFAST_ENOMEM, "workspace too small: need " + std::to_string(o.total) + " bytes");

  rfast_ctx* c = new (std::nothrow) rfast_ctx();
  if (!c) return fail(nullptr, RFAST_ENOMEM, "host allocation failed");
  c->stream = (hipStream_t)hip_stream;
  c->nnzR = nnzR;
  c->nnzC = nnzC;
  char* b = (char*)d_workspace;
  RfastDev& d = c->d;
  d.n = n; d.p = p; d.M = D + 2; d.H = D + 1; d.eR = nnzR - n; d.eC = nnzC - n;
  d.burst = burst; d.d_max = D - (burst - 1);
  d.x = (float*)(b + o.x); d.z = (float*)(b + o.z); d.g = (float*)(b + o.g);
  d.v_ring = (float*)(b + o.v_ring); d.sigma_ring = (float*)(b + o.sigma_ring); d.rho_tilde = (float*)(b + o.rho_tilde);
  d.r_ptr = (int32_t*)(b + o.r_ptr); d.r_src = (int32_t*)(b + o.r_src); d.r_dst = (int32_t*)(b + o.r_dst); d.r_w = (float*)(b + o.r_w);
  d.r_self = (float*)(b + o.r_self);
  d.c_ptr = (int32_t*)(b + o.c_ptr); d.c_src = (int32_t*)(b + o.c_src); d.c_dst = (int32_t*)(b + o.c_dst); d.c_w = (float*)(b + o.c_w); d.c_self = (float*)(b + o.c_self);
  d.co_ptr = (int32_t*)(b + o.co_ptr); d.co_eid = (int32_t*)(b + o.co_eid); d.co_w = (float*)(b + o.co_w);
  d.ro_ptr = (int32_t*)(b + o.ro_ptr); d.ro_eid = (int32_t*)(b + o.ro_eid);
  d.t = (int32_t*)(b + o.t); d.t_hist = (int32_t*)(b + o.t_hist);
  d.tau_r = (int32_t*)(b + o.tau_r); d.tau_c = (int32_t*)(b + o.tau_c);
  d.deliv_r = (unsigned long long*)(b + o.deliv_r); d.deliv_c = (unsigned long long*)(b + o.deliv_c);
  d.round_no = (int32_t*)(b + o.round_no); d.err = (int32_t*)(b + o.err);
  d.n_active = (int32_t*)(b + o.n_active); d.active_plan = (int2*)(b + o.active_plan);
  d.plan_t = (int32_t*)(b + o.plan_t); d.slot_r = (int32_t*)(b + o.slot_r); d.slot_c = (int32_t*)(b + o.slot_c);
  d.plan_c = (int32_t*)(b + o.plan_c); d.node_spill = (uint8_t*)(b + o.node_spill);
  d.blk_plan = nullptr;
  d.blk_head = nullptr;
  c->blk_plan_base = (int32_t*)(b + o.blk_plan);
  c->blk_head_base = (int32_t*)(b + o.blk_head);
  c->plan_set0 = b + o.n_active;
  c->plan_set_bytes = o.plan_set_bytes;
  c->plan_set = 0;
  d.gen_active = (uint8_t*)(b + o.gen_active); d.gen_delay_r = (int32_t*)(b + o.gen_delay_r);
  d.gen_delay_c = (int32_t*)(b + o.gen_delay_c); d.gen_drop_r = (uint8_t*)(b + o.gen_drop_r);
  d.gen_drop_c = (uint8_t*)(b + o.gen_drop_c); d.gen_batch = (int32_t*)(b + o.gen_batch);
  d.gen_cdf = (uint32_t*)(b + o.gen_cdf);
  c->gen_depth = o.gen_depth;
  d.xbar = (float*)(b + o.xbar);
  d.mom = nullptr; d.beta = 0.f; d.wd = 0.f;
  d.resid = (float*)(b + o.resid); d.gscratch = (void*)(b + o.gscratch);
  c->d_diag = (double*)(b + o.diag);
  d.prob = *prob;

  hipError_t e = rfast_static_scratch_init();  // for rfast_diagnostics_static, which may not look anything up later
  auto chk = [&](hipError_t r) { if (e == hipSuccess) e = r; };
  chk(upload(c, b, o.r_ptr, gr.ptr)); chk(upload(c, b, o.r_src, gr.src)); chk(upload(c, b, o.r_dst, gr.dst)); chk(upload(c, b, o.r_w, gr.w));
  chk(upload(c, b, o.r_self, gr.self));
  chk(upload(c, b, o.c_ptr, gc.ptr)); chk(upload(c, b, o.c_src, gc.src)); chk(upload(c, b, o.c_dst, gc.dst)); chk(upload(c, b, o.c_w, gc.w)); chk(upload(c, b, o.c_self, gc.self));
  chk(upload(c, b, o.co_ptr, gc.out_ptr)); chk(upload(c, b, o.co_eid, gc.out_eid)); chk(upload(c, b, o.co_w, gc.out_w));
  chk(upload(c, b, o.ro_ptr, gr.out_ptr)); chk(upload(c, b, o.ro_eid, gr.out_eid));
  for (int i = 0; i < n; ++i)
    c->max_degree = std::max({c->max_degree, gr.ptr[i + 1] - gr.ptr[i], gc.ptr[i + 1] - gc.ptr[i], gc.out_ptr[i + 1] - gc.out_ptr[i]});
  chk(rfast_wave_prime(c));
  chk(hipStreamSynchronize(c->stream));  // the host vectors die with this scope
  if (e != hipSuccess) {
    const int r = hipfail(nullptr, e, "uploading graph");
    delete c;
    return r;
  }
  *out = c;
  return RFAST_OK;
}

int rfast_init(rfast_ctx* c, const float* d_x0, const int32_t* d_batch_idx0) {
  if (!c) return RFAST_EINVAL;
  RfastDev& d = c->d;
  if (d.prob.kind != RFAST_OBJ_DIAG_QUADRATIC && d.prob.batch > 0 && !d_batch_idx0)
    return fail(c, RFAST_EINVAL, "initial sample rows are required when batch > 0");
  const size_t vec = (size_t)d.p * 4;
  c->sync_parity = 0;
  c->host_round = 0;
  c->needs_init = false;
  hipError_t e = hipSuccess;
  auto chk = [&](hipError_t r) { if (e == hipSuccess) e = r; };
  if (d.mom) chk(hipMemsetAsync(d.mom, 0, d.n * vec, c->stream));
  if (d_x0) chk(hipMemcpyAsync(d.x, d_x0, d.n * vec, hipMemcpyDeviceToDevice, c->stream));
  else chk(hipMemsetAsync(d.x, 0, d.n * vec, c->stream));
  chk(hipMemsetAsync(d.g, 0, 2 * d.n * vec, c->stream));
  chk(hipMemsetAsync(d.v_ring, 0, (size_t)d.n * d.M * vec, c->stream));
  chk(hipMemsetAsync(d.sigma_ring, 0, (size_t)d.n * d.M * vec, c->stream));
  if (d.eC) {
    chk(hipMemsetAsync(d.rho_tilde, 0, (size_t)d.eC * vec, c->stream));
    chk(hipMemsetAsync(d.tau_c, 0, (size_t)d.eC * 4, c->stream));
    chk(hipMemsetAsync(d.slot_c, 0xff, (size_t)d.eC * 4, c->stream));
    chk(hipMemsetAsync(d.plan_c, 0, (size_t)d.eC * 4, c->stream));
    // only version 0 (slot 0) counts as delivered
    chk(hipMemsetAsync(d.deliv_c, 0, (size_t)d.eC * 8, c->stream));
  }
  if (d.eR) {
    chk(hipMemsetAsync(d.tau_r, 0, (size_t)d.eR * 4, c->stream));
    chk(hipMemsetAsync(d.slot_r, 0xff, (size_t)d.eR * 4, c->stream));
    chk(hipMemsetAsync(d.deliv_r, 0, (size_t)d.eR * 8, c->stream));
  }
  chk(hipMemsetAsync(d.t, 0, (size_t)d.n * 4, c->stream));
  chk(hipMemsetAsync(d.t_hist, 0, (size_t)d.n * d.H * 4, c->stream));
  chk(hipMemsetAsync(d.plan_t, 0, (size_t)d.n * 4, c->stream));
  chk(hipMemsetAsync(d.round_no, 0, 4, c->stream));
  chk(hipMemsetAsync(d.err, 0, 16, c->stream));
  chk(hipMemsetAsync(d.n_active, 0, 8, c->stream));
  if (e != hipSuccess) return hipfail(c, e, "rfast_init clears");
  e = rfast_launch_init_grad(c, d_batch_idx0);
  if (e != hipSuccess) return hipfail(c, e, "initial gradient");
  return RFAST_OK;
}

// Points the per-round plan arrays of c->d at set q (the resolver writes the rounds it takes in one
// launch into consecutive sets; the kernels of a round read the set of that round).
static void use_plan_set(rfast_ctx* c, int32_t q) {
  RfastDev& d = c->d;
  const ptrdiff_t shift = (ptrdiff_t)(q - c->plan_set) * (ptrdiff_t)c->plan_set_bytes;
  auto move = [shift](auto*& ptr) { ptr = reinterpret_cast<std::remove_reference_t<decltype(ptr)>>(reinterpret_cast<char*>(ptr) + shift); };
  move(d.n_active); move(d.active_plan); move(d.plan_t); move(d.slot_r); move(d.slot_c); move(d.plan_c); move(d.node_spill);
  c->plan_set = q;
}

static int check_round_args(rfast_ctx* c, const uint8_t* d_active, const int32_t* d_delay_R, const int32_t* d_delay_C,
                            const uint8_t* d_drop_R, const uint8_t* d_drop_C, float gamma, const int32_t* d_batch_idx) {
  const RfastDev& d = c->d;
  if (!d_active || (d.eR && (!d_delay_R || !d_drop_R)) || (d.eC && (!d_delay_C || !d_drop_C)))
    return fail(c, RFAST_EINVAL, "NULL schedule pointer");
  const bool separable = d.prob.kind == RFAST_OBJ_DIAG_QUADRATIC;
  if (!separable && d.prob.batch > 0 && !d_batch_idx) return fail(c, RFAST_EINVAL, "sample rows are required when batch > 0");
  if (!std::isfinite(gamma)) return fail(c, RFAST_EINVAL, "gamma is not finite");
  if (c->needs_init) return fail(c, RFAST_EINVAL, "rfast_init must follow rfast_set_optimizer");
  return RFAST_OK;
}

static int float_round(rfast_ctx* c, float gamma, const int32_t* d_batch_idx);

int rfast_round(rfast_ctx* c, const uint8_t* d_active, const int32_t* d_delay_R, const int32_t* d_delay_C,
                const uint8_t* d_drop_R, const uint8_t* d_drop_C, float gamma, const int32_t* d_batch_idx) {
  if (!c) return RFAST_EINVAL;
  const int rc = check_round_args(c, d_active, d_delay_R, d_delay_C, d_drop_R, d_drop_C, gamma, d_batch_idx);
  if (rc != RFAST_OK) return rc;
  if (fold_sync(c) != RFAST_OK) return RFAST_EHIP;
  time_begin(c, 2);
  const hipError_t e = rfast_launch_resolve(c, d_active, d_delay_R, d_delay_C, d_drop_R, d_drop_C);
  time_end(c, 2);
  if (e != hipSuccess) return hipfail(c, e, "resolver launch");
  return float_round(c, gamma, d_batch_idx);
}

// The floating-point part of a round whose plan the resolver has written into the current plan set.
static int float_round(rfast_ctx* c, float gamma, const int32_t* d_batch_idx) {
  const bool separable = c->d.prob.kind == RFAST_OBJ_DIAG_QUADRATIC;
  gamma = gamma_now(c, gamma);
  hipError_t e;
  if (separable) {
    time_begin(c, 0);
    e = rfast_launch_state(c, RFAST_MODE_FUSED, gamma);
    time_end(c, 0);
    if (e != hipSuccess) return hipfail(c, e, "fused round launch");
    return after_round(c);
  }
  time_begin(c, 0);
  e = rfast_launch_state(c, RFAST_MODE_MIX, gamma);
  time_end(c, 0);
  if (e != hipSuccess) return hipfail(c, e, "mix launch");
  time_begin(c, 1);
  e = rfast_launch_gradient(c, d_batch_idx);
  time_end(c, 1);
  if (e != hipSuccess) return hipfail(c, e, "gradient launch");
  time_begin(c, 0);
  e = rfast_launch_state(c, RFAST_MODE_TRACK, gamma);
  time_end(c, 0);
  if (e != hipSuccess) return hipfail(c, e, "track launch");
  return after_round(c);
}

// `count` consecutive rounds of least squares or logistic regression whose plans the resolver has written into plan
// sets 0 .. count-1: two kernels per round instead of four (the lane that tracks a coordinate in one round mixes it for
// the next).  d_active, d_batch_idx: the activity flags and the rows of the first of these rounds, those of the others
// behind them.
static int chained_rounds(rfast_ctx* c, int32_t count, float gamma, const uint8_t* d_active, const int32_t* d_batch_idx) {
  const RfastDev& d = c->d;
  const size_t rows = (size_t)d.n * (size_t)d.prob.batch;
  use_plan_set(c, 0);
  time_begin(c, 0);
  hipError_t e = rfast_launch_state(c, RFAST_MODE_MIX, gamma_now(c, gamma));
  time_end(c, 0);
  if (e != hipSuccess) return hipfail(c, e, "mix launch");
  for (int32_t q = 0; q < count; ++q) {
    use_plan_set(c, q);
    const int32_t* bi = d_batch_idx ? d_batch_idx + (size_t)q * rows : nullptr;
    const uint8_t* act = d_active + (size_t)q * d.n;
    time_begin(c, 1);
    e = rfast_launch_rows(c, bi, act);
    time_end(c, 1);
    if (e != hipSuccess) return hipfail(c, e, "rows launch");
    time_begin(c, 0);
    e = rfast_launch_cols_track_mix(c, bi, act, q + 1 < count ? act + d.n : nullptr, c->plan_set_bytes,
                                    gamma_at(c, gamma, c->host_round + 1));
    time_end(c, 0);
    if (e != hipSuccess) return hipfail(c, e, "columns, track and mix launch");
    const int rc = after_round(c);
    if (rc != RFAST_OK) return rc;
  }
  return RFAST_OK;
}

// How many of the next `rounds` rounds one launch of the LDS-resident kernel should take (0: run
// the next round as one pass).  A launch holds no rebase, so it must end at the latest on the next
// multiple of the rebase interval, and it runs with one step size, so it must end with the current
// step of the step-size schedule; and it reads and writes every ring slot once, which a large
// state earns back only over enough rounds.
static int32_t block_length(const rfast_ctx* c, int32_t rounds, int64_t at_round = -1) {
  if (!c->use_blocks || !(rfast_wave_eligible(c) || rfast_block_eligible(c) || rfast_tiny_eligible(c))) return 0;
  const int64_t now = at_round >= 0 ? at_round : c->host_round;  // the round the launch would start with
  int32_t len = rounds < kBlockRounds ? rounds : kBlockRounds;
  if (c->rebase_interval > 0) {
    const int64_t to_boundary = c->rebase_interval - now % c->rebase_interval;
    if (to_boundary < len) len = (int32_t)to_boundary;
  }
  if (c->gamma_step > 0) {  // one step size per launch
    const int64_t to_decay = c->gamma_step - now % c->gamma_step;
    if (to_decay < len) len = (int32_t)to_decay;
  }
  const bool large = (double)c->d.n * (double)c->d.p * 4.0 > 8.0e6;
  return len >= (large && c->use_blocks != 2 ? kBlockMinRoundsLarge : 2) ? len : 0;
}

// Resolves `len` rounds (schedule arrays of round q at offset q of each pointer) into plan records,
// one launch, and advances them with one launch.
static int run_block(rfast_ctx* c, int32_t len, const uint8_t* d_active, const int32_t* d_delay_R,
                     const int32_t* d_delay_C, const uint8_t* d_drop_R, const uint8_t* d_drop_C, float gamma,
                     const int32_t* d_batch_idx) {
  RfastDev& d = c->d;
  if (fold_sync(c) != RFAST_OK) return RFAST_EHIP;
  RfastBlock blk;
  blk.rounds = len;
  // a rebase that falls due when these rounds are done costs the wavefront-tile kernel nothing: it shifts the
  // running sums while it writes its tiles back (the other kernel is followed by the rebase kernel)
  const bool rebase_due = c->rebase_interval > 0 && (c->host_round + len) % c->rebase_interval == 0;
  blk.rebase = rebase_due && rfast_wave_eligible(c) ? 1 : 0;
  blk.gamma = gamma_now(c, gamma);  // of the first round: a launch does not straddle a decay step
  const bool own_resolver = rfast_tiny_resolves(c);  // the one-workgroup kernel resolves its rounds itself
  hipError_t e = hipSuccess;
  d.blk_plan = c->blk_plan_base;
  d.blk_head = c->blk_head_base;
  if (!own_resolver) {
    time_begin(c, 2);
    e = rfast_launch_resolve(c, d_active, d_delay_R, d_delay_C, d_drop_R, d_drop_C, len);
    time_end(c, 2);
  }
  c->host_round += len;
  if (e == hipSuccess) {
    time_begin(c, 0);
    if (rfast_tiny_eligible(c))
      e = rfast_launch_tiny(c, blk, d_batch_idx, (int)(c->host_round - len), d_active, d_delay_R, d_delay_C, d_drop_R, d_drop_C);
    else e = rfast_wave_eligible(c) ? rfast_launch_wave(c, blk) : rfast_launch_block(c, blk);
    time_end(c, 0);
  }
  d.blk_plan = nullptr;
  d.blk_head = nullptr;
  if (e != hipSuccess) return hipfail(c, e, "multi-round launch");
  if (rebase_due && !blk.rebase) {
    e = rfast_launch_rebase(c);
    if (e != hipSuccess) return hipfail(c, e, "rebase launch");
  }
  return RFAST_OK;
}

int rfast_block_info(rfast_ctx* c, int32_t* lanes_per_node, int32_t* tile_per_wavefront) {
  if (!c || !lanes_per_node) return RFAST_EINVAL;
  const bool taken = block_length(c, kBlockRounds) > 0, wave = rfast_wave_eligible(c);
  if (taken && rfast_tiny_eligible(c)) {  // one workgroup holds the whole problem
    *lanes_per_node = 1024 / c->d.n > 0 ? 1024 / c->d.n : 1;
    if (tile_per_wavefront) *tile_per_wavefront = 0;
    return RFAST_OK;
  }
  *lanes_per_node = taken ? (wave ? rfast_wave_lanes(c) : rfast_block_lanes(c)) : 0;
  if (tile_per_wavefront) *tile_per_wavefront = taken && wave ? 1 : 0;
  return RFAST_OK;
}

int rfast_set_tile_group(rfast_ctx* c, int32_t wavefronts) {
  if (!c) return RFAST_EINVAL;
  if (wavefronts != 0 && wavefronts != 1 && wavefronts != 2 && wavefronts != 4)
    return fail(c, RFAST_EINVAL, "wavefronts per workgroup must be 0 (automatic), 1, 2 or 4");
  c->wave_group = wavefronts;
  return RFAST_OK;
}

int rfast_use_blocks(rfast_ctx* c, int32_t on) {
  if (!c) return RFAST_EINVAL;
  c->use_blocks = on == 2 ? 2 : (on != 0 ? 1 : 0);
  return RFAST_OK;
}

int rfast_run(rfast_ctx* c, int32_t rounds, const uint8_t* d_active, const int32_t* d_delay_R, const int32_t* d_delay_C,
              const uint8_t* d_drop_R, const uint8_t* d_drop_C, float gamma, const int32_t* d_batch_idx) {
  if (!c) return RFAST_EINVAL;
  if (rounds < 0) return fail(c, RFAST_EINVAL, "rounds < 0");
  const RfastDev& d = c->d;
  const size_t B = d.prob.kind == RFAST_OBJ_DIAG_QUADRATIC ? 0 : (size_t)d.prob.batch;
  for (int32_t r = 0; r < rounds; ++r) {
    // the separable objective on a small graph: tiles of coordinates stay in LDS over up to kBlockRounds rounds
    const int32_t len = block_length(c, rounds - r);
    if (len > 0) {
      if (!d_active || (d.eR && (!d_delay_R || !d_drop_R)) || (d.eC && (!d_delay_C || !d_drop_C)))
        return fail(c, RFAST_EINVAL, "NULL schedule pointer");
      if (!std::isfinite(gamma)) return fail(c, RFAST_EINVAL, "gamma is not finite");
      if (c->needs_init) return fail(c, RFAST_EINVAL, "rfast_init must follow rfast_set_optimizer");
      if (B > 0 && !d_batch_idx) return fail(c, RFAST_EINVAL, "sample rows are required when batch > 0");
      const int rc = run_block(c, len, d_active + (size_t)r * d.n, d_delay_R ? d_delay_R + (size_t)r * d.eR : nullptr,
                               d_delay_C ? d_delay_C + (size_t)r * d.eC : nullptr,
                               d_drop_R ? d_drop_R + (size_t)r * d.eR : nullptr,
                               d_drop_C ? d_drop_C + (size_t)r * d.eC : nullptr, gamma,
                               d_batch_idx ? d_batch_idx + (size_t)r * d.n * B : nullptr);
      if (rc != RFAST_OK) return rc;
      r += len - 1;
      continue;
    }
    // One pass per round: the resolver takes up to kResolveAhead rounds in one launch, into as many
    // plan sets (integer state only, so it may run ahead of the kernels); a stretch ends where a
    // multi-round launch may start and, because the rebase reads the counters, on the multiples of
    // the rebase interval.
    int32_t ahead = rounds - r < kResolveAhead ? rounds - r : kResolveAhead;
    for (int32_t q = 1; q < ahead; ++q) {
      const int64_t then = c->host_round + q;
      const bool boundary = c->rebase_interval > 0 && then % c->rebase_interval == 0;
      if (boundary || block_length(c, rounds - r - q, then) > 0) { ahead = q; break; }
    }
    int rc = check_round_args(c, d_active + (size_t)r * d.n, d_delay_R, d_delay_C, d_drop_R, d_drop_C, gamma, d_batch_idx);
    if (rc != RFAST_OK) return rc;
    if (fold_sync(c) != RFAST_OK) return RFAST_EHIP;
    use_plan_set(c, 0);
    time_begin(c, 2);
    const hipError_t e = rfast_launch_resolve(c, d_active + (size_t)r * d.n, d_delay_R ? d_delay_R + (size_t)r * d.eR : nullptr,
                                              d_delay_C ? d_delay_C + (size_t)r * d.eC : nullptr,
                                              d_drop_R ? d_drop_R + (size_t)r * d.eR : nullptr,
                                              d_drop_C ? d_drop_C + (size_t)r * d.eC : nullptr, ahead, c->plan_set_bytes);
    time_end(c, 2);
    if (e != hipSuccess) return hipfail(c, e, "resolver launch");
    if (c->use_blocks && rfast_chain_eligible(c)) {
      rc = chained_rounds(c, ahead, gamma, d_active + (size_t)r * d.n, d_batch_idx ? d_batch_idx + (size_t)r * d.n * B : nullptr);
      if (rc != RFAST_OK) return rc;
    } else {
      for (int32_t q = 0; q < ahead; ++q) {
        use_plan_set(c, q);
        rc = float_round(c, gamma, d_batch_idx ? d_batch_idx + (size_t)(r + q) * d.n * B : nullptr);
        if (rc != RFAST_OK) return rc;
      }
    }
    r += ahead - 1;
  }
  return RFAST_OK;
}

int rfast_use_graphs(rfast_ctx* c, int32_t on) {
  if (!c) return RFAST_EINVAL;
  c->use_graphs = on != 0;
  if (!on) drop_graph(c);
  return RFAST_OK;
}

int rfast_run_generated(rfast_ctx* c, int32_t rounds, uint64_t seed, const float* d_p_active, int32_t max_delay,
                        float p_drop, float gamma) {
  if (!c || !d_p_active) return RFAST_EINVAL;
  if (rounds < 0) return fail(c, RFAST_EINVAL, "rounds < 0");
  const RfastDev& d = c->d;
  if (max_delay < 0 || max_delay > d.d_max) return fail(c, RFAST_ERANGE, "max_delay must lie in [0, D - burst + 1]");
  if (!(p_drop >= 0.f && p_drop <= 1.f)) return fail(c, RFAST_ERANGE, "p_drop must lie in [0, 1]");
  if (!std::isfinite(gamma)) return fail(c, RFAST_EINVAL, "gamma is not finite");
  // A generated round takes no host argument that varies from round to round (the
  // generator reads the round number on the device), so kGraphRounds of them are
  // captured once into a HIP graph and replayed: one launch per kGraphRounds rounds.
  if (c->needs_init) return fail(c, RFAST_EINVAL, "rfast_init must follow rfast_set_optimizer");
  const bool graphs = c->use_graphs && !c->profiling;
  while (rounds > 0) {
    // a graph bakes the step size in, so a replay must not straddle a decay step of the schedule,
    // and it must hold no rebase, so it must end before the next multiple of the rebase interval
    const bool one_step_size = c->gamma_step <= 0 || c->host_round % c->gamma_step + kGraphRounds <= c->gamma_step;
    const bool no_rebase_inside =
        c->rebase_interval <= 0 || c->host_round % c->rebase_interval + kGraphRounds < c->rebase_interval;
    if (graphs && rounds >= kGraphRounds && one_step_size && no_rebase_inside) {
      if (fold_sync(c) != RFAST_OK) return RFAST_EHIP;
      const bool same = c->graph_exec && c->graph_seed == seed && c->graph_p_active == d_p_active &&
                        c->graph_max_delay == max_delay && c->graph_p_drop == p_drop && c->graph_gamma == gamma_now(c, gamma);
      if (!same) {
        const int rc = build_graph(c, seed, d_p_active, max_delay, p_drop, gamma);
        if (rc != RFAST_OK) return rc;
      }
      const hipError_t e = hipGraphLaunch(c->graph_exec, c->stream);
      if (e != hipSuccess) return hipfail(c, e, "hipGraphLaunch");
      c->host_round += kGraphRounds;
      c->gen_last = 0;
      rounds -= kGraphRounds;
      continue;
    }
    // no replay: the schedule of the next stretch of rounds in one launch, then as an uploaded one
    // (several rounds per launch where that applies, else the resolver ahead of the round kernels)
    int32_t len = rounds < c->gen_depth ? rounds : c->gen_depth;
    if (graphs && len > kGraphRounds) len = kGraphRounds;  // a replay may become possible again after a boundary
    const hipError_t e = rfast_launch_generate(c, seed, d_p_active, max_delay, p_drop, false, len);
    if (e != hipSuccess) return hipfail(c, e, "schedule generator launch");
    const int rc = rfast_run(c, len, d.gen_active, d.gen_delay_r, d.gen_delay_c, d.gen_drop_r, d.gen_drop_c, gamma, d.gen_batch);
    if (rc != RFAST_OK) return rc;
    c->gen_last = len - 1;
    rounds -= len;
  }
  return RFAST_OK;
}

int rfast_run_events(rfast_ctx* c, int32_t iterations, uint64_t seed, const float* host_weights, int32_t max_delay,
                     float p_drop, float gamma) {
  if (!c) return RFAST_EINVAL;
  if (iterations < 0) return fail(c, RFAST_EINVAL, "iterations < 0");
  const RfastDev& d = c->d;
  if (max_delay < 0 || max_delay > d.d_max) return fail(c, RFAST_ERANGE, "max_delay must lie in [0, D - burst + 1]");
  if (!(p_drop >= 0.f && p_drop <= 1.f)) return fail(c, RFAST_ERANGE, "p_drop must lie in [0, 1]");
  if (!std::isfinite(gamma)) return fail(c, RFAST_EINVAL, "gamma is not finite");
  if (c->needs_init) return fail(c, RFAST_EINVAL, "rfast_init must follow rfast_set_optimizer");
  // selection thresholds: node i is drawn when cdf[i-1] <= u < cdf[i], u a 32-bit word
  std::vector<uint32_t> cdf(d.n);
  double total = 0.0;
  for (int i = 0; i < d.n; ++i) {
    const double w = host_weights ? (double)host_weights[i] : 1.0;
    if (!(w >= 0.0) || !std::isfinite(w)) return fail(c, RFAST_ERANGE, "selection weights must be finite and >= 0");
    total += w;
  }
  if (!(total > 0.0)) return fail(c, RFAST_ERANGE, "selection weights sum to zero");
  double cum = 0.0;
  for (int i = 0; i < d.n; ++i) {
    cum += host_weights ? (double)host_weights[i] : 1.0;
    const double thr = std::floor(cum / total * 4294967296.0);
    cdf[i] = thr >= 4294967295.0 ? 0xFFFFFFFFu : (uint32_t)thr;
  }
  hipError_t e = hipMemcpyAsync(d.gen_cdf, cdf.data(), (size_t)d.n * 4, hipMemcpyHostToDevice, c->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(c->stream);  // the host vector dies with this scope
  if (e != hipSuccess) return hipfail(c, e, "uploading selection thresholds");
  // A stretch of iterations drawn by one launch, then one pass per iteration with the resolver ahead (a
  // multi-round launch, where one lane in n would work, is not what a single activation wants).
  const int32_t blocks = c->use_blocks;
  c->use_blocks = 0;
  int rc = RFAST_OK;
  for (int32_t k = 0; k < iterations && rc == RFAST_OK;) {
    const int32_t len = iterations - k < c->gen_depth ? iterations - k : c->gen_depth;
    e = rfast_launch_generate(c, seed, nullptr, max_delay, p_drop, true, len);
    if (e != hipSuccess) {
      rc = hipfail(c, e, "schedule generator launch");
      break;
    }
    rc = rfast_run(c, len, d.gen_active, d.gen_delay_r, d.gen_delay_c, d.gen_drop_r, d.gen_drop_c, gamma, d.gen_batch);
    c->gen_last = len - 1;
    k += len;
  }
  c->use_blocks = blocks;
  return rc;
}

int rfast_sync_round(rfast_ctx* c, float gamma, const int32_t* d_batch_idx) {
  if (!c) return RFAST_EINVAL;
  const RfastDev& d = c->d;
  const bool separable = d.prob.kind == RFAST_OBJ_DIAG_QUADRATIC;
  if (!separable && d.prob.batch > 0 && !d_batch_idx) return fail(c, RFAST_EINVAL, "sample rows are required when batch > 0");
  if (!std::isfinite(gamma)) return fail(c, RFAST_EINVAL, "gamma is not finite");
  if (c->needs_init) return fail(c, RFAST_EINVAL, "rfast_init must follow rfast_set_optimizer");
  gamma = gamma_now(c, gamma);
  hipError_t e;
  time_begin(c, 0);
  e = rfast_launch_sync(c, separable ? 2 : 0, gamma, c->sync_parity);
  time_end(c, 0);
  if (e != hipSuccess) return hipfail(c, e, "synchronous step launch");
  if (!separable) {
    time_begin(c, 1);
    e = rfast_launch_gradient(c, d_batch_idx);
    time_end(c, 1);
    if (e != hipSuccess) return hipfail(c, e, "gradient launch");
    time_begin(c, 0);
    e = rfast_launch_sync(c, 1, gamma, c->sync_parity);
    time_end(c, 0);
    if (e != hipSuccess) return hipfail(c, e, "synchronous tracker launch");
  }
  c->sync_parity ^= 1;
  c->host_round++;
  return RFAST_OK;
}

int rfast_sync_run(rfast_ctx* c, int32_t rounds, float gamma, const int32_t* d_batch_idx) {
  if (!c) return RFAST_EINVAL;
  if (rounds < 0) return fail(c, RFAST_EINVAL, "rounds < 0");
  const RfastDev& d = c->d;
  const size_t B = d.prob.kind == RFAST_OBJ_DIAG_QUADRATIC ? 0 : (size_t)d.prob.batch;
  const bool multi = c->use_blocks && rfast_sync_wave_eligible(c);
  const bool large = (double)d.n * (double)d.p * 4.0 > 8.0e6;
  for (int32_t r = 0; r < rounds;) {
    // several steps per launch for the separable objective on a small graph, with one step size
    int32_t len = multi ? rounds - r : 0;
    if (len > 0 && c->gamma_step > 0) {
      const int64_t to_decay = c->gamma_step - c->host_round % c->gamma_step;
      if (to_decay < len) len = (int32_t)to_decay;
    }
    if (len >= (large && c->use_blocks != 2 ? kBlockMinRoundsLarge : 2)) {
      if (!std::isfinite(gamma)) return fail(c, RFAST_EINVAL, "gamma is not finite");
      if (c->needs_init) return fail(c, RFAST_EINVAL, "rfast_init must follow rfast_set_optimizer");
      if (fold_sync(c) != RFAST_OK) return RFAST_EHIP;
      time_begin(c, 0);
      hipError_t e = rfast_launch_sync_wave(c, gamma_now(c, gamma), len);
      time_end(c, 0);
      if (e == hipSuccess) e = rfast_launch_sync_plan(c, len);
      if (e != hipSuccess) return hipfail(c, e, "multi-step synchronous launch");
      c->host_round += len;
      r += len;
      continue;
    }
    const int rc = rfast_sync_round(c, gamma, d_batch_idx ? d_batch_idx + (size_t)r * d.n * B : nullptr);
    if (rc != RFAST_OK) return rc;
    ++r;
  }
  return RFAST_OK;
}

int rfast_set_optimizer(rfast_ctx* c, float momentum, float weight_decay, float* d_momentum) {
  if (!c) return RFAST_EINVAL;
  if (!(momentum >= 0.f && momentum < 1.f)) return fail(c, RFAST_ERANGE, "momentum must lie in [0, 1)");
  if (!(weight_decay >= 0.f) || !std::isfinite(weight_decay)) return fail(c, RFAST_ERANGE, "weight_decay must be finite and >= 0");
  if (momentum != 0.f && !d_momentum) return fail(c, RFAST_EINVAL, "momentum != 0 needs a buffer of n*p floats");
  if (d_momentum && ((uintptr_t)d_momentum % 16) != 0) return fail(c, RFAST_EINVAL, "momentum buffer must be 16-byte aligned");
  drop_graph(c);  // a captured graph holds the old kernel arguments
  c->d.beta = momentum;
  c->d.wd = weight_decay;
  c->d.mom = momentum != 0.f ? d_momentum : nullptr;
  c->needs_init = true;
  const hipError_t e = rfast_wave_prime(c);  // the variant has instantiations of its own
  if (e != hipSuccess) return hipfail(c, e, "loading the multi-round kernel");
  return RFAST_OK;
}

int rfast_set_gamma_schedule(rfast_ctx* c, int32_t step_rounds, float factor) {
  if (!c) return RFAST_EINVAL;
  if (step_rounds < 0) return fail(c, RFAST_EINVAL, "step_rounds < 0");
  if (!(factor > 0.f) || !std::isfinite(factor)) return fail(c, RFAST_ERANGE, "factor must be finite and > 0");
  c->gamma_step = step_rounds;
  c->gamma_factor = factor;
  return RFAST_OK;
}

int rfast_set_rebase_interval(rfast_ctx* c, int32_t rounds) {
  if (!c || rounds < 0) return RFAST_EINVAL;
  c->rebase_interval = rounds;
  return RFAST_OK;
}

int rfast_rebase(rfast_ctx* c) {
  if (!c) return RFAST_EINVAL;
  const hipError_t e = rfast_launch_rebase(c);
  if (e != hipSuccess) return hipfail(c, e, "rebase launch");
  return RFAST_OK;
}

int rfast_check(rfast_ctx* c) {
  if (!c) return RFAST_EINVAL;
  hipError_t e = hipStreamSynchronize(c->stream);
  if (e != hipSuccess) return hipfail(c, e, "stream synchronize");
  int32_t err[4];
  e = hipMemcpy(err, c->d.err, 16, hipMemcpyDeviceToHost);
  if (e != hipSuccess) return hipfail(c, e, "reading device status");
  if (err[0] == 0) return RFAST_OK;
  static const char* kinds[] = {"delay on R edge", "delay on C edge", "sample row of node", "class label of a sample of node"};
  const char* what = err[2] >= 0 && err[2] <= 3 ? kinds[err[2]] : "value";
  return fail(c, err[0], std::string(what) + " " + std::to_string(err[3]) + " out of range in round " + std::to_string(err[1]) +
                             " (clamped on the device)");
}

int rfast_read_state(rfast_ctx* c, int32_t field, void* host_dst, size_t bytes) {
  if (!c || !host_dst) return RFAST_EINVAL;
  const size_t want = field_bytes(c, field);
  if (want == (size_t)-1) return fail(c, RFAST_EINVAL, "unknown field");
  if (bytes != want) return fail(c, RFAST_EINVAL, "field holds " + std::to_string(want) + " bytes");
  const RfastDev& d = c->d;
  if (fold_sync(c) != RFAST_OK) return RFAST_EHIP;
  hipError_t e = hipStreamSynchronize(c->stream);
  if (e != hipSuccess) return hipfail(c, e, "stream synchronize");
  if (bytes == 0) return RFAST_OK;
  const void* src = nullptr;
  switch (field) {
    case RFAST_X: src = d.x; break;
    case RFAST_Z: src = d.z; break;
    case RFAST_V_RING: src = d.v_ring; break;
    case RFAST_SIGMA_RING: src = d.sigma_ring; break;
    case RFAST_RHO_TILDE: src = d.rho_tilde; break;
    case RFAST_T_NODE: src = d.t; break;
    case RFAST_TAU_R: src = d.tau_r; break;
    case RFAST_TAU_C: src = d.tau_c; break;
    case RFAST_SLOT_R: src = d.slot_r; break;
    case RFAST_SLOT_C: src = d.slot_c; break;
    case RFAST_ROUND: src = d.round_no; break;
    case RFAST_DELIV_R: src = d.deliv_r; break;
    case RFAST_DELIV_C: src = d.deliv_c; break;
    case RFAST_T_HIST: src = d.t_hist; break;
    // the generator's arrays hold a stretch of rounds; these fields are the last round executed
    case RFAST_SCHED_ACTIVE: src = d.gen_active + (size_t)c->gen_last * d.n; break;
    case RFAST_SCHED_DELAY_R: src = d.gen_delay_r + (size_t)c->gen_last * d.eR; break;
    case RFAST_SCHED_DELAY_C: src = d.gen_delay_c + (size_t)c->gen_last * d.eC; break;
    case RFAST_SCHED_DROP_R: src = d.gen_drop_r + (size_t)c->gen_last * d.eR; break;
    case RFAST_SCHED_DROP_C: src = d.gen_drop_c + (size_t)c->gen_last * d.eC; break;
    case RFAST_SCHED_BATCH:
      src = d.gen_batch + (size_t)c->gen_last * d.n * (d.prob.kind == RFAST_OBJ_DIAG_QUADRATIC ? 0 : d.prob.batch);
      break;
    case RFAST_MOMENTUM: src = d.mom; break;
    default: break;
  }
  if (field == RFAST_RHO_RING) {
    // rho_ij = a_ij * sigma_j: expand the per-sender rings into per-edge rings
    // (fp32 product, the value the kernels consume)
    std::vector<int32_t> src_h(d.eC);
    std::vector<float> w_h(d.eC);
    e = hipMemcpy(src_h.data(), d.c_src, (size_t)d.eC * 4, hipMemcpyDeviceToHost);
    if (e == hipSuccess) e = hipMemcpy(w_h.data(), d.c_w, (size_t)d.eC * 4, hipMemcpyDeviceToHost);
    const size_t ring = (size_t)d.M * d.p;
    for (int q = 0; q < d.eC && e == hipSuccess; ++q) {
      float* dst = (float*)host_dst + (size_t)q * ring;
      e = hipMemcpy(dst, d.sigma_ring + (size_t)src_h[q] * ring, ring * 4, hipMemcpyDeviceToHost);
      for (size_t k = 0; k < ring; ++k) dst[k] = w_h[q] * dst[k];
    }
    if (e == hipSuccess) e = zero_dead_slots(c, true, (float*)host_dst, d.eC, src_h.data());
  } else if (field == RFAST_RHO_TILDE) {
    // rho~_ij = a_ij * sigma_j[tau_ij] lives in the sender's ring while tau_ij >= t_j - D and in the
    // array otherwise: put the two together
    std::vector<int32_t> src_h(d.eC), tau_h(d.eC), t_h(d.n);
    std::vector<float> w_h(d.eC);
    e = hipMemcpy(host_dst, d.rho_tilde, bytes, hipMemcpyDeviceToHost);
    if (e == hipSuccess) e = hipMemcpy(src_h.data(), d.c_src, (size_t)d.eC * 4, hipMemcpyDeviceToHost);
    if (e == hipSuccess) e = hipMemcpy(w_h.data(), d.c_w, (size_t)d.eC * 4, hipMemcpyDeviceToHost);
    if (e == hipSuccess) e = hipMemcpy(tau_h.data(), d.tau_c, (size_t)d.eC * 4, hipMemcpyDeviceToHost);
    if (e == hipSuccess) e = hipMemcpy(t_h.data(), d.t, (size_t)d.n * 4, hipMemcpyDeviceToHost);
    for (int q = 0; q < d.eC && e == hipSuccess; ++q) {
      const int j = src_h[q];
      if (tau_h[q] < t_h[j] - (d.M - 2)) continue;
      float* dst = (float*)host_dst + (size_t)q * d.p;
      e = hipMemcpy(dst, d.sigma_ring + ((size_t)j * d.M + tau_h[q] % d.M) * d.p, (size_t)d.p * 4, hipMemcpyDeviceToHost);
      for (int64_t k = 0; k < d.p; ++k) dst[k] = w_h[q] * dst[k];
    }
  } else if (field == RFAST_G) {
    // the separable objective keeps no sample in memory: write the current ones out first
    if (d.prob.kind == RFAST_OBJ_DIAG_QUADRATIC) {
      e = rfast_diag_init_gradient(c);
      if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
      if (e != hipSuccess) return hipfail(c, e, "forming the gradient samples");
    }
    // the stored sample of node i is the one of version t_i: g[t_i & 1][i]
    std::vector<int32_t> t(d.n);
    e = hipMemcpy(t.data(), d.t, (size_t)d.n * 4, hipMemcpyDeviceToHost);
    const size_t vec = (size_t)d.p * 4;
    for (int i = 0; i < d.n && e == hipSuccess; ++i)
      e = hipMemcpy((char*)host_dst + i * vec, (const char*)d.g + ((size_t)(t[i] & 1) * d.n + i) * vec, vec, hipMemcpyDeviceToHost);
  } else {
    e = hipMemcpy(host_dst, src, bytes, hipMemcpyDeviceToHost);
    if (e == hipSuccess && (field == RFAST_V_RING || field == RFAST_SIGMA_RING))
      e = zero_dead_slots(c, field == RFAST_SIGMA_RING, (float*)host_dst, d.n, nullptr);
  }
  if (e != hipSuccess) return hipfail(c, e, "copying state to host");
  return RFAST_OK;
}

int rfast_write_state(rfast_ctx* c, int32_t field, const void* host_src, size_t bytes) {
  if (!c || !host_src) return RFAST_EINVAL;
  if (field == RFAST_RHO_RING || field == RFAST_SLOT_R || field == RFAST_SLOT_C ||
      (field >= RFAST_SCHED_ACTIVE && field <= RFAST_SCHED_BATCH))
    return fail(c, RFAST_EINVAL, "this field is derived and cannot be written");
  const size_t want = field_bytes(c, field);
  if (want == (size_t)-1) return fail(c, RFAST_EINVAL, "unknown field");
  if (bytes != want) return fail(c, RFAST_EINVAL, "field holds " + std::to_string(want) + " bytes");
  const RfastDev& d = c->d;
  if (fold_sync(c) != RFAST_OK) return RFAST_EHIP;
  hipError_t e = hipStreamSynchronize(c->stream);
  if (e != hipSuccess) return hipfail(c, e, "stream synchronize");
  if (bytes == 0) return RFAST_OK;
  void* dst = nullptr;
  switch (field) {
    case RFAST_X: dst = d.x; break;
    case RFAST_Z: dst = d.z; break;
    case RFAST_V_RING: dst = d.v_ring; break;
    case RFAST_SIGMA_RING: dst = d.sigma_ring; break;
    case RFAST_RHO_TILDE: dst = d.rho_tilde; break;
    case RFAST_T_NODE: dst = d.t; break;
    case RFAST_TAU_R: dst = d.tau_r; break;
    case RFAST_TAU_C: dst = d.tau_c; break;
    case RFAST_ROUND: dst = d.round_no; break;
    case RFAST_DELIV_R: dst = d.deliv_r; break;
    case RFAST_DELIV_C: dst = d.deliv_c; break;
    case RFAST_T_HIST: dst = d.t_hist; break;
    case RFAST_MOMENTUM: dst = d.mom; break;
    default: break;
  }
  if (field == RFAST_ROUND) c->host_round = *(const int32_t*)host_src;
  if (field == RFAST_G) {
    // both parities receive the sample, so the order of restoring G and T_NODE does not matter
    e = hipMemcpy(d.g, host_src, bytes, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy((char*)d.g + bytes, host_src, bytes, hipMemcpyHostToDevice);
  } else {
    e = hipMemcpy(dst, host_src, bytes, hipMemcpyHostToDevice);
  }
  if (e != hipSuccess) return hipfail(c, e, "copying state to the device");
  return RFAST_OK;
}

int rfast_diagnostics(rfast_ctx* c, const float* d_xstar, rfast_diag* host_out) {
  if (!c || !host_out) return RFAST_EINVAL;
  if (fold_sync(c) != RFAST_OK) return RFAST_EHIP;
  hipError_t e = rfast_launch_diag(c, d_xstar, c->d_diag);
  if (e != hipSuccess) return hipfail(c, e, "diagnostics launch");
  e = hipStreamSynchronize(c->stream);
  if (e != hipSuccess) return hipfail(c, e, "stream synchronize");
  double h[8];
  e = hipMemcpy(h, c->d_diag, sizeof(h), hipMemcpyDeviceToHost);
  if (e != hipSuccess) return hipfail(c, e, "copying diagnostics");
  host_out->consensus_sq = h[0];
  host_out->z_sq = h[1];
  host_out->conservation_sq = h[2];
  host_out->gsum_sq = h[3];
  host_out->xbar_gap_sq = d_xstar ? h[4] : -1.0;
  // sum_i f_i(xbar); the l2 term of the logistic objective and the weight decay of the optimizer
  // variant each add n * coefficient/2 * ||xbar||^2
  const double l2 = (c->d.prob.kind == RFAST_OBJ_LOGISTIC ? (double)c->d.prob.lambda : 0.0) + (double)c->d.wd;
  host_out->loss_at_xbar = h[5] + 0.5 * l2 * c->d.n * h[6];
  return RFAST_OK;
}

int rfast_diagnostics_static(rfast_ctx* c, const float* d_xstar, double* d_out) {
  if (!c || !d_out) return RFAST_EINVAL;
  if (c->d.prob.kind != RFAST_OBJ_DIAG_QUADRATIC && c->d.p > rfast_static_max_coords())
    return fail(c, RFAST_ERANGE, "rfast_diagnostics_static: p = " + std::to_string(c->d.p) + " exceeds the " +
                                     std::to_string(rfast_static_max_coords()) +
                                     " coordinates its static scratch holds for this objective (use rfast_diagnostics)");
  if (fold_sync(c) != RFAST_OK) return RFAST_EHIP;
  const double l2 = (c->d.prob.kind == RFAST_OBJ_LOGISTIC ? (double)c->d.prob.lambda : 0.0) + (double)c->d.wd;
  const hipError_t e = rfast_launch_diag_static(c, d_xstar, d_out, 0.5 * l2 * c->d.n);
  if (e != hipSuccess) return hipfail(c, e, "diagnostics launch (static scratch)");
  return RFAST_OK;
}

int rfast_profile_enable(rfast_ctx* c, int32_t on) {
  if (!c) return RFAST_EINVAL;
  constexpr size_t kMax = 4096;
  if (on && c->ev[0][0].empty()) {
    for (int w = 0; w < 3; ++w)
      for (int s = 0; s < 2; ++s) {
        const size_t cnt = (w == 0 ? 2 : 1) * kMax;
        c->ev[w][s].resize(cnt);
        for (size_t k = 0; k < cnt; ++k)
          if (hipEventCreate(&c->ev[w][s][k]) != hipSuccess) return fail(c, RFAST_EHIP, "hipEventCreate failed");
      }
  }
  for (int w = 0; w < 3; ++w) c->ev_used[w] = 0;
  c->profiling = on != 0;
  return RFAST_OK;
}

int rfast_kernel_time(rfast_ctx* c, int32_t which, double* ms_sum, int64_t* launches) {
  if (!c || which < 0 || which > 2 || !ms_sum || !launches) return RFAST_EINVAL;
  hipError_t e = hipStreamSynchronize(c->stream);
  if (e != hipSuccess) return hipfail(c, e, "stream synchronize");
  double tot = 0.0;
  for (size_t k = 0; k < c->ev_used[which]; ++k) {
    float ms = 0.f;
    e = hipEventElapsedTime(&ms, c->ev[which][0][k], c->ev[which][1][k]);
    if (e != hipSuccess) return hipfail(c, e, "hipEventElapsedTime");
    tot += ms;
  }
  *ms_sum = tot;
  *launches = (int64_t)c->ev_used[which];
  return RFAST_OK;
}

const char* rfast_last_error(const rfast_ctx* c) { return c ? c->err.c_str() : g_create_error.c_str(); }

void rfast_destroy(rfast_ctx* c) {
  if (!c) return;
  (void)hipStreamSynchronize(c->stream);
  drop_graph(c);
  if (c->capture_stream) (void)hipStreamDestroy(c->capture_stream);
  for (int w = 0; w < 3; ++w)
    for (int s = 0; s < 2; ++s)
      for (hipEvent_t ev : c->ev[w][s]) (void)hipEventDestroy(ev);
  delete c;
}

}  // extern "C"
