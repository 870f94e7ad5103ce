"""TEST INFRASTRUCTURE — plain fp64 CPU oracle of R-FAST's activation round.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this file.  It shares no code with the HIP library and never imports it.

What it computes: the node update of Algorithm 1 / Algorithm 2 of the paper
(steps S1, S2a, S2b, S2c, S3, S4, S5), written out per activated node in the
paper's order and notation, with an unbounded dictionary of published versions
per node / per edge instead of a ring buffer, so that nothing here depends on
slot arithmetic.

Notation bridge.  W (row-stochastic, pull) is passed as R; A (column-
stochastic, push) is passed as C.  Both are CSR with row = receiver.
v_i^t is the t-th published copy of node i (version 0 is the zero vector,
Algorithm 1 initialisation); rho[(i, j)][t] is the running sum kept by sender
j for receiver i after j's t-th activation (S2c); rho_tilde[(i, j)] is the
receiver-side buffer (S4); tau_v / tau_rho are the largest stamps picked up so
far on each edge (S2a, S2b); t[i] is node i's local iteration counter (S5).

Readings taken where the paper is silent (each also listed in the design notes):
 * the sums over in-neighbours in S2a, S2b and over out-neighbours in S2c
   exclude the node itself; w_ii and a_ii enter through the explicit terms;
 * the "old" gradient of S2b is the stored sample, not a re-evaluation
   (Lemma 3's proof keeps the sample unchanged for inactive nodes);
 * stamps never decrease (a receiver keeps the newest one it has picked up: S2a, S2b);
 * a batched round activates a set of nodes that all read the state as of the
   start of the round; delay d on an edge means the receiver sees what the
   sender had published before round r-d;
 * a packet loss is decided when a version is sent, per edge; a lost version
   is never visible on that edge; after burst-1 consecutive losses on an edge
   the next version is delivered regardless (Assumption 3 excludes links that
   fail forever), so staleness in versions is at most D = d_max + burst - 1.

Optimizer variant (labelled: the paper's large-scale experiment lists momentum,
weight decay and a step-decayed learning rate among its hyper-parameters but
does not say where they enter Algorithm 1).  Reading taken here:
 * weight decay lambda is part of the sampled gradient, g = grad f_i(x; zeta) +
   lambda * x, at initialisation and in S2b, so it is tracked like any gradient
   (the objective becomes f_i + lambda/2 ||x||^2);
 * momentum beta is a heavy-ball buffer on the tracked direction in S1:
   m_i <- beta m_i + z_i (m_i^0 = 0), v = x_i - gamma m_i; only the node that
   is activated touches its buffer.  beta = 0 is the paper's S1;
 * the step size of round r is gamma * factor^(r div step_rounds), computed by
   the caller (step_gamma below).
With one node and no edges the recursion is textbook SGD with momentum and
weight decay, which is what the tests pin it to.
"""
from __future__ import annotations

import numpy as np


def step_gamma(gamma0, factor, step_rounds, r):
    """Step-decayed learning rate of round r (large-scale experiment, hyper-parameter ii)."""
    return gamma0 * factor ** (r // step_rounds) if step_rounds > 0 else gamma0


class RFastOracle:
    def __init__(self, n, p, R, C, D, burst, objective, x0=None, batch0=None, prune=True,
                 momentum=0.0, weight_decay=0.0):
        """R, C: objects with rowptr, col, w (CSR, row = receiver, diagonal included).
        objective: object with grad(i, x, version, batch_rows) -> float64 [p]."""
        self.n, self.p, self.D, self.burst = int(n), int(p), int(D), int(burst)
        assert self.burst >= 1 and self.D >= self.burst - 1
        self.d_max = self.D - (self.burst - 1)
        self.obj = objective
        self.prune = prune
        self.momentum, self.weight_decay = float(momentum), float(weight_decay)
        self.r_self, self.r_in = self._split(R)      # r_in[i] = [(edge id, j, w_ij)]
        self.c_self, self.c_in = self._split(C)
        self.edges_R = [(i, j) for i in range(n) for (_, j, _) in self.r_in[i]]
        self.edges_C = [(i, j) for i in range(n) for (_, j, _) in self.c_in[i]]
        # out-edges of sender j over C: (edge id, receiver l, a_lj)
        self.c_out = [[] for _ in range(n)]
        self.r_out = [[] for _ in range(n)]
        for i in range(n):
            for (e, j, w) in self.c_in[i]:
                self.c_out[j].append((e, i, w))
            for (e, j, w) in self.r_in[i]:
                self.r_out[j].append((e, i, w))
        # ---- initialisation (Algorithm 1, first line) ----
        self.x = np.zeros((n, p)) if x0 is None else np.array(x0, dtype=np.float64).reshape(n, p)
        self.t = np.zeros(n, dtype=np.int64)
        self.g = np.stack([
            self._sample(i, self.x[i], 0, None if batch0 is None else batch0[i]) for i in range(n)])
        self.z = self.g.copy()
        self.m = np.zeros((n, p))
        self.v = [{0: np.zeros(p)} for _ in range(n)]
        self.rho = [{0: np.zeros(p)} for _ in self.edges_C]
        self.rho_tilde = [np.zeros(p) for _ in self.edges_C]
        self.tau_v = np.zeros(len(self.edges_R), dtype=np.int64)
        self.tau_rho = np.zeros(len(self.edges_C), dtype=np.int64)
        self.delivered_R = [{0: True} for _ in self.edges_R]
        self.delivered_C = [{0: True} for _ in self.edges_C]
        self.t_start = [self.t.copy()]   # t_start[s] = counters at the start of round s
        self.round_no = 0
        self.last_z_half = np.zeros((n, p))

    def _sample(self, i, x, version, batch):
        g = self.obj.grad(i, x, version, batch)
        return g + self.weight_decay * x if self.weight_decay != 0.0 else g

    @staticmethod
    def _split(G):
        n = len(G.rowptr) - 1
        self_w = np.zeros(n)
        ins = [[] for _ in range(n)]
        e = 0
        for i in range(n):
            for k in range(int(G.rowptr[i]), int(G.rowptr[i + 1])):
                j = int(G.col[k])
                if j == i:
                    self_w[i] = float(G.w[k])
                else:
                    ins[i].append((e, j, float(G.w[k])))
                    e += 1
        return self_w, ins

    # ------------------------------------------------------------------ S1..S5
    def activate(self, i, stamp_v, stamp_rho, gamma, batch=None, lost_R=(), lost_C=()):
        """One activation of node i (Algorithm 2, S.1-S.5), reading version
        stamp_v[e] of v on each R in-edge e and version stamp_rho[e] of rho on
        each C in-edge e.  lost_R / lost_C: out-edge ids whose new packet is lost."""
        t = int(self.t[i])
        # S1: local descent (variant: along the heavy-ball buffer of the tracked direction)
        if self.momentum != 0.0:
            self.m[i] = self.momentum * self.m[i] + self.z[i]
            v_new = self.x[i] - gamma * self.m[i]
        else:
            v_new = self.x[i] - gamma * self.z[i]
        # S2a: pull / mix over R
        x_new = self.r_self[i] * v_new
        for (e, j, w) in self.r_in[i]:
            x_new = x_new + w * self.v[j][int(stamp_v[e])]
        # S2b: tracker sum over C with the new and the stored old gradient sample
        g_new = self._sample(i, x_new, t + 1, batch)
        z_half = self.z[i].copy()
        consumed = {}
        for (e, j, w) in self.c_in[i]:
            consumed[e] = self.rho[e][int(stamp_rho[e])]
            z_half = z_half + (consumed[e] - self.rho_tilde[e])
        z_half = z_half + g_new - self.g[i]
        # S2c: keep a_ii, push a_li to every out-neighbour l as a running sum
        z_new = self.c_self[i] * z_half
        for (e, l, w) in self.c_out[i]:
            self.rho[e][t + 1] = self.rho[e][t] + w * z_half
        # S3: publish (stamp t+1); a lost packet is simply never visible on its edge
        self.v[i][t + 1] = v_new
        for (e, l, w) in self.r_out[i]:
            self.delivered_R[e][t + 1] = self._deliver(self.delivered_R[e], t + 1, e in lost_R)
        for (e, l, w) in self.c_out[i]:
            self.delivered_C[e][t + 1] = self._deliver(self.delivered_C[e], t + 1, e in lost_C)
        # S4: buffer the consumed running sums
        for (e, j, w) in self.c_in[i]:
            self.rho_tilde[e] = consumed[e].copy()
            self.tau_rho[e] = int(stamp_rho[e])
        for (e, j, w) in self.r_in[i]:
            self.tau_v[e] = int(stamp_v[e])
        # S5: commit, bump the local counter
        self.x[i], self.z[i], self.g[i] = x_new, z_new, g_new
        self.last_z_half[i] = z_half
        self.t[i] = t + 1
        if self.prune:
            self._prune(i)

    def _deliver(self, hist, t, lost):
        if not lost:
            return True
        # forced delivery after burst-1 consecutive losses
        return all(not hist.get(t - k, True) for k in range(1, self.burst))

    def _prune(self, i):
        keep_from = int(self.t[i]) - self.D - 1
        stores = [self.v[i]] + [self.rho[e] for (e, _, _) in self.c_out[i]]
        stores += [self.delivered_C[e] for (e, _, _) in self.c_out[i]]
        stores += [self.delivered_R[e] for (e, _, _) in self.r_out[i]]
        for store in stores:
            for k in [k for k in store if k < keep_from]:
                del store[k]

    # ------------------------------------------------------------------ round
    def resolve(self, i, delay_R, delay_C):
        """Stamps node i picks up at the start of the current round: on each
        in-edge the newest delivered version the sender had published before
        round r - delay (found by scanning stamps downward from the sender's
        counter at that time), never older than the stamp already held."""
        r = self.round_no
        sv, sr = {}, {}
        for (e, j, w) in self.r_in[i]:
            u = int(self.t_start[max(r - int(delay_R[e]), 0)][j])
            cand = next(tt for tt in range(u, -1, -1) if self.delivered_R[e].get(tt, tt == 0))
            sv[e] = max(int(self.tau_v[e]), cand)
        for (e, j, w) in self.c_in[i]:
            u = int(self.t_start[max(r - int(delay_C[e]), 0)][j])
            cand = next(tt for tt in range(u, -1, -1) if self.delivered_C[e].get(tt, tt == 0))
            sr[e] = max(int(self.tau_rho[e]), cand)
        return sv, sr

    def round(self, active, delay_R, delay_C, drop_R, drop_C, gamma, batch_idx=None, order=None):
        """One batched activation round: every node with active[i] != 0 runs
        S1-S5 once, all reading the start-of-round state."""
        if np.any(np.asarray(delay_R) < 0) or np.any(np.asarray(delay_R) > self.d_max) or \
           np.any(np.asarray(delay_C) < 0) or np.any(np.asarray(delay_C) > self.d_max):
            raise ValueError("delay outside [0, d_max]")
        act = [i for i in range(self.n) if active[i]]
        plans = {i: self.resolve(i, delay_R, delay_C) for i in act}
        lost_R = {e for e in range(len(self.edges_R)) if drop_R[e]}
        lost_C = {e for e in range(len(self.edges_C)) if drop_C[e]}
        for i in (act if order is None else order):
            sv, sr = plans[i]
            self.activate(i, sv, sr, gamma, None if batch_idx is None else batch_idx[i], lost_R, lost_C)
        self.round_no += 1
        self.t_start.append(self.t.copy())

    # ------------------------------------------------------------ diagnostics
    def conservation_residual(self):
        """Lemma 3 (tracking conservation): sum_i z_i + sum_edges (latest rho -
        rho_tilde) - sum_i g_i, which is zero in exact arithmetic."""
        tot = self.z.sum(axis=0) - self.g.sum(axis=0)
        for e, (i, j) in enumerate(self.edges_C):
            tot = tot + self.rho[e][int(self.t[j])] - self.rho_tilde[e]
        return tot

    def diagnostics(self, x_star=None):
        xbar = self.x.mean(axis=0)
        out = {
            "consensus_sq": float(((self.x - xbar) ** 2).sum()),
            "z_sq": float((self.z ** 2).sum()),
            "conservation_sq": float((self.conservation_residual() ** 2).sum()),
            "gsum_sq": float((self.g.sum(axis=0) ** 2).sum()),
        }
        if x_star is not None:
            out["xbar_gap_sq"] = float(((xbar - x_star) ** 2).sum())
            out["x_gap_sq"] = float(((self.x - x_star) ** 2).sum())
        if hasattr(self.obj, "loss"):
            # objective of the run: with weight decay each f_i carries lambda/2 ||x||^2
            out["loss_at_xbar"] = float(sum(self.obj.loss(i, xbar) for i in range(self.n))
                                        + 0.5 * self.weight_decay * self.n * (xbar ** 2).sum())
        return out

    def slots(self):
        """Ring-buffer view of the integer state for M = D + 2 slots."""
        M = self.D + 2
        return {"t": self.t.copy(), "tau_v": self.tau_v.copy(), "tau_rho": self.tau_rho.copy(),
                "slot_v": self.tau_v % M, "slot_rho": self.tau_rho % M}
