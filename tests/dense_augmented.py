"""Matrix-only second formulation of single-node R-FAST activations, built from
the paper's augmented systems (appendices "augmented graph of G(W)" and
"augmented graph of G(A)"): the row-stochastic matrix W-hat^k acting on
h = [x; v^k; v^(k-1); ...; v^(k-D)] and the column-stochastic sum/push
matrices S^k, P^k acting on z-hat = [z; edge masses at age 0..D].

Used only to pin the event-driven oracle; it knows nothing of stamps, running
sums rho or buffers rho-tilde.
"""
import numpy as np


class DenseAugmented:
    def __init__(self, Wd, Ad, D, x0, g0):
        self.W, self.A, self.D = np.asarray(Wd, float), np.asarray(Ad, float), int(D)
        n = self.n = self.W.shape[0]
        p = x0.shape[1]
        # C-edges (receiver i, sender j), receiver-major, sender ascending
        self.edges = [(i, j) for i in range(n) for j in range(n) if j != i and self.A[i, j] != 0.0]
        self.E = len(self.edges)
        self.eid = {ed: k for k, ed in enumerate(self.edges)}
        self.h = np.zeros(((D + 2) * n, p))
        self.h[:n] = x0
        self.S = n + (D + 1) * self.E
        self.zhat = np.zeros((self.S, p))
        self.zhat[:n] = g0

    def vnode(self, e, d):
        return self.n + d * self.E + e

    def W_hat(self, i, d_v):
        n, D = self.n, self.D
        N = (D + 2) * n
        M = np.zeros((N, N))
        M[i, i] = self.W[i, i]
        for j, d in d_v.items():
            M[i, j + (d + 1) * n] += self.W[i, j]
        for r in range(2 * n):
            if r != i and r != i + n:
                M[r, r] = 1.0
        for r in list(range(2 * n, N)) + [i + n]:
            M[r, r - n] = 1.0
        return M

    def S_mat(self, i, d_rho):
        M = np.eye(self.S)
        for j, d0 in d_rho.items():
            e = self.eid[(i, j)]
            for d in range(d0, self.D + 1):
                m = self.vnode(e, d)
                M[m, m] = 0.0
                M[i, m] = 1.0
        return M

    def P_mat(self, i):
        n, D = self.n, self.D
        M = np.zeros((self.S, self.S))
        for l in range(n):
            if l != i:
                M[l, l] = 1.0
        M[i, i] = self.A[i, i]
        for (recv, send), e in self.eid.items():
            if send == i:
                M[self.vnode(e, 0), i] = self.A[recv, i]
            for d in range(D):
                M[self.vnode(e, d + 1), self.vnode(e, d)] = 1.0
            M[self.vnode(e, D), self.vnode(e, D)] = 1.0
        return M

    def step(self, i, d_v, d_rho, gamma, grad):
        """grad(i, x) -> gradient sample; returns nothing, advances h and z-hat."""
        n = self.n
        Wh = self.W_hat(i, d_v)
        g_old = grad(i, self.h[i])
        hh = self.h.copy()
        hh[i] -= gamma * self.zhat[i]
        self.h = Wh @ hh
        eps = grad(i, self.h[i]) - g_old
        Sm, Pm = self.S_mat(i, d_rho), self.P_mat(i)
        zh = Sm @ self.zhat
        zh[i] += eps
        self.zhat = Pm @ zh
        return Wh, Sm, Pm
