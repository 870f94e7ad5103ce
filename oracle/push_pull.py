"""TEST INFRASTRUCTURE — fp64 oracle of the synchronous push-pull recursion that
R-FAST is developed from (eq. (2) of the paper, "Push-Pull Protocol"):

    x_i^{t+1} = sum_j w_ij (x_j^t - gamma^t z_j^t)
    z_i^{t+1} = sum_j a_ij z_j^t + grad f_i(x_i^{t+1}) - grad f_i(x_i^t),   z^0 = grad f(x^0)

with W row-stochastic and A column-stochastic (both sums include j = i).  Written
with dense matrices, exactly as printed.  Stochastic variants pass a sample: the
gradient at x^{t+1} is drawn with stamp t+1 and kept as the "old" gradient of
the next step (the same convention as the asynchronous oracle).  The labelled
optimizer variant of the asynchronous oracle carries over: weight decay is part
of the gradient, momentum replaces z by the buffer m <- beta m + z in the
descent term.  Only tests may import this file; it shares no code with the HIP
library.
"""
import numpy as np


class PushPullOracle:
    def __init__(self, W, A, objective, x0=None, batch0=None, momentum=0.0, weight_decay=0.0):
        self.momentum, self.weight_decay = float(momentum), float(weight_decay)
        self.W = np.asarray(W, dtype=np.float64)
        self.A = np.asarray(A, dtype=np.float64)
        self.n = self.W.shape[0]
        self.obj = objective
        p = objective.p if x0 is None else np.asarray(x0).shape[1]
        self.x = np.zeros((self.n, p)) if x0 is None else np.array(x0, dtype=np.float64)
        self.t = 0
        self.g = self._grad(self.x, 0, batch0)
        self.z = self.g.copy()
        self.m = np.zeros_like(self.x)

    def _grad(self, x, stamp, batch):
        g = np.stack([self.obj.grad(i, x[i], stamp, None if batch is None else batch[i]) for i in range(self.n)])
        return g + self.weight_decay * x

    def step(self, gamma, batch=None):
        if self.momentum != 0.0:
            self.m = self.momentum * self.m + self.z
            x_new = self.W @ (self.x - gamma * self.m)
        else:
            x_new = self.W @ (self.x - gamma * self.z)
        g_new = self._grad(x_new, self.t + 1, batch)
        self.z = self.A @ self.z + g_new - self.g
        self.x, self.g = x_new, g_new
        self.t += 1
