"""Synthetic logistic-regression problem for the training-loop tests: nb samples of `dim` features, one per
block of `block` slots at offset `off` (plain input construction, no scheme arithmetic)."""
import numpy as np

import workloads as wl


class Problem:
    def __init__(self, n_slots: int, block: int = 64, dim: int = 40, off: int = 4, seed: int = 7):
        self.n, self.block, self.dim, self.off = n_slots, block, dim, off
        self.nb = n_slots // block
        g = wl.rng(seed)
        self.X = np.clip(g.normal(0, 0.5, (self.nb, dim)), -3, 3)
        self.w0 = g.normal(0, 0.05, dim)
        wstar = g.normal(0, 0.3, dim)
        self.y = (self.X @ wstar > 0).astype(np.float64)

    def slots_x(self):
        z = np.zeros(self.n)
        for b in range(self.nb):
            z[b * self.block + self.off: b * self.block + self.off + self.dim] = self.X[b]
        return z

    def slots_w(self, w):
        z = np.zeros(self.n)
        for b in range(self.nb):
            z[b * self.block + self.off: b * self.block + self.off + self.dim] = w
        return z

    def slots_y(self):
        return np.repeat(self.y, self.block)

    def plain_iteration(self, w, v, a, lr, gamma, c15=None):
        """The same polynomial step in fp64: returns (w_next, v_next).  a: monomial coefficients in x of the
        degree-7 polynomial; c15: monomial coefficients in x/12 of the degree-15 one (used if given)."""
        z = self.X @ w
        p = sum(a[k] * z**k for k in range(8)) if c15 is None else np.polyval(np.asarray(c15)[::-1], z / 12.0)
        vn = w - lr * ((p - self.y)[:, None] * self.X).sum(0) / self.nb
        return (1 + gamma) * vn - gamma * v, vn
