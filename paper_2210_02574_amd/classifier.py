"""Encrypted linear classifier on packed embeddings: host-side sequencing of library calls.

The paper's method (Section 2.2, Section 3.1) runs logistic regression on CKKS ciphertexts of
768-dimensional sentence embeddings: logits are inner products <w, x> under encryption, the
logistic function is a polynomial, multi-class is one-vs-rest.  This module only orders calls of
the device library (hmult_relin, hrot, hrot_many, rescale, rotate_sum, pmult, cmult, add, sub);
all arithmetic runs in the HIP kernels.

Packing (a reading: the paper gives sizes only; its ciphertext sizes imply 768 values padded to
1024 slots): a ciphertext holds N/2 / 1024 samples, sample b in the 1024-slot block b with its
features at block offsets 4 .. 771 and zeros elsewhere.
"""
from __future__ import annotations

from typing import Dict, List, Sequence

import numpy as np

BLOCK = 1024
OFFSET = 4
DIM = 768


def pack_samples(X: np.ndarray, n_slots: int) -> np.ndarray:
    """[n_slots/1024][768] -> slot vector with features at offsets 4..771 of each block."""
    nb = n_slots // BLOCK
    assert X.shape == (nb, DIM)
    z = np.zeros(n_slots)
    for b in range(nb):
        z[b * BLOCK + OFFSET: b * BLOCK + OFFSET + DIM] = X[b]
    return z


def weight_diagonals(W: np.ndarray, n_slots: int) -> List[np.ndarray]:
    """The four plaintext diagonals d_i[1024 b + j] = W[j mod 4][j + i - 4] (0 where j+i is outside 4..771)."""
    classes = W.shape[0]
    assert classes == 4 and W.shape[1] == DIM
    nb = n_slots // BLOCK
    out = []
    j = np.arange(BLOCK)
    for i in range(4):
        f = j + i - OFFSET
        ok = (f >= 0) & (f < DIM)
        d = np.where(ok, W[j % 4, np.clip(f, 0, DIM - 1)], 0.0)
        out.append(np.tile(d, nb))
    return out


INFER_HOISTED = (1, 2, 3)
INFER_SUM_SHIFTS = tuple(4 << k for k in range(8))  # 4 .. 512


class EncryptedInference:
    """logits[b][c] = <W[c], x_b> for every sample of one ciphertext (3 hoisted rotations, 4 plaintext
    products, one rescale, 8 sequential rotations): the result sits in slots 1024 b + c, c < 4."""

    def __init__(self, he, level: int):
        self.he, self.level = he, level
        self.pt_scale = float(he.q[level - 1])  # the rescale then returns exactly the input scale

    def make_keys(self, sk, seed: int) -> Dict[int, object]:
        shifts = list(INFER_HOISTED) + list(INFER_SUM_SHIFTS)
        return {r: self.he.keygen_rot(sk, r, seed + k) for k, r in enumerate(shifts)}

    def encode_weights(self, W: np.ndarray):
        he = self.he
        return [he.to_device(he.plain_to_ntt(he.encode(d, self.pt_scale), self.level))
                for d in weight_diagonals(W, he.n)]

    def run(self, ct, pts, keys):
        """ct: device ciphertext at self.level, scale s; returns a level-1 lower ciphertext at scale s."""
        he = self.he
        rots = he.hrot_many([keys[r] for r in INFER_HOISTED], ct)
        out = he.rescale(he.pmult_sum([ct] + list(rots), pts))
        he.rotate_sum([keys[r] for r in INFER_SUM_SHIFTS], out)
        return out


def logits_from_slots(z: np.ndarray, classes: int = 4) -> np.ndarray:
    nb = z.shape[0] // BLOCK
    return np.stack([z[b * BLOCK: b * BLOCK + classes].real for b in range(nb)])


# ---- one encrypted gradient-descent step of one-vs-rest logistic regression ----------------------------

def sigmoid_ls_coeffs(degree: int = 7, radius: float = 8.0) -> np.ndarray:
    """Monomial coefficients in t = x/radius of the least-squares polynomial approximation of the
    logistic function on [-radius, radius] (continuous L2, by Legendre projection).  The paper evaluates
    the logistic function through a polynomial (Section 2.2: minimax, degree 15 on [-12, 12]); the training
    workload here prescribes degree 7, least squares, on [-8, 8]."""
    from numpy.polynomial import legendre as leg

    xs, ws = leg.leggauss(400)
    f = 1.0 / (1.0 + np.exp(-radius * xs))
    c = [(2 * k + 1) / 2.0 * np.sum(ws * f * leg.legval(xs, [0] * k + [1])) for k in range(degree + 1)]
    mono = leg.leg2poly(c)
    mono[0] = 0.5
    mono[2::2] = 0.0  # logistic - 1/2 is odd: the even terms vanish up to quadrature round-off
    return mono


TRAIN_SUM_SHIFTS = tuple(1 << k for k in range(10))          # block sum: +1 .. +512
TRAIN_FILL_SHIFTS = tuple(-(1 << k) for k in range(10))      # replicate slot 0 of a block: -1 .. -512
TRAIN_BLOCK_SHIFTS = tuple(BLOCK << k for k in range(5))     # sum over the 32 blocks: 1024 .. 16384


class TrainPlan:
    """Levels and scales of every intermediate of one step, fixed by the parameter set."""

    def __init__(self, q: Sequence[int], level: int, scale: float, lr: float, n_samples: int, coeffs=None,
                 degree: int = 7):
        """degree 7: least-squares polynomial on [-8, 8] (coeffs: monomial coefficients in x/8).  degree 15: the
        paper's minimax polynomial on [-12, 12] (coeffs: monomial coefficients in x/12), one level deeper."""
        qf = [float(v) for v in q]
        self.level, self.scale, self.degree = level, scale, degree
        l = level
        self.s1 = scale * scale / qf[l - 1]                 # x*w, level l-1
        self.mask_scale = qf[l - 2]                         # mask product rescales back to s1, level l-2
        self.step = lr / n_samples
        if degree == 15:
            self.mask_value = 1.0 / 12.0                    # the mask also maps z to t = z / 12
            self.c15 = minimax_logistic_coeffs()[0] if coeffs is None else np.asarray(coeffs, dtype=np.float64)
            l0, s = l - 2, self.s1                          # t at level l-2
            self.s_y = s * s / qf[l0 - 1]                   # y = t^2
            self.s_y2 = self.s_y * self.s_y / qf[l0 - 2]
            self.s_y4 = self.s_y2 * self.s_y2 / qf[l0 - 3]
            self.t_hi = s                                   # c13 + c15 y
            self.t_b = self.s_y2 * self.t_hi / qf[l0 - 3]   # B
            self.t_q = self.s_y4 * self.t_b / qf[l0 - 4]    # Q = y^4 B + A
            self.t_hi_a = self.t_q * qf[l0 - 3] / self.s_y2
            self.t_p = s * self.t_q / qf[l0 - 5]            # p(t), level l-7
            self.label_level, self.label_scale = l - 7, self.t_p
            self.t_g = self.t_p * scale / qf[l - 8]
            self.c_w = scale * qf[l - 9] / self.t_g
            self.out_level = l - 9
            return
        self.mask_value = 1.0
        self.s2 = self.s1 * self.s1 / qf[l - 3]             # z^2, level l-3
        self.s4 = self.s2 * self.s2 / qf[l - 4]             # z^4, level l-4
        self.t_u = scale                                    # a7 z^2 + a5, level l-4
        self.c_u = self.t_u * qf[l - 4] / self.s2
        self.t_v = self.s4 * self.t_u / qf[l - 5]           # z^4 * u and a3 z^2 + a1, level l-5
        self.c_v = self.t_v * qf[l - 4] / self.s2
        self.t_p = self.s1 * self.t_v / qf[l - 6]           # p(z), level l-6
        self.label_level, self.label_scale = l - 6, self.t_p
        self.t_g = self.t_p * scale / qf[l - 7]             # gradient after rescale, level l-7
        self.c_w = scale * qf[l - 8] / self.t_g             # update constant; result at level l-8, `scale`
        self.out_level = l - 8
        c = sigmoid_ls_coeffs() if coeffs is None else coeffs  # monomial coefficients in t = x/8
        self.a1, self.a3, self.a5, self.a7 = c[1] / 8.0, c[3] / 8.0**3, c[5] / 8.0**5, c[7] / 8.0**7


def _residues(value: float, scale: float, q: Sequence[int], level: int) -> List[int]:
    v = int(round(value * scale))
    return [v % int(q[i]) for i in range(level)]


class EncryptedTrainStep:
    """W_c <- W_c - (lr/n) sum_samples (p(<x, w_c>) - y_c) x for every class c, all under encryption.

    X[i]: ciphertexts of packed samples (level `level`, scale `scale`); W[c]: weights replicated in every
    block at the feature offsets (same level and scale); Y[c][i]: labels replicated over each block at
    plan.label_level / plan.label_scale.  Per (class, ciphertext): 6 HMult and 20 HRot; per class 5 more HRot."""

    def __init__(self, he, level: int, scale: float, lr: float, n_samples: int, coeffs=None, block: int = BLOCK,
                 degree: int = 7):
        """block: slots per sample (a power of two; the paper's layout is 1024).  degree: 7 or 15 (see TrainPlan)."""
        self.he = he
        self.plan = TrainPlan(he.q, level, scale, lr, n_samples, coeffs, degree)
        assert block & (block - 1) == 0 and block <= he.n
        self.block = block
        lb, lnb = block.bit_length() - 1, (he.n // block).bit_length() - 1
        self.sum_shifts = tuple(1 << k for k in range(lb))           # block sum
        self.fill_shifts = tuple(-(1 << k) for k in range(lb))       # replicate slot 0 of a block
        self.block_shifts = tuple(block << k for k in range(lnb))    # sum over the blocks

    def rotation_shifts(self):
        return list(self.sum_shifts) + list(self.fill_shifts) + list(self.block_shifts)

    def make_keys(self, sk, seed: int):
        rot = {r: self.he.keygen_rot(sk, r, seed + 1 + k) for k, r in enumerate(self.rotation_shifts())}
        return self.he.keygen_relin(sk, seed), rot

    def mask_slots(self) -> np.ndarray:
        m = np.zeros(self.he.n)
        m[::self.block] = self.plan.mask_value
        return m

    def encode_mask(self):
        he, p = self.he, self.plan
        return he.to_device(he.plain_to_ntt(he.encode(self.mask_slots(), p.mask_scale), p.level - 1))

    def _mul(self, relin, a, b):
        return self.he.hmult_relin_rescale(relin, a, b)

    def _affine(self, ct, coeff: float, c_scale: float, const: float, t_scale: float):
        """rescale(coeff * ct) + const, landing on scale t_scale one level down."""
        he = self.he
        level = int(ct.shape[1])
        out = he.rescale(he.cmult(ct, _residues(coeff, c_scale, he.q, level)))
        return he.add_const(out, _residues(const, t_scale, he.q, level - 1), out=out)

    def logistic(self, relin, z):
        """p(z) for z at level l-2, scale s1 -> level l-6, scale t_p (degree 15: z / 12 in, level l-7 out)."""
        he, p = self.he, self.plan
        if p.degree == 15:
            return self._logistic15_b(relin, z.unsqueeze(0))[0]
        z2 = self._mul(relin, z, z)
        z4 = self._mul(relin, z2, z2)
        u = self._affine(z2, p.a7, p.c_u, p.a5, p.t_u)
        zu = self._mul(relin, z4, u)
        v = he.moddrop(self._affine(z2, p.a3, p.c_v, p.a1, p.t_v), p.level - 5)
        inner = he.add(zu, v, out=zu)
        out = self._mul(relin, he.moddrop(z, p.level - 5), inner)
        return he.add_const(out, _residues(0.5, p.t_p, he.q, p.level - 6), out=out)

    def gradient_term(self, relin, rot, mask_pt, x, x_low, w, y):
        """(p(<x, w>) - y) * x for one ciphertext of samples: level l-6, scale t_p * scale, not rescaled."""
        he = self.he
        m = self._mul(relin, x, w)
        he.rotate_sum([rot[r] for r in self.sum_shifts], m)
        z = he.rescale(he.pmult(m, mask_pt))
        he.rotate_sum([rot[r] for r in self.fill_shifts], z)
        e = self.logistic(relin, z)
        he.sub(e, y, out=e)
        return he.hmult_relin(relin, e, x_low)

    def run(self, relin, rot, mask_pt, X, W, Y):
        he, p = self.he, self.plan
        X_low = [he.moddrop(x, p.label_level) for x in X]
        out = []
        for c, w in enumerate(W):
            G = None
            for i, x in enumerate(X):
                g = self.gradient_term(relin, rot, mask_pt, x, X_low[i], w, Y[c][i])
                G = g if G is None else he.add(G, g, out=G)
            G = he.rescale(G)
            he.rotate_sum([rot[r] for r in self.block_shifts], G)
            level = int(G.shape[1])
            upd = he.rescale(he.cmult(G, _residues(p.step, p.c_w, he.q, level)))
            out.append(he.sub(he.moddrop(w, p.out_level), upd))
        return out

    # ---- the same step with all ciphertexts of a class processed as one batch per library call ----------------

    def _mul_b(self, relin, a, b):
        return self.he.hmult_relin_rescale_batch(relin, a, b)

    def _affine_b(self, cts, coeff: float, c_scale: float, const: float, t_scale: float):
        he = self.he
        level = int(cts.shape[2])
        out = he.rescale_batch(he.cmult_batch(cts, _residues(coeff, c_scale, he.q, level)))
        return he.add_const_batch(out, _residues(const, t_scale, he.q, level - 1), out=out)

    def _lin_b(self, y, c0: float, c1: float, target: float, s_in: float):
        """rescale(c1 y) + c0 at scale `target`, one level below y."""
        he = self.he
        level = int(y.shape[2])
        out = he.rescale_batch(he.cmult_batch(y, _residues(c1, target * float(he.q[level - 1]) / s_in, he.q, level)))
        return he.add_const_batch(out, _residues(c0, target, he.q, level - 1), out=out)

    def _logistic15_b(self, relin, t):
        """1/2 + t Q(t^2) with the degree-15 minimax coefficients, t = z / 12 at level l-2 -> level l-7."""
        he, p, c = self.he, self.plan, self.plan.c15
        l0 = p.level - 2
        y = self._mul_b(relin, t, t)
        y2 = self._mul_b(relin, y, y)
        y4 = self._mul_b(relin, y2, y2)
        a_hi = self._lin_b(y, c[5], c[7], p.t_hi_a, p.s_y)
        b_hi = self._lin_b(y, c[13], c[15], p.t_hi, p.s_y)
        a_lo = he.moddrop_batch(self._lin_b(y, c[1], c[3], p.t_q, p.s_y), l0 - 3)
        b_lo = he.moddrop_batch(self._lin_b(y, c[9], c[11], p.t_b, p.s_y), l0 - 3)
        A = self._mul_b(relin, y2, a_hi)
        he.add_batch(A, a_lo, out=A)
        B = self._mul_b(relin, y2, b_hi)
        he.add_batch(B, b_lo, out=B)
        Q = self._mul_b(relin, y4, B)
        he.add_batch(Q, he.moddrop_batch(A, l0 - 4), out=Q)
        out = self._mul_b(relin, he.moddrop_batch(t, l0 - 4), Q)
        return he.add_const_batch(out, _residues(0.5, p.t_p, he.q, l0 - 5), out=out)

    def _logistic_b(self, relin, z):
        he, p = self.he, self.plan
        if p.degree == 15:
            return self._logistic15_b(relin, z)
        z2 = self._mul_b(relin, z, z)
        z4 = self._mul_b(relin, z2, z2)
        u = self._affine_b(z2, p.a7, p.c_u, p.a5, p.t_u)
        zu = self._mul_b(relin, z4, u)
        v = he.moddrop_batch(self._affine_b(z2, p.a3, p.c_v, p.a1, p.t_v), p.level - 5)
        inner = he.add_batch(zu, v, out=zu)
        out = self._mul_b(relin, he.moddrop_batch(z, p.level - 5), inner)
        return he.add_const_batch(out, _residues(0.5, p.t_p, he.q, p.level - 6), out=out)

    def run_batched(self, relin, rot, mask_pt, X, W, Y):
        """X: [n][2][level][N]; W: list of [2][level][N]; Y: list (per class) of [n][2][label_level][N].
        Same arithmetic as run(); the sum over the ciphertexts is a pairwise tree (modular addition is
        associative, so the residues are identical)."""
        he, p = self.he, self.plan
        n = int(X.shape[0])
        X_low = he.moddrop_batch(X, p.label_level)
        out = []
        for c, w in enumerate(W):
            wb = w.unsqueeze(0).expand(n, -1, -1, -1).contiguous()
            m = self._mul_b(relin, X, wb)
            he.rotate_sum_batch([rot[r] for r in self.sum_shifts], m)
            z = he.rescale_batch(he.pmult_batch(m, mask_pt))
            he.rotate_sum_batch([rot[r] for r in self.fill_shifts], z)
            e = self._logistic_b(relin, z)
            he.sub_batch(e, Y[c], out=e)
            g = he.hmult_relin_batch(relin, e, X_low)
            k = n
            while k > 1:  # pairwise sum over the batch
                h = k // 2
                he.add_batch(g[:h], g[k - h:k], out=g[:h])
                k -= h
            G = he.rescale(g[0])
            he.rotate_sum([rot[r] for r in self.block_shifts], G)
            level = int(G.shape[1])
            upd = he.rescale(he.cmult(G, _residues(p.step, p.c_w, he.q, level)))
            out.append(he.sub(he.moddrop(w, p.out_level), upd))
        return out


# ---- the paper's logistic approximation: odd minimax polynomial of degree 15 on [-12, 12] -------------------

def minimax_logistic_coeffs(degree: int = 15, radius: float = 12.0, iters: int = 60):
    """Remez exchange for the odd polynomial sum_k c_k t^(2k+1), t = x/radius, that minimises the maximum
    error against 1/(1+exp(-x)) - 1/2 on [-radius, radius] (Section 2.2 of the paper uses degree 15 on
    [-12, 12] and quotes an error within 0.00614).  Returns (monomial coefficients in t, degree+1 long with
    the constant 1/2, sup error)."""
    m = (degree + 1) // 2
    n = m + 1

    def g(t):
        return 1.0 / (1.0 + np.exp(-radius * t)) - 0.5

    x = np.sort(np.cos(np.pi * np.arange(n)[::-1] / (2 * n - 1)))
    grid = np.linspace(0.0, 1.0, 200001)
    powers = np.stack([grid ** (2 * k + 1) for k in range(m)], axis=1)
    c = np.zeros(m)
    for _ in range(iters):
        A = np.zeros((n, n))
        for k in range(m):
            A[:, k] = x ** (2 * k + 1)
        A[:, m] = (-1.0) ** np.arange(n)
        sol = np.linalg.solve(A, g(x))
        c = sol[:m]
        err = powers @ c - g(grid)
        d = np.diff(err)
        ext = [i + 1 for i in range(len(d) - 1) if d[i] * d[i + 1] < 0] + [len(grid) - 1]
        sel = []
        for i in ext:  # keep one extremum per sign run
            if sel and np.sign(err[i]) == np.sign(err[sel[-1]]):
                if abs(err[i]) > abs(err[sel[-1]]):
                    sel[-1] = i
            else:
                sel.append(i)
        while len(sel) > n:
            sel = sel[1:] if abs(err[sel[0]]) < abs(err[sel[-1]]) else sel[:-1]
        if len(sel) < n:
            break
        new_x = grid[sel]
        done = np.max(np.abs(new_x - x)) < 1e-9
        x = new_x
        if done:
            break
    mono = np.zeros(degree + 1)
    mono[0] = 0.5
    mono[1::2] = c
    sup = float(np.abs(powers @ c - g(grid)).max())
    return mono, sup


class EncryptedLogistic15:
    """p(t) = 1/2 + t Q(t^2), Q of degree 7, on a ciphertext holding t = x/12 (level l0, scale s): 7 HMult and
    4 scalar products, five levels.  Q(y) = A(y) + y^4 B(y), A = (c1 + c3 y) + y^2 (c5 + c7 y),
    B = (c9 + c11 y) + y^2 (c13 + c15 y)."""

    def __init__(self, he, level: int, scale: float, coeffs=None):
        self.he, self.level, self.scale = he, level, scale
        self.c = minimax_logistic_coeffs()[0] if coeffs is None else np.asarray(coeffs, dtype=np.float64)
        q = [float(v) for v in he.q]
        l, s = level, scale
        self.s_y = s * s / q[l - 1]                    # y = t^2, level l-1
        self.s_y2 = self.s_y * self.s_y / q[l - 2]     # y^2, level l-2
        self.s_y4 = self.s_y2 * self.s_y2 / q[l - 3]   # y^4, level l-3
        self.t_hi = s                                  # c13 + c15 y, level l-2
        self.t_b = self.s_y2 * self.t_hi / q[l - 3]    # B, level l-3
        self.t_q = self.s_y4 * self.t_b / q[l - 4]     # Q = y^4 B + A, level l-4: A is built at exactly this scale
        self.t_hi_a = self.t_q * q[l - 3] / self.s_y2  # c5 + c7 y, level l-2
        self.t_p = s * self.t_q / q[l - 5]             # p, level l-5
        self.out_level, self.out_scale = l - 5, self.t_p

    def _lin(self, y, c0: float, c1: float, target: float, s_in: float):
        """rescale(c1 * y) + c0 at scale `target`, one level below y."""
        he = self.he
        level = int(y.shape[1])
        q_drop = float(he.q[level - 1])
        out = he.rescale(he.cmult(y, _residues(c1, target * q_drop / s_in, he.q, level)))
        return he.add_const(out, _residues(c0, target, he.q, level - 1), out=out)

    def _mul(self, relin, a, b):
        return self.he.hmult_relin_rescale(relin, a, b)

    def run(self, relin, t):
        he, c, l = self.he, self.c, self.level
        y = self._mul(relin, t, t)
        y2 = self._mul(relin, y, y)
        y4 = self._mul(relin, y2, y2)
        a_hi = self._lin(y, c[5], c[7], self.t_hi_a, self.s_y)
        b_hi = self._lin(y, c[13], c[15], self.t_hi, self.s_y)
        a_lo = he.moddrop(self._lin(y, c[1], c[3], self.t_q, self.s_y), l - 3)
        b_lo = he.moddrop(self._lin(y, c[9], c[11], self.t_b, self.s_y), l - 3)
        A = self._mul(relin, y2, a_hi)
        he.add(A, a_lo, out=A)
        B = self._mul(relin, y2, b_hi)
        he.add(B, b_lo, out=B)
        Q = self._mul(relin, y4, B)
        he.add(Q, he.moddrop(A, l - 4), out=Q)
        p = self._mul(relin, he.moddrop(t, l - 4), Q)
        return he.add_const(p, _residues(0.5, self.t_p, he.q, l - 5), out=p)
