"""Oracle-side composition of the encrypted classifier workloads (test infrastructure only).

Written directly from the definitions, with the oracle's own packing helpers: sample b of a
ciphertext occupies the 1024-slot block b, feature f at block offset f + 4.  The logits are
slot-wise products with four "diagonal" weight vectors applied to the input rotated by 0..3,
followed by a stride-4 rotate-and-sum: slot 1024 b + c ends up holding <W[c], x_b>.
"""
from __future__ import annotations

import numpy as np


def pack(X, n_slots):
    z = np.zeros(n_slots)
    for b in range(n_slots // 1024):
        for f in range(768):
            z[1024 * b + 4 + f] = X[b][f]
    return z


def diagonal(W, i, n_slots):
    """d_i[1024 b + j] = W[j mod 4][j + i - 4] when 0 <= j + i - 4 < 768, else 0."""
    d = np.zeros(n_slots)
    for b in range(n_slots // 1024):
        for j in range(1024):
            f = j + i - 4
            if 0 <= f < 768:
                d[1024 * b + j] = W[j % 4][f]
    return d


def infer(o, ct, W, level, rot_keys):
    """rot_keys: dict shift -> oracle switching key.  Returns the level-1 ciphertext of the logits."""
    q_last = float(o.q[level - 1])
    acc = None
    for i in range(4):
        x_i = ct if i == 0 else o.hrot(ct, rot_keys[i], i)
        pt = o.coeffs_to_ntt(o.encode(diagonal(W, i, o.n), q_last), level)
        term = o.pmult(x_i, pt)
        acc = term if acc is None else o.add(acc, term)
    out = o.rescale(acc)
    for k in range(8):
        out = o.add(out, o.hrot(out, rot_keys[4 << k], 4 << k))
    return out


# ---- one gradient-descent step of logistic regression, oracle composition ----------------------------------

def logistic_poly_coeffs():
    """Least-squares degree-7 polynomial of 1/(1+exp(-x)) on [-8,8], as monomial coefficients in x.
    Normal equations of the continuous L2 problem in t = x/8 with the monomial basis 1, t, .., t^7,
    integrals by a fine composite Simpson rule."""
    n = 200001
    t = np.linspace(-1.0, 1.0, n)
    w = np.ones(n)
    w[1:-1:2] = 4.0
    w[2:-1:2] = 2.0
    w *= (t[1] - t[0]) / 3.0
    f = 1.0 / (1.0 + np.exp(-8.0 * t))
    A = np.array([[np.sum(w * t ** (i + j)) for j in range(8)] for i in range(8)])
    b = np.array([np.sum(w * f * t**i) for i in range(8)])
    c = np.linalg.solve(A, b)
    return [c[k] / 8.0**k for k in range(8)]


def _const(o, value, scale, level):
    v = int(round(value * scale))
    return [v % o.q[i] for i in range(level)]


def train_step(o, X, W, Y, relin, rot, level, scale, lr, n_samples, a=None, block=1024, c15=None):
    """X: list of ciphertexts, W: list (per class), Y[c][i]; rot: dict shift -> key.  Returns new W list.
    Same level/scale schedule as the device driver, derived here from the rescale rule
    (scale after a rescale = scale before / dropped prime).  block = slots per sample.
    c15: monomial coefficients (in x/12) of a degree-15 polynomial; if given it replaces the degree-7 one, the
    mask then also divides by 12, and the step is one level deeper."""
    q = [float(v) for v in o.q]
    a = logistic_poly_coeffs() if a is None else a  # monomial coefficients in x
    mask = np.zeros(o.n)
    mask[::block] = 1.0 if c15 is None else 1.0 / 12.0
    lb = block.bit_length() - 1
    lnb = (o.n // block).bit_length() - 1
    new_w = []
    for c, w in enumerate(W):
        G = None
        for i, x in enumerate(X):
            # logits: block sums of x*w
            m = o.rescale(o.hmult_relin(x, w, relin))  # level-1
            s1 = scale * scale / q[level - 1]
            for k in range(lb):
                m = o.add(m, o.hrot(m, rot[1 << k], 1 << k))
            pt = o.coeffs_to_ntt(o.encode(mask, q[level - 2]), level - 1)
            z = o.rescale(o.pmult(m, pt))  # level-2, scale s1
            for k in range(lb):
                z = o.add(z, o.hrot(z, rot[-(1 << k)], -(1 << k)))
            if c15 is not None:
                p, tp = logistic15(o, z, relin, level - 2, s1, c15)  # level-7
                e = o.sub(p, Y[c][i])
                g = o.hmult_relin(e, o.moddrop(x, level - 7), relin)
                G = g if G is None else o.add(G, g)
                continue
            # polynomial 0.5 + z (a1 + a3 z^2 + a5 z^4 + a7 z^6) = 0.5 + z ((a1 + a3 z^2) + z^4 (a5 + a7 z^2))
            z2 = o.rescale(o.hmult_relin(z, z, relin))  # level-3
            s2 = s1 * s1 / q[level - 3]
            z4 = o.rescale(o.hmult_relin(z2, z2, relin))  # level-4
            s4 = s2 * s2 / q[level - 4]
            tu = scale
            u = o.rescale(o.cmult(z2, _const(o, a[7], tu * q[level - 4] / s2, level - 3)))
            u = o.add_const(u, _const(o, a[5], tu, level - 4))
            zu = o.rescale(o.hmult_relin(z4, u, relin))  # level-5
            tv = s4 * tu / q[level - 5]
            v = o.rescale(o.cmult(z2, _const(o, a[3], tv * q[level - 4] / s2, level - 3)))
            v = o.add_const(v, _const(o, a[1], tv, level - 4))
            inner = o.add(zu, o.moddrop(v, level - 5))
            p = o.rescale(o.hmult_relin(o.moddrop(z, level - 5), inner, relin))  # level-6
            tp = s1 * tv / q[level - 6]
            p = o.add_const(p, _const(o, 0.5, tp, level - 6))
            e = o.sub(p, Y[c][i])
            g = o.hmult_relin(e, o.moddrop(x, level - 6), relin)
            G = g if G is None else o.add(G, g)
        lg = G.shape[1]  # level-6, or level-7 with the degree-15 polynomial
        G = o.rescale(G)
        tg = tp * scale / q[lg - 1]
        for k in range(lnb):
            G = o.add(G, o.hrot(G, rot[block << k], block << k))
        upd = o.rescale(o.cmult(G, _const(o, lr / n_samples, scale * q[lg - 2] / tg, lg - 1)))
        new_w.append(o.sub(o.moddrop(w, lg - 2), upd))
    return new_w


# ---- degree-15 odd minimax approximation of the logistic function on [-12, 12] ----------------------------

def minimax15_by_linear_program(radius=12.0, grid=1201):
    """The same minimax problem posed on a grid as a linear program (scipy): minimise E subject to
    |sum_k c_k t^(2k+1) - (sigma(radius t) - 1/2)| <= E at every grid point of [0, 1].
    Returns (coefficients c_k of t^(2k+1), E)."""
    from scipy.optimize import linprog

    t = np.linspace(0.0, 1.0, grid)
    g = 1.0 / (1.0 + np.exp(-radius * t)) - 0.5
    P = np.stack([t ** (2 * k + 1) for k in range(8)], axis=1)
    ones = np.ones((grid, 1))
    A = np.vstack([np.hstack([P, -ones]), np.hstack([-P, -ones])])
    b = np.concatenate([g, -g])
    cost = np.zeros(9)
    cost[8] = 1.0
    res = linprog(cost, A_ub=A, b_ub=b, bounds=[(None, None)] * 8 + [(0, None)], method="highs")
    return res.x[:8], float(res.x[8])


def minimax15_coeffs(radius=12.0):
    """Monomial coefficients in t = x/radius (length 16, constant 1/2, even powers zero) of the odd degree-15
    minimax approximation of the logistic function, from the linear program on a 4801-point grid: the oracle
    side's own derivation of the polynomial the paper uses (Section 2.2; its sup error is within the printed
    0.00614)."""
    c, _ = minimax15_by_linear_program(radius, grid=4801)
    mono = np.zeros(16)
    mono[0] = 0.5
    mono[1::2] = c
    return mono


def logistic15(o, t, relin, level, scale, c):
    """1/2 + t Q(t^2) on a ciphertext of t at (level, scale); c = monomial coefficients (length 16).
    Horner-free split: Q = A + y^4 B with A = (c1 + c3 y) + y^2 (c5 + c7 y), B = (c9 + c11 y) + y^2 (c13 + c15 y)."""
    q = [float(v) for v in o.q]

    def mul(a, b):
        return o.rescale(o.hmult_relin(a, b, relin))

    def const(v, s, lvl):
        iv = int(round(v * s))
        return [iv % o.q[i] for i in range(lvl)]

    def lin(y, lvl, s_in, c0, c1, target):
        out = o.rescale(o.cmult(y, const(c1, target * q[lvl - 1] / s_in, lvl)))
        return o.add_const(out, const(c0, target, lvl - 1))

    l = level
    y = mul(t, t)
    s_y = scale * scale / q[l - 1]
    y2 = mul(y, y)
    s_y2 = s_y * s_y / q[l - 2]
    y4 = mul(y2, y2)
    s_y4 = s_y2 * s_y2 / q[l - 3]
    # scales: B is built at t_b, Q = y^4 B + A lands at t_q, so A is built at exactly t_q
    t_hi = scale
    t_b = s_y2 * t_hi / q[l - 3]
    t_q = s_y4 * t_b / q[l - 4]
    t_hi_a = t_q * q[l - 3] / s_y2
    a_hi = lin(y, l - 1, s_y, c[5], c[7], t_hi_a)
    b_hi = lin(y, l - 1, s_y, c[13], c[15], t_hi)
    a_lo = o.moddrop(lin(y, l - 1, s_y, c[1], c[3], t_q), l - 3)
    b_lo = o.moddrop(lin(y, l - 1, s_y, c[9], c[11], t_b), l - 3)
    A = o.add(mul(y2, a_hi), a_lo)
    B = o.add(mul(y2, b_hi), b_lo)
    Q = o.add(mul(y4, B), o.moddrop(A, l - 4))
    t_p = scale * t_q / q[l - 5]
    p = mul(o.moddrop(t, l - 4), Q)
    return o.add_const(p, const(0.5, t_p, l - 5)), t_p
