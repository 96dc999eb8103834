"""Bootstrap (Section 2.2 of the paper lists it as the operation that refreshes a ciphertext's level) for
sparsely packed ciphertexts, driven from Python over the library's device entry points.

Construction (the published one for CKKS): ModRaise, trace onto the subring of the packed slots, one
baby-step/giant-step matrix product that moves coefficients into slots, exp(i theta) by a Taylor polynomial
and r squarings for the reduction modulo q0, and the inverse matrix product.  The two real halves of the
coefficient vector go through the polynomial part as one batch of two ciphertexts.

A ciphertext with `ns` packed slots holds a slot vector of period ns (the paper's weight vectors, one
1024-slot block repeated, are of this kind).
"""
from __future__ import annotations

import math
from typing import Dict, List

import numpy as np

COS_TAYLOR = [(-1) ** k / math.factorial(2 * k) for k in range(5)]      # in y = theta^2, up to theta^8
SIN_TAYLOR = [(-1) ** k / math.factorial(2 * k + 1) for k in range(5)]  # theta * (.), up to theta^9


def _residues(value: float, scale: float, q, level: int) -> List[int]:
    v = int(round(value * scale))
    return [v % int(q[i]) for i in range(level)]


class Bootstrapper:
    def __init__(self, he, ns: int, r: int = 8, level: int = None):
        assert ns >= 2 and ns & (ns - 1) == 0 and ns <= he.n
        self.he, self.ns, self.r = he, ns, r
        self.L = he.L if level is None else level
        self.gap = he.n // ns
        bits = ns.bit_length() - 1
        self.g1 = 1 << ((bits + 1) // 2)   # baby steps 0 .. g1-1
        self.g2 = ns // self.g1            # giant steps 0, g1, .. (g2-1) g1
        self.trace_shifts = [ns << k for k in range(self.gap.bit_length() - 1)]
        self.out_level = self.L - 7 - r
        assert self.out_level >= 1, "not enough levels for this r"
        self._mono: Dict = {}
        self._pts: Dict = {}

    # ---- keys and plaintexts ----------------------------------------------------------------------------------

    def rotation_shifts(self) -> List[int]:
        giant = [self.g1 * b for b in range(1, self.g2)]
        return sorted(set(self.trace_shifts) | set(range(1, self.g1)) | set(giant))

    def make_keys(self, sk, seed: int):
        he = self.he
        rot = {sh: he.keygen_rot(sk, sh, seed + 10 + i) for i, sh in enumerate(self.rotation_shifts())}
        return {"relin": he.keygen_relin(sk, seed), "conj": he.keygen_conj(sk, seed + 1), "rot": rot}

    def dft(self) -> np.ndarray:
        """U[j][k] = xi_j^k with xi_j = exp(2 pi i 5^j / (4 ns)): slots of a polynomial in X^(N/2ns) from its
        coefficient pairs t_k + i t_(k+ns)."""
        ns = self.ns
        powers = np.empty(ns, dtype=np.int64)
        e = 1
        for j in range(ns):
            powers[j] = e
            e = (e * 5) % (4 * ns)
        return np.exp((0.5j * np.pi / ns) * powers[:, None] * np.arange(ns)[None, :])

    def cts_matrix(self) -> np.ndarray:
        # (1/ns) conj(U)^T inverts U; 1/gap undoes the trace; pi / 2^r turns (w + conj w) into 2 pi Re(w) / 2^r
        return (math.pi / (self.gap * 2.0**self.r * self.ns)) * self.dft().conj().T

    def stc_matrix(self, gain: float = 1.0) -> np.ndarray:
        # sin / (2 pi), and the 1/2 of the imaginary-part extraction
        return (gain / (4.0 * math.pi)) * self.dft()

    def natural_factor(self) -> float:
        """Output scale over input scale at gain 1: the scale of exp(i theta) after the squarings over q0."""
        q = [float(v) for v in self.he.q]
        lvl = self.L - 6
        s = q[0] * q[0] / q[lvl]
        for _ in range(self.r):
            s = s * s / q[lvl - 1]
            lvl -= 1
        return s / q[0]

    def gain_for(self, delta_in: float, target_scale: float) -> float:
        """Gain of the last matrix that makes the refreshed ciphertext land exactly on target_scale."""
        return target_scale / (delta_in * self.natural_factor())

    def diagonal_slots(self, M: np.ndarray):
        """[b][a]: slot vector (length n) of diagonal g1 b + a of M, rotated right by g1 b."""
        ns, g1 = self.ns, self.g1
        rows = np.arange(ns)
        out = []
        for b in range(self.g2):
            src = (rows - g1 * b) % ns
            out.append([np.tile(M[src, (rows + a) % ns], self.he.n // ns) for a in range(g1)])
        return out

    def _plain(self, coeffs: np.ndarray, level: int):
        """Integer polynomial -> device plaintext [level][N] in the NTT domain (residues on the host, NTT on the GPU)."""
        he = self.he
        c = np.asarray(coeffs, dtype=np.int64)
        limbs = np.stack([np.mod(c, np.int64(he.q[i])).astype(np.uint64) for i in range(level)])
        d = he.to_device(limbs)
        he.ntt(d, list(range(level)))
        return d

    def encode_matrix(self, M: np.ndarray, level: int):
        he = self.he
        scale = float(he.q[level - 1])
        return [[self._plain(he.encode(v, scale), level) for v in row] for row in self.diagonal_slots(M)]

    def prepare(self, gain: float = 1.0):
        """Encodes the plaintext diagonals of both matrix products once (they depend only on ns, r, the moduli
        and the gain of the last matrix)."""
        if "cts" not in self._pts:
            self._pts["cts"] = self.encode_matrix(self.cts_matrix(), self.L)
            for lvl in (self.L - 1, self.L - 6, self.out_level + 1):
                for sign in (1, -1):
                    self.monomial(lvl, sign)
        if ("stc", gain) not in self._pts:
            self._pts[("stc", gain)] = self.encode_matrix(self.stc_matrix(gain), self.out_level + 1)
        return self._pts["cts"], self._pts[("stc", gain)]

    def monomial(self, level: int, sign: int):
        """Plaintext of +-X^(N/2): every slot times +-i, exactly, at no cost in scale or level."""
        key = (level, sign)
        if key not in self._mono:
            c = np.zeros(self.he.N, dtype=np.int64)
            c[self.he.N // 2] = sign
            self._mono[key] = self._plain(c, level)
        return self._mono[key]

    # ---- building blocks ----------------------------------------------------------------------------------------

    def linear_transform(self, ct, pts, rot):
        """Matrix product on the packed slots (baby steps hoisted), then rescale."""
        he, g1 = self.he, self.g1
        babies = [ct] + (he.hrot_many([rot[a] for a in range(1, g1)], ct) if g1 > 1 else [])
        acc = None
        for b in range(self.g2):
            inner = he.pmult_sum(babies, pts[b])
            if b:
                inner = he.hrot(rot[g1 * b], inner)
            acc = inner if acc is None else he.add(acc, inner, out=acc)
        return he.rescale(acc)

    def _lin(self, y, level: int, s_in: float, c0: float, c1: float, target: float):
        he = self.he
        out = he.rescale_batch(he.cmult_batch(y, _residues(c1, target * float(he.q[level - 1]) / s_in, he.q, level)))
        return he.add_const_batch(out, _residues(c0, target, he.q, level - 1), out=out)

    def _quartic(self, relin, y, y2, l: int, s_y: float, s_y2: float, c, target: float):
        """c0 + c1 y + .. + c4 y^4 as (c0 + c1 y) + y2 ((c2 + c3 y) + c4 y2): y at level l, y2 = y^2 at l-1;
        result at level l-3, scale `target`."""
        he = self.he
        q = [float(v) for v in he.q]
        t_in = target * q[l - 3] / s_y2
        inner = he.moddrop_batch(self._lin(y, l, s_y, c[2], c[3], t_in), l - 2)
        top = he.rescale_batch(he.cmult_batch(y2, _residues(c[4], t_in * q[l - 2] / s_y2, he.q, l - 1)))
        he.add_batch(inner, top, out=inner)
        prod = he.hmult_relin_rescale_batch(relin, he.moddrop_batch(y2, l - 2), inner)
        low = he.moddrop_batch(self._lin(y, l, s_y, c[0], c[1], target), l - 3)
        return he.add_batch(prod, low, out=prod)

    def exp_i(self, relin, theta, level: int, scale: float):
        """theta: batch of ciphertexts with real slots at (level, scale) -> exp(i 2^r theta), level - 5 - r."""
        he, l = self.he, level
        q = [float(v) for v in he.q]
        y = he.hmult_relin_rescale_batch(relin, theta, theta)
        s_y = scale * scale / q[l - 1]
        y2 = he.hmult_relin_rescale_batch(relin, y, y)
        s_y2 = s_y * s_y / q[l - 2]
        t_p = scale
        t_s = scale * t_p / q[l - 5]
        P = self._quartic(relin, y, y2, l - 1, s_y, s_y2, SIN_TAYLOR, t_p)
        C = self._quartic(relin, y, y2, l - 1, s_y, s_y2, COS_TAYLOR, t_s)
        S = he.hmult_relin_rescale_batch(relin, he.moddrop_batch(theta, l - 4), P)
        E = he.pmult_batch(S, self.monomial(l - 5, 1))
        he.add_batch(E, he.moddrop_batch(C, l - 5), out=E)
        lvl, s = l - 5, t_s
        for _ in range(self.r):
            E = he.hmult_relin_rescale_batch(relin, E, E)
            s = s * s / q[lvl - 1]
            lvl -= 1
        return E, lvl, s

    # ---- the whole operation ------------------------------------------------------------------------------------

    def run(self, ct1, keys, pts_cts=None, pts_stc=None, gain: float = 1.0):
        """ct1: device ciphertext at level 1 (scale delta, slot vector of period ns).  Returns (ct, level, factor):
        the same slots at `level` and scale delta * factor.  gain multiplies the last matrix and the factor
        (see gain_for); explicit plaintexts must have been encoded with the same gain."""
        import torch

        he, L = self.he, self.L
        relin, conj, rot = keys["relin"], keys["conj"], keys["rot"]
        if pts_cts is None or pts_stc is None:
            pts_cts, pts_stc = self.prepare(gain)
        ct = he.modraise(ct1, L)
        he.rotate_sum([rot[sh] for sh in self.trace_shifts], ct)
        scale = float(he.q[0])  # read as a ciphertext of t / q0
        w = self.linear_transform(ct, pts_cts, rot)
        wc = he.hconj(conj, w)
        th = torch.stack([he.add(w, wc), he.pmult(he.sub(w, wc), self.monomial(L - 1, -1))])
        E, lvl, s = self.exp_i(relin, th, L - 1, scale)
        iE2 = he.pmult(E[1], self.monomial(lvl, 1))
        plus, minus = he.add(E[0], iE2), he.sub(E[0], iE2)
        F = he.pmult(he.sub(plus, he.hconj(conj, minus)), self.monomial(lvl, -1))
        out = self.linear_transform(F, pts_stc, rot)
        return out, lvl - 1, gain * s / float(he.q[0])
