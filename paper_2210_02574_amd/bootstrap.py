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


class DiagonalLayout:
    """A matrix on the packed slots whose non-zero diagonals lie on an arithmetic progression
    first + step * e, e = 0 .. count - 1 (offsets read in (-ns/2, ns/2]), cut into baby steps e mod baby and
    giant steps e // baby.  diag_d[j] = M[j][(j + d) mod ns]."""

    def __init__(self, M: np.ndarray):
        ns = M.shape[0]
        rows = np.arange(ns)
        present = [d for d in range(ns) if np.abs(M[rows, (rows + d) % ns]).max() > 1e-12]
        signed = sorted(d if d <= ns // 2 else d - ns for d in present)
        self.ns, self.present = ns, set(signed)
        self.first = signed[0]
        gaps = [d - self.first for d in signed[1:]]
        self.step = int(np.gcd.reduce(gaps)) if gaps else 1
        self.count = (signed[-1] - self.first) // self.step + 1
        self.baby = int(math.ceil(math.sqrt(self.count)))
        self.giant = -(-self.count // self.baby)

    def giant_shift(self, b: int) -> int:
        return self.first + self.step * self.baby * b

    def shifts(self) -> List[int]:
        return [self.step * a for a in range(1, self.baby)] + [self.giant_shift(b) for b in range(self.giant)]

    def slot_vectors(self, M: np.ndarray, n: int):
        """{(b, a): diagonal first + step (baby b + a) as a length-n slot vector, rotated right by giant_shift(b)}."""
        ns = self.ns
        rows = np.arange(ns)
        out = {}
        for b in range(self.giant):
            back = (rows - self.giant_shift(b)) % ns
            for a in range(self.baby):
                d = self.giant_shift(b) + self.step * a
                if d in self.present:
                    out[(b, a)] = np.tile(M[back, (back + d) % ns], n // ns)
        return out


class Bootstrapper:
    def __init__(self, he, ns: int, r: int = 8, level: int = None, groups: int = 1):
        """groups = 1: CoeffToSlot and SlotToCoeff are one dense ns x ns matrix each (one level each).
        groups >= 2: each is a product of that many sparse factors, groups of consecutive butterfly stages of
        the special FFT (one level per factor; far fewer rotations and plaintexts, and better precision because
        every factor's entries are large against the rounding of its encoding)."""
        assert ns >= 2 and ns & (ns - 1) == 0 and ns <= he.n
        self.he, self.ns, self.r, self.groups = he, ns, r, groups
        self.L = he.L if level is None else level
        self.gap = he.n // ns
        bits = ns.bit_length() - 1
        self.g1 = 1 << ((bits + 1) // 2)   # baby steps 0 .. g1-1
        self.g2 = ns // self.g1            # giant steps 0, g1, .. (g2-1) g1
        self.trace_shifts = [ns << k for k in range(self.gap.bit_length() - 1)]
        self.out_level = self.L - 5 - r - 2 * groups
        assert self.out_level >= 1, "not enough levels for this r"
        self._mono: Dict = {}
        self._pts: Dict = {}
        self._factors = None

    # ---- keys and plaintexts ----------------------------------------------------------------------------------

    def rotation_shifts(self) -> List[int]:
        if self.groups == 1:
            giant = [self.g1 * b for b in range(1, self.g2)]
            return sorted(set(self.trace_shifts) | set(range(1, self.g1)) | set(giant))
        shifts = set(self.trace_shifts)
        for G in self.factors():  # the inverse of a factor has the same diagonals
            shifts |= set(DiagonalLayout(G).shifts())
        shifts.discard(0)
        return sorted(shifts)

    def butterflies(self, length: int) -> np.ndarray:
        """Stage of the special FFT on blocks of `length`: (u, v) -> (u + D v, u - D v), D_j = exp(2 pi i 5^j / (4 length))."""
        ns, half = self.ns, length // 2
        B = np.zeros((ns, ns), dtype=np.complex128)
        tw = np.array([np.exp(0.5j * np.pi * pow(5, j, 4 * length) / length) for j in range(half)])
        for start in range(0, ns, length):
            top = np.arange(start, start + half)
            B[top, top] = 1.0
            B[top, top + half] = tw
            B[top + half, top] = 1.0
            B[top + half, top + half] = -tw
        return B

    def factors(self):
        """[G_1 .. G_groups] with U = G_groups .. G_1 R, R the bit-reversal permutation of the packed slots."""
        if self._factors is None:
            lengths = [2 << s for s in range(self.ns.bit_length() - 1)]
            per = -(-len(lengths) // self.groups)
            self._factors = []
            for g in range(self.groups):
                G = np.eye(self.ns, dtype=np.complex128)
                for ln in lengths[g * per:(g + 1) * per]:
                    G = self.butterflies(ln) @ G
                self._factors.append(G)
        return self._factors

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
        lvl = self.L - self.groups - 5
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

    def encode_sparse(self, M: np.ndarray, level: int):
        """(layout, {(b, a): device plaintext}) of a sparse-diagonal matrix at scale q_(level-1)."""
        he = self.he
        lay = DiagonalLayout(M)
        scale = float(he.q[level - 1])
        return lay, {k: self._plain(he.encode(v, scale), level) for k, v in lay.slot_vectors(M, he.n).items()}

    def prepare(self, gain: float = 1.0):
        """Encodes the plaintext diagonals of both matrix products once (they depend only on ns, r, the moduli
        and the gain of the last matrix)."""
        g, L = self.groups, self.L
        top = self.out_level + g  # level at which the way back starts
        if "cts" not in self._pts:
            if g == 1:
                self._pts["cts"] = self.encode_matrix(self.cts_matrix(), L)
            else:
                c = (math.pi / (self.gap * 2.0**self.r)) ** (1.0 / g)
                self._pts["cts"] = [self.encode_sparse(c * np.linalg.inv(G), L - (g - 1 - i))
                                    for i, G in enumerate(self.factors())]
            for lvl in (L - g, L - g - 5, top):
                for sign in (1, -1):
                    self.monomial(lvl, sign)
        if ("stc", gain) not in self._pts:
            if g == 1:
                self._pts[("stc", gain)] = self.encode_matrix(self.stc_matrix(gain), top)
            else:
                c = (gain / (4.0 * math.pi)) ** (1.0 / g)
                self._pts[("stc", gain)] = [self.encode_sparse(c * G, top - i) for i, G in enumerate(self.factors())]
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

    def _giant_steps(self, items, rot):
        """sum over items (shift, cts, pts) of Rotate(sum_k cts[k] pts[k], shift).  The rotations are independent,
        so the inner sums with a non-zero shift are written back to back and go through one call with one key
        each; modular addition makes the order of the outer sum immaterial."""
        he = self.he
        acc = None
        moving = [it for it in items if it[0] % he.n]
        for shift, cts, pts in items:
            if shift % he.n == 0:
                inner = he.pmult_sum(cts, pts)
                acc = inner if acc is None else he.add(acc, inner, out=acc)
        if moving:
            batch = he.empty_batch(len(moving), he._level(moving[0][1][0]))
            for k, (_, cts, pts) in enumerate(moving):
                he.pmult_sum(cts, pts, out=batch[k])
            rotated = he.hrot_batch_keys([rot[shift] for shift, _, _ in moving], batch)
            for k in range(len(moving)):
                acc = rotated[k] if acc is None else he.add(acc, rotated[k], out=acc)
        return acc

    def linear_transform(self, ct, pts, rot):
        """Matrix product on the packed slots (baby steps hoisted, giant steps in one call), then rescale."""
        he, g1 = self.he, self.g1
        babies = [ct] + (he.hrot_many([rot[a] for a in range(1, g1)], ct) if g1 > 1 else [])
        return he.rescale(self._giant_steps([(g1 * b, babies, pts[b]) for b in range(self.g2)], rot))

    def sparse_transform(self, ct, lay: DiagonalLayout, pts, rot):
        """Product with a sparse-diagonal matrix (baby steps hoisted, inner sums in one pass each, giant steps in
        one call), then rescale."""
        he = self.he
        used = [a for a in range(1, lay.baby) if any((b, a) in pts for b in range(lay.giant))]
        rotated = he.hrot_many([rot[lay.step * a] for a in used], ct) if used else []
        babies = {0: ct}
        babies.update(dict(zip(used, rotated)))
        items = []
        for b in range(lay.giant):
            terms = [a for a in range(lay.baby) if (b, a) in pts]
            if terms:
                items.append((lay.giant_shift(b), [babies[a] for a in terms], [pts[(b, a)] for a in terms]))
        return he.rescale(self._giant_steps(items, rot))

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
        g = self.groups
        ct = he.modraise(ct1, L)
        he.rotate_sum([rot[sh] for sh in self.trace_shifts], ct)
        scale = float(he.q[0])  # read as a ciphertext of t / q0
        if g == 1:
            w = self.linear_transform(ct, pts_cts, rot)
        else:
            # U^-1 = R^-1 G_1^-1 .. G_g^-1 without the permutation: the slots come out bit-reversed, which the
            # slot-wise middle part does not see and the way back (G_g .. G_1, again without R) undoes
            w = ct
            for lay, pts in reversed(pts_cts):
                w = self.sparse_transform(w, lay, pts, rot)
        wc = he.hconj(conj, w)
        th = torch.stack([he.add(w, wc), he.pmult(he.sub(w, wc), self.monomial(L - g, -1))])
        E, lvl, s = self.exp_i(relin, th, L - g, scale)
        iE2 = he.pmult(E[1], self.monomial(lvl, 1))
        plus, minus = he.add(E[0], iE2), he.sub(E[0], iE2)
        F = he.pmult(he.sub(plus, he.hconj(conj, minus)), self.monomial(lvl, -1))
        if g == 1:
            out = self.linear_transform(F, pts_stc, rot)
        else:
            out = F
            for lay, pts in pts_stc:
                out = self.sparse_transform(out, lay, pts, rot)
        return out, lvl - g, gain * s / float(he.q[0])
