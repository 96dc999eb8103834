"""Ciphertexts with their metadata.  The library leaves level and scale to the caller (a level is the number
of limbs of the device buffer, the scale a double that Mult multiplies and rescale divides by the dropped
prime, Section 2.2 of the paper); this thin wrapper carries both and keeps them consistent.  Every operation
is one or two calls of the device library."""
from __future__ import annotations

from typing import Dict, Optional, Sequence

import numpy as np


class Evaluator:
    """The public material an evaluating party holds: relinearisation key, rotation keys by shift, and
    optionally the conjugation key."""

    def __init__(self, he, relin=None, rot: Optional[Dict[int, object]] = None, conj=None):
        self.he, self.relin, self.rot, self.conj = he, relin, dict(rot or {}), conj

    @classmethod
    def generate(cls, he, sk, seed: int, shifts: Sequence[int] = (), with_conj: bool = False):
        rot = {r: he.keygen_rot(sk, r, seed + 2 + i) for i, r in enumerate(shifts)}
        return cls(he, he.keygen_relin(sk, seed), rot, he.keygen_conj(sk, seed + 1) if with_conj else None)

    def encrypt(self, sk, z, level: int, scale: float, seed: int) -> "Ciphertext":
        he = self.he
        return Ciphertext(self, he.to_device(he.encrypt_coeffs(sk, he.encode(z, scale), level, seed)), scale)

    def decrypt(self, sk, ct: "Ciphertext") -> np.ndarray:
        return self.he.decrypt(sk, self.he.to_host(ct.data), ct.scale)


class Ciphertext:
    """data: device tensor [2][level][N]; scale: the factor between slot values and the encoded integers."""

    SCALE_RTOL = 1e-9  # two scales this close count as equal (they differ by float rounding of the same formula)

    def __init__(self, ev: Evaluator, data, scale: float):
        self.ev, self.data, self.scale = ev, data, float(scale)

    @property
    def level(self) -> int:
        return int(self.data.shape[1])

    def _like(self, data, scale=None) -> "Ciphertext":
        return Ciphertext(self.ev, data, self.scale if scale is None else scale)

    def moddrop(self, level: int) -> "Ciphertext":
        return self if level == self.level else self._like(self.ev.he.moddrop(self.data, level))

    def _aligned(self, other: "Ciphertext"):
        level = min(self.level, other.level)
        return self.moddrop(level), other.moddrop(level)

    def _check_scale(self, other: "Ciphertext"):
        if abs(self.scale - other.scale) > self.SCALE_RTOL * self.scale:
            raise ValueError(f"scales differ: {self.scale!r} vs {other.scale!r}; bring them together with mul_const")

    def __add__(self, other: "Ciphertext") -> "Ciphertext":
        a, b = self._aligned(other)
        a._check_scale(b)
        return a._like(self.ev.he.add(a.data, b.data))

    def __sub__(self, other: "Ciphertext") -> "Ciphertext":
        a, b = self._aligned(other)
        a._check_scale(b)
        return a._like(self.ev.he.sub(a.data, b.data))

    def __mul__(self, other: "Ciphertext") -> "Ciphertext":
        """Mult of Section 2.2: slot-wise product, one level lower."""
        a, b = self._aligned(other)
        he = self.ev.he
        out = he.hmult_relin_rescale(self.ev.relin, a.data, b.data)
        return a._like(out, a.scale * b.scale / float(he.q[a.level - 1]))

    def mul_const(self, value: float, target_scale: Optional[float] = None) -> "Ciphertext":
        """Times a real constant, one level lower; the constant is encoded so that the result lands on
        target_scale (default: the scale this ciphertext has now)."""
        he = self.ev.he
        target = self.scale if target_scale is None else target_scale
        c_scale = target * float(he.q[self.level - 1]) / self.scale
        v = int(round(value * c_scale))
        out = he.rescale(he.cmult(self.data, [v % int(he.q[i]) for i in range(self.level)]))
        return self._like(out, target)

    def add_const(self, value: float) -> "Ciphertext":
        he = self.ev.he
        v = int(round(value * self.scale))
        return self._like(he.add_const(self.data, [v % int(he.q[i]) for i in range(self.level)]))

    def mul_plain(self, z) -> "Ciphertext":
        """Times a plaintext slot vector, one level lower, scale unchanged."""
        he = self.ev.he
        q_last = float(he.q[self.level - 1])
        pt = he.to_device(he.plain_to_ntt(he.encode(z, q_last), self.level))
        return self._like(he.rescale(he.pmult(self.data, pt)))

    def rotate(self, r: int) -> "Ciphertext":
        """Slot j of the result is slot j + r of this ciphertext."""
        if r % self.ev.he.n == 0:
            return self
        return self._like(self.ev.he.hrot(self.ev.rot[r], self.data))

    def conj(self) -> "Ciphertext":
        return self._like(self.ev.he.hconj(self.ev.conj, self.data))
