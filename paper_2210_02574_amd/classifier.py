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
        acc = he.pmult(ct, pts[0])
        for r, pt in zip(rots, pts[1:]):
            he.add(acc, he.pmult(r, pt), out=acc)
        out = he.rescale(acc)
        he.rotate_sum([keys[r] for r in INFER_SUM_SHIFTS], out)
        return out


def logits_from_slots(z: np.ndarray, classes: int = 4) -> np.ndarray:
    nb = z.shape[0] // BLOCK
    return np.stack([z[b * BLOCK: b * BLOCK + classes].real for b in range(nb)])
