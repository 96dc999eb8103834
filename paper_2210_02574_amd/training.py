"""Encrypted training loop: the paper's recipe (Section 3.1: logistic regression on encrypted embeddings, the
logistic function as a polynomial, stochastic gradient descent with Nesterov momentum, Bootstrap to keep
going) as a sequence of library calls.

One iteration, per class, with the weights W at the level Bootstrap returns (l) and scale S:
  V' = W - (lr / n) sum_samples (p(<x, W>) - y) x        gradient step, eight levels (classifier.EncryptedTrainStep)
  W' = (1 + gamma) V' - gamma V                           Nesterov's update in its look-ahead form, one level
  W' <- W' / 2^6                                          one level, down to level 1: Bootstrap wants |m| << q0
  W  <- Bootstrap(W'), with the gain that lands on S      5 + r + 2 groups levels, back to level l
The divisor trades the two error sources of Bootstrap against each other: the sine's own error grows with
(|m| / q0)^3, while the rounding of the CoeffToSlot plaintexts is amplified by q0 / |m|; 2^6 with r = 7 keeps
both near 1e-4 for weights up to about 3 at 1024 packed slots.
The labels and samples stay at level l and scale S, so nothing else changes from one iteration to the next.
"""
from __future__ import annotations

import numpy as np

from .bootstrap import Bootstrapper
from .classifier import EncryptedTrainStep, _residues


class EncryptedTrainer:
    def __init__(self, he, block: int, lr: float, gamma: float, n_samples: int, scale: float = 2.0**50, r: int = 7,
                 coeffs=None, shrink_bits: int = 6, groups: int = 2, degree: int = 7):
        """degree: 7 (least squares on [-8, 8]) or 15 (the paper's minimax polynomial on [-12, 12], one more level)."""
        self.he, self.block, self.gamma, self.scale = he, block, gamma, scale
        self.boot = Bootstrapper(he, block, r, groups=groups)
        self.level = self.boot.out_level
        need = (9 if degree == 15 else 8) + 3
        assert self.level >= need, "the gradient step, the momentum update (1) and the division (1) end at level 1"
        self.step = EncryptedTrainStep(he, self.level, scale, lr, n_samples, coeffs, block, degree)
        self.shrink = int(round(he.q[1] / 2.0**shrink_bits))       # divides by ~2^shrink_bits when followed by a rescale
        self.delta_in = scale * self.shrink / float(he.q[1])       # scale of the ciphertext Bootstrap receives
        self.gain = self.boot.gain_for(self.delta_in, scale)

    def rotation_shifts(self):
        return sorted(set(self.step.rotation_shifts()) | set(self.boot.rotation_shifts()))

    def make_keys(self, sk, seed: int):
        he = self.he
        rot = {sh: he.keygen_rot(sk, sh, seed + 10 + i) for i, sh in enumerate(self.rotation_shifts())}
        return {"relin": he.keygen_relin(sk, seed), "conj": he.keygen_conj(sk, seed + 1), "rot": rot}

    def momentum(self, v_new, v_old):
        """(1 + gamma) v_new - gamma v_old, one level down, same scale."""
        he = self.he
        level = int(v_new.shape[1])
        q_drop = float(he.q[level - 1])
        a = he.cmult(v_new, _residues(1.0 + self.gamma, q_drop, he.q, level))
        b = he.cmult(he.moddrop(v_old, level) if int(v_old.shape[1]) > level else v_old,
                     _residues(self.gamma, q_drop, he.q, level))
        return he.rescale(he.sub(a, b, out=a))

    def refresh(self, keys, w, pts_cts=None, pts_stc=None):
        """Level >= 2, scale S -> level self.level, scale S."""
        he = self.he
        w2 = he.moddrop(w, 2) if int(w.shape[1]) > 2 else w
        small = he.rescale(he.cmult(w2, [self.shrink % int(he.q[0]), self.shrink % int(he.q[1])]))
        out, level, _ = self.boot.run(small, keys, pts_cts, pts_stc, gain=self.gain)
        assert level == self.level
        return out

    def iterate(self, keys, mask_pt, X, W, V, Y, boot_pts=(None, None)):
        """X: [n][2][level][N]; W, V: per class (V at the step's output level or above); Y: per class [n][2][label_level][N].
        Returns (W, V) of the next iteration."""
        v_new = self.step.run_batched(keys["relin"], keys["rot"], mask_pt, X, W, Y)
        w_new = [self.refresh(keys, self.momentum(vn, vo), *boot_pts) for vn, vo in zip(v_new, V)]
        return w_new, v_new

    def fit(self, keys, mask_pt, batches, W, V, epochs: int = 1, boot_pts=(None, None)):
        """Mini-batch stochastic gradient descent (Section 3.1): `epochs` passes over `batches`, a list of (X, Y)
        as for iterate(), each of the n_samples this trainer was built for; one Bootstrap per iteration and class.
        Returns the last (W, V)."""
        for _ in range(epochs):
            for X, Y in batches:
                W, V = self.iterate(keys, mask_pt, X, W, V, Y, boot_pts)
        return W, V
