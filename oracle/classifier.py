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
