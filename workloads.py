"""Seeded synthetic inputs and parameter sets shared by the tests, the benchmark and the smoke check.

This module holds configuration data and random input generators only: none of the
scheme's arithmetic lives here.  Both the CPU oracle and the HIP library are fed
from these generators so that they see identical inputs.

Parameter sets follow the rule "the c largest primes congruent to 1 mod 2N below
2^b, in descending order" (checked against an independent primality routine in
the tests).  Moduli are written as 2^b - delta.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List

import numpy as np


@dataclass(frozen=True)
class Params:
    name: str
    logN: int
    q: tuple  # ciphertext primes q_0 .. q_{L-1}
    p: tuple  # special primes p_0 .. p_{K-1}
    dnum: int

    @property
    def N(self) -> int:
        return 1 << self.logN

    @property
    def L(self) -> int:
        return len(self.q)

    @property
    def K(self) -> int:
        return len(self.p)

    @property
    def alpha(self) -> int:
        return -(-self.L // self.dnum)

    @property
    def moduli(self) -> List[int]:
        return list(self.q) + list(self.p)


_C1_Q = tuple(2**40 - d for d in (147455, 237567, 368639))
_C1_P = (2**50 - 16383,)

_N16_Q = tuple(
    2**50 - d
    for d in (
        3014655, 4718591, 19529727, 20447231, 21102591, 22675455, 22806527, 23199743,
        23461887, 23855103, 27131903, 28966911, 36438015, 36831231, 40894463, 42336255,
        44826623, 45088767, 47579135, 54263807, 55312383, 60817407, 62128127, 63176703,
    )
)
_N16_P = tuple(2**60 - d for d in (262143, 8126463, 9830399, 10878975))

# Tiny configuration, as stated: N=2^12, three ~40-bit primes, one ~50-bit special prime, dnum=1.
C1 = Params("C1", 12, _C1_Q, _C1_P, 1)
# Same primes with one prime per digit (special modulus larger than every digit), used wherever
# a decrypted result has to be meaningful.
C1B = Params("C1B", 12, _C1_Q, _C1_P, 3)
# N=2^16, 24 ~50-bit primes, 4 ~60-bit special primes, dnum=6: the throughput configuration.
N16 = Params("N16", 16, _N16_Q, _N16_P, 6)
# The same prime chain on a small ring (the primes are 1 mod 2^17, hence 1 mod 2^13): 24 levels at N=2^12, deep
# enough to run a whole bootstrapping where the oracle finishes in seconds.
B12 = Params("B12", 12, _N16_Q, _N16_P, 6)
# The paper's ring degree (Section 3.1: N = 2^17, a 1540-bit modulus, level 29): 30 primes just below 2^50
# (1500 bits; 2^50 is the limit of the floating-point kernels), 4 special primes below 2^60, dnum = 8.
_P17_Q = tuple(
    2**50 - d
    for d in (
        4718591, 20447231, 22806527, 23855103, 36438015, 40894463, 44826623, 45088767, 54263807, 55312383,
        60817407, 62128127, 63176703, 64749567, 66322431, 72351743, 72613887, 75497471, 75759615, 78118911,
        84148223, 84410367, 84934655, 88080383, 89915391, 96206847, 99876863, 106954751, 110886911, 114294783,
    )
)
_P17_P = tuple(2**60 - d for d in (262143, 8126463, 14417919, 25427967))
P17 = Params("P17", 17, _P17_Q, _P17_P, 8)
# Small rings that put ciphertext primes on the integer path of the device kernels (2^50 and above): all three
# of I12; every other one of M12, where 55-bit and 45-bit primes alternate so that floating-point limbs take
# sources of 2^50 and above in both base conversions.
_W55 = tuple(2**55 - d for d in (311295, 434175, 696319))
_W45 = tuple(2**45 - d for d in (204799, 385023))
_W60 = tuple(2**60 - d for d in (16383, 98303))
I12 = Params("I12", 12, _W55, _W60[:1], 3)
M12 = Params("M12", 12, (_W55[0], _W45[0], _W55[1], _W45[1]), _W60, 2)
# Digits of six primes and five special primes (alpha = 6, K = 5): the base conversions then run in their
# forms for five to eight source limbs.
_W_P = _N16_P + (2**60 - 14417919,)
W12 = Params("W12", 12, _N16_Q[:12], _W_P, 2)
W16 = Params("W16", 16, _N16_Q[:12], _W_P, 2)
# Four more primes of the same rule: 28 levels, enough for one training iteration (9 levels), the division
# before bootstrapping (1), a bootstrapping with two-factor matrix products (16) and the level it starts from;
# dnum = 7 keeps 4 primes per digit.
_T_Q = _N16_Q + (2**50 - 64356351, 2**50 - 64749567, 2**50 - 65667071, 2**50 - 66322431)
T16 = Params("T16", 16, _T_Q, _N16_P, 7)
T12 = Params("T12", 12, _T_Q, _N16_P, 7)


def active_mod_idx(params: Params, level: int) -> List[int]:
    """Modulus indices of the level + K limbs a key switch works on."""
    return list(range(level)) + [params.L + k for k in range(params.K)]


def rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def uniform_limbs(seed: int, params: Params, mod_idx) -> np.ndarray:
    """[len(mod_idx)][N] uint64, limb b uniform in [0, modulus[mod_idx[b]])."""
    g = rng(seed)
    mods = params.moduli
    out = np.empty((len(mod_idx), params.N), dtype=np.uint64)
    for b, mi in enumerate(mod_idx):
        out[b] = g.integers(0, mods[mi], size=params.N, dtype=np.uint64)
    return out


def uniform_ct(seed: int, params: Params, level: int, comps: int = 2) -> np.ndarray:
    """[comps][level][N] uniform residues: a ciphertext-shaped buffer with no decryption meaning."""
    mi = list(range(level)) * comps
    return uniform_limbs(seed, params, mi).reshape(comps, level, params.N)


def uniform_evk(seed: int, params: Params) -> np.ndarray:
    """[dnum][2][L+K][N] uniform residues: a key-shaped buffer for throughput runs."""
    mi = list(range(params.L + params.K)) * (2 * params.dnum)
    return uniform_limbs(seed, params, mi).reshape(params.dnum, 2, params.L + params.K, params.N)


def slots_uniform(seed: int, n: int, lo: float = -1.0, hi: float = 1.0) -> np.ndarray:
    """n real slot values uniform in [lo, hi]."""
    return rng(seed).uniform(lo, hi, size=n)


def small_coeffs(seed: int, N: int, bound: int) -> np.ndarray:
    """int64[N] uniform in [-bound, bound]: an already-encoded plaintext polynomial."""
    return rng(seed).integers(-bound, bound + 1, size=N, dtype=np.int64)


def embeddings(seed: int, samples: int, dim: int = 768) -> np.ndarray:
    """Stand-in for sentence embeddings: fp64 N(0, 0.5^2) clipped to [-3, 3]."""
    return np.clip(rng(seed).normal(0.0, 0.5, size=(samples, dim)), -3.0, 3.0)


def weights(seed: int, classes: int = 4, dim: int = 768) -> np.ndarray:
    """Classifier weights: fp64 N(0, 0.05^2)."""
    return rng(seed).normal(0.0, 0.05, size=(classes, dim))


def mixed_levels(seed: int, count: int, lo: int = 8, hi: int = 24, max_log_offset: int = 14):
    """Levels uniform in [lo, hi] and rotation offsets uniform in {2^0 .. 2^max_log_offset}."""
    g = rng(seed)
    levels = g.integers(lo, hi + 1, size=count)
    offs = 1 << g.integers(0, max_log_offset + 1, size=count)
    return [int(v) for v in levels], [int(v) for v in offs]
