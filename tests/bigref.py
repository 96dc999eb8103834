"""Big-integer reference helpers for the tests (Python ints, tiny sizes).

Written straight from the mathematical definitions so that the C oracle can be
pinned against something other than itself.
"""
from __future__ import annotations

import sympy


def ntt_primes(logN: int, bits: int, count: int):
    """The `count` largest primes congruent to 1 mod 2N below 2^bits, descending (sympy primality)."""
    twoN = 2 << logN
    out = []
    c = ((2**bits - 2) // twoN) * twoN + 1
    while len(out) < count and c > twoN:
        if sympy.isprime(c):
            out.append(c)
        c -= twoN
    return out


def brv(x: int, bits: int) -> int:
    r = 0
    for i in range(bits):
        r |= ((x >> i) & 1) << (bits - 1 - i)
    return r


def ntt_definition(a, psi: int, q: int, logN: int):
    """out[k] = sum_j a[j] * psi^((2*brv(k)+1)*j) mod q."""
    N = 1 << logN
    out = []
    for k in range(N):
        e = 2 * brv(k, logN) + 1
        x = pow(psi, e, q)
        out.append(sum(int(a[j]) * pow(x, j, q) for j in range(N)) % q)
    return out


def negacyclic_mul(a, b, q=None):
    """Schoolbook product in Z[X]/(X^N+1) (optionally mod q)."""
    N = len(a)
    out = [0] * N
    for i in range(N):
        ai = int(a[i])
        if ai == 0:
            continue
        for j in range(N):
            k = i + j
            if k < N:
                out[k] += ai * int(b[j])
            else:
                out[k - N] -= ai * int(b[j])
    if q is not None:
        out = [v % q for v in out]
    return out


def automorph(a, g: int):
    """a(X) -> a(X^g) in Z[X]/(X^N+1), on signed/plain integers."""
    N = len(a)
    out = [0] * N
    for j in range(N):
        e = (j * g) % (2 * N)
        if e < N:
            out[e] += int(a[j])
        else:
            out[e - N] -= int(a[j])
    return out


def crt(residues, moduli):
    """Integer in [0, prod moduli) with the given residues."""
    Q = 1
    for m in moduli:
        Q *= m
    v = 0
    for r, m in zip(residues, moduli):
        Qi = Q // m
        v += int(r) * Qi * pow(Qi, -1, m)
    return v % Q


def centre(v: int, Q: int) -> int:
    v %= Q
    return v - Q if v > Q // 2 else v


def prod(xs):
    r = 1
    for x in xs:
        r *= int(x)
    return r
