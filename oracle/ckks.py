"""CPU oracle for the RNS-CKKS hot path -- test infrastructure only.

Thin ctypes front end over ``ckks_oracle.c`` (plain C, ``unsigned __int128``
products and ``%``), plus the two steps that are easier to read in Python:
the discrete-Gaussian threshold table (high-precision ``decimal``) and the CRT
reconstruction used by decryption (Python integers).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this package.  It shares no code with the HIP library and never imports it.

Conventions (the readings of the scheme are listed in the design document):
level = number of limbs; ciphertext ``[2][level][N]`` uint64 in the NTT domain
(bit-reversed evaluation order); switching key ``[dnum][2][L+K][N]``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from decimal import Decimal, getcontext

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ckks_oracle.c")
_LIB = os.path.join(_HERE, "libckks_oracle.so")

_u64p = ctypes.POINTER(ctypes.c_uint64)
_i64p = ctypes.POINTER(ctypes.c_int64)
_i8p = ctypes.POINTER(ctypes.c_int8)
_i32p = ctypes.POINTER(ctypes.c_int32)
_f64p = ctypes.POINTER(ctypes.c_double)


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP over independent limbs)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(
            ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-std=gnu11", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.orc_ctx_create.restype = ctypes.c_void_p
        lib.orc_ctx_create.argtypes = [ctypes.c_int, ctypes.c_int, _u64p, ctypes.c_int, _u64p, ctypes.c_int]
        lib.orc_modulus.restype = ctypes.c_uint64
        lib.orc_psi.restype = ctypes.c_uint64
        lib.orc_least_primitive_root.restype = ctypes.c_uint64
        lib.orc_least_primitive_root.argtypes = [ctypes.c_uint64]
        lib.orc_ntt_direct_at.restype = ctypes.c_uint64
        lib.orc_stream_word.restype = ctypes.c_uint64
        lib.orc_stream_word.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64]
        lib.orc_galois_element.restype = ctypes.c_uint64
        _lib = lib
    return _lib


def _p(a, ty):
    return a.ctypes.data_as(ty)


def gaussian_cdt(sigma: str = "3.2", tail: int = 19, prec: int = 120):
    """Cumulative thresholds of the discrete Gaussian on [-tail, tail]:
    C_i = floor(2^64 * sum_{t<=-tail+i} rho(t) / sum rho), rho(t)=exp(-t^2/(2 sigma^2)),
    for i = 0 .. 2*tail-1 (the last cumulative value, 2^64, is left out)."""
    getcontext().prec = prec
    s = Decimal(sigma)
    rho = [(-(Decimal(t) ** 2) / (2 * s * s)).exp() for t in range(-tail, tail + 1)]
    tot = sum(rho)
    out, acc = [], Decimal(0)
    for i in range(2 * tail):
        acc += rho[i]
        out.append(int((acc / tot * Decimal(2**64)).to_integral_value(rounding="ROUND_FLOOR")))
    return out


class Oracle:
    """One CKKS context: ring degree 2^logN, ciphertext primes q, special primes p, dnum digits."""

    def __init__(self, logN: int, q, p, dnum: int):
        lib = _load()
        self.lib = lib
        self.logN, self.N, self.n = logN, 1 << logN, 1 << (logN - 1)
        self.q, self.p = [int(x) for x in q], [int(x) for x in p]
        self.L, self.K, self.dnum = len(self.q), len(self.p), dnum
        self.M = self.L + self.K
        self.alpha = -(-self.L // dnum)
        qa = (ctypes.c_uint64 * self.L)(*self.q)
        pa = (ctypes.c_uint64 * self.K)(*self.p)
        self.ctx = ctypes.c_void_p(lib.orc_ctx_create(logN, self.L, qa, self.K, pa, dnum))
        self.moduli = self.q + self.p
        self.cdt = gaussian_cdt()
        lib.orc_set_cdt(self.ctx, (ctypes.c_uint64 * 38)(*self.cdt))

    def __del__(self):
        try:
            self.lib.orc_ctx_destroy(self.ctx)
        except Exception:
            pass

    # ---- tables -----------------------------------------------------------------
    def psi(self, mi: int) -> int:
        return int(self.lib.orc_psi(self.ctx, mi))

    def galois_element(self, r: int) -> int:
        return int(self.lib.orc_galois_element(self.ctx, ctypes.c_int64(r)))

    def active_moduli(self, level: int):
        return list(range(level)) + [self.L + k for k in range(self.K)]

    # ---- NTT --------------------------------------------------------------------
    def _mi(self, mod_idx, B):
        mi = np.ascontiguousarray(np.broadcast_to(np.asarray(mod_idx, dtype=np.int32), (B,)))
        return mi

    def ntt(self, limbs: np.ndarray, mod_idx) -> np.ndarray:
        a = np.array(limbs, dtype=np.uint64, copy=True).reshape(-1, self.N)
        mi = self._mi(mod_idx, a.shape[0])
        self.lib.orc_ntt_batch(self.ctx, _p(a, _u64p), _p(mi, _i32p), a.shape[0])
        return a.reshape(np.shape(limbs))

    def intt(self, limbs: np.ndarray, mod_idx) -> np.ndarray:
        a = np.array(limbs, dtype=np.uint64, copy=True).reshape(-1, self.N)
        mi = self._mi(mod_idx, a.shape[0])
        self.lib.orc_intt_batch(self.ctx, _p(a, _u64p), _p(mi, _i32p), a.shape[0])
        return a.reshape(np.shape(limbs))

    def ntt_direct_at(self, limb: np.ndarray, mod_idx: int, k: int) -> int:
        a = np.ascontiguousarray(limb, dtype=np.uint64)
        return int(self.lib.orc_ntt_direct_at(self.ctx, mod_idx, _p(a, _u64p), ctypes.c_uint64(k)))

    # ---- randomness ---------------------------------------------------------------
    def stream_word(self, seed: int, tag: int, i: int) -> int:
        return int(self.lib.orc_stream_word(seed, tag, i))

    def sample_uniform(self, seed: int, tag: int, q: int, n: int) -> np.ndarray:
        out = np.empty(n, dtype=np.uint64)
        self.lib.orc_sample_uniform(
            ctypes.c_uint64(seed), ctypes.c_uint64(tag), ctypes.c_uint64(q), _p(out, _u64p), ctypes.c_uint64(n)
        )
        return out

    def sample_ternary(self, seed: int, tag: int, n: int) -> np.ndarray:
        out = np.empty(n, dtype=np.int8)
        self.lib.orc_sample_ternary(ctypes.c_uint64(seed), ctypes.c_uint64(tag), _p(out, _i8p), ctypes.c_uint64(n))
        return out

    def sample_gauss(self, seed: int, tag: int, n: int) -> np.ndarray:
        out = np.empty(n, dtype=np.int8)
        self.lib.orc_sample_gauss(
            self.ctx, ctypes.c_uint64(seed), ctypes.c_uint64(tag), _p(out, _i8p), ctypes.c_uint64(n)
        )
        return out

    # ---- encode / decode ------------------------------------------------------------
    def encode(self, z, scale: float) -> np.ndarray:
        """Slots (length <= N/2, zero padded) -> integer coefficients (int64[N])."""
        z = np.asarray(z)
        re = np.zeros(self.n, dtype=np.float64)
        im = np.zeros(self.n, dtype=np.float64)
        re[: z.shape[0]] = z.real
        if np.iscomplexobj(z):
            im[: z.shape[0]] = z.imag
        out = np.empty(self.N, dtype=np.int64)
        self.lib.orc_encode(self.ctx, _p(re, _f64p), _p(im, _f64p), ctypes.c_double(scale), _p(out, _i64p))
        return out

    def decode(self, coeffs, scale: float) -> np.ndarray:
        m = np.ascontiguousarray(np.asarray(coeffs, dtype=np.float64))
        re = np.empty(self.n, dtype=np.float64)
        im = np.empty(self.n, dtype=np.float64)
        self.lib.orc_decode(self.ctx, _p(m, _f64p), ctypes.c_double(scale), _p(re, _f64p), _p(im, _f64p))
        return re + 1j * im

    def coeffs_to_ntt(self, coeffs, level: int) -> np.ndarray:
        """Integer polynomial -> NTT-domain plaintext [level][N] (residues of the signed coefficients)."""
        out = np.empty((level, self.N), dtype=np.uint64)
        c = [int(v) for v in np.asarray(coeffs).tolist()]
        for i in range(level):
            qi = self.q[i]
            out[i] = np.array([v % qi for v in c], dtype=np.uint64)
        return self.ntt(out, list(range(level)))

    # ---- keys -----------------------------------------------------------------------
    def keygen_secret(self, seed: int) -> np.ndarray:
        s = np.empty(self.N, dtype=np.int8)
        self.lib.orc_keygen_secret(self.ctx, ctypes.c_uint64(seed), _p(s, _i8p))
        return s

    def small_to_ntt(self, s: np.ndarray, mod_idx: int) -> np.ndarray:
        out = np.empty(self.N, dtype=np.uint64)
        s = np.ascontiguousarray(s, dtype=np.int8)
        self.lib.orc_small_to_ntt(self.ctx, mod_idx, _p(s, _i8p), _p(out, _u64p))
        return out

    def _keygen_switch(self, s, sp_ntt, seed):
        evk = np.empty((self.dnum, 2, self.M, self.N), dtype=np.uint64)
        s = np.ascontiguousarray(s, dtype=np.int8)
        sp = np.ascontiguousarray(sp_ntt, dtype=np.uint64)
        self.lib.orc_keygen_switch(self.ctx, _p(s, _i8p), _p(sp, _u64p), ctypes.c_uint64(seed), _p(evk, _u64p))
        return evk

    def keygen_relin(self, s: np.ndarray, seed: int) -> np.ndarray:
        """Switching key from s^2 to s."""
        sp = np.empty((self.L, self.N), dtype=np.uint64)
        for i in range(self.L):
            sp[i] = self._sq_limb(self.small_to_ntt(s, i), i)
        return self._keygen_switch(s, sp, seed)

    def _sq_limb(self, sh, i):
        mi = np.array([i], dtype=np.int32)
        out = np.empty_like(sh)
        self.lib.orc_limbwise(self.ctx, 2, _p(sh, _u64p), _p(sh, _u64p), _p(out, _u64p), _p(mi, _i32p), 1)
        return out

    def keygen_rot(self, s: np.ndarray, r: int, seed: int) -> np.ndarray:
        """Switching key from sigma_g(s) to s, g = 5^r mod 2N."""
        g = self.galois_element(r)
        s = np.ascontiguousarray(s, dtype=np.int8)
        sg = np.empty(self.N, dtype=np.int8)
        self.lib.orc_automorph_small(self.ctx, ctypes.c_uint64(g), _p(s, _i8p), _p(sg, _i8p))
        sp = np.stack([self.small_to_ntt(sg, i) for i in range(self.L)])
        return self._keygen_switch(s, sp, seed)

    def keygen_galois(self, s: np.ndarray, g: int, seed: int) -> np.ndarray:
        """Switching key from sigma_g(s) to s for any odd g."""
        s = np.ascontiguousarray(s, dtype=np.int8)
        sg = np.empty(self.N, dtype=np.int8)
        self.lib.orc_automorph_small(self.ctx, ctypes.c_uint64(g), _p(s, _i8p), _p(sg, _i8p))
        sp = np.stack([self.small_to_ntt(sg, i) for i in range(self.L)])
        return self._keygen_switch(s, sp, seed)

    def keygen_conj(self, s: np.ndarray, seed: int) -> np.ndarray:
        """Key for complex conjugation of the slots: the automorphism X -> X^(2N-1) = X^-1."""
        return self.keygen_galois(s, 2 * self.N - 1, seed)

    # ---- public-key encryption (stream kinds 6, 7: key; 8, 9, 10: encryption) -------------------------
    @staticmethod
    def _tag(kind: int, digit: int = 0, modidx: int = 0) -> int:
        return (kind << 32) | (digit << 16) | modidx

    def _mul_limb(self, a, b, i):
        mi = np.array([i], dtype=np.int32)
        out = np.empty(self.N, dtype=np.uint64)
        a = np.ascontiguousarray(a, dtype=np.uint64)
        b = np.ascontiguousarray(b, dtype=np.uint64)
        self.lib.orc_limbwise(self.ctx, 2, _p(a, _u64p), _p(b, _u64p), _p(out, _u64p), _p(mi, _i32p), 1)
        return out

    def keygen_public(self, s: np.ndarray, seed: int) -> np.ndarray:
        """pk = (b, a) on the L ciphertext moduli, NTT domain: a uniform, b = -a s + e, e Gaussian."""
        e = self.sample_gauss(seed, self._tag(7), self.N)
        pk = np.empty((2, self.L, self.N), dtype=np.uint64)
        for i in range(self.L):
            qi = self.q[i]
            a = self.sample_uniform(seed, self._tag(6, 0, i), qi, self.N)
            as_ = self._mul_limb(a, self.small_to_ntt(s, i), i)
            eh = self.small_to_ntt(e, i)
            pk[0, i] = (eh + (np.uint64(qi) - as_)) % np.uint64(qi)
            pk[1, i] = a
        return pk

    def encrypt_public_coeffs(self, pk: np.ndarray, coeffs, level: int, seed: int) -> np.ndarray:
        """c0 = v b + e0 + m, c1 = v a + e1 with v ternary, e0 and e1 Gaussian."""
        v = self.sample_ternary(seed, self._tag(8), self.N)
        e0 = self.sample_gauss(seed, self._tag(9), self.N)
        e1 = self.sample_gauss(seed, self._tag(10), self.N)
        m = [int(x) for x in np.asarray(coeffs).tolist()]
        ct = np.empty((2, level, self.N), dtype=np.uint64)
        for i in range(level):
            qi = self.q[i]
            vh = self.small_to_ntt(v, i)
            me = np.array([(m[k] + int(e0[k])) % qi for k in range(self.N)], dtype=np.uint64)
            meh = self.ntt(me[None, :], [i])[0]
            e1h = self.small_to_ntt(e1, i)
            ct[0, i] = (self._mul_limb(vh, pk[0, i], i) + meh) % np.uint64(qi)
            ct[1, i] = (self._mul_limb(vh, pk[1, i], i) + e1h) % np.uint64(qi)
        return ct

    # ---- encrypt / decrypt -------------------------------------------------------------
    def encrypt_coeffs(self, s: np.ndarray, coeffs: np.ndarray, level: int, seed: int) -> np.ndarray:
        ct = np.empty((2, level, self.N), dtype=np.uint64)
        s = np.ascontiguousarray(s, dtype=np.int8)
        m = np.ascontiguousarray(coeffs, dtype=np.int64)
        self.lib.orc_encrypt(self.ctx, _p(s, _i8p), _p(m, _i64p), level, ctypes.c_uint64(seed), _p(ct, _u64p))
        return ct

    def decrypt_residues(self, s: np.ndarray, ct: np.ndarray) -> np.ndarray:
        level = ct.shape[1]
        ct = np.ascontiguousarray(ct, dtype=np.uint64)
        s = np.ascontiguousarray(s, dtype=np.int8)
        out = np.empty((level, self.N), dtype=np.uint64)
        self.lib.orc_decrypt_residues(self.ctx, _p(s, _i8p), _p(ct, _u64p), level, _p(out, _u64p))
        return out

    def crt_centred(self, residues: np.ndarray):
        """CRT over all given limbs, centred lift in (-Q/2, Q/2]; list of Python ints."""
        level = residues.shape[0]
        qs = self.q[:level]
        Q = 1
        for v in qs:
            Q *= v
        terms = []
        for i, qi in enumerate(qs):
            Qi = Q // qi
            terms.append(Qi * pow(Qi, -1, qi))
        cols = [residues[i].tolist() for i in range(level)]
        out = []
        half = Q // 2
        for n in range(self.N):
            v = 0
            for i in range(level):
                v += cols[i][n] * terms[i]
            v %= Q
            if v > half:
                v -= Q
            out.append(v)
        return out

    def decrypt_coeffs(self, s: np.ndarray, ct: np.ndarray):
        """c0 + c1*s, iNTT, CRT over all limbs, centred: list of Python ints."""
        return self.crt_centred(self.decrypt_residues(s, ct))

    def decrypt(self, s: np.ndarray, ct: np.ndarray, scale: float) -> np.ndarray:
        m = np.array([float(v) for v in self.decrypt_coeffs(s, ct)], dtype=np.float64)
        return self.decode(m, scale)

    # ---- homomorphic ops ----------------------------------------------------------------
    def _limbwise(self, op, a, b):
        a = np.ascontiguousarray(a, dtype=np.uint64)
        b = np.ascontiguousarray(b, dtype=np.uint64)
        assert a.shape == b.shape and a.shape[0] == 2
        level = a.shape[1]
        mi = np.array(list(range(level)) * 2, dtype=np.int32)
        out = np.empty_like(a)
        self.lib.orc_limbwise(self.ctx, op, _p(a, _u64p), _p(b, _u64p), _p(out, _u64p), _p(mi, _i32p), 2 * level)
        return out

    def add(self, a, b):
        return self._limbwise(0, a, b)

    def sub(self, a, b):
        return self._limbwise(1, a, b)

    def pmult(self, ct, pt_ntt):
        ct = np.ascontiguousarray(ct, dtype=np.uint64)
        pt = np.ascontiguousarray(pt_ntt, dtype=np.uint64)
        level = ct.shape[1]
        assert pt.shape == (level, self.N)
        out = np.empty_like(ct)
        self.lib.orc_pmult(self.ctx, _p(ct, _u64p), _p(pt, _u64p), level, _p(out, _u64p))
        return out

    def cmult(self, ct, scalars):
        ct = np.ascontiguousarray(ct, dtype=np.uint64)
        level = ct.shape[1]
        sc = np.array([int(v) for v in scalars], dtype=np.uint64)
        assert sc.shape == (level,)
        out = np.empty_like(ct)
        self.lib.orc_cmult(self.ctx, _p(ct, _u64p), _p(sc, _u64p), level, _p(out, _u64p))
        return out

    def add_const(self, ct, scalars):
        ct = np.ascontiguousarray(ct, dtype=np.uint64)
        level = ct.shape[1]
        sc = np.array([int(v) for v in scalars], dtype=np.uint64)
        assert sc.shape == (level,)
        out = np.empty_like(ct)
        self.lib.orc_add_const(self.ctx, _p(ct, _u64p), _p(sc, _u64p), level, _p(out, _u64p))
        return out

    @staticmethod
    def moddrop(ct, level):
        """Keep the first `level` limbs of both components."""
        return np.ascontiguousarray(ct[:, :level])

    def tensor(self, a, b):
        a = np.ascontiguousarray(a, dtype=np.uint64)
        b = np.ascontiguousarray(b, dtype=np.uint64)
        level = a.shape[1]
        out = np.empty((3, level, self.N), dtype=np.uint64)
        self.lib.orc_tensor(self.ctx, _p(a, _u64p), _p(b, _u64p), level, _p(out, _u64p))
        return out

    def set_exact(self, exact: bool):
        """Selects the corrected base conversions (ModUp to [x]_D, ModDown to the rounded quotient) for every
        key switch of this context; off by default."""
        self.lib.orc_set_exact(self.ctx, 1 if exact else 0)

    def modup(self, x_coeff):
        x = np.ascontiguousarray(x_coeff, dtype=np.uint64)
        level = x.shape[0]
        beta = -(-level // self.alpha)
        out = np.empty((beta, level + self.K, self.N), dtype=np.uint64)
        self.lib.orc_modup(self.ctx, _p(x, _u64p), level, _p(out, _u64p))
        return out

    def moddown(self, u_ntt, level):
        u = np.ascontiguousarray(u_ntt, dtype=np.uint64)
        assert u.shape == (level + self.K, self.N)
        out = np.empty((level, self.N), dtype=np.uint64)
        self.lib.orc_moddown(self.ctx, _p(u, _u64p), level, _p(out, _u64p))
        return out

    def automorph_coeff(self, limb, mod_idx, g):
        a = np.ascontiguousarray(limb, dtype=np.uint64)
        out = np.empty_like(a)
        self.lib.orc_automorph_coeff(self.ctx, mod_idx, ctypes.c_uint64(g), _p(a, _u64p), _p(out, _u64p))
        return out

    def keyswitch(self, d, evk, g: int = 1, want_intermediates: bool = False):
        d = np.ascontiguousarray(d, dtype=np.uint64)
        evk = np.ascontiguousarray(evk, dtype=np.uint64)
        level = d.shape[0]
        beta = -(-level // self.alpha)
        k = np.empty((2, level, self.N), dtype=np.uint64)
        raised = u = None
        rp = up = None
        if want_intermediates:
            raised = np.empty((beta, level + self.K, self.N), dtype=np.uint64)
            u = np.empty((2, level + self.K, self.N), dtype=np.uint64)
            rp, up = _p(raised, _u64p), _p(u, _u64p)
        self.lib.orc_keyswitch(
            self.ctx, _p(d, _u64p), level, _p(evk, _u64p), ctypes.c_uint64(g), _p(k[0], _u64p), _p(k[1], _u64p), rp, up
        )
        if want_intermediates:
            return k, raised, u
        return k

    def hmult_relin(self, a, b, evk):
        a = np.ascontiguousarray(a, dtype=np.uint64)
        b = np.ascontiguousarray(b, dtype=np.uint64)
        evk = np.ascontiguousarray(evk, dtype=np.uint64)
        level = a.shape[1]
        out = np.empty_like(a)
        self.lib.orc_hmult_relin(self.ctx, _p(a, _u64p), _p(b, _u64p), level, _p(evk, _u64p), _p(out, _u64p))
        return out

    def rescale(self, ct):
        ct = np.ascontiguousarray(ct, dtype=np.uint64)
        level = ct.shape[1]
        assert level >= 2
        out = np.empty((2, level - 1, self.N), dtype=np.uint64)
        self.lib.orc_rescale(self.ctx, _p(ct, _u64p), level, _p(out, _u64p))
        return out

    def hrot(self, ct, evk, r: int):
        """Left rotation of the slot vector by r: out_slot[j] = in_slot[(j+r) mod n]."""
        ct = np.ascontiguousarray(ct, dtype=np.uint64)
        evk = np.ascontiguousarray(evk, dtype=np.uint64)
        level = ct.shape[1]
        out = np.empty_like(ct)
        g = self.galois_element(r)
        self.lib.orc_hrot(self.ctx, _p(ct, _u64p), level, _p(evk, _u64p), ctypes.c_uint64(g), _p(out, _u64p))
        return out

    def hconj(self, ct, evk):
        """Complex conjugation of every slot (key from keygen_conj)."""
        ct = np.ascontiguousarray(ct, dtype=np.uint64)
        evk = np.ascontiguousarray(evk, dtype=np.uint64)
        out = np.empty_like(ct)
        self.lib.orc_hrot(self.ctx, _p(ct, _u64p), ct.shape[1], _p(evk, _u64p), ctypes.c_uint64(2 * self.N - 1),
                          _p(out, _u64p))
        return out

    def rotate_sum(self, ct, evks, shift0: int):
        """for k < len(evks): ct <- ct + HRot(ct, shift0 * 2^k); evks[k] is the key for that shift."""
        for k, evk in enumerate(evks):
            ct = self.add(ct, self.hrot(ct, evk, shift0 << k))
        return ct
