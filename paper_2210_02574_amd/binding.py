"""ctypes binding of the C ABI declared in include/he.h.

Argument marshalling only: every computation runs inside the shared library.  Device buffers
are torch int64 tensors on the GPU (their bits are the uint64 residues); host buffers are
numpy arrays.  The library is loaded from the package directory and a missing build is an
error, never a fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhe_gfx950.so")

HE_OK = 0
ERRORS = {
    -1: "HE_EINVAL", -2: "HE_ELEVEL", -3: "HE_ENOKEY", -4: "HE_EWORKSPACE",
    -5: "HE_EHIP", -6: "HE_ENODEV", -7: "HE_ENOMEM", -8: "HE_ESCRATCH",
}

# every symbol include/he.h declares
SYMBOLS = [
    "he_ctx_create", "he_ctx_destroy", "he_strerror", "he_last_hip_error", "he_ctx_modulus",
    "he_galois_element", "he_gauss_cdt", "he_workspace_bytes", "he_ctx_set_conversion",
    "he_keygen_secret", "he_sk_destroy", "he_sk_coeffs", "he_keygen_relin", "he_keygen_rot",
    "he_keygen_conj", "he_keygen_public", "he_encrypt_public_coeffs", "he_keygen_secret_sparse", "he_modraise", "he_pmult_sum",
    "he_evk_from_host", "he_evk_to_host", "he_evk_destroy",
    "he_encode", "he_decode", "he_plain_to_ntt", "he_encrypt_coeffs", "he_decrypt_coeffs", "he_decrypt",
    "he_ntt", "he_intt", "he_add", "he_sub", "he_pmult", "he_cmult", "he_add_const", "he_moddrop",
    "he_hmult_relin", "he_hmult_relin_rescale", "he_rescale", "he_hrot", "he_hrot_many", "he_rotate_sum",
    "he_add_batch", "he_sub_batch", "he_pmult_batch", "he_cmult_batch", "he_add_const_batch", "he_moddrop_batch",
    "he_hmult_relin_batch", "he_hmult_relin_rescale_batch", "he_rescale_batch", "he_hrot_batch", "he_hrot_batch_keys", "he_hrot_batch_levels", "he_rotate_sum_batch",
    "he_hrot_noalloc",
    "he_profile_start", "he_profile_stop",
]


class HeError(RuntimeError):
    def __init__(self, code: int, where: str, detail: str = ""):
        self.code = code
        super().__init__(f"{where}: {ERRORS.get(code, code)}" + (f" ({detail})" if detail else ""))


class he_kernel_stat(ctypes.Structure):
    _fields_ = [
        ("name", ctypes.c_char * 48), ("launches", ctypes.c_int64), ("total_ms", ctypes.c_double),
        ("bytes", ctypes.c_double),
    ]


class he_params(ctypes.Structure):
    _fields_ = [
        ("logN", ctypes.c_int32), ("L", ctypes.c_int32), ("K", ctypes.c_int32), ("dnum", ctypes.c_int32),
        ("q", ctypes.POINTER(ctypes.c_uint64)), ("p", ctypes.POINTER(ctypes.c_uint64)),
    ]


_lib = None


def load_library() -> ctypes.CDLL:
    """Loads the in-tree HIP library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2210_02574_amd.build` "
                "(hipcc --offload-arch=gfx950); there is no fallback path"
            )
        from .build import is_stale

        if is_stale() and not os.environ.get("HE_ALLOW_STALE_LIB"):
            raise ImportError(
                f"{LIB_PATH} was built from other sources than the present ones: rebuild it with "
                "`python -m paper_2210_02574_amd.build` (or set HE_ALLOW_STALE_LIB=1 to load it anyway)"
            )
        # torch first: it brings its own HIP runtime, and a process must not end up with the system's runtime
        # initialised by this library and torch's by torch (the second one then finds no GPU)
        import torch  # noqa: F401

        lib = ctypes.CDLL(LIB_PATH)
        vp, i32, u64, sz, dbl = ctypes.c_void_p, ctypes.c_int32, ctypes.c_uint64, ctypes.c_size_t, ctypes.c_double
        sig = {
            "he_ctx_create": [ctypes.POINTER(he_params), i32, ctypes.POINTER(vp)],
            "he_ctx_destroy": [vp],
            "he_strerror": [i32],
            "he_last_hip_error": [vp],
            "he_ctx_modulus": [vp, i32, ctypes.POINTER(u64), ctypes.POINTER(u64)],
            "he_ctx_set_conversion": [vp, i32],
            "he_galois_element": [vp, i32, ctypes.POINTER(u64)],
            "he_gauss_cdt": [vp],
            "he_workspace_bytes": [vp, i32, i32, ctypes.POINTER(sz)],
            "he_keygen_secret": [vp, u64, ctypes.POINTER(vp)],
            "he_sk_destroy": [vp],
            "he_sk_coeffs": [vp, vp],
            "he_keygen_relin": [vp, vp, u64, ctypes.POINTER(vp)],
            "he_keygen_rot": [vp, vp, i32, u64, ctypes.POINTER(vp)],
            "he_keygen_conj": [vp, vp, u64, ctypes.POINTER(vp)],
            "he_keygen_secret_sparse": [vp, u64, i32, ctypes.POINTER(vp)],
            "he_modraise": [vp, vp, vp, i32, vp, sz, vp],
            "he_pmult_sum": [vp, vp, vp, i32, vp, i32, vp],
            "he_keygen_public": [vp, vp, u64, vp],
            "he_encrypt_public_coeffs": [vp, vp, vp, i32, u64, vp],
            "he_evk_from_host": [vp, vp, u64, ctypes.POINTER(vp)],
            "he_evk_to_host": [vp, vp],
            "he_evk_destroy": [vp],
            "he_encode": [vp, vp, vp, i32, dbl, vp],
            "he_decode": [vp, vp, dbl, vp, vp],
            "he_plain_to_ntt": [vp, vp, i32, vp],
            "he_encrypt_coeffs": [vp, vp, vp, i32, u64, vp],
            "he_decrypt_coeffs": [vp, vp, vp, i32, vp],
            "he_decrypt": [vp, vp, vp, i32, dbl, vp, vp],
            "he_ntt": [vp, vp, vp, i32, vp],
            "he_intt": [vp, vp, vp, i32, vp],
            "he_add": [vp, vp, vp, vp, i32, vp],
            "he_sub": [vp, vp, vp, vp, i32, vp],
            "he_pmult": [vp, vp, vp, vp, i32, vp],
            "he_cmult": [vp, vp, vp, vp, i32, vp],
            "he_add_const": [vp, vp, vp, vp, i32, vp],
            "he_moddrop": [vp, vp, i32, vp, i32, vp],
            "he_hmult_relin": [vp, vp, vp, vp, vp, i32, vp, sz, vp],
            "he_hmult_relin_rescale": [vp, vp, vp, vp, vp, i32, vp, sz, vp],
            "he_rescale": [vp, vp, vp, i32, vp, sz, vp],
            "he_hrot": [vp, vp, vp, vp, i32, vp, sz, vp],
            "he_hrot_noalloc": [vp, vp, vp, vp, i32, vp],
            "he_hrot_many": [vp, vp, i32, vp, vp, i32, vp, sz, vp],
            "he_rotate_sum": [vp, vp, i32, vp, i32, vp, sz, vp],
            "he_add_batch": [vp, vp, vp, vp, i32, i32, vp],
            "he_sub_batch": [vp, vp, vp, vp, i32, i32, vp],
            "he_pmult_batch": [vp, vp, vp, vp, i32, i32, vp],
            "he_cmult_batch": [vp, vp, vp, vp, i32, i32, vp],
            "he_add_const_batch": [vp, vp, vp, vp, i32, i32, vp],
            "he_moddrop_batch": [vp, vp, i32, vp, i32, i32, vp],
            "he_hmult_relin_batch": [vp, vp, vp, vp, vp, i32, i32, vp, sz, vp],
            "he_hmult_relin_rescale_batch": [vp, vp, vp, vp, vp, i32, i32, vp, sz, vp],
            "he_rescale_batch": [vp, vp, vp, i32, i32, vp, sz, vp],
            "he_hrot_batch": [vp, vp, vp, vp, i32, i32, vp, sz, vp],
            "he_hrot_batch_keys": [vp, vp, vp, vp, i32, i32, vp, sz, vp],
            "he_hrot_batch_levels": [vp, vp, vp, vp, vp, i32, vp, sz, vp],
            "he_rotate_sum_batch": [vp, vp, i32, vp, i32, i32, vp, sz, vp],
            "he_profile_start": [vp],
            "he_profile_stop": [vp, vp, i32, ctypes.POINTER(i32)],
        }
        for name in SYMBOLS:
            fn = getattr(lib, name)
            fn.argtypes = sig[name]
            fn.restype = i32
        lib.he_strerror.restype = ctypes.c_char_p
        lib.he_last_hip_error.restype = ctypes.c_char_p
        for name in ("he_ctx_destroy", "he_sk_destroy", "he_evk_destroy"):
            getattr(lib, name).restype = None
        _lib = lib
    return _lib


def _hp(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


class SecretKey:
    def __init__(self, he, handle):
        self.he, self.handle = he, handle

    def coeffs(self) -> np.ndarray:
        out = np.empty(self.he.N, dtype=np.int8)
        self.he._chk(self.he.lib.he_sk_coeffs(self.handle, _hp(out)), "he_sk_coeffs")
        return out

    def __del__(self):
        try:
            self.he.lib.he_sk_destroy(self.handle)
        except Exception:
            pass


class EvalKey:
    def __init__(self, he, handle):
        self.he, self.handle = he, handle

    def to_host(self) -> np.ndarray:
        he = self.he
        out = np.empty((he.dnum, 2, he.M, he.N), dtype=np.uint64)
        he._chk(he.lib.he_evk_to_host(self.handle, _hp(out)), "he_evk_to_host")
        return out

    def __del__(self):
        try:
            self.he.lib.he_evk_destroy(self.handle)
        except Exception:
            pass


class HE:
    """One library context.  device = -1: host functions only; device >= 0: that GPU."""

    def __init__(self, logN: int, q: Sequence[int], p: Sequence[int], dnum: int, device: int = -1):
        self.lib = load_library()
        self.logN, self.N, self.n = logN, 1 << logN, 1 << (logN - 1)
        self.q, self.p = [int(v) for v in q], [int(v) for v in p]
        self.L, self.K, self.M, self.dnum = len(self.q), len(self.p), len(self.q) + len(self.p), dnum
        self.alpha = -(-self.L // dnum)
        self.device = device
        self._qa = (ctypes.c_uint64 * self.L)(*self.q)
        self._pa = (ctypes.c_uint64 * self.K)(*self.p)
        prm = he_params(logN, self.L, self.K, dnum, self._qa, self._pa)
        h = ctypes.c_void_p()
        if device >= 0:
            import torch

            torch.cuda.init()  # torch owns device memory and streams: its runtime comes up before the library's
        rc = self.lib.he_ctx_create(ctypes.byref(prm), device, ctypes.byref(h))
        if rc != HE_OK:
            raise HeError(rc, "he_ctx_create")
        self.ctx = h
        self._ws = None

    @classmethod
    def from_params(cls, params, device: int = -1):
        return cls(params.logN, params.q, params.p, params.dnum, device)

    def __del__(self):
        try:
            self._ws = None
            self.lib.he_ctx_destroy(self.ctx)
        except Exception:
            pass

    def _chk(self, rc: int, where: str):
        if rc != HE_OK:
            detail = self.lib.he_last_hip_error(self.ctx).decode() if rc == -5 else ""
            raise HeError(rc, where, detail)

    # ---- context queries --------------------------------------------------------------------
    def modulus(self, i: int):
        m, psi = ctypes.c_uint64(), ctypes.c_uint64()
        self._chk(self.lib.he_ctx_modulus(self.ctx, i, ctypes.byref(m), ctypes.byref(psi)), "he_ctx_modulus")
        return int(m.value), int(psi.value)

    def set_exact_conversion(self, exact: bool):
        """Selects the corrected base conversions (True) or the fast ones (False, the default) for later calls."""
        self._chk(self.lib.he_ctx_set_conversion(self.ctx, 1 if exact else 0), "he_ctx_set_conversion")

    def galois_element(self, r: int) -> int:
        g = ctypes.c_uint64()
        self._chk(self.lib.he_galois_element(self.ctx, r, ctypes.byref(g)), "he_galois_element")
        return int(g.value)

    def gauss_cdt(self) -> List[int]:
        out = np.empty(38, dtype=np.uint64)
        self._chk(self.lib.he_gauss_cdt(_hp(out)), "he_gauss_cdt")
        return [int(v) for v in out]

    def workspace_bytes(self, level: int, count: int = 1) -> int:
        out = ctypes.c_size_t()
        self._chk(self.lib.he_workspace_bytes(self.ctx, level, count, ctypes.byref(out)), "he_workspace_bytes")
        return int(out.value)

    # ---- host: keys ----------------------------------------------------------------------------
    def keygen_secret(self, seed: int) -> SecretKey:
        h = ctypes.c_void_p()
        self._chk(self.lib.he_keygen_secret(self.ctx, seed, ctypes.byref(h)), "he_keygen_secret")
        return SecretKey(self, h)

    def keygen_secret_sparse(self, seed: int, h: int) -> SecretKey:
        """Secret with exactly h non-zero coefficients (bootstrapping)."""
        hd = ctypes.c_void_p()
        self._chk(self.lib.he_keygen_secret_sparse(self.ctx, seed, h, ctypes.byref(hd)), "he_keygen_secret_sparse")
        return SecretKey(self, hd)

    def keygen_relin(self, sk: SecretKey, seed: int) -> EvalKey:
        h = ctypes.c_void_p()
        self._chk(self.lib.he_keygen_relin(self.ctx, sk.handle, seed, ctypes.byref(h)), "he_keygen_relin")
        return EvalKey(self, h)

    def keygen_rot(self, sk: SecretKey, r: int, seed: int) -> EvalKey:
        h = ctypes.c_void_p()
        self._chk(self.lib.he_keygen_rot(self.ctx, sk.handle, r, seed, ctypes.byref(h)), "he_keygen_rot")
        return EvalKey(self, h)

    def keygen_conj(self, sk: SecretKey, seed: int) -> EvalKey:
        """Key of slot-wise complex conjugation; apply it with hrot / hconj."""
        h = ctypes.c_void_p()
        self._chk(self.lib.he_keygen_conj(self.ctx, sk.handle, seed, ctypes.byref(h)), "he_keygen_conj")
        return EvalKey(self, h)

    def keygen_public(self, sk: SecretKey, seed: int) -> np.ndarray:
        pk = np.empty((2, self.L, self.N), dtype=np.uint64)
        self._chk(self.lib.he_keygen_public(self.ctx, sk.handle, seed, _hp(pk)), "he_keygen_public")
        return pk

    def encrypt_public_coeffs(self, pk: np.ndarray, coeffs: np.ndarray, level: int, seed: int) -> np.ndarray:
        pk = np.ascontiguousarray(pk, dtype=np.uint64)
        assert pk.shape == (2, self.L, self.N)
        m = np.ascontiguousarray(coeffs, dtype=np.int64)
        assert m.shape == (self.N,)
        out = np.empty((2, level, self.N), dtype=np.uint64)
        self._chk(self.lib.he_encrypt_public_coeffs(self.ctx, _hp(pk), _hp(m), level, seed, _hp(out)),
                  "he_encrypt_public_coeffs")
        return out

    def evk_from_host(self, evk: np.ndarray, g: int = 1) -> EvalKey:
        evk = np.ascontiguousarray(evk, dtype=np.uint64)
        assert evk.shape == (self.dnum, 2, self.M, self.N)
        h = ctypes.c_void_p()
        self._chk(self.lib.he_evk_from_host(self.ctx, _hp(evk), g, ctypes.byref(h)), "he_evk_from_host")
        return EvalKey(self, h)

    # ---- host: encode / encrypt / decrypt -----------------------------------------------------------
    def encode(self, z, scale: float) -> np.ndarray:
        z = np.asarray(z)
        re = np.ascontiguousarray(z.real, dtype=np.float64)
        im = np.ascontiguousarray(z.imag, dtype=np.float64) if np.iscomplexobj(z) else None
        out = np.empty(self.N, dtype=np.int64)
        self._chk(
            self.lib.he_encode(self.ctx, _hp(re), _hp(im) if im is not None else None, re.shape[0], scale, _hp(out)),
            "he_encode",
        )
        return out

    def decode(self, coeffs, scale: float) -> np.ndarray:
        m = np.ascontiguousarray(coeffs, dtype=np.float64)
        re, im = np.empty(self.n), np.empty(self.n)
        self._chk(self.lib.he_decode(self.ctx, _hp(m), scale, _hp(re), _hp(im)), "he_decode")
        return re + 1j * im

    def plain_to_ntt(self, coeffs: np.ndarray, level: int) -> np.ndarray:
        m = np.ascontiguousarray(coeffs, dtype=np.int64)
        out = np.empty((level, self.N), dtype=np.uint64)
        self._chk(self.lib.he_plain_to_ntt(self.ctx, _hp(m), level, _hp(out)), "he_plain_to_ntt")
        return out

    def encrypt_coeffs(self, sk: SecretKey, coeffs: np.ndarray, level: int, seed: int) -> np.ndarray:
        m = np.ascontiguousarray(coeffs, dtype=np.int64)
        assert m.shape == (self.N,)
        out = np.empty((2, level, self.N), dtype=np.uint64)
        self._chk(self.lib.he_encrypt_coeffs(self.ctx, sk.handle, _hp(m), level, seed, _hp(out)), "he_encrypt_coeffs")
        return out

    def decrypt_coeffs(self, sk: SecretKey, ct: np.ndarray) -> np.ndarray:
        ct = np.ascontiguousarray(ct, dtype=np.uint64)
        level = ct.shape[1]
        out = np.empty(self.N, dtype=np.float64)
        self._chk(self.lib.he_decrypt_coeffs(self.ctx, sk.handle, _hp(ct), level, _hp(out)), "he_decrypt_coeffs")
        return out

    def decrypt(self, sk: SecretKey, ct: np.ndarray, scale: float) -> np.ndarray:
        ct = np.ascontiguousarray(ct, dtype=np.uint64)
        level = ct.shape[1]
        re, im = np.empty(self.n), np.empty(self.n)
        self._chk(self.lib.he_decrypt(self.ctx, sk.handle, _hp(ct), level, scale, _hp(re), _hp(im)), "he_decrypt")
        return re + 1j * im

    # ---- device plumbing (torch: memory and streams only) ----------------------------------------------
    def to_device(self, a: np.ndarray):
        import torch

        a = np.ascontiguousarray(a, dtype=np.uint64)
        return torch.from_numpy(a.view(np.int64)).to(f"cuda:{self.device}")

    @staticmethod
    def to_host(t) -> np.ndarray:
        return t.detach().cpu().contiguous().numpy().view(np.uint64)

    def empty_ct(self, level: int):
        import torch

        return torch.empty((2, level, self.N), dtype=torch.int64, device=f"cuda:{self.device}")

    def _stream(self):
        import torch

        return ctypes.c_void_p(torch.cuda.current_stream(self.device).cuda_stream)

    def _workspace(self, level: int, count: int = 1):
        """One workspace per stream: calls enqueued on different streams may run concurrently."""
        import torch

        need = self.workspace_bytes(level, count)
        key = torch.cuda.current_stream(self.device).cuda_stream
        if self._ws is None:
            self._ws = {}
        ws = self._ws.get(key)
        if ws is None or ws.numel() * 8 < need:
            self._ws[key] = None
            ws = self._ws[key] = torch.empty(need // 8, dtype=torch.int64, device=f"cuda:{self.device}")
        return ctypes.c_void_p(ws.data_ptr()), ws.numel() * 8

    @staticmethod
    def _dp(t):
        assert t.is_cuda and t.is_contiguous() and t.element_size() == 8
        return ctypes.c_void_p(t.data_ptr())

    # ---- device: polynomial arithmetic --------------------------------------------------------------------
    def ntt(self, limbs, mod_idx: Sequence[int]):
        mi = np.ascontiguousarray(mod_idx, dtype=np.int32)
        assert limbs.numel() == mi.shape[0] * self.N
        self._chk(self.lib.he_ntt(self.ctx, self._dp(limbs), _hp(mi), mi.shape[0], self._stream()), "he_ntt")
        return limbs

    def intt(self, limbs, mod_idx: Sequence[int]):
        mi = np.ascontiguousarray(mod_idx, dtype=np.int32)
        assert limbs.numel() == mi.shape[0] * self.N
        self._chk(self.lib.he_intt(self.ctx, self._dp(limbs), _hp(mi), mi.shape[0], self._stream()), "he_intt")
        return limbs

    def _level(self, ct) -> int:
        assert ct.dim() == 3 and ct.shape[0] == 2 and ct.shape[2] == self.N
        return int(ct.shape[1])

    def add(self, a, b, out=None):
        level = self._level(a)
        assert b.shape == a.shape
        out = self.empty_ct(level) if out is None else out
        self._chk(self.lib.he_add(self.ctx, self._dp(a), self._dp(b), self._dp(out), level, self._stream()), "he_add")
        return out

    def sub(self, a, b, out=None):
        level = self._level(a)
        assert b.shape == a.shape
        out = self.empty_ct(level) if out is None else out
        self._chk(self.lib.he_sub(self.ctx, self._dp(a), self._dp(b), self._dp(out), level, self._stream()), "he_sub")
        return out

    def pmult(self, ct, pt, out=None):
        level = self._level(ct)
        assert tuple(pt.shape) == (level, self.N)
        out = self.empty_ct(level) if out is None else out
        self._chk(
            self.lib.he_pmult(self.ctx, self._dp(ct), self._dp(pt), self._dp(out), level, self._stream()), "he_pmult"
        )
        return out

    def cmult(self, ct, scalars: Sequence[int], out=None):
        level = self._level(ct)
        sc = np.array([int(v) for v in scalars], dtype=np.uint64)
        assert sc.shape == (level,)
        out = self.empty_ct(level) if out is None else out
        self._chk(self.lib.he_cmult(self.ctx, self._dp(ct), _hp(sc), self._dp(out), level, self._stream()), "he_cmult")
        return out

    def add_const(self, ct, scalars: Sequence[int], out=None):
        level = self._level(ct)
        sc = np.array([int(v) for v in scalars], dtype=np.uint64)
        assert sc.shape == (level,)
        out = self.empty_ct(level) if out is None else out
        self._chk(
            self.lib.he_add_const(self.ctx, self._dp(ct), _hp(sc), self._dp(out), level, self._stream()), "he_add_const"
        )
        return out

    def moddrop(self, ct, level: int, out=None):
        in_level = self._level(ct)
        if level == in_level and out is None:
            return ct
        out = self.empty_ct(level) if out is None else out
        self._chk(
            self.lib.he_moddrop(self.ctx, self._dp(ct), in_level, self._dp(out), level, self._stream()), "he_moddrop"
        )
        return out

    # ---- device: hot path ----------------------------------------------------------------------------------------
    def hmult_relin(self, relin: EvalKey, a, b, out=None):
        level = self._level(a)
        assert b.shape == a.shape
        out = self.empty_ct(level) if out is None else out
        ws, wsb = self._workspace(level)
        self._chk(
            self.lib.he_hmult_relin(
                self.ctx, relin.handle, self._dp(a), self._dp(b), self._dp(out), level, ws, wsb, self._stream()
            ),
            "he_hmult_relin",
        )
        return out

    def hmult_relin_rescale(self, relin: EvalKey, a, b, out=None):
        """rescale(hmult_relin(a, b)) in one call (same residues)."""
        level = self._level(a)
        assert b.shape == a.shape
        out = self.empty_ct(level - 1) if out is None else out
        ws, wsb = self._workspace(level)
        self._chk(
            self.lib.he_hmult_relin_rescale(
                self.ctx, relin.handle, self._dp(a), self._dp(b), self._dp(out), level, ws, wsb, self._stream()
            ),
            "he_hmult_relin_rescale",
        )
        return out

    def rescale(self, ct, out=None):
        level = self._level(ct)
        out = self.empty_ct(level - 1) if out is None else out
        ws, wsb = self._workspace(level)
        self._chk(
            self.lib.he_rescale(self.ctx, self._dp(ct), self._dp(out), level, ws, wsb, self._stream()), "he_rescale"
        )
        return out

    def pmult_sum(self, cts, pts, out=None):
        """sum_k cts[k] * pts[k] in one pass (at most 64 terms per call; longer lists are chunked and added)."""
        assert len(cts) == len(pts) and len(cts) >= 1
        level = self._level(cts[0])
        out = self.empty_ct(level) if out is None else out
        acc = None
        for lo in range(0, len(cts), 64):
            c, p = cts[lo:lo + 64], pts[lo:lo + 64]
            ca = (ctypes.c_void_p * len(c))(*[t.data_ptr() for t in c])
            pa = (ctypes.c_void_p * len(p))(*[t.data_ptr() for t in p])
            dst = out if acc is None else self.empty_ct(level)
            self._chk(self.lib.he_pmult_sum(self.ctx, ca, pa, len(c), self._dp(dst), level, self._stream()),
                      "he_pmult_sum")
            acc = dst if acc is None else self.add(acc, dst, out=acc)
        return out

    def modraise(self, ct, level_out: int, out=None):
        """Level-1 ciphertext -> level_out limbs of the same centred coefficients (first step of bootstrapping)."""
        assert self._level(ct) == 1
        out = self.empty_ct(level_out) if out is None else out
        ws, wsb = self._workspace(level_out)
        self._chk(self.lib.he_modraise(self.ctx, self._dp(ct), self._dp(out), level_out, ws, wsb, self._stream()),
                  "he_modraise")
        return out

    def hconj(self, conj: EvalKey, ct, out=None):
        """Complex conjugation of every slot (key from keygen_conj)."""
        return self.hrot(conj, ct, out=out)

    def hrot(self, rot: EvalKey, ct, out=None):
        level = self._level(ct)
        out = self.empty_ct(level) if out is None else out
        ws, wsb = self._workspace(level)
        self._chk(
            self.lib.he_hrot(self.ctx, rot.handle, self._dp(ct), self._dp(out), level, ws, wsb, self._stream()),
            "he_hrot",
        )
        return out

    def hrot_noalloc(self, rot: EvalKey, ct, out):
        """hrot on the library's static scratch array: no workspace, no allocation (the caller passes `out`)."""
        level = self._level(ct)
        assert tuple(out.shape) == tuple(ct.shape)
        self._chk(
            self.lib.he_hrot_noalloc(self.ctx, rot.handle, self._dp(ct), self._dp(out), level, self._stream()),
            "he_hrot_noalloc",
        )
        return out

    def hrot_many(self, rots: Sequence[EvalKey], ct, outs=None):
        level = self._level(ct)
        n = len(rots)
        outs = [self.empty_ct(level) for _ in range(n)] if outs is None else outs
        keys = (ctypes.c_void_p * n)(*[k.handle for k in rots])
        ptrs = (ctypes.c_void_p * n)(*[o.data_ptr() for o in outs])
        ws, wsb = self._workspace(level, min(n, 32))  # room for all rotations: they then share every launch
        self._chk(
            self.lib.he_hrot_many(self.ctx, keys, n, self._dp(ct), ptrs, level, ws, wsb, self._stream()),
            "he_hrot_many",
        )
        return outs

    def rotate_sum(self, rots: Sequence[EvalKey], ct):
        level = self._level(ct)
        n = len(rots)
        keys = (ctypes.c_void_p * n)(*[k.handle for k in rots])
        ws, wsb = self._workspace(level)
        self._chk(
            self.lib.he_rotate_sum(self.ctx, keys, n, self._dp(ct), level, ws, wsb, self._stream()), "he_rotate_sum"
        )
        return ct

    # ---- device: batches [count][2][level][N] ---------------------------------------------------------------------
    def _blevel(self, cts):
        assert cts.dim() == 4 and cts.shape[1] == 2 and cts.shape[3] == self.N and cts.is_contiguous()
        return int(cts.shape[2]), int(cts.shape[0])

    def empty_batch(self, count: int, level: int):
        import torch

        return torch.empty((count, 2, level, self.N), dtype=torch.int64, device=f"cuda:{self.device}")

    def add_batch(self, a, b, out=None):
        level, count = self._blevel(a)
        assert b.shape == a.shape
        out = self.empty_batch(count, level) if out is None else out
        self._chk(self.lib.he_add_batch(self.ctx, self._dp(a), self._dp(b), self._dp(out), level, count, self._stream()),
                  "he_add_batch")
        return out

    def sub_batch(self, a, b, out=None):
        level, count = self._blevel(a)
        assert b.shape == a.shape
        out = self.empty_batch(count, level) if out is None else out
        self._chk(self.lib.he_sub_batch(self.ctx, self._dp(a), self._dp(b), self._dp(out), level, count, self._stream()),
                  "he_sub_batch")
        return out

    def pmult_batch(self, cts, pt, out=None):
        level, count = self._blevel(cts)
        assert tuple(pt.shape) == (level, self.N)
        out = self.empty_batch(count, level) if out is None else out
        self._chk(self.lib.he_pmult_batch(self.ctx, self._dp(cts), self._dp(pt), self._dp(out), level, count,
                                          self._stream()), "he_pmult_batch")
        return out

    def cmult_batch(self, cts, scalars: Sequence[int], out=None):
        level, count = self._blevel(cts)
        sc = np.array([int(v) for v in scalars], dtype=np.uint64)
        assert sc.shape == (level,)
        out = self.empty_batch(count, level) if out is None else out
        self._chk(self.lib.he_cmult_batch(self.ctx, self._dp(cts), _hp(sc), self._dp(out), level, count, self._stream()),
                  "he_cmult_batch")
        return out

    def add_const_batch(self, cts, scalars: Sequence[int], out=None):
        level, count = self._blevel(cts)
        sc = np.array([int(v) for v in scalars], dtype=np.uint64)
        assert sc.shape == (level,)
        out = self.empty_batch(count, level) if out is None else out
        self._chk(self.lib.he_add_const_batch(self.ctx, self._dp(cts), _hp(sc), self._dp(out), level, count,
                                              self._stream()), "he_add_const_batch")
        return out

    def moddrop_batch(self, cts, level: int, out=None):
        in_level, count = self._blevel(cts)
        if level == in_level and out is None:
            return cts
        out = self.empty_batch(count, level) if out is None else out
        self._chk(self.lib.he_moddrop_batch(self.ctx, self._dp(cts), in_level, self._dp(out), level, count,
                                            self._stream()), "he_moddrop_batch")
        return out

    def hmult_relin_batch(self, relin: EvalKey, a, b, out=None):
        level, count = self._blevel(a)
        assert b.shape == a.shape
        out = self.empty_batch(count, level) if out is None else out
        ws, wsb = self._workspace(level, count)
        self._chk(self.lib.he_hmult_relin_batch(self.ctx, relin.handle, self._dp(a), self._dp(b), self._dp(out), level,
                                                count, ws, wsb, self._stream()), "he_hmult_relin_batch")
        return out

    def hmult_relin_rescale_batch(self, relin: EvalKey, a, b, out=None):
        level, count = self._blevel(a)
        assert b.shape == a.shape
        out = self.empty_batch(count, level - 1) if out is None else out
        ws, wsb = self._workspace(level, count)
        self._chk(self.lib.he_hmult_relin_rescale_batch(self.ctx, relin.handle, self._dp(a), self._dp(b), self._dp(out),
                                                        level, count, ws, wsb, self._stream()),
                  "he_hmult_relin_rescale_batch")
        return out

    def rescale_batch(self, cts, out=None):
        level, count = self._blevel(cts)
        out = self.empty_batch(count, level - 1) if out is None else out
        ws, wsb = self._workspace(level, count)
        self._chk(self.lib.he_rescale_batch(self.ctx, self._dp(cts), self._dp(out), level, count, ws, wsb,
                                            self._stream()), "he_rescale_batch")
        return out

    def hrot_batch(self, rot: EvalKey, cts, out=None):
        level, count = self._blevel(cts)
        out = self.empty_batch(count, level) if out is None else out
        ws, wsb = self._workspace(level, count)
        self._chk(self.lib.he_hrot_batch(self.ctx, rot.handle, self._dp(cts), self._dp(out), level, count, ws, wsb,
                                         self._stream()), "he_hrot_batch")
        return out

    def hrot_batch_keys(self, rots: Sequence[EvalKey], cts, out=None):
        """Rotate ciphertext o of the batch with key rots[o]."""
        level, count = self._blevel(cts)
        if len(rots) != count:
            raise ValueError("one key per ciphertext")
        out = self.empty_batch(count, level) if out is None else out
        keys = (ctypes.c_void_p * count)(*[k.handle for k in rots])
        ws, wsb = self._workspace(level, min(count, 32))
        self._chk(self.lib.he_hrot_batch_keys(self.ctx, keys, self._dp(cts), self._dp(out), level, count, ws, wsb,
                                              self._stream()), "he_hrot_batch_keys")
        return out

    def hrot_batch_levels(self, rots: Sequence[EvalKey], levels: Sequence[int], packed, out=None):
        """Rotate ciphertexts of mixed levels packed back to back (`packed`: flat [sum 2 level_o][N] tensor),
        operation o with key rots[o]; returns the results packed the same way."""
        import torch

        lv = np.ascontiguousarray(levels, dtype=np.int32)
        count = lv.shape[0]
        if len(rots) != count:
            raise ValueError("one key per ciphertext")
        assert packed.dim() == 2 and packed.shape[1] == self.N and int(packed.shape[0]) == 2 * int(lv.sum())
        out = torch.empty_like(packed) if out is None else out
        keys = (ctypes.c_void_p * count)(*[k.handle for k in rots])
        ws, wsb = self._workspace(int(lv.max()), min(count, 32))
        self._chk(self.lib.he_hrot_batch_levels(self.ctx, keys, _hp(lv), self._dp(packed), self._dp(out), count, ws, wsb,
                                                self._stream()), "he_hrot_batch_levels")
        return out

    def rotate_sum_batch(self, rots: Sequence[EvalKey], cts):
        level, count = self._blevel(cts)
        n = len(rots)
        keys = (ctypes.c_void_p * n)(*[k.handle for k in rots])
        ws, wsb = self._workspace(level, count)
        self._chk(self.lib.he_rotate_sum_batch(self.ctx, keys, n, self._dp(cts), level, count, ws, wsb, self._stream()),
                  "he_rotate_sum_batch")
        return cts

    # ---- measurement -------------------------------------------------------------------------------------------------
    def profile_start(self):
        self._chk(self.lib.he_profile_start(self.ctx), "he_profile_start")

    def profile_stop(self):
        """Per-kernel {name: (launches, total_ms, bytes)} since profile_start."""
        buf = (he_kernel_stat * 32)()
        n = ctypes.c_int32()
        self._chk(self.lib.he_profile_stop(self.ctx, buf, 32, ctypes.byref(n)), "he_profile_stop")
        return {buf[i].name.decode(): (int(buf[i].launches), float(buf[i].total_ms), float(buf[i].bytes))
                for i in range(n.value)}
