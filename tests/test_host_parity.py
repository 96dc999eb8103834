"""Host side of the library against the oracle (no GPU): tables, samplers, keys, encryption are
bit-exact from the same seeds; encode agrees to one unit; decryption agrees with the big-integer CRT.
Also checks that the shared library exports every symbol the header declares."""
import ctypes
import os
import re

import numpy as np
import pytest

import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2210_02574_amd as pkg

    return pkg


def test_library_exports_every_declared_symbol(lib):
    text = open(os.path.join(ROOT, "include", "he.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(he_[a-z0-9_]+)\s*\(", text))
    assert declared == set(lib.SYMBOLS)
    dll = ctypes.CDLL(lib.LIB_PATH)
    for name in declared:
        assert hasattr(dll, name), name


def test_device_functions_refuse_a_host_only_context(lib):
    he = lib.HE.from_params(wl.C1)
    mi = np.zeros(1, dtype=np.int32)
    rc = he.lib.he_ntt(he.ctx, ctypes.c_void_p(16), ctypes.c_void_p(mi.ctypes.data), 1, None)
    assert rc == -6
    rc = he.lib.he_rescale(he.ctx, ctypes.c_void_p(16), ctypes.c_void_p(32), 3, ctypes.c_void_p(64), 1 << 30, None)
    assert rc == -6


def test_context_rejects_bad_parameters(lib):
    with pytest.raises(lib.HeError):
        lib.HE(12, [2**40 - 147455 + 2], [2**50 - 16383], 1)  # not 1 mod 2N
    with pytest.raises(lib.HeError):
        lib.HE(12, list(wl.C1.q), list(wl.C1.p), 4)  # more digits than primes
    with pytest.raises(lib.HeError):
        lib.HE(12, [wl.C1.q[0], wl.C1.q[0]], list(wl.C1.p), 1)  # repeated modulus
    he = lib.HE.from_params(wl.C1)
    with pytest.raises(lib.HeError):
        he.workspace_bytes(0)
    with pytest.raises(lib.HeError):
        he.workspace_bytes(4)


@pytest.mark.parametrize("params", [wl.C1, wl.C1B, wl.M12, wl.W12], ids=lambda p: p.name)
def test_tables_keys_and_encryption_bit_exact(lib, oracle_mod, params):
    he = lib.HE.from_params(params)
    o = oracle_mod.Oracle(params.logN, params.q, params.p, params.dnum)
    for i, t in enumerate(params.moduli):
        assert he.modulus(i) == (t, o.psi(i))
    assert he.gauss_cdt() == oracle_mod.gaussian_cdt()
    for r in (1, 5, -3, 2047, 2048 + 7):
        assert he.galois_element(r) == o.galois_element(r)
    sk = he.keygen_secret(11)
    s = o.keygen_secret(11)
    assert np.array_equal(sk.coeffs(), s)
    assert np.array_equal(he.keygen_relin(sk, 12).to_host(), o.keygen_relin(s, 12))
    for r in (1, 64, -1):
        assert np.array_equal(he.keygen_rot(sk, r, 13 + r).to_host(), o.keygen_rot(s, r, 13 + r))
    assert np.array_equal(he.keygen_conj(sk, 16).to_host(), o.keygen_conj(s, 16))
    m = wl.small_coeffs(14, params.N, 2**35)
    for level in (3, 1):
        a, b = he.encrypt_coeffs(sk, m, level, 15), o.encrypt_coeffs(s, m, level, 15)
        assert np.array_equal(a, b)
    pk = he.keygen_public(sk, 17)
    assert np.array_equal(pk, o.keygen_public(s, 17))
    for level in (3, 2):
        assert np.array_equal(he.encrypt_public_coeffs(pk, m, level, 18), o.encrypt_public_coeffs(pk, m, level, 18))
    assert np.array_equal(he.plain_to_ntt(m, 2), o.coeffs_to_ntt(m, 2))


def test_encode_decode_decrypt_against_oracle(lib, oracle_mod):
    params = wl.C1B
    he = lib.HE.from_params(params)
    o = oracle_mod.Oracle(params.logN, params.q, params.p, params.dnum)
    g = wl.rng(21)
    z = g.uniform(-1, 1, he.n) + 1j * g.uniform(-1, 1, he.n)
    for scale in (2.0**30, 2.0**50):
        a, b = he.encode(z, scale), o.encode(z, scale)
        assert np.abs(a - b).max() <= 1
    a = he.encode(z[:100].real, 2.0**30)
    assert np.abs(a - o.encode(z[:100].real, 2.0**30)).max() <= 1
    m = o.encode(z, 2.0**30)
    assert np.abs(he.decode(m.astype(np.float64), 2.0**30) - o.decode(m, 2.0**30)).max() < 1e-9
    sk, s = he.keygen_secret(5), o.keygen_secret(5)
    # products of two encodings reach ~2^60 * N: needs two to three limbs in the reconstruction
    big = wl.rng(6).integers(-(2**62), 2**62, size=he.N, dtype=np.int64)
    for level, msg in ((3, big), (2, big), (1, wl.small_coeffs(7, he.N, 2**37))):
        ct = o.encrypt_coeffs(s, msg, level, 31)
        want = np.array([float(v) for v in o.decrypt_coeffs(s, ct)])
        got = he.decrypt_coeffs(sk, ct)
        assert np.array_equal(got, want)
    # a value wider than two limbs: multiply the ciphertext by a 45-bit scalar
    ct = o.encrypt_coeffs(s, big, 3, 32)
    c = 2**45 + 12345
    ct = o.cmult(ct, [c % q for q in params.q])
    want = np.array([float(v) for v in o.decrypt_coeffs(s, ct)])
    assert np.abs(want).max() > 2.0**100
    assert np.array_equal(he.decrypt_coeffs(sk, ct), want)
    ct = o.encrypt_coeffs(s, o.encode(z, 2.0**30), 3, 33)
    assert np.abs(he.decrypt(sk, ct, 2.0**30) - z).max() < 2.0**-18


def test_missing_library_is_an_import_error(monkeypatch, tmp_path):
    """No fallback: without the built library the binding raises instead of computing anything."""
    from paper_2210_02574_amd import binding

    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libhe_missing.so"))
    with pytest.raises(ImportError) as ei:
        binding.load_library()
    assert "no fallback" in str(ei.value)
