"""GPU parity: every device entry point, called through the C ABI, against the CPU oracle on the
same seeded inputs -- bit-exact on every residue.  Sizes: the tiny configuration (N=2^12, literal
dnum=1 and the one-prime-per-digit variant) in full, and N=2^16 / L=24 / dnum=6 at several levels
including partial last digits; the paper-scale ring N=2^17 / L=30 / dnum=8 at three levels."""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pkg():
    import torch

    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2210_02574_amd as p

    return p


class Env:
    def __init__(self, pkg, oracle_mod, params):
        self.params = params
        self.he = pkg.HE.from_params(params, device=0)
        self.o = oracle_mod.Oracle(params.logN, params.q, params.p, params.dnum)
        self._keys = {}

    def synth_key(self, seed, g):
        """A key-shaped buffer of uniform residues, wrapped for the Galois element g."""
        if (seed, g) not in self._keys:
            evk = wl.uniform_evk(seed, self.params)
            self._keys[(seed, g)] = (self.he.evk_from_host(evk, g), evk)
        return self._keys[(seed, g)]


@pytest.fixture(scope="module", params=["C1", "C1B", "N16", "I12", "M12", "P17"])
def env(request, pkg, oracle_mod):
    return Env(pkg, oracle_mod, getattr(wl, request.param))


def _sync():
    import torch

    torch.cuda.synchronize()


def test_ntt_intt_all_moduli(env):
    he, o, p = env.he, env.o, env.params
    M = p.L + p.K
    mod_idx = [b % M for b in range(M + 5)]
    if p.logN == 12:
        mod_idx = [b % M for b in range(8)]  # the 8 polynomials of the tiny workload
    a = wl.uniform_limbs(101, p, mod_idx)
    d = he.to_device(a)
    he.ntt(d, mod_idx)
    f = he.to_host(d)
    want = o.ntt(a, mod_idx)
    assert np.array_equal(f, want)
    he.intt(d, mod_idx)
    assert np.array_equal(he.to_host(d), a)
    # inverse alone, from oracle-made NTT values
    d2 = he.to_device(want)
    he.intt(d2, mod_idx)
    assert np.array_equal(he.to_host(d2), a)


def test_ntt_edge_values(env):
    """All-zero, all q-1, and a monomial: extremes of the lazy-reduction ranges."""
    he, o, p = env.he, env.o, env.params
    mods = p.moduli
    mod_idx = [0, p.L - 1, p.L, p.L + p.K - 1]
    a = np.zeros((4, p.N), dtype=np.uint64)
    a[1] = mods[mod_idx[1]] - 1
    a[2][1] = 1
    a[3] = mods[mod_idx[3]] - 1
    d = he.to_device(a)
    he.ntt(d, mod_idx)
    assert np.array_equal(he.to_host(d), o.ntt(a, mod_idx))
    d = he.to_device(a)
    he.intt(d, mod_idx)
    assert np.array_equal(he.to_host(d), o.intt(a, mod_idx))


def _levels(p):
    if p.logN == 12:
        return list(range(p.L, 0, -1))
    if p.logN == 17:
        return [30, 7, 1]
    return [24, 23, 21, 9, 4, 1]


def test_elementwise(env):
    he, o, p = env.he, env.o, env.params
    for level in _levels(p)[:2]:
        a, b = wl.uniform_ct(201, p, level), wl.uniform_ct(202, p, level)
        da, db = he.to_device(a), he.to_device(b)
        assert np.array_equal(he.to_host(he.add(da, db)), o.add(a, b))
        assert np.array_equal(he.to_host(he.sub(da, db)), o.sub(a, b))
        pt = wl.uniform_limbs(203, p, list(range(level)))
        assert np.array_equal(he.to_host(he.pmult(da, he.to_device(pt))), o.pmult(a, pt))
        sc = [int(v) for v in wl.uniform_limbs(204, p, list(range(level)))[:, 0]]
        assert np.array_equal(he.to_host(he.cmult(da, sc)), o.cmult(a, sc))
        # in place
        he.add(da, db, out=da)
        assert np.array_equal(he.to_host(da), o.add(a, b))


def test_pmult_sum(env):
    """sum_k ct_k * pt_k in one pass against the oracle's products and sums (70 terms: more than one call)."""
    he, o, p = env.he, env.o, env.params
    level = min(3, p.L) if p.logN == 12 else 9
    terms = 70 if p.logN == 12 else 5
    cts = [wl.uniform_ct(2000 + k, p, level) for k in range(terms)]
    pts = [wl.uniform_limbs(2100 + k, p, list(range(level))) for k in range(terms)]
    want = None
    for c, t in zip(cts, pts):
        term = o.pmult(c, t)
        want = term if want is None else o.add(want, term)
    got = he.pmult_sum([he.to_device(c) for c in cts], [he.to_device(t) for t in pts])
    assert np.array_equal(he.to_host(got), want)


def test_hmult_relin_and_rescale(env):
    he, o, p = env.he, env.o, env.params
    key, evk = env.synth_key(301, 1)
    for level in _levels(p):
        a, b = wl.uniform_ct(302 + level, p, level), wl.uniform_ct(402 + level, p, level)
        da, db = he.to_device(a), he.to_device(b)
        got = he.to_host(he.hmult_relin(key, da, db))
        want = o.hmult_relin(a, b, evk)
        assert np.array_equal(got, want), level
        if level >= 2:
            rs = he.to_host(he.rescale(he.to_device(want)))
            assert np.array_equal(rs, o.rescale(want)), level
    # output aliasing an input
    level = _levels(p)[0]
    a, b = wl.uniform_ct(310, p, level), wl.uniform_ct(311, p, level)
    da, db = he.to_device(a), he.to_device(b)
    he.hmult_relin(key, da, db, out=da)
    assert np.array_equal(he.to_host(da), o.hmult_relin(a, b, evk))


def test_hmult_relin_rescale_in_one_call(env):
    """The fused Mult + rescale against the oracle's rescale(hmult_relin(a, b)) on every residue, and the
    batched form against the single one."""
    import torch

    he, o, p = env.he, env.o, env.params
    key, evk = env.synth_key(301, 1)
    for level in [l for l in _levels(p) if l >= 2]:
        a, b = wl.uniform_ct(1402 + level, p, level), wl.uniform_ct(1502 + level, p, level)
        da, db = he.to_device(a), he.to_device(b)
        got = he.to_host(he.hmult_relin_rescale(key, da, db))
        want = o.rescale(o.hmult_relin(a, b, evk))
        assert got.shape == (2, level - 1, p.N)
        assert np.array_equal(got, want), level
    level = _levels(p)[0]
    count = 3
    a = torch.stack([he.to_device(wl.uniform_ct(1600 + i, p, level)) for i in range(count)])
    b = torch.stack([he.to_device(wl.uniform_ct(1700 + i, p, level)) for i in range(count)])
    outb = he.hmult_relin_rescale_batch(key, a, b)
    for i in range(count):
        assert torch.equal(outb[i], he.rescale(he.hmult_relin(key, a[i], b[i]))), i
    with pytest.raises(Exception) as ei:
        one = he.to_device(wl.uniform_ct(1800, p, 1))
        he.hmult_relin_rescale(key, one, one, out=he.empty_ct(1))
    assert "HE_ELEVEL" in str(ei.value)


def test_hrot_single_and_hoisted(env):
    import torch

    he, o, p = env.he, env.o, env.params
    rots = [1, 5, p.N // 4] if p.logN == 12 else [1, 1 << 14]
    keys = [env.synth_key(500 + r, o.galois_element(r)) for r in rots]
    for level in _levels(p)[:4]:
        ct = wl.uniform_ct(600 + level, p, level)
        d = he.to_device(ct)
        singles = []
        for r, (key, evk) in zip(rots, keys):
            got = he.to_host(he.hrot(key, d))
            assert np.array_equal(got, o.hrot(ct, evk, r)), (level, r)
            singles.append(got)
        outs = he.hrot_many([k for k, _ in keys], d)
        for got, want in zip(outs, singles):
            assert np.array_equal(he.to_host(got), want)
        assert np.array_equal(he.to_host(d), ct)  # input untouched
        if p.logN == 12:  # the same through a workspace for one and for two operations (three rotations)
            import ctypes

            handles = (ctypes.c_void_p * len(keys))(*[k.handle for k, _ in keys])
            for fit in (1, 2):
                outs2 = [he.empty_ct(level) for _ in keys]
                ptrs = (ctypes.c_void_p * len(keys))(*[t.data_ptr() for t in outs2])
                ws, _ = he._workspace(level, 2)
                rc = he.lib.he_hrot_many(he.ctx, handles, len(keys), ctypes.c_void_p(d.data_ptr()), ptrs, level, ws,
                                         he.workspace_bytes(level, fit), None)
                assert rc == 0
                for got, want in zip(outs2, singles):
                    assert np.array_equal(he.to_host(got), want), (level, fit)
        # one key per ciphertext of a batch: two different inputs, against the oracle
        ct2 = wl.uniform_ct(650 + level, p, level)
        both = he.hrot_batch_keys([k for k, _ in keys[:2]], torch.stack([d, he.to_device(ct2)]))
        assert np.array_equal(he.to_host(both[0]), singles[0])
        assert np.array_equal(he.to_host(both[1]), o.hrot(ct2, keys[1][1], rots[1])), level


def test_hrot_every_digit_count_at_full_size(env):
    """One rotation per level 20, 16, 12, 8, 4, 1 at N = 2^16 (5, 4, 3, 2, 1 digits and a one-limb digit), beyond
    the levels of the test above (6, 6, 6 and 3 digits)."""
    he, o, p = env.he, env.o, env.params
    if p.name != "N16":
        pytest.skip("the other parameter sets run every level in test_hrot_single_and_hoisted")
    for k, level in enumerate((20, 16, 12, 8, 4, 1)):
        r = 1 << (2 * k + 1)
        key, evk = env.synth_key(520 + k, o.galois_element(r))
        ct = wl.uniform_ct(680 + level, p, level)
        assert np.array_equal(he.to_host(he.hrot(key, he.to_device(ct))), o.hrot(ct, evk, r)), level


def test_hrot_mixed_levels_in_one_call(env):
    """Rotations at different levels through one call (shared launches, buffers laid out for the largest level of
    a group): every output against the oracle's rotation of that ciphertext at its own level.  Levels span full and
    partial last digits, a one-limb ciphertext, repeated keys next to each other, and the largest level not first."""
    import torch

    he, o, p = env.he, env.o, env.params
    if p.logN == 16:
        levels, rots = [17, 24, 24, 12, 8, 3, 1, 9, 21], [1, 1, 64, 64, 64, 1 << 14, 2, 2, 1]
    elif p.logN == 17:
        levels, rots = [7, 30, 1, 12], [1, 1, 4, 4]
    else:
        levels = [min(l, p.L) for l in (2, 3, 1, 3, 2)]
        rots = [1, 1, 5, 5, p.N // 4]
    keys = {r: env.synth_key(540 + k, o.galois_element(r)) for k, r in enumerate(sorted(set(rots)))}
    cts = [wl.uniform_ct(690 + k, p, lv) for k, lv in enumerate(levels)]
    packed = torch.cat([he.to_device(c).reshape(-1, p.N) for c in cts])
    out = he.hrot_batch_levels([keys[r][0] for r in rots], levels, packed)
    got = he.to_host(out)
    at = 0
    for k, (lv, r, ct) in enumerate(zip(levels, rots, cts)):
        want = o.hrot(ct, keys[r][1], r)
        assert np.array_equal(got[at:at + 2 * lv].reshape(2, lv, p.N), want), (k, lv, r)
        at += 2 * lv
    assert np.array_equal(he.to_host(packed), np.concatenate([c.reshape(-1, p.N) for c in cts]))  # inputs untouched
    # a workspace that holds one operation only: groups of one, same results
    import ctypes

    lv32 = np.ascontiguousarray(levels, dtype=np.int32)
    handles = (ctypes.c_void_p * len(levels))(*[keys[r][0].handle for r in rots])
    out1 = torch.zeros_like(packed)
    ws, _ = he._workspace(max(levels), 1)
    rc = he.lib.he_hrot_batch_levels(he.ctx, handles, ctypes.c_void_p(lv32.ctypes.data), ctypes.c_void_p(packed.data_ptr()),
                                     ctypes.c_void_p(out1.data_ptr()), len(levels), ws, he.workspace_bytes(max(levels), 1), None)
    assert rc == 0
    assert torch.equal(out1, out)


def test_patterned_inputs_through_the_key_switch(env):
    """Residues at the ends of their ranges (all q-1, all (q-1)/2, alternating 0 / q-1, within 1000 of q) through
    Mult, the fused Mult + rescale and Rotate: the lazy ranges of both arithmetic paths at their widest."""
    he, o, p = env.he, env.o, env.params
    relin, relin_h = env.synth_key(301, 1)
    rkey, rkey_h = env.synth_key(500 + 1, o.galois_element(1))
    g = wl.rng(4242)

    def patterned(kind, level):
        ct = np.empty((2, level, p.N), dtype=np.uint64)
        for i in range(level):
            q = p.q[i]
            if kind == 0:
                ct[:, i] = q - 1
            elif kind == 1:
                ct[:, i] = (q - 1) // 2
            elif kind == 2:
                ct[:, i, ::2], ct[:, i, 1::2] = 0, q - 1
            else:
                ct[:, i] = g.integers(q - 1000, q, size=(2, p.N), dtype=np.uint64)
        return ct

    levels = _levels(p)
    cases = [(0, 0, levels[0]), (2, 3, levels[0]), (1, 2, levels[1]), (3, 0, levels[-2])]
    for ka, kb, level in (cases if p.logN == 12 else cases[:2]):
        a, b = patterned(ka, level), patterned(kb, level)
        da, db = he.to_device(a), he.to_device(b)
        want = o.hmult_relin(a, b, relin_h)
        assert np.array_equal(he.to_host(he.hmult_relin(relin, da, db)), want), (ka, kb, level)
        if level >= 2:
            assert np.array_equal(he.to_host(he.hmult_relin_rescale(relin, da, db)), o.rescale(want)), (ka, kb, level)
        assert np.array_equal(he.to_host(he.hrot(rkey, da)), o.hrot(a, rkey_h, 1)), (ka, level)


def test_rotate_sum(env):
    he, o, p = env.he, env.o, env.params
    level = 2 if p.logN == 12 else 6
    shifts = [4, 8, 16]
    keys = [env.synth_key(700 + r, o.galois_element(r)) for r in shifts]
    ct = wl.uniform_ct(701, p, level)
    d = he.to_device(ct)
    he.rotate_sum([k for k, _ in keys], d)
    want = o.rotate_sum(ct, [e for _, e in keys], 4)
    assert np.array_equal(he.to_host(d), want)


def test_real_keys_and_decryption(env):
    """Keys and ciphertexts from the library's own host side: parity with the oracle's from the same
    seeds, then HMult / HRot on the device decrypt to the slot-wise product / the shifted vector."""
    he, o, p = env.he, env.o, env.params
    if p.name == "C1":
        pytest.skip("dnum=1 with P << Q: key-switch noise swamps the message (parity only)")
    level = 3 if p.logN == 12 else 5
    scale = 2.0**30 if p.name == "C1B" else 2.0**45
    sk, s = he.keygen_secret(801), o.keygen_secret(801)
    relin = he.keygen_relin(sk, 802)
    rot = he.keygen_rot(sk, 3, 803)
    assert np.array_equal(relin.to_host(), o.keygen_relin(s, 802))
    assert np.array_equal(rot.to_host(), o.keygen_rot(s, 3, 803))
    z1, z2 = wl.slots_uniform(804, he.n), wl.slots_uniform(805, he.n)
    m1, m2 = o.encode(z1, scale), o.encode(z2, scale)
    assert np.abs(he.encode(z1, scale) - m1).max() <= 1
    c1, c2 = he.encrypt_coeffs(sk, m1, level, 806), he.encrypt_coeffs(sk, m2, level, 807)
    assert np.array_equal(c1, o.encrypt_coeffs(s, m1, level, 806))
    d1, d2 = he.to_device(c1), he.to_device(c2)
    prod = he.rescale(he.hmult_relin(relin, d1, d2))
    want = o.rescale(o.hmult_relin(c1, c2, o.keygen_relin(s, 802)))
    assert np.array_equal(he.to_host(prod), want)
    out_scale = scale * scale / p.q[level - 1]
    err = np.abs(he.decrypt(sk, he.to_host(prod), out_scale) - z1 * z2).max()
    tol = 2.0**-15 * max(1.0, 2.0**40 / out_scale) * (16 if p.logN == 12 else 1)
    assert err <= tol, (err, tol)
    r = he.hrot(rot, d1)
    err = np.abs(he.decrypt(sk, he.to_host(r), scale) - np.roll(z1, -3)).max()
    assert err <= 2.0**-15 * max(1.0, 2.0**40 / scale), err


def test_conjugation_and_public_key_encryption(env):
    """Conjugation is Rotate with the key of X -> X^(2N-1): bit-exact against the oracle on uniform residues,
    and on a public-key encryption it decrypts to the conjugated slots."""
    he, o, p = env.he, env.o, env.params
    g = 2 * p.N - 1
    key, evk = env.synth_key(950, g)
    for level in _levels(p)[:3]:
        ct = wl.uniform_ct(951 + level, p, level)
        got = he.to_host(he.hconj(key, he.to_device(ct)))
        assert np.array_equal(got, o.hconj(ct, evk)), level
    if p.name == "C1":
        return  # dnum=1 with P << Q: key-switch noise swamps the message
    level = 3 if p.logN == 12 else 4
    scale = 2.0**30 if p.logN == 12 else 2.0**40
    sk, s = he.keygen_secret(960), o.keygen_secret(960)
    ck = he.keygen_conj(sk, 961)
    assert np.array_equal(ck.to_host(), o.keygen_conj(s, 961))
    pk = he.keygen_public(sk, 962)
    rng = wl.rng(963)
    z = rng.uniform(-1, 1, he.n) + 1j * rng.uniform(-1, 1, he.n)
    m = o.encode(z, scale)
    ct = he.encrypt_public_coeffs(pk, m, level, 964)
    assert np.array_equal(ct, o.encrypt_public_coeffs(o.keygen_public(s, 962), m, level, 964))
    out = he.to_host(he.hconj(ck, he.to_device(ct)))
    err = np.abs(he.decrypt(sk, out, scale) - np.conj(z)).max()
    tol = 2.0**-15 * max(1.0, 2.0**40 / scale) * 4
    assert err <= tol, (err, tol)


@pytest.mark.parametrize("name", ["W12", "W16"])
def test_conversions_with_more_than_four_sources(pkg, oracle_mod, name):
    """alpha = 6 and K = 5: ModUp, ModDown and the fused ModDown + rescale in their forms for up to eight source
    limbs, at a full and at a partial last digit, against the oracle on every residue."""
    import torch

    p = getattr(wl, name)
    assert p.alpha == 6 and p.K == 5
    env = Env(pkg, oracle_mod, p)
    he, o = env.he, env.o
    relin, relin_h = env.synth_key(3301, 1)
    rkey, rkey_h = env.synth_key(3302, o.galois_element(3))
    for level in (12, 8, 5):
        a, b = wl.uniform_ct(3310 + level, p, level), wl.uniform_ct(3330 + level, p, level)
        da, db = he.to_device(a), he.to_device(b)
        prod = o.hmult_relin(a, b, relin_h)
        assert np.array_equal(he.to_host(he.hmult_relin(relin, da, db)), prod), level
        assert np.array_equal(he.to_host(he.hmult_relin_rescale(relin, da, db)), o.rescale(prod)), level
        assert np.array_equal(he.to_host(he.hrot(rkey, da)), o.hrot(a, rkey_h, 3)), level
        both = he.hrot_batch_keys([rkey, rkey], torch.stack([da, db]))
        assert np.array_equal(he.to_host(both[1]), o.hrot(b, rkey_h, 3)), level
    _sync()


@pytest.mark.parametrize("name", ["C1", "C1B", "N16", "I12", "M12", "W12", "W16", "P17"])
def test_corrected_conversions_match_the_oracle(pkg, oracle_mod, name):
    """The selectable variant with corrected base conversions (ModUp to the digit's own residue, ModDown to the
    rounded quotient, the multiples estimated in double precision as specified): Mult, the fused Mult + rescale,
    Rotate and a mixed-level call against the oracle with the same variant selected, on every residue -- on the
    floating-point and the integer path, split sources, and conversions of five to eight sources.  Where the
    corrections are non-trivial the residues differ from the default form's."""
    import torch

    p = getattr(wl, name)
    env = Env(pkg, oracle_mod, p)
    he, o = env.he, env.o
    relin, relin_h = env.synth_key(3401, 1)
    rkey, rkey_h = env.synth_key(3402, o.galois_element(3))
    levels = {12: [p.L, max(1, p.L - 1), 1], 16: [p.L, p.L - 3, 9, 2], 17: [30, 7]}[p.logN]
    he.set_exact_conversion(True)
    o.set_exact(True)
    try:
        for level in sorted(set(levels), reverse=True):
            a, b = wl.uniform_ct(3410 + level, p, level), wl.uniform_ct(3440 + level, p, level)
            da, db = he.to_device(a), he.to_device(b)
            prod = o.hmult_relin(a, b, relin_h)
            assert np.array_equal(he.to_host(he.hmult_relin(relin, da, db)), prod), level
            if level >= 2:
                assert np.array_equal(he.to_host(he.hmult_relin_rescale(relin, da, db)), o.rescale(prod)), level
            rot = o.hrot(a, rkey_h, 3)
            assert np.array_equal(he.to_host(he.hrot(rkey, da)), rot), level
            if level == max(levels) and p.alpha > 1 and p.K > 1:
                o.set_exact(False)
                assert not np.array_equal(rot, o.hrot(a, rkey_h, 3))
                o.set_exact(True)
        cts = [wl.uniform_ct(3470 + k, p, lv) for k, lv in enumerate(levels)]
        packed = torch.cat([he.to_device(c).reshape(-1, p.N) for c in cts])
        got = he.to_host(he.hrot_batch_levels([rkey] * len(levels), levels, packed))
        at = 0
        for lv, ct in zip(levels, cts):
            assert np.array_equal(got[at:at + 2 * lv].reshape(2, lv, p.N), o.hrot(ct, rkey_h, 3)), lv
            at += 2 * lv
    finally:
        he.set_exact_conversion(False)
        o.set_exact(False)
    # back to the default form
    a = wl.uniform_ct(3499, p, levels[0])
    assert np.array_equal(he.to_host(he.hrot(rkey, he.to_device(a))), o.hrot(a, rkey_h, 3))
    _sync()


def test_unbuilt_conversion_sizes_are_refused(pkg):
    """Digits of more than four primes at N = 2^17, and of more than eight anywhere, have no kernel: a device
    context for them is refused instead of running a smaller one."""
    with pytest.raises(Exception) as ei:
        pkg.HE.from_params(wl.Params("X17", 17, wl.P17.q[:12], wl.P17.p, 2), device=0)
    assert "HE_EINVAL" in str(ei.value)
    with pytest.raises(Exception) as ei:
        pkg.HE.from_params(wl.Params("X12", 12, wl.N16.q[:18], wl.N16.p, 2), device=0)
    assert "HE_EINVAL" in str(ei.value)
    pkg.HE.from_params(wl.Params("X12h", 12, wl.N16.q[:18], wl.N16.p, 2), device=-1)  # the host functions do not care


def test_error_codes_on_device_context(env):
    import ctypes

    he, p = env.he, env.params
    key, _ = env.synth_key(301, 1)
    rkey, _ = env.synth_key(901, env.o.galois_element(1))
    a = he.to_device(wl.uniform_ct(902, p, 1))
    with pytest.raises(Exception) as ei:
        he.rescale(a)
    assert "HE_ELEVEL" in str(ei.value)
    with pytest.raises(Exception) as ei:
        he.hrot(key, a)  # relinearisation key is not a rotation key
    assert "HE_ENOKEY" in str(ei.value)
    with pytest.raises(Exception) as ei:
        he.hmult_relin(rkey, a, a)
    assert "HE_ENOKEY" in str(ei.value)
    with pytest.raises(Exception) as ei:
        he.modraise(a, 1, out=he.empty_ct(1))  # ModRaise goes to at least two limbs
    assert "HE_ELEVEL" in str(ei.value)
    ptrs = (ctypes.c_void_p * 65)(*([a.data_ptr()] * 65))
    rc = he.lib.he_pmult_sum(he.ctx, ptrs, ptrs, 65, ctypes.c_void_p(a.data_ptr()), 1, None)
    assert rc == -1  # more than 64 terms in one call
    rc = he.lib.he_hrot(he.ctx, rkey.handle, ctypes.c_void_p(a.data_ptr()), ctypes.c_void_p(a.data_ptr() + 8),
                        1, ctypes.c_void_p(a.data_ptr()), 16, None)
    assert rc == -4  # workspace too small
    with pytest.raises(Exception) as ei:
        he.hrot_batch_keys([rkey, key], he.empty_batch(2, 1))  # second key is not a rotation key
    assert "HE_ENOKEY" in str(ei.value)
    with pytest.raises(ValueError):
        he.hrot_batch_keys([rkey], he.empty_batch(2, 1))  # one key per ciphertext
    ws, wsb = he._workspace(1, 1)
    keys = (ctypes.c_void_p * 1)(rkey.handle)
    rc = he.lib.he_hrot_batch_keys(he.ctx, keys, ctypes.c_void_p(a.data_ptr() + 8), ctypes.c_void_p(he.empty_ct(1).data_ptr()),
                                   1, 1, ws, wsb, None)
    assert rc == -1  # input not 16-byte aligned: refused before any launch
    too_many = 65536  # count x workspace limbs no longer fits the 16-bit limb slots of a launch
    rc = he.lib.he_hrot_batch(he.ctx, rkey.handle, ctypes.c_void_p(a.data_ptr()), ctypes.c_void_p(he.empty_ct(1).data_ptr()),
                              1, too_many, ws, ctypes.c_size_t(1 << 62), None)
    assert rc == -1
    _sync()


def test_batched_calls_equal_single_calls(env):
    """Every batched entry point on [count][2][level][N] gives, ciphertext by ciphertext, the bits of the
    single-ciphertext call (which the other tests compare with the oracle)."""
    import ctypes

    import torch

    he, o, p = env.he, env.o, env.params
    level = 3 if p.logN == 12 else 23  # partial last digit at N = 2^16
    count = 5
    relin, _ = env.synth_key(301, 1)
    rkeys = [env.synth_key(700 + r, o.galois_element(r))[0] for r in (4, 8)]
    a = torch.stack([he.to_device(wl.uniform_ct(1100 + i, p, level)) for i in range(count)])
    b = torch.stack([he.to_device(wl.uniform_ct(1200 + i, p, level)) for i in range(count)])
    pt = he.to_device(wl.uniform_limbs(1300, p, list(range(level))))
    sc = [int(v) for v in wl.uniform_limbs(1301, p, list(range(level)))[:, 0]]

    def same(batched, single):
        for i in range(count):
            assert torch.equal(batched[i], single(i)), i

    same(he.add_batch(a, b), lambda i: he.add(a[i], b[i]))
    same(he.sub_batch(a, b), lambda i: he.sub(a[i], b[i]))
    same(he.pmult_batch(a, pt), lambda i: he.pmult(a[i], pt))
    same(he.cmult_batch(a, sc), lambda i: he.cmult(a[i], sc))
    same(he.add_const_batch(a, sc), lambda i: he.add_const(a[i], sc))
    if level > 1:
        same(he.moddrop_batch(a, level - 1), lambda i: he.moddrop(a[i], level - 1))
        same(he.rescale_batch(a), lambda i: he.rescale(a[i]))
    same(he.hmult_relin_batch(relin, a, b), lambda i: he.hmult_relin(relin, a[i], b[i]))
    same(he.hrot_batch(rkeys[0], a), lambda i: he.hrot(rkeys[0], a[i]))
    mixed = [rkeys[i % 2] for i in range(count)]
    same(he.hrot_batch_keys(mixed, a), lambda i: he.hrot(mixed[i], a[i]))
    if p.logN == 12:  # more operations than one group of launches holds (32), and a workspace for fewer still
        many = torch.stack([he.to_device(wl.uniform_ct(1400 + i, p, level)) for i in range(35)])
        mkeys = [rkeys[(i // 3) % 2] for i in range(35)]
        got = he.hrot_batch_keys(mkeys, many)
        for i in range(35):
            assert torch.equal(got[i], he.hrot(mkeys[i], many[i])), i
        ws, wsb = he._workspace(level, 3)
        small = he.workspace_bytes(level, 3)
        out = he.empty_batch(35, level)
        keys = (ctypes.c_void_p * 35)(*[k.handle for k in mkeys])
        rc = he.lib.he_hrot_batch_keys(he.ctx, keys, ctypes.c_void_p(many.data_ptr()), ctypes.c_void_p(out.data_ptr()),
                                       level, 35, ws, small, None)
        assert rc == 0
        assert torch.equal(out, got)
    rs = he.rotate_sum_batch(rkeys, a.clone())
    same(rs, lambda i: he.rotate_sum(rkeys, a[i].clone()))
    # in place
    c = a.clone()
    he.hmult_relin_batch(relin, c, b, out=c)
    same(c, lambda i: he.hmult_relin(relin, a[i], b[i]))
