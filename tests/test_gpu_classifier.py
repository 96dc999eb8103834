"""Encrypted inference (the C4 workload): 32 synthetic 768-dimensional embeddings in one ciphertext at
N=2^16, level 24, scale 2^40, four classes.  The device sequence is compared bit for bit with the oracle's
own composition and the decrypted logits with the fp64 product X W^T (bound 2^-15 at scale 2^40)."""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


def test_inference_matches_oracle_and_plaintext(oracle_mod):
    import torch

    import paper_2210_02574_amd as pkg
    from oracle import classifier as oc
    from paper_2210_02574_amd import classifier as cl

    assert torch.cuda.is_available()
    p = wl.N16
    he = pkg.HE.from_params(p, device=0)
    o = oracle_mod.Oracle(p.logN, p.q, p.p, p.dnum)
    level, scale = 24, 2.0**40
    X = wl.embeddings(41, he.n // 1024)
    W = wl.weights(42)
    sk, s = he.keygen_secret(43), o.keygen_secret(43)
    inf = cl.EncryptedInference(he, level)
    keys = inf.make_keys(sk, 100)
    okeys = {r: o.keygen_rot(s, r, 100 + k) for k, r in enumerate(list(cl.INFER_HOISTED) + list(cl.INFER_SUM_SHIFTS))}
    z = cl.pack_samples(X, he.n)
    assert np.array_equal(z, oc.pack(X, o.n))
    m = o.encode(z, scale)
    ct = he.encrypt_coeffs(sk, m, level, 44)
    assert np.array_equal(ct, o.encrypt_coeffs(s, m, level, 44))
    pts = inf.encode_weights(W)
    # plaintext diagonals: both encoders, within one unit; the device run uses the oracle's encodings
    for i, pt in enumerate(pts):
        want = o.encode(oc.diagonal(W, i, o.n), float(p.q[level - 1]))
        got = he.encode(cl.weight_diagonals(W, he.n)[i], float(p.q[level - 1]))
        assert np.abs(got - want).max() <= 1
        pts[i] = he.to_device(o.coeffs_to_ntt(want, level))
    out = inf.run(he.to_device(ct), pts, keys)
    got = he.to_host(out)
    want = oc.infer(o, ct, W, level, okeys)
    assert got.shape == (2, level - 1, p.N)
    assert np.array_equal(got, want)
    logits = cl.logits_from_slots(he.decrypt(sk, got, scale))
    ref = X @ W.T
    err = np.abs(logits - ref).max()
    print("inference max abs error %.3g (bound %.3g)" % (err, 2.0**-15))
    assert err <= 2.0**-15


def test_train_step_slice_matches_oracle_and_plaintext(oracle_mod):
    """One gradient step of one class on one ciphertext of 32 samples (6 HMult, 25 HRot, levels 24 -> 16,
    scale 2^50): bit-exact against the oracle's own composition, and the decrypted updated weights against
    the fp64 evaluation of the same polynomial step."""
    import torch

    import paper_2210_02574_amd as pkg
    from oracle import classifier as oc
    from paper_2210_02574_amd import classifier as cl

    assert torch.cuda.is_available()
    p = wl.N16
    he = pkg.HE.from_params(p, device=0)
    o = oracle_mod.Oracle(p.logN, p.q, p.p, p.dnum)
    level, scale, lr = 24, 2.0**50, 1.0
    nb = he.n // 1024
    n_samples = nb
    X = wl.embeddings(51, nb)
    W0 = wl.weights(52)[:1]
    Wstar = wl.weights(53)
    labels = (np.argmax(X @ Wstar.T, axis=1) == 0).astype(np.float64)
    coeffs = cl.sigmoid_ls_coeffs()
    step = cl.EncryptedTrainStep(he, level, scale, lr, n_samples, coeffs)
    plan = step.plan
    sk, s = he.keygen_secret(54), o.keygen_secret(54)
    relin, rot = step.make_keys(sk, 200)
    orelin = o.keygen_relin(s, 200)
    orot = {r: o.keygen_rot(s, r, 201 + k) for k, r in enumerate(step.rotation_shifts())}
    zx = cl.pack_samples(X, he.n)
    zw = np.tile(np.concatenate([np.zeros(4), W0[0], np.zeros(1024 - 772)]), nb)
    zy = np.repeat(labels, 1024)
    cx = o.encrypt_coeffs(s, o.encode(zx, scale), level, 55)
    cw = o.encrypt_coeffs(s, o.encode(zw, scale), level, 56)
    cy = o.encrypt_coeffs(s, o.encode(zy, plan.label_scale), plan.label_level, 57)
    mask_pt = he.to_device(o.coeffs_to_ntt(o.encode(step.mask_slots(), plan.mask_scale), level - 1))
    a_x = [coeffs[k] / 8.0**k for k in range(8)]
    got = step.run(relin, rot, mask_pt, [he.to_device(cx)], [he.to_device(cw)], [[he.to_device(cy)]])
    got = he.to_host(got[0])
    want = oc.train_step(o, [cx], [cw], [[cy]], orelin, orot, level, scale, lr, n_samples, a_x)[0]
    assert got.shape == (2, plan.out_level, p.N)
    assert np.array_equal(got, want)
    dec = he.decrypt(sk, got, scale).real
    z = X @ W0[0]
    pz = np.polyval(coeffs[::-1], z / 8.0)
    ref = W0[0] - lr / n_samples * ((pz - labels) @ X)
    w_new = dec[4:772]
    err = np.abs(w_new - ref).max()
    print("train-step slice: max abs error of updated weights %.3g (bound %.3g)" % (err, 2.0**-15))
    assert err <= 2.0**-15
    # every block carries the same updated weights
    assert np.abs(dec[1024 + 4: 1024 + 772] - ref).max() <= 2.0**-15


@pytest.mark.timeout(600)
def test_full_shape_train_step_of_one_class(oracle_mod):
    """The training step at the shape that is timed (Section 3.1; 1024 samples x 768 features in 32 ciphertexts,
    one class, the batched driver, cross-ciphertext gradient sum and cross-block rotate-and-sum, levels 24 -> 16,
    scale 2^50) with real keys: the decrypted updated weights against the fp64 step over all 1024 samples within
    2^-15, and the same driver on the first two ciphertexts bit for bit against the oracle's composition (which
    runs 52 rotations and 12 Mult for them)."""
    import torch

    import paper_2210_02574_amd as pkg
    from oracle import classifier as oc
    from paper_2210_02574_amd import classifier as cl

    assert torch.cuda.is_available()
    p = wl.N16
    he = pkg.HE.from_params(p, device=0)
    o = oracle_mod.Oracle(p.logN, p.q, p.p, p.dnum)
    level, scale, lr = 24, 2.0**50, 1.0
    nb, ncts = he.n // 1024, 32
    n_samples = nb * ncts
    X = wl.embeddings(71, n_samples)
    W0 = wl.weights(72)[0]
    labels = (np.argmax(X @ wl.weights(73).T, axis=1) == 0).astype(np.float64)
    a_x = oc.logistic_poly_coeffs()  # the oracle's derivation (monomial coefficients in x); an input of the driver
    coeffs = np.array([a_x[k] * 8.0**k for k in range(8)])
    step = cl.EncryptedTrainStep(he, level, scale, lr, n_samples, coeffs)
    plan = step.plan
    sk, s = he.keygen_secret(74), o.keygen_secret(74)
    relin, rot = step.make_keys(sk, 300)
    zw = np.tile(np.concatenate([np.zeros(4), W0, np.zeros(1024 - 772)]), nb)

    def x_slots(i):
        return cl.pack_samples(X[i * nb:(i + 1) * nb], he.n)

    def y_slots(i):
        return np.repeat(labels[i * nb:(i + 1) * nb], 1024)

    # (a) all 32 ciphertexts, the library's own encodings and encryptions
    Xb = torch.stack([he.to_device(he.encrypt_coeffs(sk, he.encode(x_slots(i), scale), level, 400 + i)) for i in range(ncts)])
    Yb = torch.stack([he.to_device(he.encrypt_coeffs(sk, he.encode(y_slots(i), plan.label_scale), plan.label_level, 500 + i))
                      for i in range(ncts)])
    Wd = he.to_device(he.encrypt_coeffs(sk, he.encode(zw, scale), level, 600))
    out = step.run_batched(relin, rot, step.encode_mask(), Xb, [Wd], [Yb])[0]
    assert tuple(out.shape) == (2, plan.out_level, p.N)
    dec = he.decrypt(sk, he.to_host(out), scale).real
    pz = np.polyval(coeffs[::-1], (X @ W0) / 8.0)
    ref = W0 - lr / n_samples * ((pz - labels) @ X)
    err = np.abs(dec[4:772] - ref).max()
    print("full-shape train step (32 ciphertexts): max abs error of updated weights %.3g (bound %.3g), step size %.3g"
          % (err, 2.0**-15, np.abs(ref - W0).max()))
    assert err <= 2.0**-15
    assert np.abs(dec[31 * 1024 + 4: 31 * 1024 + 772] - ref).max() <= 2.0**-15  # every block carries the update
    assert np.abs(ref - W0).max() > 2.0**-10  # the step moved the weights by far more than the bound
    del Xb, Yb, out
    # (b) the first two ciphertexts through the same batched driver, bit for bit against the oracle
    orelin = o.keygen_relin(s, 300)
    orot = {r: o.keygen_rot(s, r, 301 + k) for k, r in enumerate(step.rotation_shifts())}
    cx = [o.encrypt_coeffs(s, o.encode(x_slots(i), scale), level, 400 + i) for i in range(2)]
    cy = [o.encrypt_coeffs(s, o.encode(y_slots(i), plan.label_scale), plan.label_level, 500 + i) for i in range(2)]
    cw = o.encrypt_coeffs(s, o.encode(zw, scale), level, 600)
    mask_pt = he.to_device(o.coeffs_to_ntt(o.encode(step.mask_slots(), plan.mask_scale), level - 1))
    got = step.run_batched(relin, rot, mask_pt, torch.stack([he.to_device(c) for c in cx]), [he.to_device(cw)],
                           [torch.stack([he.to_device(c) for c in cy])])[0]
    want = oc.train_step(o, cx, [cw], [cy], orelin, orot, level, scale, lr, n_samples, a_x)[0]
    assert np.array_equal(he.to_host(got), want)


def test_batched_train_step_equals_sequential():
    """The batched driver (one library call per step over all ciphertexts of a class) gives the bits of
    the sequential driver, on three ciphertexts of uniform residues (odd count: uneven pairwise sum)."""
    import torch

    import paper_2210_02574_amd as pkg
    from paper_2210_02574_amd import classifier as cl

    p = wl.N16
    he = pkg.HE.from_params(p, device=0)
    step = cl.EncryptedTrainStep(he, p.L, 2.0**50, 1.0, 96)
    plan = step.plan
    relin = he.evk_from_host(wl.uniform_evk(1, p), 1)
    rot = {r: he.evk_from_host(wl.uniform_evk(2 + k, p), he.galois_element(r))
           for k, r in enumerate(step.rotation_shifts())}
    X = [he.to_device(wl.uniform_ct(100 + i, p, plan.level)) for i in range(3)]
    W = [he.to_device(wl.uniform_ct(200, p, plan.level))]
    Y = [[he.to_device(wl.uniform_ct(300 + i, p, plan.label_level)) for i in range(3)]]
    mask = he.to_device(wl.uniform_limbs(400, p, list(range(plan.level - 1))))
    seq = step.run(relin, rot, mask, X, W, Y)
    bat = step.run_batched(relin, rot, mask, torch.stack(X), W, [torch.stack(Y[0])])
    assert torch.equal(seq[0], bat[0])


def test_logistic15_matches_oracle_and_the_paper_bound(oracle_mod):
    """The paper's activation (Section 2.2): the degree-15 minimax polynomial on [-12, 12], evaluated under
    encryption on t = x/12 (7 HMult, five levels).  Bit-exact against the oracle's own composition with the
    same coefficients; the decrypted values follow the fp64 polynomial to 1e-6 and the true logistic function
    to the paper's 0.00614."""
    import torch

    import paper_2210_02574_amd as pkg
    from oracle import classifier as oc
    from paper_2210_02574_amd import classifier as cl

    assert torch.cuda.is_available()
    p = wl.N16
    he = pkg.HE.from_params(p, device=0)
    o = oracle_mod.Oracle(p.logN, p.q, p.p, p.dnum)
    level, scale = 8, 2.0**50
    coeffs = oc.minimax15_coeffs()  # the oracle's own derivation; the device run takes the same numbers as an input
    sup = np.abs(np.polyval(coeffs[::-1], np.linspace(-1, 1, 48001)) - 1 / (1 + np.exp(-12 * np.linspace(-1, 1, 48001)))).max()
    sk, s = he.keygen_secret(61), o.keygen_secret(61)
    relin, orelin = he.keygen_relin(sk, 62), o.keygen_relin(s, 62)
    x = 12.0 * wl.slots_uniform(63, he.n).real
    x[:5] = [-12.0, 12.0, 0.0, 11.3, -0.4]
    t = (x / 12.0).astype(np.complex128)
    m = o.encode(t, scale)
    ct = he.encrypt_coeffs(sk, m, level, 64)
    ev = cl.EncryptedLogistic15(he, level, scale, coeffs)
    got = he.to_host(ev.run(relin, he.to_device(ct)))
    want, want_scale = oc.logistic15(o, ct, orelin, level, scale, coeffs)
    assert got.shape == (2, level - 5, p.N)
    assert ev.out_scale == want_scale
    assert np.array_equal(got, want)
    dec = he.decrypt(sk, got, ev.out_scale).real
    poly = np.polyval(coeffs[::-1], x / 12.0)
    err_poly = np.abs(dec - poly).max()
    err_sig = np.abs(dec - 1.0 / (1.0 + np.exp(-x))).max()
    print("logistic15: vs fp64 polynomial %.3g, vs logistic function %.4g (minimax error %.4g)" % (err_poly, err_sig, sup))
    assert err_poly <= 1e-6
    assert err_sig <= 0.00614 + 1e-6
