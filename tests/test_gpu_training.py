"""Encrypted training loop on the device (paper_2210_02574_amd/training.py) against the oracle's composition:
one iteration bit-exact on every residue (shared plaintext encodings), three iterations against the fp64
iteration of the same polynomial step."""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("degree", [7, 15])
def test_training_iterations_match_oracle_and_plaintext(oracle_mod, degree):
    import torch

    import paper_2210_02574_amd as pkg
    from oracle import bootstrap as ob
    from oracle import classifier as oc
    from oracle import training as ot
    from paper_2210_02574_amd.training import EncryptedTrainer
    from training_common import Problem

    assert torch.cuda.is_available()
    p = wl.T12
    he = pkg.HE.from_params(p, device=0)
    o = oracle_mod.Oracle(p.logN, p.q, p.p, p.dnum)
    pr = Problem(o.n)
    S, lr, gamma = 2.0**50, 1.0, 0.5
    a = oc.logistic_poly_coeffs()
    c15 = None
    if degree == 7:
        tr = EncryptedTrainer(he, pr.block, lr, gamma, pr.nb, S, coeffs=np.array([a[k] * 8.0**k for k in range(8)]))
    else:  # the paper's activation: degree-15 minimax polynomial on [-12, 12], same coefficients on both sides
        c15 = oc.minimax15_coeffs()  # the oracle's own derivation, an input of the device driver
        tr = EncryptedTrainer(he, pr.block, lr, gamma, pr.nb, S, coeffs=c15, degree=15)
    plan = ob.Plan(o, pr.block, 7, groups=2)
    level = tr.level
    assert level == plan.out_level == 12 and tr.rotation_shifts() == sorted(
        set([1 << k for k in range(6)] + [-(1 << k) for k in range(6)] + [pr.block << k for k in range(5)])
        | set(plan.rotation_shifts()))
    sk, s = he.keygen_secret_sparse(1, 64), ob.sparse_secret(o, 1, 64)
    keys = tr.make_keys(sk, 100)
    okeys = {"relin": o.keygen_relin(s, 100), "conj": o.keygen_conj(s, 101),
             "rot": {sh: o.keygen_rot(s, sh, 110 + i) for i, sh in enumerate(tr.rotation_shifts())}}
    tp = tr.step.plan
    x_ct = o.encrypt_coeffs(s, o.encode(pr.slots_x(), S), level, 200)
    w_ct = o.encrypt_coeffs(s, o.encode(pr.slots_w(pr.w0), S), level, 201)
    y_ct = o.encrypt_coeffs(s, o.encode(pr.slots_y(), tp.label_scale), tp.label_level, 202)
    # oracle iteration and its plaintext encodings (mask, both Bootstrap matrices)
    g = plan.groups
    c_in = (np.pi / (plan.gap * 2.0**plan.r)) ** (1.0 / g)
    c_out = (tr.gain / (4.0 * np.pi)) ** (1.0 / g)
    cts_o = [ob.encode_sparse(o, c_in * np.linalg.inv(plan.factors[i]), plan.L - (g - 1 - i)) for i in range(g)]
    stc_o = [ob.encode_sparse(o, c_out * plan.factors[i], level + g - i) for i in range(g)]
    v_level = tp.out_level
    W1, V1 = ot.iterate(o, [x_ct], [w_ct], [o.moddrop(w_ct, v_level)], [[y_ct]], okeys, plan, pr.block, S, lr, gamma,
                        pr.nb, a, cts_o, stc_o, c15=c15)
    mask = np.zeros(o.n)
    mask[::pr.block] = tp.mask_value
    mask_pt = he.to_device(o.coeffs_to_ntt(o.encode(mask, float(o.q[level - 2])), level - 1))
    from paper_2210_02574_amd.bootstrap import DiagonalLayout

    def to_dev(encoded, mats):  # the driver's own layout of the same matrices, the oracle's encodings
        return [(DiagonalLayout(M), {k: he.to_device(v) for k, v in pts.items()}) for (_, pts), M in zip(encoded, mats)]

    X = he.to_device(x_ct).unsqueeze(0).contiguous()
    Y = [he.to_device(y_ct).unsqueeze(0).contiguous()]
    W = [he.to_device(w_ct)]
    V = [he.moddrop(W[0], v_level)]
    fac = tr.boot.factors()
    boot_pts = (to_dev(cts_o, [c_in * np.linalg.inv(G) for G in fac]), to_dev(stc_o, [c_out * G for G in fac]))
    Wn, Vn = tr.iterate(keys, mask_pt, X, W, V, Y, boot_pts)
    assert np.array_equal(he.to_host(Vn[0]), V1[0])
    assert np.array_equal(he.to_host(Wn[0]), W1[0])
    # two more iterations with the driver's own plaintexts; compare with the fp64 iteration
    wp, vp = pr.plain_iteration(pr.w0, pr.w0, a, lr, gamma, c15)
    mask_own = tr.step.encode_mask()
    for it in range(2):
        Wn, Vn = tr.iterate(keys, mask_own, X, Wn, Vn, Y)
        wp, vp = pr.plain_iteration(wp, vp, a, lr, gamma, c15)
        dec = he.decrypt(sk, he.to_host(Wn[0]), S).real
        err = np.abs(dec[pr.off:pr.off + pr.dim] - wp).max()
        print("iteration %d: max weight error %.3g (|w| up to %.3g)" % (it + 2, err, np.abs(wp).max()))
        assert err < 2e-4


def test_minibatch_epochs_follow_the_plaintext_recipe():
    """Two mini-batches, two epochs (four iterations with a Bootstrap each) with the driver's own keys and
    plaintexts: the decrypted weights follow the fp64 run of the same mini-batch schedule."""
    import torch

    import paper_2210_02574_amd as pkg
    from oracle import classifier as oc
    from paper_2210_02574_amd.training import EncryptedTrainer
    from training_common import Problem

    assert torch.cuda.is_available()
    p = wl.T12
    he = pkg.HE.from_params(p, device=0)
    probs = [Problem(he.n, seed=7), Problem(he.n, seed=8)]
    S, lr, gamma = 2.0**50, 2.0, 0.1  # the paper's ciphertext hyperparameters for its multi-class set
    a = oc.logistic_poly_coeffs()
    tr = EncryptedTrainer(he, probs[0].block, lr, gamma, probs[0].nb, S, coeffs=np.array([a[k] * 8.0**k for k in range(8)]))
    sk = he.keygen_secret_sparse(1, 64)
    keys = tr.make_keys(sk, 100)
    tp = tr.step.plan
    batches = []
    for i, pr in enumerate(probs):
        X = he.to_device(he.encrypt_coeffs(sk, he.encode(pr.slots_x(), S), tr.level, 500 + i)).unsqueeze(0).contiguous()
        Y = [he.to_device(he.encrypt_coeffs(sk, he.encode(pr.slots_y(), tp.label_scale), tp.label_level, 510 + i))
             .unsqueeze(0).contiguous()]
        batches.append((X, Y))
    w0 = probs[0].w0
    W = [he.to_device(he.encrypt_coeffs(sk, he.encode(probs[0].slots_w(w0), S), tr.level, 520))]
    V = [he.moddrop(W[0], tp.out_level)]
    W, V = tr.fit(keys, tr.step.encode_mask(), batches, W, V, epochs=2)
    wp, vp = w0, w0
    for _ in range(2):
        for pr in probs:
            wp, vp = pr.plain_iteration(wp, vp, a, lr, gamma)
    pr = probs[0]
    dec = he.decrypt(sk, he.to_host(W[0]), S).real
    err = np.abs(dec[pr.off:pr.off + pr.dim] - wp).max()
    print("four iterations: max weight error %.3g (|w| up to %.3g)" % (err, np.abs(wp).max()))
    assert err < 2e-4
    # every block of the packed weight vector holds the same weights
    assert np.abs(dec[pr.block + pr.off:pr.block + pr.off + pr.dim] - wp).max() < 2e-4


@pytest.mark.timeout(600)
def test_full_size_training_iteration():
    """The paper's recipe at full size (Section 3.1): N = 2^16, 28 primes, one sample per 1024-slot block, 1024
    samples x 768 features in 32 ciphertexts, one class; gradient step, Nesterov look-ahead and a Bootstrap of the
    1024-slot weight vector per iteration, real keys (sparse secret), the driver's own plaintexts.  Two iterations
    against the fp64 iteration of the same polynomial step: max weight error <= 1e-5."""
    import torch

    import paper_2210_02574_amd as pkg
    from oracle import classifier as oc
    from paper_2210_02574_amd.training import EncryptedTrainer

    assert torch.cuda.is_available()
    p = wl.T16
    he = pkg.HE.from_params(p, device=0)
    block, dim, off, ncts = 1024, 768, 4, 32
    nb = he.n // block
    n_samples = nb * ncts
    S, lr, gamma = 2.0**50, 1.0, 0.5
    a = oc.logistic_poly_coeffs()
    tr = EncryptedTrainer(he, block, lr, gamma, n_samples, S, coeffs=np.array([a[k] * 8.0**k for k in range(8)]))
    level, tp = tr.level, tr.step.plan
    assert level == 12 and tp.out_level == 4
    sk = he.keygen_secret_sparse(1, 64)
    keys = tr.make_keys(sk, 100)
    tr.boot.prepare(tr.gain)
    X = wl.embeddings(81, n_samples)
    w0 = wl.weights(82)[0]
    y = (X @ wl.weights(83)[0] > 0).astype(np.float64)

    def blocks(rows):
        z = np.zeros(he.n)
        for b in range(nb):
            z[b * block + off: b * block + off + dim] = rows[b]
        return z

    Xc = torch.stack([he.to_device(he.encrypt_coeffs(sk, he.encode(blocks(X[i * nb:(i + 1) * nb]), S), level, 200 + i))
                      for i in range(ncts)])
    Yc = [torch.stack([he.to_device(he.encrypt_coeffs(sk, he.encode(np.repeat(y[i * nb:(i + 1) * nb], block), tp.label_scale),
                                                      tp.label_level, 300 + i)) for i in range(ncts)])]
    W = [he.to_device(he.encrypt_coeffs(sk, he.encode(blocks([w0] * nb), S), level, 400))]
    V = [he.moddrop(W[0], tp.out_level)]
    mask = tr.step.encode_mask()
    wp, vp = w0.copy(), w0.copy()
    for it in range(2):
        W, V = tr.iterate(keys, mask, Xc, W, V, Yc)
        z = X @ wp
        pz = sum(a[k] * z**k for k in range(8))
        vn = wp - lr * ((pz - y)[:, None] * X).sum(0) / n_samples
        wp, vp = (1 + gamma) * vn - gamma * vp, vn
        assert tuple(W[0].shape) == (2, level, p.N)
        dec = he.decrypt(sk, he.to_host(W[0]), S).real
        err = np.abs(dec[off:off + dim] - wp).max()
        print("full-size iteration %d: max weight error %.3g (|w| up to %.3g)" % (it + 1, err, np.abs(wp).max()))
        assert err <= 1e-5
        assert np.abs(dec[5 * block + off: 5 * block + off + dim] - wp).max() <= 1e-5  # every block holds the weights
    assert np.abs(wp - w0).max() > 1e-2
