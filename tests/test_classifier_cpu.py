"""CPU-side checks of the classifier drivers: polynomial coefficients and packing helpers."""
import numpy as np

import workloads as wl


def test_sigmoid_coefficients():
    """Degree-7 least-squares fit of the logistic function on [-8,8]: two derivations (Legendre projection in
    the library's driver, normal equations in the oracle) agree with each other and with the values worked
    out by hand for this fit: 0.5 + 1.735165 t - 4.195716 t^3 + 5.437381 t^5 - 2.509360 t^7, sup error 0.0322."""
    from oracle import classifier as oc
    from paper_2210_02574_amd import classifier as cl

    c = cl.sigmoid_ls_coeffs()
    a = oc.logistic_poly_coeffs()
    assert np.allclose([a[k] * 8.0**k for k in range(8)], c, atol=1e-9)
    assert np.allclose(c[1::2], [1.735165, -4.195716, 5.437381, -2.509360], atol=5e-7)
    assert np.allclose(cl.sigmoid_ls_coeffs(degree=3)[1::2], [1.200963, -0.815625], atol=5e-7)
    t = np.linspace(-1, 1, 4001)
    sup = np.abs(np.polyval(c[::-1], t) - 1 / (1 + np.exp(-8 * t))).max()
    assert abs(sup - 0.0322) < 2e-4


def test_packing_and_diagonals_reproduce_the_logits():
    """Plaintext check of the packing: the diagonal products summed with stride 4 give X W^T in slots
    1024 b + c, for both sides' helpers."""
    from oracle import classifier as oc
    from paper_2210_02574_amd import classifier as cl

    n = 4096
    X = wl.embeddings(1, n // 1024)
    W = wl.weights(2)
    z = cl.pack_samples(X, n)
    assert np.array_equal(z, oc.pack(X, n))
    t = np.zeros(n)
    for i, d in enumerate(cl.weight_diagonals(W, n)):
        assert np.array_equal(d, oc.diagonal(W, i, n))
        t += d * np.roll(z, -i)
    for k in range(8):
        t = t + np.roll(t, -(4 << k))
    assert np.allclose(cl.logits_from_slots(t), X @ W.T, atol=1e-12)


def test_minimax15_matches_the_paper():
    """Degree-15 minimax polynomial of the logistic function on [-12, 12]: the paper (Section 2.2) states an
    error within 0.00614.  Remez exchange (library driver) and a linear program on a grid (oracle side)
    agree, and the sup error sits just under the printed bound."""
    from oracle import classifier as oc
    from paper_2210_02574_amd import classifier as cl

    mono, sup = cl.minimax_logistic_coeffs()
    assert 0.00605 < sup <= 0.00614
    t = np.linspace(-1, 1, 48001)
    err = np.abs(np.polyval(mono[::-1], t) - 1 / (1 + np.exp(-12 * t)))
    assert abs(err.max() - sup) < 1e-7
    c_lp, e_lp = oc.minimax15_by_linear_program()
    assert abs(e_lp - sup) < 2e-5
    # the coefficients every oracle leg uses: inside the printed bound, and close to the library's Remez result
    c_o = oc.minimax15_coeffs()
    err_o = np.abs(np.polyval(c_o[::-1], t) - 1 / (1 + np.exp(-12 * t))).max()
    assert err_o <= 0.00614 and abs(err_o - sup) < 2e-6
    assert np.abs(np.polyval(c_o[::-1], t) - np.polyval(mono[::-1], t)).max() < 1e-5
    err_lp = np.abs(sum(c_lp[k] * t ** (2 * k + 1) for k in range(8)) + 0.5 - 1 / (1 + np.exp(-12 * t))).max()
    assert abs(err_lp - sup) < 1e-4


def test_oracle_logistic15_decrypts_to_the_logistic_function():
    """The oracle's encrypted degree-15 evaluation at N=2^16 decrypts to the fp64 polynomial (1e-6) and so to
    the logistic function within the paper's 0.00614 on [-12, 12] (Section 2.2)."""
    import workloads as wl
    from oracle import classifier as oc
    from oracle.ckks import Oracle

    p = wl.N16
    o = Oracle(p.logN, p.q, p.p, p.dnum)
    coeffs = oc.minimax15_coeffs()
    s = o.keygen_secret(61)
    relin = o.keygen_relin(s, 62)
    x = 12.0 * wl.slots_uniform(63, o.n).real
    x[:3] = [-12.0, 12.0, 0.0]
    ct = o.encrypt_coeffs(s, o.encode((x / 12.0).astype(np.complex128), 2.0**50), 8, 64)
    out, sc = oc.logistic15(o, ct, relin, 8, 2.0**50, coeffs)
    assert out.shape == (2, 3, p.N)
    dec = o.decrypt(s, out, sc).real
    assert np.abs(dec - np.polyval(coeffs[::-1], x / 12.0)).max() <= 1e-6
    assert np.abs(dec - 1.0 / (1.0 + np.exp(-x))).max() <= 0.00614 + 1e-6
