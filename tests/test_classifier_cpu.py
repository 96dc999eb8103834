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
