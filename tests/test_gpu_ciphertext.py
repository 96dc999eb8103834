"""The (tensor, level, scale) wrapper: an expression evaluated under encryption against numpy, with levels and
scales tracked by the wrapper alone."""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


def test_expression_with_tracked_levels_and_scales():
    import torch

    import paper_2210_02574_amd as pkg

    assert torch.cuda.is_available()
    p = wl.N16
    he = pkg.HE.from_params(p, device=0)
    sk = he.keygen_secret(31)
    ev = pkg.Evaluator.generate(he, sk, 32, shifts=(1, -2), with_conj=True)
    g = wl.rng(33)
    x = g.uniform(-1, 1, he.n) + 1j * g.uniform(-1, 1, he.n)
    y = g.uniform(-1, 1, he.n)
    m = g.uniform(-1, 1, he.n)
    scale = 2.0**45
    cx, cy = ev.encrypt(sk, x, 6, scale, 34), ev.encrypt(sk, y, 5, scale, 35)
    assert (cx.level, cy.level) == (6, 5)
    # (x * y) * 0.75 + rot(x, 1) * m - conj(x) * 0.5, all terms brought to one scale by the constants
    xy = cx * cy                                   # level 4, scale 2^90 / q
    assert xy.level == 4 and abs(xy.scale - scale * scale / p.q[4]) < 1e-3
    t1 = xy.mul_const(0.75, target_scale=scale)    # level 3, scale 2^45
    t2 = cx.rotate(1).mul_plain(m)                 # level 5, scale 2^45
    t3 = cx.conj().mul_const(0.5)                  # level 5
    out = t1 + t2 - t3
    assert out.level == 3 and out.scale == scale
    want = x * y * 0.75 + np.roll(x, -1) * m - np.conj(x) * 0.5
    err = np.abs(ev.decrypt(sk, out) - want).max()
    assert err < 2.0**-20, err
    # a square and a constant: scale follows Mult, add_const uses it
    sq = (out * out).add_const(1.25)
    assert sq.level == 2
    assert np.abs(ev.decrypt(sk, sq) - (want * want + 1.25)).max() < 2.0**-18
    with pytest.raises(ValueError):
        _ = xy + cx  # scales 2^90/q and 2^45
    assert np.abs(ev.decrypt(sk, cx.rotate(-2)) - np.roll(x, 2)).max() < 2.0**-20
