"""The rotation that allocates nothing (he_hrot_noalloc, the library's static scratch array in place of a
workspace) against he_hrot through the C ABI: same residues, on two calls in a row, the second one smaller.
Collected last on purpose: a failure here must not hide the parity tests."""
import ctypes

import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


def _hrot_both(he, key, ct):
    import torch

    d = he.to_device(ct)
    want = he.to_host(he.hrot(key, d))
    out = torch.empty_like(d)
    before = torch.cuda.memory_allocated()
    rc = he.lib.he_hrot_noalloc(he.ctx, key.handle, ctypes.c_void_p(d.data_ptr()), ctypes.c_void_p(out.data_ptr()),
                                int(d.shape[1]), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == 0, rc
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    return he.to_host(out), want


@pytest.mark.parametrize("name,levels", [("N16", (9, 3)), ("B12", (24, 5)), ("C1B", (3, 1))])
def test_hrot_noalloc_equals_hrot(name, levels, oracle_mod):
    import torch

    assert torch.cuda.is_available(), "this test needs the MI355X"
    import paper_2210_02574_amd as pkg

    p = getattr(wl, name)
    he = pkg.HE.from_params(p, device=0)
    evk = wl.uniform_evk(901, p)
    g = he.galois_element(3)
    key = he.evk_from_host(evk, g)
    for k, level in enumerate(levels):  # the second call is the smaller one and finds the first one's leftovers
        ct = wl.uniform_ct(910 + k, p, level)
        got, want = _hrot_both(he, key, ct)
        assert np.array_equal(got, want), (name, level)
    if name == "C1B":  # and against the oracle, where it finishes at once
        o = oracle_mod.Oracle(p.logN, p.q, p.p, p.dnum)
        assert np.array_equal(got, o.hrot(ct, evk, 3)), name


def test_hrot_noalloc_refuses_what_does_not_fit():
    import torch

    import paper_2210_02574_amd as pkg

    p = wl.N16
    he = pkg.HE.from_params(p, device=0)
    key = he.evk_from_host(wl.uniform_evk(902, p), he.galois_element(1))
    assert he.workspace_bytes(10) > 64 << 20 >= he.workspace_bytes(9)
    d = he.to_device(wl.uniform_ct(903, p, 10))
    out = torch.zeros_like(d)
    with pytest.raises(pkg.HeError) as e:
        he.hrot_noalloc(key, d, out)
    assert e.value.code == -8
    torch.cuda.synchronize()
    assert int(out.abs().sum()) == 0  # nothing was launched
