"""Parity at the benchmark's full sizes and launch configuration: the step that bench.py times
(N=2^16, L=24, dnum=6) is run once on a reduced count of operations and whole outputs of each kind of
operation are compared with the oracle bit for bit."""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n_streams", [1, 3])
def test_bench_step_outputs_match_oracle(oracle_mod, n_streams):
    import torch

    import bench
    import paper_2210_02574_amd as pkg

    assert torch.cuda.is_available()
    p = wl.N16
    he = pkg.HE.from_params(p, device=0)
    o = oracle_mod.Oracle(p.logN, p.q, p.p, p.dnum)
    w = bench.Workload(he, seed=2, n_hmult=3, n_single=6, n_ntt=56, n_streams=n_streams, hm_chunk=2)
    ntt_in = he.to_host(w.ntt_limbs).copy()
    w.step()
    torch.cuda.synchronize()
    # NTT followed by iNTT returns the input; the forward result itself is checked on a second pass
    assert np.array_equal(he.to_host(w.ntt_limbs), ntt_in)
    he.ntt(w.ntt_limbs, w.ntt_mods)
    fwd = he.to_host(w.ntt_limbs)
    for b in (0, 23, 24, 27, 55):
        assert np.array_equal(fwd[b], o.ntt(ntt_in[b], w.ntt_mods[b])), b
    he.intt(w.ntt_limbs, w.ntt_mods)
    relin = wl.uniform_evk(1000, p)
    for i in (1, 2):
        a, b = he.to_host(w.hm_a[i]), he.to_host(w.hm_b[i])
        assert np.array_equal(he.to_host(w.rs_out[i]), o.rescale(o.hmult_relin(a, b, relin))), i
    ct = he.to_host(w.hoist_in)
    for k in (0, 7, 14):
        evk = wl.uniform_evk(1001 + k, p)
        assert np.array_equal(he.to_host(w.hoist_out[k]), o.hrot(ct, evk, w.offsets[k])), k
    for i in (0, 5):
        k = w.single_keys[i]
        evk = wl.uniform_evk(1001 + k, p)
        got = he.to_host(w.single_out[i])
        assert got.shape[1] == w.single_levels[i]
        assert np.array_equal(got, o.hrot(he.to_host(w.single_in[i]), evk, w.offsets[k])), i


def test_full_batches_span_several_launches(oracle_mod):
    """The batch sizes that bench.py times: 16 products per call (2304 raised limbs, more than one launch of the
    conversion passes can carry, so the list is split) and 32 mixed-level rotations per call.  Operations on both sides
    of every split, the first and the last are compared with the oracle bit for bit."""
    import torch

    import bench
    import paper_2210_02574_amd as pkg

    p = wl.N16
    he = pkg.HE.from_params(p, device=0)
    o = oracle_mod.Oracle(p.logN, p.q, p.p, p.dnum)
    w = bench.Workload(he, seed=2, n_hmult=16, n_single=32, n_ntt=1, n_streams=1, hm_chunk=16, single_chunk=32)
    assert len(w.single_groups) == 1
    w.step()
    torch.cuda.synchronize()
    relin = wl.uniform_evk(1000, p)
    for i in (0, 7, 8, 15):
        a, b = he.to_host(w.hm_a[i]), he.to_host(w.hm_b[i])
        assert np.array_equal(he.to_host(w.rs_out[i]), o.rescale(o.hmult_relin(a, b, relin))), i
    # the call's order is by key, then by level: take its first and last operation and four in between
    order = sorted(range(w.n_single), key=lambda i: (w.single_keys[i], -w.single_levels[i]))
    for pos in (0, 9, 15, 16, 22, 31):
        i = order[pos]
        k = w.single_keys[i]
        evk = wl.uniform_evk(1001 + k, p)
        got = he.to_host(w.single_out[i])
        assert got.shape[1] == w.single_levels[i]
        assert np.array_equal(got, o.hrot(he.to_host(w.single_in[i]), evk, w.offsets[k])), (pos, i)
