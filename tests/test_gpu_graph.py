"""The library only enqueues kernels and copies on the caller's stream, so a sequence of calls can be captured in
a HIP graph: a captured rotation, HMult + rescale and rotate-and-sum replay to the bits of the eager calls, on
every replay, with eager work in between."""
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


def test_captured_sequence_replays_to_the_eager_result():
    import torch

    import paper_2210_02574_amd as pkg

    p = wl.C1B
    he = pkg.HE.from_params(p, device=0)
    level = p.L
    relin = he.evk_from_host(wl.uniform_evk(11, p), 1)
    rots = [he.evk_from_host(wl.uniform_evk(12 + k, p), he.galois_element(1 << k)) for k in range(3)]
    a, b = he.to_device(wl.uniform_ct(21, p, level)), he.to_device(wl.uniform_ct(22, p, level))

    def sequence():
        prod = he.hmult_relin_rescale(relin, a, b)
        rot = he.hrot(rots[0], prod)
        he.rotate_sum(rots, rot)  # three steps: ends with the copy back from the workspace
        return rot

    want = sequence().clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        sequence()  # the binding's workspace of the capture stream exists before the capture starts
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        got = sequence()
    torch.cuda.synchronize()
    for replay in range(3):
        got.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(got, want), replay
        he.hrot(rots[1], he.to_device(wl.uniform_ct(30 + replay, p, level)))  # eager work between replays
        torch.cuda.synchronize()
