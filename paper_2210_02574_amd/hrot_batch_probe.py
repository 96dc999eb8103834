"""Three batched rotations with one key on uniform residues: a short, fixed target for per-kernel hardware counters
and traces (`rocprofv3 --pmc <counters> -- python3 paper_2210_02574_amd/hrot_batch_probe.py`).  Default: eight
level-24 ciphertexts at N = 2^16, L = 24, K = 4, dnum = 6; arguments: parameter set, level, count (for example
`P17 30 4`: the paper's ring degree)."""
import os
import sys

import torch

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

import workloads as wl  # noqa: E402
import paper_2210_02574_amd as pkg  # noqa: E402


def main():
    p = getattr(wl, sys.argv[1]) if len(sys.argv) > 1 else wl.N16
    he = pkg.HE.from_params(p, device=0)
    level = int(sys.argv[2]) if len(sys.argv) > 2 else p.L
    count = int(sys.argv[3]) if len(sys.argv) > 3 else 8
    key = he.evk_from_host(wl.uniform_evk(1, p), he.galois_element(1))
    cts = torch.stack([he.to_device(wl.uniform_ct(30 + i, p, level)) for i in range(count)])
    out = he.empty_batch(count, level)
    for _ in range(3):
        he.hrot_batch(key, cts, out=out)
    torch.cuda.synchronize()
    print("3 x hrot_batch of %d ciphertexts at level %d" % (count, level))


if __name__ == "__main__":
    main()
