#!/usr/bin/env python3
"""Benchmark of the RNS-CKKS hot path on one MI355X.

One step = one pass of the whole hot path at N=2^16, L=24, K=4, dnum=6 over synthetic residues:
  * 256 limb NTT + iNTT pairs (limb b modulo modulus b mod 28),
  * 64 independent HMult + relinearisation + rescale on level-24 ciphertexts,
  * 15 hoisted rotations of one level-24 ciphertext by 2^0 .. 2^14,
  * 128 single rotations at mixed levels 8..24.
Every step therefore performs 64 + 15 + 128 = 207 key switches; `value` is key switches per
second over the whole step with all inputs resident in HBM.  All operations of a step are independent;
with more than one stream they are issued round-robin to the streams without joins between the four kinds
(`detail` times the kinds one after the other in a separate pass).  The line also carries the roofline
of the kernel that takes the most time (measured with HIP events inside the library over a
repeat of the timed steps) and the CPU oracle timed on a bounded sample of the same workload.

Contract: python bench.py --gpus 1 --steps K --warmup W  -> one JSON line on stdout.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import workloads as wl  # noqa: E402

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published

# Published peaks of one MI355X: HBM3E bandwidth, and the vector ALU rate that bounds the instruction-bound kernels:
# 256 compute units x 4 SIMDs x 16 lanes x 2.4 GHz lane-instructions per second (one FP64 multiply-add or one
# 32-bit integer multiply-add per lane and cycle: 78.6 TFLOP/s of FP64).
ALU_PEAK_TLIPS = 256 * 4 * 16 * 2.4e9 / 1e12

# Hardware-counter figures per launch of each kernel come from the committed rocprofv3 summary below (its header
# names the commit and the commands): scaled HBM traffic (2 x FETCH_SIZE + WRITE_SIZE, see the calibration there)
# and vector instructions issued (64 x SQ_INSTS_VALU lane-instructions), both averaged over the launches of this
# benchmark's step.  They are re-measured whenever a kernel changes; a missing file gives null fields.
COUNTER_SUMMARY = os.path.join("profiles", "bench_step_N16_L24_counters.md")


def load_counter_summary():
    """{library kernel name: (traffic bytes, lane-instructions, algorithmic bytes), each per launch of the profiled
    run} and the summary's source line."""
    path = os.path.join(ROOT, COUNTER_SUMMARY)
    table, source = {}, None
    if not os.path.exists(path):
        return table, source
    source = COUNTER_SUMMARY
    with open(path) as fh:
        for line in fh:
            if line.startswith("Measured at commit"):
                source = COUNTER_SUMMARY + " (" + line.strip().rstrip(".") + ")"
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            if len(cells) >= 7 and cells[0].startswith("k_") and cells[0] != "kernel":
                try:
                    table[cells[0]] = (float(cells[4]), float(cells[5]), float(cells[6]))
                except ValueError:
                    pass
    return table, source


class Workload:
    """Device-resident synthetic inputs of one step and the step itself."""

    N_NTT = 256
    N_HMULT = 64
    N_SINGLE = 128

    def __init__(self, he, seed: int = 2, n_hmult: int = None, n_single: int = None, n_ntt: int = None,
                 n_streams: int = 1, hm_chunk: int = 16, single_mode: str = "levels", single_chunk: int = 32):
        import torch

        self.torch = torch
        self.he = he
        # independent operations are spread over this many HIP streams (default priority)
        self.streams = [torch.cuda.Stream(device=he.device) for _ in range(n_streams)] if n_streams > 1 else []
        p = self.params = wl.N16
        self.n_hmult = self.N_HMULT if n_hmult is None else n_hmult
        self.n_single = self.N_SINGLE if n_single is None else n_single
        self.n_ntt = self.N_NTT if n_ntt is None else n_ntt
        self.dev = torch.device(f"cuda:{he.device}")
        self.gen = torch.Generator(device=self.dev)
        self.gen.manual_seed(seed)
        M = p.L + p.K
        self.ntt_mods = [b % M for b in range(self.n_ntt)]
        self.ntt_limbs = self._uniform(self.ntt_mods)
        L = p.L
        # the independent HMult operands, stored back to back so that one batched call covers them
        self.hm_a = torch.stack([self._uniform_ct(L) for _ in range(self.n_hmult)])
        self.hm_b = torch.stack([self._uniform_ct(L) for _ in range(self.n_hmult)])
        self.rs_out = he.empty_batch(self.n_hmult, L - 1)
        self.hm_chunk = hm_chunk
        # keys: uniform residues in key layout (throughput does not depend on the values)
        self.key_host = {}
        self.relin = self._key(1000, 1)
        self.offsets = [1 << k for k in range(15)]
        self.rot = [self._key(1001 + k, he.galois_element(r)) for k, r in enumerate(self.offsets)]
        self.hoist_in = self._uniform_ct(L)
        self.hoist_out = [he.empty_ct(L) for _ in self.offsets]
        levels, offs = wl.mixed_levels(seed + 1, self.n_single)
        self.single_levels = levels
        self.single_keys = [self.offsets.index(o) for o in offs]
        self.single_in = [self._uniform_ct(lv) for lv in levels]
        self.single_out = [he.empty_ct(lv) for lv in levels]
        # The single rotations are independent (own ciphertext, level and key each).  They are issued as a server
        # would batch independent requests: sorted by key and packed back to back, 32 per call of the mixed-level
        # entry point ("levels", the default: every launch is shared by the 32 operations, and neighbours with the
        # same key share its memory traffic); or one call per level with one key per ciphertext ("per-level"); or
        # one he_hrot call each ("each").
        self.single_groups = []
        self.single_mode = single_mode
        if single_mode == "levels":
            order = sorted(range(self.n_single), key=lambda i: (self.single_keys[i], -levels[i]))
            for lo in range(0, self.n_single, single_chunk):
                idx = order[lo:lo + single_chunk]
                packed = torch.cat([self.single_in[i].reshape(-1, p.N) for i in idx])
                outs = torch.empty_like(packed)
                at = 0
                for i in idx:
                    n = 2 * levels[i]
                    self.single_in[i] = packed[at:at + n].view(2, levels[i], p.N)
                    self.single_out[i] = outs[at:at + n].view(2, levels[i], p.N)
                    at += n
                self.single_groups.append(([self.rot[self.single_keys[i]] for i in idx], [int(levels[i]) for i in idx],
                                           packed, outs))
        elif single_mode == "per-level":
            for lv in sorted(set(levels), reverse=True):
                # rotations that share a key sit next to each other: the inner product then reads that key once
                idx = sorted((i for i in range(self.n_single) if levels[i] == lv), key=lambda i: self.single_keys[i])
                cts = torch.stack([self.single_in[i] for i in idx])
                outs = he.empty_batch(len(idx), lv)
                for k, i in enumerate(idx):
                    self.single_in[i], self.single_out[i] = cts[k], outs[k]
                self.single_groups.append(([self.rot[self.single_keys[i]] for i in idx], None, cts, outs))
        self.key_switches = self.n_hmult + len(self.offsets) + self.n_single

    def _uniform(self, mod_idx):
        torch = self.torch
        mods = self.params.moduli
        out = torch.empty((len(mod_idx), self.params.N), dtype=torch.int64, device=self.dev)
        for b, mi in enumerate(mod_idx):
            out[b].random_(0, mods[mi], generator=self.gen)
        return out

    def _uniform_ct(self, level):
        return self._uniform(list(range(level)) * 2).view(2, level, self.params.N)

    def _key(self, seed, g):
        evk = wl.uniform_evk(seed, self.params)
        return self.he.evk_from_host(evk, g)

    def step(self, marks=None, serial=False):
        """serial: every operation on the current stream, one after the other (each kernel alone on the GPU)."""
        he = self.he

        def mark(name):
            if marks is not None:
                ev = self.torch.cuda.Event(enable_timing=True)
                ev.record()
                marks.append((name, ev))

        if marks is None and self.streams and not serial:
            return self._step_overlapped()
        mark("start")
        he.ntt(self.ntt_limbs, self.ntt_mods)
        he.intt(self.ntt_limbs, self.ntt_mods)
        mark("ntt_pairs")
        for lo in range(0, self.n_hmult, self.hm_chunk):  # batched calls of hm_chunk ciphertext pairs
            hi = min(lo + self.hm_chunk, self.n_hmult)
            he.hmult_relin_rescale_batch(self.relin, self.hm_a[lo:hi], self.hm_b[lo:hi], out=self.rs_out[lo:hi])
        mark("hmult_relin_rescale")
        he.hrot_many(self.rot, self.hoist_in, outs=self.hoist_out)
        mark("hrot_hoisted")
        n_jobs = len(self.single_groups) or self.n_single
        if serial:
            for i in range(n_jobs):
                self._single_one(i)
        else:
            self._spread(n_jobs, self._single_one)
        mark("hrot_single")

    def _step_overlapped(self):
        """The same operations as step(), all of them independent, dealt to the side streams without joins
        between the four kinds: the NTT pairs and the hoisted rotations first, then the HMult batches and the
        single rotations round-robin."""
        he, torch = self.he, self.torch
        jobs = [lambda: (he.ntt(self.ntt_limbs, self.ntt_mods), he.intt(self.ntt_limbs, self.ntt_mods)),
                lambda: he.hrot_many(self.rot, self.hoist_in, outs=self.hoist_out)]
        for lo in range(0, self.n_hmult, self.hm_chunk):
            hi = min(lo + self.hm_chunk, self.n_hmult)
            jobs.append(lambda lo=lo, hi=hi: he.hmult_relin_rescale_batch(self.relin, self.hm_a[lo:hi], self.hm_b[lo:hi],
                                                                          out=self.rs_out[lo:hi]))
        jobs += [lambda i=i: self._single_one(i) for i in range(len(self.single_groups) or self.n_single)]
        self._spread(len(jobs), lambda k: jobs[k]())

    def _single_one(self, i):
        if self.single_groups:
            keys, lv, cts, outs = self.single_groups[i]
            if lv is None:
                self.he.hrot_batch_keys(keys, cts, out=outs)
            else:
                self.he.hrot_batch_levels(keys, lv, cts, out=outs)
        else:
            self.he.hrot(self.rot[self.single_keys[i]], self.single_in[i], out=self.single_out[i])

    def _spread(self, count, fn):
        """Runs fn(0..count-1); with side streams the independent calls are dealt round-robin to them and
        joined back into the current stream."""
        torch = self.torch
        if not self.streams:
            for i in range(count):
                fn(i)
            return
        cur = torch.cuda.current_stream(self.he.device)
        for st in self.streams:
            st.wait_stream(cur)
        for i in range(count):
            with torch.cuda.stream(self.streams[i % len(self.streams)]):
                fn(i)
        for st in self.streams:
            cur.wait_stream(st)


def train_step_ms(he, w: "Workload") -> float:
    """One full encrypted gradient-descent step (4 classes x 32 ciphertexts of 32 samples = 1024 samples x 768
    features, degree-7 polynomial logistic function, levels 24 -> 16) on uniform residues: 768 HMult and
    2580 HRot.  Returns milliseconds for the step."""
    import torch

    from paper_2210_02574_amd import classifier as cl

    step = cl.EncryptedTrainStep(he, wl.N16.L, 2.0**50, 1.0, 1024)
    plan = step.plan
    rot = {}
    for k, r in enumerate(w.offsets):  # +2^0 .. +2^14 cover the block-sum and cross-block shifts
        rot[r] = w.rot[k]
    for k, r in enumerate(cl.TRAIN_FILL_SHIFTS):
        rot[r] = w._key(2000 + k, he.galois_element(r))
    X = [w._uniform_ct(plan.level) for _ in range(32)]
    W = [w._uniform_ct(plan.level) for _ in range(4)]
    Y = [[w._uniform_ct(plan.label_level) for _ in range(32)] for _ in range(4)]
    mask = w._uniform(list(range(plan.level - 1)))
    Xb = torch.stack(X)
    Yb = [torch.stack(y) for y in Y]
    del X, Y
    step.run_batched(w.relin, rot, mask, Xb, W[:1], Yb[:1])  # warm-up: one class
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    step.run_batched(w.relin, rot, mask, Xb, W, Yb)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3


def inference_ms(he, w: "Workload", reps: int = 10) -> float:
    """Latency of one encrypted inference (32 samples x 768 features -> 4 logits each at level 24: 3 hoisted and
    8 sequential rotations, 4 plaintext products, one rescale) on uniform residues.  Milliseconds per call."""
    import torch

    from paper_2210_02574_amd import classifier as cl

    inf = cl.EncryptedInference(he, wl.N16.L)
    keys = {}
    for k, r in enumerate(w.offsets):  # 1, 2, 4 .. 512 are among the power-of-two keys
        keys[r] = w.rot[k]
    keys[3] = w._key(3000, he.galois_element(3))
    ct = w._uniform_ct(wl.N16.L)
    pts = [w._uniform(list(range(wl.N16.L))) for _ in range(4)]
    inf.run(ct, pts, keys)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        inf.run(ct, pts, keys)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / reps


def bootstrap_ms(he, w: "Workload", ns: int = 1024, reps: int = 3) -> float:
    """One Bootstrap of a sparsely packed ciphertext (ns slots, level 1 -> 8 of 24; ModRaise, trace, matrix products
    as two sparse factors each with hoisted baby steps, degree-9 Taylor polynomial and 7 squarings on a batch of
    two) on uniform residues with the real plaintext diagonals.  Milliseconds per call, plaintexts prepared
    beforehand."""
    import torch

    from paper_2210_02574_amd.bootstrap import Bootstrapper

    bs = Bootstrapper(he, ns, r=7, groups=2)
    rot = {sh: w._key(4000 + i, he.galois_element(sh)) for i, sh in enumerate(bs.rotation_shifts())}
    keys = {"relin": w.relin, "conj": w._key(3999, 2 * wl.N16.N - 1), "rot": rot}
    bs.prepare()
    ct1 = w._uniform_ct(1)
    bs.run(ct1, keys)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        bs.run(ct1, keys)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / reps


def train_iteration_ms(reps: int = 2) -> float:
    """One iteration of the paper's training recipe (Section 3.1) for one class at full size, on uniform residues
    with the real plaintexts: N = 2^16, 28 primes (dnum = 7), 1024 samples x 768 features in 32 ciphertexts of
    1024-slot blocks; gradient step with the degree-7 polynomial (batched over the 32 ciphertexts), Nesterov
    look-ahead, division, Bootstrap of the 1024-slot weight vector (level 1 -> 12).  Milliseconds per iteration."""
    import torch

    import paper_2210_02574_amd as pkg
    from paper_2210_02574_amd.training import EncryptedTrainer

    p = wl.T16
    he = pkg.HE.from_params(p, device=0)
    tr = EncryptedTrainer(he, 1024, 1.0, 0.5, 1024, 2.0**50)
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(16)

    def uniform_batch(count, level):
        out = torch.empty((count, 2, level, p.N), dtype=torch.int64, device=dev)
        for i in range(level):
            out[:, :, i].random_(0, p.q[i], generator=gen)
        return out

    def key(seed, g):
        return he.evk_from_host(wl.uniform_evk(seed, p), g)

    keys = {"relin": key(5000, 1), "conj": key(5001, 2 * p.N - 1),
            "rot": {sh: key(5002 + i, he.galois_element(sh)) for i, sh in enumerate(tr.rotation_shifts())}}
    tr.boot.prepare(tr.gain)
    tp = tr.step.plan
    X = uniform_batch(32, tr.level)
    Y = [uniform_batch(32, tp.label_level)]
    W = [uniform_batch(1, tr.level)[0]]
    V = [uniform_batch(1, tp.out_level)[0]]
    mask = tr.step.encode_mask()
    W, V = tr.iterate(keys, mask, X, W, V, Y)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        W, V = tr.iterate(keys, mask, X, W, V, Y)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / reps


def probe(args) -> None:
    """Short fixed targets for hardware counters and traces (`rocprofv3 ... -- python3 bench.py --probe ...`).
    `hrot-batch [SET LEVEL COUNT]`: three batched rotations with one key on uniform residues (default: eight
    level-24 ciphertexts of the N = 2^16 set; `P17 30 4` is the paper's ring degree).  `copy`: five plain
    device-to-device copies of 256 MiB, the launch of known size (262144 KiB read and written) against which the
    profiler's HBM traffic counters are scaled."""
    import torch

    import paper_2210_02574_amd as pkg

    if args[0] == "copy":
        a = torch.empty(32 * 1024 * 1024, dtype=torch.int64, device="cuda").random_()
        b = torch.empty_like(a)
        for _ in range(5):
            b.copy_(a)
        torch.cuda.synchronize()
        print("copied 5 x 256 MiB")
        return
    if args[0] != "hrot-batch":
        print("bench.py: unknown probe %r (hrot-batch, copy)" % args[0], file=sys.stderr)
        sys.exit(2)
    p = getattr(wl, args[1]) if len(args) > 1 else wl.N16
    he = pkg.HE.from_params(p, device=0)
    level = int(args[2]) if len(args) > 2 else p.L
    count = int(args[3]) if len(args) > 3 else 8
    key = he.evk_from_host(wl.uniform_evk(1, p), he.galois_element(1))
    cts = torch.stack([he.to_device(wl.uniform_ct(30 + i, p, level)) for i in range(count)])
    out = he.empty_batch(count, level)
    for _ in range(3):
        he.hrot_batch(key, cts, out=out)
    torch.cuda.synchronize()
    print("3 x hrot_batch of %d ciphertexts at level %d" % (count, level))


def paper_scale_rates(reps: int = 5) -> dict:
    """The paper's ring degree (N = 2^17, 30 primes below 2^50, 4 special primes, dnum = 8) on uniform residues:
    rotations in batches of four and Mult + rescale in batches of four at level 30."""
    import torch

    import paper_2210_02574_amd as pkg

    p = wl.P17
    he = pkg.HE.from_params(p, device=0)
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(17)

    def uniform_batch(count):
        out = torch.empty((count, 2, p.L, p.N), dtype=torch.int64, device=dev)
        for i in range(p.L):
            out[:, :, i].random_(0, p.q[i], generator=gen)
        return out

    rot = he.evk_from_host(wl.uniform_evk(1701, p), he.galois_element(1))
    relin = he.evk_from_host(wl.uniform_evk(1702, p), 1)
    a, b = uniform_batch(4), uniform_batch(4)
    out = he.empty_batch(4, p.L)
    out2 = he.empty_batch(4, p.L - 1)
    res = {}
    for name, fn in (("hrot_per_s", lambda: he.hrot_batch(rot, a, out=out)),
                     ("hmult_relin_rescale_per_s", lambda: he.hmult_relin_rescale_batch(relin, a, b, out=out2))):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        res[name] = 4 * reps / (time.perf_counter() - t0)
    res["workload"] = "N=2^17, L=30, K=4, dnum=8, level 30, batches of 4"
    return res


def cpu_baseline(sample_hrot: int = 32, sample_hmult: int = 16, sample_ntt: int = 112):
    """The oracle, as it stands, on a bounded sample of the step: NTT/iNTT pairs, HMult+relin+rescale
    and HRot at level 24; reported in key switches per second."""
    import oracle

    p = wl.N16
    o = oracle.Oracle(p.logN, p.q, p.p, p.dnum)
    cores = int(o.lib.orc_num_threads())
    mods = [b % (p.L + p.K) for b in range(sample_ntt)]
    limbs = wl.uniform_limbs(11, p, mods)
    evk = wl.uniform_evk(12, p)
    a, b = wl.uniform_ct(13, p, p.L), wl.uniform_ct(14, p, p.L)
    t0 = time.perf_counter()
    f = o.ntt(limbs, mods)
    o.intt(f, mods)
    t_ntt = time.perf_counter() - t0
    t0 = time.perf_counter()
    for _ in range(sample_hmult):
        o.rescale(o.hmult_relin(a, b, evk))
    t_hm = time.perf_counter() - t0
    t0 = time.perf_counter()
    for _ in range(sample_hrot):
        o.hrot(a, evk, 1)
    t_rot = time.perf_counter() - t0
    ks = sample_hmult + sample_hrot
    return {
        "value": ks / (t_hm + t_rot),
        "unit": "key-switches/s",
        "cores": cores,
        "kind": "oracle",
        "sample": f"{sample_hmult} HMult+relin+rescale and {sample_hrot} HRot at level 24 (N=2^16, dnum=6), "
                  f"plus {sample_ntt} limb NTT+iNTT pairs",
        "seconds": round(t_ntt + t_hm + t_rot, 3),
        "ntt_pairs_per_s": sample_ntt / t_ntt,
        "hmult_relin_rescale_per_s": sample_hmult / t_hm,
        "hrot_per_s": sample_hrot / t_rot,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-train-step", action="store_true")
    ap.add_argument("--hmult-batch", type=int, default=16, help="ciphertext pairs per batched HMult call")
    ap.add_argument("--single-mode", choices=["levels", "per-level", "each"], default="levels",
                    help="how the 128 single rotations are issued: 32 per mixed-level call, one call per level, or one call each")
    ap.add_argument("--single-chunk", type=int, default=32, help="single rotations per call in --single-mode levels")
    ap.add_argument("--streams", type=int, default=1, help="HIP streams for the independent operations of a step")
    ap.add_argument("--probe", nargs="+", metavar="ARG",
                    help="run a short profiling target instead of the benchmark: hrot-batch [SET LEVEL COUNT] | copy")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2210_02574_amd.build import ensure_built

    ensure_built()
    import paper_2210_02574_amd as pkg

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    if args.probe:
        probe(args.probe)
        return
    he = pkg.HE.from_params(wl.N16, device=0)
    w = Workload(he, n_streams=args.streams, hm_chunk=args.hmult_batch, single_mode=args.single_mode,
                 single_chunk=args.single_chunk)
    for _ in range(args.warmup):
        w.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        w.step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    # the four kinds of operation one after the other (same steps again, outside the timed region): segment
    # times from events on the launch stream
    marks = []
    for _ in range(args.steps):
        w.step(marks)
    torch.cuda.synchronize()
    seg = {}
    for (n0, e0), (n1, e1) in zip(marks[:-1], marks[1:]):
        if n1 != "start":
            seg[n1] = seg.get(n1, 0.0) + e0.elapsed_time(e1)
    p = wl.N16
    limb_bytes = p.N * 8
    seg_s = {k: v / 1e3 / args.steps for k, v in seg.items()}
    detail = {
        "ntt_pairs_per_s": w.n_ntt / seg_s["ntt_pairs"],
        # read + write of every limb, forward and inverse: the definition's bytes
        "ntt_effective_GBps": w.n_ntt * 2 * 2 * limb_bytes / seg_s["ntt_pairs"] / 1e9,
        "hmult_relin_rescale_per_s": w.n_hmult / seg_s["hmult_relin_rescale"],
        "hrot_hoisted_per_s": len(w.offsets) / seg_s["hrot_hoisted"],
        "hrot_single_mixed_levels_per_s": w.n_single / seg_s["hrot_single"],
        "segment_ms": {k: round(v * 1e3, 3) for k, v in seg_s.items()},
    }

    # the same steps again with per-kernel HIP events inside the library: once as timed (operations overlapping
    # on the streams, so a kernel's duration includes its share of the contention) and once with every
    # operation on one stream, where each kernel has the GPU to itself: the roofline is taken from the latter
    he.profile_start()
    for _ in range(args.steps):
        w.step()
    stats_conc = he.profile_stop()
    he.profile_start()
    for _ in range(args.steps):
        w.step(serial=True)
    stats = he.profile_stop()
    counters, counter_source = load_counter_summary()

    def kernel_entry(k, v, conc=None):
        launches, total_ms, nbytes = v
        avg_s = total_ms / 1e3 / launches if launches else 0.0
        gbps = nbytes / (total_ms / 1e3) / 1e9 if total_ms else None
        # counter figures of the profiled run, carried over in proportion to the algorithmic bytes per launch
        traffic, lane_insts = None, None
        if k in counters and counters[k][2] > 0 and launches:
            scale = nbytes / launches / counters[k][2]
            traffic, lane_insts = counters[k][0] * scale, counters[k][1] * scale
        e = {
            "launches": launches, "total_ms": round(total_ms, 3), "avg_launch_us": round(avg_s * 1e6, 2),
            "GBps": round(gbps, 1) if gbps else None,
            "frac": round(gbps / HBM_PEAK_GBS, 4) if gbps else None,              # algorithmic bytes / own time / 8 TB/s
            "traffic": traffic,                                                     # counter bytes per launch
            "frac_counter": round(traffic / avg_s / 1e9 / HBM_PEAK_GBS, 4) if traffic and avg_s else None,
            "alu_frac": round(lane_insts / avg_s / 1e12 / ALU_PEAK_TLIPS, 4) if lane_insts and avg_s else None,
        }
        fc, fa = e["frac_counter"] or e["frac"] or 0.0, e["alu_frac"] or 0.0
        e["bound"] = "alu" if fa > fc else "hbm"
        return e

    kernels = {k: kernel_entry(k, v) for k, v in sorted(stats.items(), key=lambda kv: -kv[1][1])}
    name = next(iter(kernels))
    dom = kernels[name]
    launches, total_ms, nbytes = stats[name]
    conc = stats_conc.get(name)
    roofline = {
        "kernel": name,
        "pass": "serial (each kernel alone on the GPU; same operations as the timed steps)",
        "frac_while_overlapped": (conc[2] / (conc[1] / 1e3) / 1e9 / HBM_PEAK_GBS) if conc and conc[1] else None,
        "bound": "hbm",
        "achieved": dom["GBps"],
        "peak": HBM_PEAK_GBS,
        "unit": "GB/s",
        "frac": dom["frac"],                  # algorithmic bytes (each operand once per launch) / kernel time / peak
        "frac_counter": dom["frac_counter"],  # counter-measured HBM traffic / kernel time / peak
        "traffic": dom["traffic"],
        "traffic_source": counter_source,
        "launches": launches,
        "avg_launch_us": total_ms * 1e3 / launches,
        "bytes_per_launch": nbytes / launches,
    }
    # the kernel with the most time among those bound by instruction issue rather than by memory
    alu_name = next((k for k, e in kernels.items() if e["bound"] == "alu"), None)
    roofline_alu = None
    if alu_name:
        e = kernels[alu_name]
        roofline_alu = {
            "kernel": alu_name, "bound": "alu", "achieved": round(e["alu_frac"] * ALU_PEAK_TLIPS, 2), "peak": round(ALU_PEAK_TLIPS, 2),
            "unit": "T lane-instructions/s", "frac": e["alu_frac"], "frac_hbm": e["frac"], "frac_hbm_counter": e["frac_counter"],
            "source": counter_source,
        }

    out = {
        "metric": "HRot key-switches/sec at N=2^16 L=24 (whole step: NTT pairs + HMult+relin+rescale + hoisted and "
                  "single HRot)",
        "value": w.key_switches * args.steps / dt,
        "unit": "key-switches/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u64",
        "data": "synthetic",
        "config": {
            "workload": "N=2^16, L=24, K=4, dnum=6: 256 limb NTT+iNTT pairs, 64 HMult+relin+rescale at level 24, "
                        "15 hoisted HRot (2^0..2^14) at level 24, 128 single HRot at levels 8..24",
            "key_switches_per_step": w.key_switches,
            "streams": args.streams,
            "hmult_batch": args.hmult_batch,
            "single_hrot_calls": {"levels": "%d rotations of mixed levels per call, sorted by key" % args.single_chunk,
                                  "per-level": "one call per level (one key per ciphertext)",
                                  "each": "one call each"}[args.single_mode],
        },
        "detail": detail,
        "roofline": roofline,
        "roofline_alu": roofline_alu,
        "kernels": kernels,
    }
    if not args.no_train_step:
        out["detail"]["inference_ms"] = inference_ms(he, w)
        out["detail"]["inference_workload"] = "32 samples x 768 features, 4 classes, 11 HRot, level 24"
        out["detail"]["train_step_ms"] = train_step_ms(he, w)
        out["detail"]["paper_scale"] = paper_scale_rates()
        out["detail"]["bootstrap_ms"] = bootstrap_ms(he, w)
        out["detail"]["bootstrap_workload"] = ("1024 packed slots (the block of the paper's weight vectors), level 1 -> 8, "
                                               "5 + 4 x 14 HRot, 2 conjugations, 24 HMult")
        out["detail"]["train_step_workload"] = "1024 samples x 768 features, 4 classes, 768 HMult + 2580 HRot"
        del w
        torch.cuda.empty_cache()
        out["detail"]["train_iteration_ms"] = train_iteration_ms()
        out["detail"]["train_iteration_workload"] = ("per class: N=2^16, L=28, dnum=7, 1024 samples x 768 features in 32 "
                                                     "ciphertexts, gradient step + Nesterov update + Bootstrap of 1024 slots")
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
