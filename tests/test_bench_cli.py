"""bench.py on the command line, without a GPU: the cases it must refuse."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""  # no JSON line for a run that did not happen


def test_counter_summary_is_read_for_every_kernel_of_the_step():
    """bench.py takes measured traffic and instruction counts per launch from the committed profile summary: every
    kernel of the benchmark step must be there with positive figures, and the summary must say where it comes from."""
    import bench

    table, source = bench.load_counter_summary()
    assert source and "Measured at commit" in source
    for k in ("k_inner_blocks", "k_ntt_fwd_cols_modup", "k_ntt_fwd_blocks_fin", "k_ntt_fwd_cols_moddown",
              "k_ntt_fwd_cols_moddown_rescale", "k_ntt_inv_cols", "k_ntt_inv_blocks", "k_ntt_fwd_blocks", "k_tensor",
              "k_ntt_fwd_cols"):
        traffic, instr, alg = table[k]
        assert traffic > 0 and instr > 0 and alg > 0
        # measured traffic within a factor of two of the bytes the step has to move
        assert 0.5 < traffic / alg < 2.0, (k, traffic, alg)
