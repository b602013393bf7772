"""CPU-only checks of bench.py's bookkeeping (no device call)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402
import workloads as WL  # noqa: E402


def test_byte_model():
    # fused quadratic step: x, y, c read and x+, y+ written; round 0 does not read y
    assert bench.chain_bytes("quad_center", 2, [1, 2, 3, 4]) == (20.0, 28.0)
    assert bench.chain_bytes("quad_center", 2, [0]) == (16.0, 24.0)
    assert bench.chain_bytes("quad_center", 1, [0, 1, 2, 3, 4]) == (19.2, 19.2)
    assert bench.chain_bytes("gossip", 2, [1]) == (16.0, 20.0)
    assert bench.chain_bytes("gossip", 1, [0]) == (12.0, 12.0)
    assert bench.minibatch_bytes(16) == (80.0, 164.0)


def test_row_pitch_is_256_byte_aligned():
    for d in (1, 10, 1000, 4096, 25_557_032):
        ld = bench._ld(d)
        assert ld >= d and ld % 64 == 0 and ld - d < 64


def test_traffic_summary_parses_and_goes_stale_with_the_launch_shape():
    import paper_2306_00256_amd as P
    from paper_2306_00256_amd import binding as Bn
    t, note = bench.measured_traffic(P, "quad31_2p", 50, 5)
    alg = 19.2 * WL.SPECS["quad31_2p"].n * WL.SPECS["quad31_2p"].d
    assert alg < t < 1.1 * alg          # measured HBM bytes sit a few per cent above the algorithmic count
    assert bench.measured_traffic(P, "lsq5_2p", 50, 5)[0] is None
    for name in ("quad30_1p", "gossip100_1p", "gossip100_2p", "logistic1023_2p"):
        assert bench.measured_traffic(P, name, 50, 5)[0] is not None, name
    # a launch shape other than the one the counters were read with: the stored bytes are refused
    P.ceca_set_option(Bn.OPT_BAND, 64)
    try:
        t, note = bench.measured_traffic(P, "quad31_2p", 50, 5)
        assert t is None and note.startswith("stale")
    finally:
        P.ceca_reset_options()
    assert bench.measured_traffic(P, "quad31_2p", 50, 5)[0] is not None


def test_cpu_sample_runs_the_oracle_on_a_block():
    units, el, iters, what = bench._cpu_sample("lsq5_2p", 1, 0.05)
    assert iters >= 1 and units == 5 * 1000 * iters and el > 0 and "agents" in what


def test_more_than_one_gpu_is_refused():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0 and "one GPU" in p.stderr
