"""CPU checks of bench.py's contract and of the synthetic input recipe (no GPU)."""
import importlib.util
import os
import subprocess
import sys

import numpy as np

from paper_2401_16677_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench_module():
    spec = importlib.util.spec_from_file_location("bench_under_test", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in (r.stderr + r.stdout)
    assert not r.stdout.strip().startswith("{")          # no result line for a run it refuses


def test_algorithmic_bytes_closed_forms():
    b = _bench_module()
    w = wl.WORKLOADS["gpt3_outproj"]
    M, N, K, P = w.M, w.N, w.K, w.tp
    direct = 2 * M * K + 2 * K * N + 4 * M * N + 4 * M * N      # A, B, incoming in, sums out
    assert b.algorithmic_bytes(w, True) == direct == 452984832
    fwd_elems = M * N * (P - 1) // P
    assert b.algorithmic_bytes(w, False) == direct + 8 * fwd_elems     # copy: read + write again
    assert b.algorithmic_bytes(w, True, True) == direct - 2 * fwd_elems   # 2-byte forward slots
    assert abs(b.PEAK_BF16_TFLOPS - 256 * 2.4e9 * 4096 / 1e12) < 0.1 and b.PEAK_HBM_GBS == 8000.0
    # the transcribed-traffic table only names workloads that exist, and says where it is from
    assert all(k[0] in wl.WORKLOADS and k[1] in ("direct", "copy") for k in b.PROFILED_TRAFFIC_BYTES)
    assert "profiles/" in b.PROFILED_TRAFFIC_SOURCE and "transcribed" in b.PROFILED_TRAFFIC_SOURCE
    # the headline is the largest configuration; every configuration gets a record
    assert b.HEADLINE == "wide_fc2" and set(b.CONFIGS) == {
        "tiny_outproj", "gpt3_outproj", "gpt3_fc2", "wide_fc2", "hightp_outproj"}
    assert max(b.CONFIGS, key=lambda n: wl.WORKLOADS[n].flop) == b.HEADLINE


def test_named_configurations_have_the_stated_shapes():
    want = {"tiny_outproj": (256, 1024, 256, 4, 0), "gpt3_outproj": (4096, 12288, 1536, 8, 3),
            "gpt3_fc2": (4096, 12288, 6144, 8, 5), "wide_fc2": (2048, 20480, 10240, 8, 7),
            "hightp_outproj": (8192, 18432, 1152, 16, 9)}
    for name, shape in want.items():
        w = wl.WORKLOADS[name]
        assert (w.M, w.N, w.K, w.tp, w.rank) == shape and w.N % w.tp == 0
        assert w.flop == 2.0 * w.M * w.N * w.K
    assert (wl.WORKLOADS["wide_fc2"].tile_m, wl.WORKLOADS["wide_fc2"].tile_n) == (128, 256)
    assert wl.WORKLOADS["gpt3_fc2"].a_dist == "halfnormal"
    for w in wl.PAPER_SHAPES.values():       # H/TP or 4H/TP slices of the hidden size N
        assert w.K * w.tp in (w.N, 4 * w.N) and w.N % w.tp == 0


def test_input_recipe_distributions_and_seeding():
    w = wl.make_shape("r", 192, 512, 1024, 4, 1, 128, 128)
    a, b, inc = wl.make_inputs(w, seed=3)
    a2, b2, inc2 = wl.make_inputs(w, seed=3)
    assert np.array_equal(a, a2) and np.array_equal(b, b2) and np.array_equal(inc, inc2)
    assert not np.array_equal(a, wl.make_inputs(w, seed=4)[0])
    af, bf = wl.bf16_bits_to_f32(a), wl.bf16_bits_to_f32(b)
    sigma = w.K ** -0.25                                   # variance 1/sqrt(K)
    assert abs(af.std() / sigma - 1) < 0.02 and abs(bf.std() / sigma - 1) < 0.02
    assert abs(af.mean()) < 0.01 * sigma
    assert abs(inc.std() / np.sqrt(w.tp - 1) - 1) < 0.02     # sqrt(P-1) x std(C), std(C) = 1
    c = af.astype(np.float64) @ bf.astype(np.float64).T
    assert abs(c.std() - 1) < 0.03
    # ReLU-like A: half exact zeros, the rest positive; C's variance halves
    wh = wl.make_shape("h", 192, 512, 1024, 4, 1, 128, 128, a_dist="halfnormal")
    ah, bh, inch = wl.make_inputs(wh, seed=3)
    ahf = wl.bf16_bits_to_f32(ah)
    assert abs((ahf == 0).mean() - 0.5) < 0.01 and ahf.min() == 0.0
    ch = ahf.astype(np.float64) @ wl.bf16_bits_to_f32(bh).astype(np.float64).T
    assert abs(ch.std() / np.sqrt(0.5) - 1) < 0.05 and abs(wl.std_c(wh) ** 2 - 0.5) < 1e-12


def test_integer_inputs_are_exact_in_fp32():
    a, b, inc = wl.make_integer_inputs(64, 96, 200, seed=1)
    af, bf = wl.bf16_bits_to_f32(a), wl.bf16_bits_to_f32(b)
    assert np.all(af == np.round(af)) and np.all(np.abs(af) <= 2) and np.all(inc == np.round(inc))
    exact = af.astype(np.int64) @ bf.astype(np.int64).T + inc.astype(np.int64)
    assert np.abs(exact).max() < 2 ** 24
