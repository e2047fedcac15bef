"""Host-side checks of the benchmark driver and the seeded input generators (no GPU)."""
import os
import subprocess
import sys

import numpy as np

from paper_2402_12399_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_inputs_are_seeded_and_shaped():
    w = wl.C1
    a, b = wl.make_inputs(w), wl.make_inputs(w)
    for name in ("x", "w_router", "w1", "w2"):
        assert np.array_equal(a[name], b[name]), name
    assert a["x"].shape == (w.T, w.d_model) and a["w_router"].shape == (w.E, w.d_model)
    assert a["w1"].shape == (w.E, w.d_ff, w.d_model) and a["w2"].shape == (w.E, w.d_model, w.d_ff)
    assert a["w_router"].dtype == np.float32
    other = wl.make_inputs(wl.Workload("c1b", w.T, w.d_model, w.d_ff, w.E, w.G, w.k, w.capacity_factor, w.dtype, w.act,
                                       w.bias, w.seed + 1))
    assert not np.array_equal(a["x"], other["x"])


def test_bf16_storage_round_trip():
    rng = np.random.default_rng(0)
    v = rng.standard_normal(4096).astype(np.float32)
    bits = wl._store(v, "bf16")
    back = wl.values_f32(bits, "bf16")
    assert bits.dtype == np.uint16 and back.dtype == np.float32
    # round to nearest even: at most half a bf16 ulp (2^-9 relative), and idempotent
    assert np.all(np.abs(back - v) <= np.abs(v) * 2.0 ** -8)
    assert np.array_equal(wl._store(back, "bf16"), bits)


def test_synthetic_logits_recipe():
    a = wl.synthetic_logits(5000, 16, seed=3, bias_std=1.0, ties=True)
    b = wl.synthetic_logits(5000, 16, seed=3, bias_std=1.0, ties=True)
    assert a.dtype == np.float32 and a.shape == (5000, 16) and np.array_equal(a, b)
    assert np.isfinite(a).all()
    # the tie recipe really produces equal scores inside rows and across tokens
    assert (np.sort(a, axis=1)[:, 1:] == np.sort(a, axis=1)[:, :-1]).any()
    assert len(np.unique(a)) < a.size // 2
    c = wl.synthetic_logits(5000, 16, seed=3, bias_std=1.0, ties=False)
    assert len(np.unique(c)) > 0.9 * c.size


def test_zipf_bias_skews_expert_popularity():
    w = wl.Workload("z", 4096, 64, 64, 16, 4, 1, 1.0, "f32", "gelu", "zipf:1.5", 9)
    inp = wl.make_inputs(w)
    top1 = np.argmax(inp["x"].astype(np.float64) @ inp["w_router"].astype(np.float64).T + inp["bias"], axis=1)
    counts = np.bincount(top1, minlength=w.E)
    assert counts.max() > 4 * max(1, np.sort(counts)[w.E // 2])  # a few experts take most tokens
