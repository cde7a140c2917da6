"""The seeded input generators: determinism, formats, and that the realised routing has the
skew each workload names (checked through the oracle's router, at reduced sizes).  CPU only."""
import numpy as np

import moe_workloads as W
from oracle import moe_oracle as O


def test_bf16_round_trip_and_rounding():
    a = np.array([1.0, -2.5, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 3.1415927], dtype=np.float32)
    bits = W.f32_to_bf16_bits(a)
    back = W.bf16_bits_to_f32(bits)
    assert back[0] == 1.0 and back[1] == -2.5
    assert back[2] == 1.0 and back[3] == np.float32(1.0 + 2.0 ** -6)     # ties to even
    assert abs(back[4] - a[4]) <= 2.0 ** -7 * 2
    assert np.array_equal(W.f32_to_bf16_bits(back), bits)                # idempotent
    assert np.array_equal(O.to_f64(bits), back.astype(np.float64))       # the oracle reads the same values


def test_generators_are_deterministic_and_shaped():
    wl = W.WORKLOADS["c1"]
    a, b = W.make_inputs(wl), W.make_inputs(wl)
    assert sorted(a) == ["W1", "W2", "W_g", "b", "x"]
    for n in a:
        assert np.array_equal(a[n], b[n])
    assert a["x"].shape == (256, 64) and a["x"].dtype == np.float32
    assert a["W1"].shape == (8, 64, 128) and a["W2"].shape == (8, 128, 64)
    assert np.allclose(a["b"], 1.5 * np.log(1.0 / np.arange(1, 9)))
    small = W.WORKLOADS["c3"].scaled(T=64, d=32, F=48, E=6, shared_F=16)
    s = W.make_inputs(small)
    assert s["x"].dtype == np.uint16 and s["Wg"].shape == (6, 32, 48) and s["Wd"].shape == (6, 48, 32)
    assert s["sWg"].shape == (32, 16) and s["sWd"].shape == (16, 32)
    assert abs(float(np.std(W.bf16_bits_to_f32(s["Wd"]))) - 48 ** -0.5) < 0.01
    # a different seed gives different data; one tensor can be drawn alone
    assert not np.array_equal(W.activations(small, 1), W.activations(small, 2))
    assert np.array_equal(W.expert_weights(small, 3)["Wu"], s["Wu"][3])


def test_zipf_first_choice_loads():
    wl = W.WORKLOADS["c2"].scaled(T=8192, d=256, E=32)
    inp = W.make_inputs(wl, weights=False)
    idx, _, _ = O.route_topk(inp["x"], inp["W_g"], inp["b"], 1, 0)
    counts = np.bincount(idx[:, 0], minlength=wl.E)
    target = W.zipf_shares(wl.E, wl.zipf_s, wl.seed()) * wl.T
    order = np.argsort(-target)
    assert np.argmax(counts) == order[0]
    big = target >= 256
    assert np.all(np.abs(counts[big] - target[big]) / target[big] < 0.25)
    assert counts[order[:4]].sum() > 0.4 * wl.T and counts.sum() == wl.T


def test_hot_expert_share():
    wl = W.WORKLOADS["c4"].scaled(T=4096, d=256)
    inp = W.make_inputs(wl, weights=False)
    idx, w, _ = O.route_topk(inp["x"], inp["W_g"], inp["b"], 2, 1)
    counts = np.bincount(idx.reshape(-1), minlength=wl.E)
    assert 0.44 <= counts.max() / (2 * wl.T) <= 0.50        # one expert holds almost half of all assignments
    assert np.allclose(w.sum(axis=1), 1.0, atol=1e-6)


def test_pre_routed_ids_and_alpha_skew():
    wl = W.WORKLOADS["c5"]
    ids = W.routed_ids(wl)
    assert ids.shape == (wl.T,) and ids.min() >= 0 and ids.max() < wl.E
    foreign = float(np.mean(ids >= wl.n_local))
    assert abs(foreign - 0.30) < 0.02
    c = np.sort(np.bincount(ids[ids < wl.n_local], minlength=wl.n_local))[::-1]
    assert 2.2 < c[0] / c[1] < 3.6                           # Zipf(1.5): first/second = 2^1.5
    a = W.alpha_skew_ids(20000, 128, 0.9, 10, 1)
    assert abs(float(np.mean(a < 10)) - 0.9) < 0.01
    u = W.alpha_skew_ids(20000, 16, 0.0, 1, 1)
    assert np.bincount(u, minlength=16)[0] == 0


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asked for more it says so and exits without touching a device."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
