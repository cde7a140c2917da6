"""Pins for the CPU oracle: each check ties an oracle function to something other than itself --
a value the paper prints, a hand-worked example, a closed form, a brute-force loop on tiny
inputs, or a library routine that is the textbook form of the same thing.  CPU only."""
import math
import os

import numpy as np
import pytest

from oracle import moe_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            out[key] = [int(v) for v in vals]
    return out


# ------------------------------------------------------------------------------------ formats
def test_bf16_widening_exact_values():
    # 0x3F80 = 1.0, 0xC000 = -2.0, 0x3FC0 = 1.5, 0x0000 = 0, 0x7F80 = +inf (bfloat16 format)
    bits = np.array([0x3F80, 0xC000, 0x3FC0, 0x0000, 0x7F80], dtype=np.uint16)
    assert O.to_f64(bits).tolist() == [1.0, -2.0, 1.5, 0.0, float("inf")]


def test_round_to_bf16_ties_to_even():
    # bf16 has 8 significand bits: spacing at 1.0 is 2^-7.  1 + 2^-8 is a tie -> even (1.0);
    # 1 + 3*2^-8 is a tie -> even (1 + 2^-6); just above a tie rounds up.
    assert O.round_to_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert O.round_to_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    assert O.round_to_bf16(np.array([1.0 + 2.0 ** -8 + 2.0 ** -20]))[0] == 1.0 + 2.0 ** -7
    assert O.round_to_bf16(np.array([-3.0]))[0] == -3.0


# ------------------------------------------------------------------------------------ routing
def _route_brute(x, Wg, b, k, renorm):
    """Pure-Python loops: logits by explicit sums, full sort of (-logit, index) pairs, softmax
    with math.exp."""
    T, d = x.shape
    E = Wg.shape[1]
    idx, w = [], []
    for t in range(T):
        l = [math.fsum(float(x[t, i]) * float(Wg[i, e]) for i in range(d)) + float(b[e]) for e in range(E)]
        order = sorted(range(E), key=lambda e: (-l[e], e))
        m = max(l)
        ex = [math.exp(v - m) for v in l]
        s = math.fsum(ex)
        p = [v / s for v in ex]
        sel = order[:k]
        ws = [p[e] for e in sel]
        if renorm:
            tot = math.fsum(ws)
            ws = [v / tot for v in ws]
        idx.append(sel)
        w.append(ws)
    return np.array(idx), np.array(w)


@pytest.mark.parametrize("k,renorm", [(1, 0), (2, 1), (3, 0), (5, 1)])
def test_route_matches_brute_force(k, renorm):
    r = np.random.default_rng(7)
    T, d, E = 48, 12, 5
    x = r.standard_normal((T, d)).astype(np.float32)
    Wg = r.standard_normal((d, E)).astype(np.float32)
    b = r.standard_normal(E).astype(np.float32)
    idx, w, _ = O.route_topk(x, Wg, b, k, renorm)
    bi, bw = _route_brute(x, Wg, b, k, renorm)
    assert np.array_equal(idx, bi)
    assert np.allclose(w, bw, rtol=0, atol=1e-7)


def test_route_one_hot_tokens_read_rows_of_Wg():
    # x = e_i picks row i of W_g, so the logits are known by construction (catches a transposed
    # operand: W_g is d x E with d != E and distinct rows/columns).
    d, E = 6, 4
    Wg = np.arange(d * E, dtype=np.float32).reshape(d, E)
    Wg[:, [0, 3]] = Wg[:, [3, 0]]          # per row: col 0 largest, then 2, 1, 3
    x = np.eye(d, dtype=np.float32)
    idx, w, l = O.route_topk(x, Wg, None, 2, 1)
    assert np.array_equal(l, Wg.astype(np.float64))
    assert np.array_equal(idx, np.tile([0, 2], (d, 1)))
    # renormalised pair = softmax over the two selected logits: gap is 1 -> 1/(1+e^-1)
    assert np.allclose(w[:, 0], 1.0 / (1.0 + math.exp(-1.0)), atol=1e-7)
    assert np.allclose(w.sum(axis=1), 1.0, atol=1e-6)


def test_route_bias_is_added_per_expert_and_dominant_bias_wins():
    r = np.random.default_rng(3)
    x = r.standard_normal((64, 16)).astype(np.float32)
    Wg = (r.standard_normal((16, 8)) / 4).astype(np.float32)
    b = np.zeros(8, dtype=np.float32)
    b[5] = 30.0
    idx, w, l = O.route_topk(x, Wg, b, 2, 0)
    assert np.all(idx[:, 0] == 5)
    assert np.all(w[:, 0] > 0.999999)
    assert np.allclose(l[:, 5] - (x.astype(np.float64) @ Wg.astype(np.float64))[:, 5], 30.0)


def test_route_ties_go_to_lower_index_and_k_equals_E_is_full_softmax():
    x = np.ones((3, 4), dtype=np.float32)
    Wg = np.zeros((4, 6), dtype=np.float32)          # all logits equal
    idx, w, _ = O.route_topk(x, Wg, None, 4, 0)
    assert np.array_equal(idx, np.tile(np.arange(4), (3, 1)))
    assert np.allclose(w, 1.0 / 6.0)
    r = np.random.default_rng(11)
    x = r.standard_normal((20, 9)).astype(np.float32)
    Wg = r.standard_normal((9, 7)).astype(np.float32)
    idx, w, l = O.route_topk(x, Wg, None, 7, 0)
    assert np.allclose(w.sum(axis=1), 1.0, atol=1e-6)            # k = E: whole softmax
    assert all(sorted(row) == list(range(7)) for row in idx.tolist())
    assert np.all(np.diff(np.take_along_axis(l, idx.astype(np.int64), 1), axis=1) <= 0)   # descending
    # renormalised weights are the softmax over the k selected logits alone (closed form)
    idx3, w3, l3 = O.route_topk(x, Wg, None, 3, 1)
    sel = np.take_along_axis(l3, idx3.astype(np.int64), 1)
    ref = np.exp(sel - sel.max(1, keepdims=True))
    ref /= ref.sum(1, keepdims=True)
    assert np.allclose(w3, ref, atol=1e-7)


def test_route_uniform_router_loads_within_multinomial_bounds():
    r = np.random.default_rng(5)
    T, d, E = 8192, 64, 16
    x = r.standard_normal((T, d)).astype(np.float32)
    Wg = (r.standard_normal((d, E)) / 8).astype(np.float32)
    idx, _, _ = O.route_topk(x, Wg, None, 1, 0)
    counts = np.bincount(idx[:, 0], minlength=E)
    # loads are not exactly multinomial(1/E) (column norms differ), so allow a wide band
    assert counts.sum() == T and counts.min() > 0.5 * T / E and counts.max() < 1.6 * T / E


def test_decision_gaps():
    l = np.array([[3.0, 1.0, 2.5, -1.0], [0.0, 0.0, 5.0, 4.0]])
    assert np.allclose(O.decision_gaps(l, 1), [0.5, 1.0])
    assert np.allclose(O.decision_gaps(l, 2), [0.5, 1.0])
    assert np.allclose(O.decision_gaps(l, 3), [0.5, 0.0])


# ------------------------------------------------------------------------------------ permute
@pytest.mark.parametrize("T,k,E", [(1, 1, 1), (37, 2, 5), (200, 4, 9), (64, 1, 130)])
def test_permute_is_the_stable_counting_sort(T, k, E):
    r = np.random.default_rng(T + k + E)
    idx = r.integers(0, E, size=(T, k)).astype(np.int32)
    if E >= 3:
        idx[idx == 1] = 2                               # an empty expert
    p = O.permute(idx, E)
    flat = idx.reshape(-1)
    A = T * k
    assert np.array_equal(p["counts"], np.bincount(flat, minlength=E))
    assert np.array_equal(p["offsets"], np.concatenate([[0], np.cumsum(np.bincount(flat, minlength=E))]))
    assert np.array_equal(p["perm"], np.argsort(flat, kind="stable"))
    assert p["counts"].sum() == A and p["offsets"][-1] == A
    assert sorted(p["perm"].tolist()) == list(range(A))                  # bijection
    assert np.array_equal(p["inv_perm"][p["perm"]], np.arange(A))
    assert np.all(np.diff(flat[p["perm"]]) >= 0)                         # grouped by expert
    for e in range(E):                                                    # ascending inside an expert
        seg = p["perm"][p["offsets"][e]:p["offsets"][e + 1]]
        assert np.all(np.diff(seg) > 0)


def test_permute_hand_example_and_empty():
    # assignments (t,j): experts 2,0 | 1,2 | 0,2  -> flat [2,0,1,2,0,2]
    p = O.permute(np.array([[2, 0], [1, 2], [0, 2]]), 3)
    assert p["counts"].tolist() == [2, 1, 3]
    assert p["offsets"].tolist() == [0, 2, 3, 6]
    assert p["perm"].tolist() == [1, 4, 2, 0, 3, 5]
    assert p["inv_perm"].tolist() == [3, 0, 2, 4, 1, 5]
    x = np.arange(6, dtype=np.float32).reshape(3, 2)
    assert O.gather_rows(x, p["perm"], 2).tolist() == [[0, 1], [4, 5], [2, 3], [0, 1], [2, 3], [4, 5]]
    z = O.permute(np.zeros((0, 2), dtype=np.int32), 4)
    assert z["counts"].tolist() == [0, 0, 0, 0] and z["perm"].size == 0
    with pytest.raises(ValueError):
        O.permute(np.array([[4]]), 4)


# ------------------------------------------------------------------------------------ expert FFN
def test_ffn_hand_worked_relu():
    # x=[1,2]; W1=[[1,-1],[0,2]] -> xW1=[1,3]; W1b=[[1,-1],[-2,0]] -> [-3,-1] -> relu 0
    x = np.array([[1.0, 2.0]])
    W2 = np.array([[1.0, 0.0, 2.0], [2.0, 1.0, 0.0]])          # F=2 x d_out=3
    y = O.expert_ffn(x, {"W1": np.array([[1.0, -1.0], [0.0, 2.0]]), "W2": W2}, "relu")
    assert y.tolist() == [[7.0, 3.0, 2.0]]
    y0 = O.expert_ffn(x, {"W1": np.array([[1.0, -1.0], [-2.0, 0.0]]), "W2": W2}, "relu")
    assert y0.tolist() == [[0.0, 0.0, 0.0]]


def test_ffn_hand_worked_swiglu():
    # silu(ln 3) = ln3 * 3/4 ; silu(0) = 0 ; silu(-ln 3) = -ln3 / 4
    ln3 = math.log(3.0)
    x = np.array([[1.0, 1.0]])
    Wg = np.array([[ln3, 0.0, -ln3], [0.0, 0.0, 0.0]])
    Wu = np.array([[2.0, 5.0, 4.0], [0.0, 1.0, 0.0]])          # x Wu = [2, 6, 4]
    Wd = np.array([[1.0, 0.0], [1.0, 1.0], [0.0, 2.0]])
    y = O.expert_ffn(x, {"Wg": Wg, "Wu": Wu, "Wd": Wd}, "swiglu")
    h = [ln3 * 0.75 * 2.0, 0.0, -ln3 * 0.25 * 4.0]
    assert np.allclose(y, [[h[0] + h[1], h[1] + 2 * h[2]]], atol=1e-15)


def test_ffn_brute_force_triple_loop():
    r = np.random.default_rng(21)
    n, d, F = 5, 4, 6
    x = r.standard_normal((n, d))
    W1, W2 = r.standard_normal((d, F)), r.standard_normal((F, d))
    Wu = r.standard_normal((d, F))
    for act in ("relu", "swiglu"):
        ref = np.zeros((n, d))
        for i in range(n):
            h = []
            for f in range(F):
                a = math.fsum(x[i, c] * W1[c, f] for c in range(d))
                if act == "relu":
                    h.append(max(a, 0.0))
                else:
                    u = math.fsum(x[i, c] * Wu[c, f] for c in range(d))
                    h.append(a / (1.0 + math.exp(-a)) * u)
            for c in range(d):
                ref[i, c] = math.fsum(h[f] * W2[f, c] for f in range(F))
        w = {"W1": W1, "W2": W2} if act == "relu" else {"Wg": W1, "Wu": Wu, "Wd": W2}
        assert np.allclose(O.expert_ffn(x, w, act), ref, atol=1e-13)


def test_ffn_relu_power_of_two_homogeneity_and_rounded_hidden_modes():
    r = np.random.default_rng(2)
    x = r.standard_normal((7, 8))
    w = {"W1": r.standard_normal((8, 16)), "W2": r.standard_normal((16, 8))}
    assert np.array_equal(O.expert_ffn(2 * x, w, "relu"), 2 * O.expert_ffn(x, w, "relu"))
    a, b = O.expert_ffn(x, w, "relu"), O.expert_ffn(x, w, "relu", h_round="bf16")
    c = O.expert_ffn(x, w, "relu", h_round="f16")
    rms = np.sqrt(np.mean(a ** 2))
    assert 0 < np.abs(a - b).max() < 2e-2 * rms          # differs, by about bf16 rounding of h
    assert 0 < np.abs(a - c).max() < 2e-2 / 8 * rms      # half keeps three more bits
    # hidden activations that half holds exactly leave the result untouched
    xi = r.integers(-4, 5, (7, 8)).astype(np.float64)
    wi = {"W1": r.integers(-3, 4, (8, 16)).astype(np.float64), "W2": w["W2"]}
    assert np.array_equal(O.expert_ffn(xi, wi, "relu"), O.expert_ffn(xi, wi, "relu", h_round="f16"))


# ------------------------------------------------------------------------------------ layer
def _scaling_experts(E, d, c):
    """Expert e multiplies non-negative inputs by c[e]: W1 = I, W2 = c[e] I (ReLU)."""
    W1 = np.tile(np.eye(d), (E, 1, 1))
    W2 = np.stack([c[e] * np.eye(d) for e in range(E)])
    return {"W1": W1, "W2": W2}


def test_layer_closed_form_with_scaling_experts():
    r = np.random.default_rng(9)
    T, d, E, k = 30, 4, 5, 2
    x = np.abs(r.standard_normal((T, d)))
    c = np.array([1.0, 2.0, 4.0, 8.0, 16.0])
    idx = np.stack([r.permutation(E)[:k] for _ in range(T)])
    gw = r.random((T, k))
    y = O.moe_layer(x, idx, gw, _scaling_experts(E, d, c), "relu")
    ref = (gw * c[idx]).sum(axis=1, keepdims=True) * x
    assert np.allclose(y, ref, atol=1e-13)
    # subset of tokens = the same rows
    sub = [3, 29, 0, 7]
    assert np.allclose(O.moe_layer(x, idx, gw, _scaling_experts(E, d, c), "relu", tokens=sub), ref[sub], atol=1e-13)


def test_layer_identical_experts_equals_dense_ffn_and_shared_adds():
    r = np.random.default_rng(10)
    T, d, F, E, k = 40, 6, 10, 4, 2
    x = r.standard_normal((T, d)).astype(np.float32)
    one = {"Wg": r.standard_normal((d, F)), "Wu": r.standard_normal((d, F)), "Wd": r.standard_normal((F, d))}
    w = {n: np.tile(a, (E, 1, 1)) for n, a in one.items()}
    Wg = r.standard_normal((d, E)).astype(np.float32)
    idx, gw, _ = O.route_topk(x, Wg, None, k, 1)
    dense = O.expert_ffn(x, one, "swiglu")
    y = O.moe_layer(x, idx, gw, w, "swiglu")
    assert np.allclose(y, dense, atol=1e-6 * np.abs(dense).max())       # weights sum to 1 (fp32)
    sh = {"Wg": r.standard_normal((d, 3)), "Wu": r.standard_normal((d, 3)), "Wd": r.standard_normal((3, d))}
    y2 = O.moe_layer(x, idx, gw, w, "swiglu", shared=sh)
    assert np.allclose(y2 - y, O.expert_ffn(x, sh, "swiglu"), atol=1e-12)


def test_layer_uniform_routing_equals_per_token_dense_loop():
    r = np.random.default_rng(12)
    T, d, F, E = 33, 5, 7, 4
    x = r.standard_normal((T, d))
    w = {"W1": r.standard_normal((E, d, F)), "W2": r.standard_normal((E, F, d))}
    idx = (np.arange(T) % E).reshape(T, 1)               # round-robin: every expert the same load
    gw = np.ones((T, 1))
    y = O.moe_layer(x, idx, gw, w, "relu")
    for t in range(T):
        e = t % E
        ref = np.maximum(x[t] @ w["W1"][e], 0) @ w["W2"][e]
        assert np.allclose(y[t], ref, atol=1e-13)


def test_direct_and_permuted_forms_agree():
    r = np.random.default_rng(13)
    T, d, F, E, k = 50, 6, 8, 7, 3
    x = r.standard_normal((T, d)).astype(np.float32)
    w = {"Wg": r.standard_normal((E, d, F)), "Wu": r.standard_normal((E, d, F)), "Wd": r.standard_normal((E, F, d))}
    idx, gw, _ = O.route_topk(x, r.standard_normal((d, E)).astype(np.float32), None, k, 1)
    p = O.permute(idx, E)
    xp = O.gather_rows(x, p["perm"], k)
    yp = O.grouped_ffn(xp, p["offsets"], w, "swiglu")
    y_perm_form = O.combine(yp, p["inv_perm"], gw)
    y_direct = O.moe_layer(x, idx, gw, w, "swiglu")
    assert np.abs(y_perm_form - y_direct).max() < 1e-12 * max(1.0, np.abs(y_direct).max())


def test_combine_identity_and_weights():
    r = np.random.default_rng(14)
    T, d, E = 25, 3, 4
    x = r.standard_normal((T, d)).astype(np.float32)
    idx = r.integers(0, E, size=(T, 1))
    p = O.permute(idx, E)
    xp = O.gather_rows(x, p["perm"], 1)
    assert np.array_equal(O.combine(xp, p["inv_perm"], np.ones((T, 1))), x.astype(np.float64))
    # k = 2, hand-checkable: y[t] = w0*row + w1*row
    yp = np.array([[1.0], [10.0], [100.0], [1000.0]])
    inv = np.array([2, 0, 3, 1])                 # token0 -> rows 2,0 ; token1 -> rows 3,1
    gw = np.array([[0.5, 0.25], [2.0, 1.0]])
    sh = np.array([[0.125], [0.0]])
    assert O.combine(yp, inv, gw, sh).tolist() == [[50.0 + 0.25 + 0.125], [2000.0 + 10.0]]


def test_half_hidden_diagnostic_mode_saturates():
    # hand numbers: h = relu([1] . [[70000, 3, -5]]) = [70000, 3, 0]; as half with saturation
    # [65504, 3, 0]; times a column of ones -> 65507.  2049 is not a half value (spacing 2 there):
    # it rounds to even, 2048.
    w = {"W1": np.array([[70000.0, 3.0, -5.0]]), "W2": np.ones((3, 1))}
    assert O.expert_ffn(np.array([[1.0]]), w, "relu")[0, 0] == 70003.0
    assert O.expert_ffn(np.array([[1.0]]), w, "relu", h_round="f16")[0, 0] == 65507.0
    w = {"W1": np.array([[2049.0, -70000.0]]), "W2": np.array([[1.0], [1.0]])}
    assert O.expert_ffn(np.array([[1.0]]), w, "relu", h_round="f16")[0, 0] == 2048.0
    wg = {"Wg": np.array([[50.0]]), "Wu": np.array([[-90000.0]]), "Wd": np.array([[1.0]])}     # silu(50) = 50 to 1e-20
    assert O.expert_ffn(np.array([[1.0]]), wg, "swiglu", h_round="f16")[0, 0] == -65504.0


# ------------------------------------------------------------------------------------ Alg. 2
def test_rebalance_paper_example():
    g = _golden("alg2_example.txt")
    m_all = np.array([g["m_all_row0"], g["m_all_row1"], g["m_all_row2"]])
    S0 = O.initial_assign(m_all, g["home"], 3)
    assert S0.sum(axis=(0, 1)).tolist() == g["naive_loads"]
    S = O.rebalance(S0, g["q"][0])
    assert S.sum(axis=(0, 1)).tolist() == g["balanced_loads"]
    assert np.array_equal(S.sum(axis=2), m_all)                  # nothing lost, nothing re-routed to another expert
    assert S[:, 2, 0].sum() == g["expert2_tokens_on_gpu0"][0]
    assert S[:, 2, 1].sum() == g["expert2_tokens_on_gpu1"][0]
    assert S[:, 0, 1:].sum() == 0 and S[:, 1, 0].sum() == 0 and S[:, 1, 2].sum() == 0


def test_rebalance_threshold_and_degenerate_cases():
    g = _golden("alg2_example.txt")
    m_all = np.array([g["m_all_row0"], g["m_all_row1"], g["m_all_row2"]])
    S0 = O.initial_assign(m_all, g["home"], 3)
    # the largest (source, expert) block going to GPU 2 holds 4 tokens: q = 5 forbids any move
    assert np.array_equal(O.rebalance(S0, 5), S0)
    # q = 4: first block (4 tokens) may move, but GPU 0 has room for 3 < q -> no feasible transfer
    assert np.array_equal(O.rebalance(S0, 4), S0)
    # q = 3: the first move (3 tokens) happens, the second (1 token) does not
    assert O.rebalance(S0, 3).sum(axis=(0, 1)).tolist() == [5, 4, 6]
    # one GPU: nothing to do
    S1 = O.initial_assign(np.array([[3, 4]]), [0, 0], 1)
    assert np.array_equal(O.rebalance(S1, 1), S1)
    with pytest.raises(ValueError):
        O.rebalance(S0, 0)


def test_rebalance_invariants_random():
    r = np.random.default_rng(15)
    for trial in range(60):
        G = int(r.integers(2, 9))
        E = int(r.integers(G, 40))
        q = int(r.integers(1, 20))
        m_all = (r.zipf(1.6, size=(G, E)) % 200).astype(np.int64)
        home = [e * G // E for e in range(E)]                 # contiguous blocks of experts per GPU
        S0 = O.initial_assign(m_all, home, G)
        S = O.rebalance(S0, q)
        assert np.array_equal(S.sum(axis=2), m_all) and S.min() >= 0
        t0, t1 = S0.sum(axis=(0, 1)), S.sum(axis=(0, 1))
        t_avg = m_all.sum() // G
        assert t1.max() <= t0.max()
        assert np.all(t1[t0 <= t_avg] <= t_avg)               # a receiver is never pushed above the average
        # Receivers never pass the average, so they never become donors: an entry of S that grew
        # only ever grew, by whole moves, and every move carries at least q tokens
        # (t_s = min(t_move, room) with t_move >= q and room >= q).
        moves = []
        assert np.array_equal(O.rebalance(S0, q, moves=moves), S)
        assert all(n >= q for *_, n in moves)
        gains = (S - S0)[(S - S0) > 0]
        assert gains.size == 0 or gains.min() >= q
        replay = S0.copy()
        for s_, e_, donor, recv, n in moves:
            assert home[e_] == donor or replay[s_, e_, donor] > 0
            replay[s_, e_, donor] -= n
            replay[s_, e_, recv] += n
        assert np.array_equal(replay, S)
        # stopping: balanced, or the next candidate is too small, or the emptiest GPU has no room for q
        if t1.max() > t_avg:
            with pytest.raises(O._NoMove) as why:
                O.pick_move(S, [int(v) for v in t1], int(t_avg), q)
            assert why.value.reason in ("small", "no_room")


def _schedule(G_src, E, G, entries):
    S = np.zeros((G_src, E, G), dtype=np.int64)
    for (s_, e_, g_), n in entries.items():
        S[s_, e_, g_] = n
    return S


def test_rebalance_source_is_chosen_by_its_sum_over_experts():
    """Hand-worked, Alg. 2: the source GPU is the one that sends the most tokens to the fullest
    GPU summed over all experts, NOT the one holding the largest single block.
    3 sources, 4 experts, 3 GPUs; experts 2 and 3 both live on GPU 2.  q = 1.
        tokens per (source, expert):  source 0: 1 1 4 6 | source 1: 1 1 7 0 | source 2: 0 1 1 1
    Loads 2, 3, 19; total 24, average 8.
    Move 1: fullest GPU 2.  Sources send it 10, 7, 2 -> source 0 (its largest block is 6, while
            source 1 holds a block of 7).  Expert 3 (6 tokens).  Emptiest GPU 0 has room 8-2 = 6
            -> all 6 go.  Loads 8, 3, 13.
    Move 2: fullest GPU 2.  Sources send it 4, 7, 2 -> source 1, expert 2 (7 tokens).  Emptiest
            GPU 1 has room 5 -> 5 go.  Loads 8, 8, 8: balanced."""
    m_all = np.array([[1, 1, 4, 6], [1, 1, 7, 0], [0, 1, 1, 1]])
    home = [0, 1, 2, 2]
    S0 = O.initial_assign(m_all, home, 3)
    assert S0.sum(axis=(0, 1)).tolist() == [2, 3, 19]
    expected = _schedule(3, 4, 3, {
        (0, 0, 0): 1, (0, 1, 1): 1, (0, 2, 2): 4, (0, 3, 0): 6,
        (1, 0, 0): 1, (1, 1, 1): 1, (1, 2, 1): 5, (1, 2, 2): 2,
        (2, 1, 1): 1, (2, 2, 2): 1, (2, 3, 2): 1})
    moves = []
    S = O.rebalance(S0, 1, moves=moves)
    assert np.array_equal(S, expected)
    assert moves == [(0, 3, 2, 0, 6), (1, 2, 2, 1, 5)]
    assert S.sum(axis=(0, 1)).tolist() == [8, 8, 8]


def test_rebalance_equal_values_go_to_the_lowest_index():
    """Hand-worked tables for the reading "among equals, the lowest index" (the paper's argmax /
    argmin say nothing about ties), one case per choice of Alg. 2."""
    # (a) two equally full GPUs: GPU 0 gives first.  One source, expert e on GPU e, counts 6 6 0,
    #     average 4.  Move 1: donor 0 (6 = 6), receiver 2 (empty), min(6, 4) = 4 of expert 0.
    #     Loads 2 6 4.  Move 2: donor 1, receiver 0 (2), room 2: 2 of expert 1.  Loads 4 4 4.
    S0 = O.initial_assign(np.array([[6, 6, 0]]), [0, 1, 2], 3)
    moves = []
    S = O.rebalance(S0, 1, moves=moves)
    assert S[0].tolist() == [[2, 0, 4], [2, 4, 0], [0, 0, 0]]
    assert moves == [(0, 0, 0, 2, 4), (0, 1, 1, 0, 2)]
    # (b) two equally empty GPUs: GPU 1 receives first.  Experts 0 (5 tokens) and 1 (4 tokens) on
    #     GPU 0, nothing elsewhere; average 3.  Move 1: expert 0's block of 5, receiver 1 (0 = 0),
    #     room 3 -> 3 tokens.  Loads 6 3 0.  Move 2: blocks left on GPU 0 are 2 and 4 -> expert 1,
    #     receiver 2, room 3 -> 3 tokens.  Loads 3 3 3.
    S0 = O.initial_assign(np.array([[5, 4]]), [0, 0], 3)
    moves = []
    S = O.rebalance(S0, 1, moves=moves)
    assert S[0].tolist() == [[2, 3, 0], [1, 0, 3]]
    assert moves == [(0, 0, 0, 1, 3), (0, 1, 0, 2, 3)]
    # (c) two equally large blocks: the lower expert moves.  Experts 0 and 1, 4 tokens each, both on
    #     GPU 0 of 2; average 4.  One move: expert 0, all 4 tokens, to GPU 1.
    S0 = O.initial_assign(np.array([[4, 4]]), [0, 0], 2)
    assert O.rebalance(S0, 1)[0].tolist() == [[0, 4], [4, 0]]
    # (d) two sources sending equally much: the lower source.  Both send 3 tokens of expert 0 to
    #     GPU 0 of 2; average 3.  One move: source 0's block, 3 tokens, to GPU 1.
    S0 = O.initial_assign(np.array([[3], [3]]), [0], 2)
    S = O.rebalance(S0, 1)
    assert S[0].tolist() == [[0, 3]] and S[1].tolist() == [[3, 0]]


def test_rebalance_floor_average_and_stop_reasons():
    # total 14 on 3 GPUs: the average is floor(14/3) = 4; counts 9 3 2 with expert e on GPU e.
    # Move 1: 9 -> receiver 2 (2), room 2: loads 7 3 4.  Move 2: receiver 1 (3), room 1: 6 4 4.
    # GPU 0 is still above 4 but the emptiest GPU (1, with 4) has no room: stop.
    S0 = O.initial_assign(np.array([[9, 3, 2]]), [0, 1, 2], 3)
    moves = []
    S = O.rebalance(S0, 1, moves=moves)
    assert S[0].tolist() == [[6, 1, 2], [0, 3, 0], [0, 0, 2]]
    assert moves == [(0, 0, 0, 2, 2), (0, 0, 0, 1, 1)]
    for load, S_, q, reason in (([4, 4, 4], S, 1, "balanced"), ([6, 4, 4], S, 1, "no_room"),
                                ([9, 3, 2], S0, 10, "small"), ([9, 3, 2], S0, 3, "no_room")):
        with pytest.raises(O._NoMove) as why:
            O.pick_move(S_, load, 4, q)
        assert why.value.reason == reason, (load, q)
    # the amount is the block when the block is the smaller one: loads 3 0 with average 1 and a
    # block of 1 -> only that block moves even though there is room for one... and exactly one
    S0 = O.initial_assign(np.array([[1, 1, 1]]), [0, 0, 0], 2)          # average floor(3/2) = 1
    assert O.pick_move(S0, [3, 0], 1, 1) == (0, 0, 0, 1, 1)


def test_even_split_and_round_robin_hand_tables():
    """Section 5.3.2.  Even Split: a tokens of an expert over four GPUs -> a/4 each; the remainder
    (which the paper's example leaves open) one token each to the lowest-numbered GPUs.
    Round-robin: experts dealt to the GPUs in turn, no rebalancing."""
    S = O.schedule_even_split([7, 3, 0, 8, 1], 4)
    assert S.tolist() == [[2, 2, 2, 1], [1, 1, 1, 0], [0, 0, 0, 0], [2, 2, 2, 2], [1, 0, 0, 0]]
    assert O.round_robin_home(7, 3) == [0, 1, 2, 0, 1, 2, 0]
    S = O.schedule_round_robin([5, 0, 2, 9, 1, 4, 3], 3)
    assert S.tolist() == [[5, 0, 0], [0, 0, 0], [0, 0, 2], [9, 0, 0], [0, 1, 0], [0, 0, 4], [3, 0, 0]]
    assert S.sum(axis=0).tolist() == [17, 1, 6]
    # contiguous placement of the same counts, for contrast (Fig. 2: neighbours share a GPU)
    assert O.schedule_static([5, 0, 2, 9, 1, 4, 3], 3).sum(axis=0).tolist() == [7, 10, 7]


# ------------------------------------------------------------------------------------ threshold q
def test_threshold_q_formulas_and_paper_sizes():
    c = _golden("paper_constants.txt")
    assert O.expert_bytes(768, 3072, 4) == c["switch_expert_bytes"][0]
    assert 3 * 2048 * 1408 * 4 == c["qwen_expert_bytes"][0]      # three matrices (gated FFN)
    assert 8 * 128 * 4 == c["metadata_bytes"][0]
    # Eq. 3 against an explicit count: a dot product of length n costs n mults + (n-1) adds
    q, m, p = 5, 7, 11
    assert O.expert_flops(q, m, p) == q * p * (m + m - 1) + q * m * (p + p - 1)
    # Eq. 4 is Eq. 1 with the small terms dropped: within 0.1 % at the Switch expert's shape
    phi, beta = 15.7e12, 16e9
    q4 = O.token_threshold_q(phi, 4, beta)
    qx = O.token_threshold_q_exact(phi, 4, beta, 768, 3072)
    assert abs(q4 - qx) / qx < 1e-3
    # at q = qx the two sides of Eq. 1 are equal
    assert math.isclose(O.expert_flops(1, 768, 3072) * qx / phi, O.expert_bytes(768, 3072, 4) / beta, rel_tol=1e-12)
    assert math.isclose(q4, phi * 4 / (2 * beta))


# ------------------------------------------------------------------------------------ one-GPU schedule
def test_schedule_without_weights_is_alg2():
    # by_cost=False: weights are row counts and one row is the granule, so the loop must be
    # Alg. 2 itself.  Start both from the same placement by making it unambiguous: one expert
    # per bin and strictly falling counts (heaviest-first placement = contiguous homes).
    r = np.random.default_rng(31)
    for G in (2, 3, 5, 8):
        counts = np.sort(r.integers(1, 500, size=G))[::-1] * 2 + np.arange(G, 0, -1)
        for q in (1, 7, 64):
            a = O.schedule_balanced(counts, G, q, tile_m=1, by_cost=False)
            b = O.schedule_harmoeny(counts, G, q)
            assert np.array_equal(a, b), (G, q)
    # the paper's example again, through the one-source interface: loads 2,4,9 -> 5,5,5
    assert O.schedule_harmoeny([2, 4, 9], 3, 1).sum(axis=0).tolist() == [5, 5, 5]


def test_schedule_policies_invariants():
    r = np.random.default_rng(32)
    for trial in range(40):
        E = int(r.integers(1, 70))
        G = int(r.integers(1, 9))
        q = int(r.integers(1, 400))
        tile_m = int(r.choice([16, 64, 128]))
        counts = (r.zipf(1.3, size=E) * 13 % 3000).astype(np.int64)
        counts[r.random(E) < 0.2] = 0
        offsets = np.concatenate([[0], np.cumsum(counts)])
        for S in (O.schedule_balanced(counts, G, q, tile_m), O.schedule_harmoeny(counts, G, q),
                  O.schedule_static(counts, G), O.schedule_even_split(counts, G)):
            assert S.shape == (E, G) and S.min() >= 0
            assert np.array_equal(S.sum(axis=1), counts)                       # every row scheduled once
            tiles, bin_start = O.tiles_from_schedule(S, offsets, tile_m)
            O.validate_tiles(tiles, bin_start, counts, offsets, tile_m, G)
            assert len(tiles) <= -(-int(counts.sum()) // tile_m) + E * G
        Sb = O.schedule_balanced(counts, G, q, tile_m)
        tiles_of = lambda n: -(-int(n) // tile_m)
        per_bin = np.array([[tiles_of(n) for n in row] for row in Sb]).sum(axis=0)
        assert per_bin.max() - per_bin.min() <= 1                              # equal tile counts
        assert per_bin.sum() <= sum(tiles_of(c) for c in counts)               # splitting in whole tiles adds none
        for e in range(E):                                                      # at most one ragged part per expert
            parts = Sb[e][Sb[e] > 0]
            assert (parts % tile_m != 0).sum() <= 1
        Se = O.schedule_even_split(counts, G)
        assert np.all(Se.max(axis=1) - Se.min(axis=1) <= 1)


def test_block_order_spreads_long_blocks_among_short_ones():
    """Hand-worked listings (tile_m = 128: a block of more than 128 rows is long)."""
    # L = 2 long (keys 1/2, 3/2), M = 4 short (keys 1/4, 3/4, 5/4, 7/4)
    assert O.block_order({0: 300, 1: 200, 2: 50, 3: 40, 4: 30, 5: 20}, 128) == [2, 0, 3, 4, 1, 5]
    # equal keys: the long block first
    assert O.block_order({0: 5, 1: 200}, 128) == [1, 0]
    assert O.block_order({7: 129, 3: 500, 1: 128, 2: 128}, 128) == [3, 1, 7, 2]
    # long blocks outnumber the short ones, or one kind is missing: falling rows, then expert id
    assert O.block_order({0: 300, 1: 300, 2: 10}, 128) == [0, 1, 2]
    assert O.block_order({4: 20, 2: 20, 9: 128}, 128) == [9, 2, 4]
    assert O.block_order({4: 200, 2: 2000}, 128) == [2, 4]
    assert O.block_order({}, 128) == []
    # any input: a permutation that keeps each kind in its own order
    r = np.random.default_rng(12)
    for _ in range(200):
        tile_m = int(r.choice([16, 128, 256]))
        rows = {int(e): int(n) for e, n in zip(r.permutation(40)[:r.integers(1, 30)], r.integers(1, 4 * tile_m, 30))}
        order = O.block_order(rows, tile_m)
        assert sorted(order) == sorted(rows)
        for kind in (True, False):
            sub = [e for e in order if (rows[e] > tile_m) == kind]
            assert sub == sorted(sub, key=lambda e: (-rows[e], e))


def test_schedule_balanced_splits_hot_expert_and_balances():
    # one expert with half of all rows, 8 bins: its rows must be spread, tile counts equal
    counts = np.array([8192, 2600, 1500, 1100, 900, 800, 700, 592])
    q, tile_m, G = 313, 128, 8
    S = O.schedule_balanced(counts, G, q, tile_m)
    assert (S[0] > 0).sum() >= 4
    per_bin = np.array([[-(-int(n) // tile_m) for n in row] for row in S]).sum(axis=0)
    assert per_bin.max() - per_bin.min() <= 1 and per_bin.sum() == sum(-(-int(c) // tile_m) for c in counts)
    assert np.all(np.sort(S[0][S[0] > 0])[:-1] % tile_m == 0)   # moved parts are whole tiles
    # worked by hand: tiles 4, 1, 1 on 2 bins -> LPT gives (4 | 1+1), one move of floor(2/2) = 1 tile
    S = O.schedule_balanced(np.array([400, 100, 60]), 2, 1, 100)
    assert S.tolist() == [[300, 100], [0, 100], [0, 60]]
    # uniform small experts: nothing to split, experts dealt evenly
    S = O.schedule_balanced(np.full(128, 128), 8, 313, 128)
    assert np.all((S > 0).sum(axis=1) == 1) and np.all((S > 0).sum(axis=0) == 16)
    # all rows on one expert: spread over all bins in whole tiles
    S = O.schedule_balanced(np.array([4096, 0, 0, 0]), 8, 313, 128)
    assert (S[0] > 0).sum() == 8 and S[0].sum() == 4096 and np.all(S[0] == 512)
    # static placement never splits; contiguous homes
    assert O.contiguous_home(6, 3) == [0, 0, 1, 1, 2, 2]
