"""GPU parity: every stage of the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.  Integer outputs (expert indices, counts, offsets, permutation, the
schedule and its tile table, packed-weight bytes, gathered rows) must match bit for bit;
floating-point outputs within max|err| <= 1e-4 * RMS (fp32) or 2e-2 * RMS (bf16)."""
import numpy as np
import pytest

import moe_workloads as W
from oracle import moe_oracle as O
from gpu_util import TOL, expert_dict, make_layer, max_err_over_rms, shared_dict, to_numpy

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch


def _note(msg):
    print("[case] " + msg, flush=True)


ROUTE_CASES = [
    ("c1", {}),
    ("c1", dict(T=1, E=2, k=2)),
    ("c1", dict(T=67, d=72, E=5, k=5)),
    ("c2", dict(T=1000, d=256, E=128)),
    ("c2", dict(T=4096, d=768, E=128)),
    ("c3", dict(T=777, d=512, E=60, shared_F=0)),
    ("c4", dict(T=512, d=1024)),
    ("c2", dict(T=300, d=128, E=200, k=3)),
    ("c2u", dict(T=513, d=64, E=16, k=2, renorm=1)),
]


@pytest.mark.parametrize("packed", [False, True])
@pytest.mark.parametrize("name,over", ROUTE_CASES)
def test_route_topk(torch_gpu, name, over, packed):
    """packed=False: moe_route_topk on W_g as given; packed=True: moe_pack_router once, then
    moe_route_topk_packed (bf16 with d % 64 == 0 only; the other cases run the plain entry point)."""
    torch = torch_gpu
    wl = W.WORKLOADS[name].scaled(**over)
    _note("route %s %s packed=%s" % (name, over, packed))
    inp = W.make_inputs(wl, weights=False)
    idx_o, w_o, l_o = O.route_topk(inp["x"], inp["W_g"], inp["b"], wl.k, wl.renorm)
    layer = make_layer(wl, inp)
    layer.load_router(inp["W_g"], inp["b"], packed=packed)
    if packed and wl.dtype == "bf16" and wl.d % 64 == 0:
        assert layer.packed_router
        ref_t = np.ascontiguousarray(np.asarray(inp["W_g"]).T)
        assert np.array_equal(to_numpy(layer.W_gt), ref_t)             # W_g^T, bit for bit
        n2 = (O.to_f64(inp["W_g"]) ** 2).sum(axis=0)
        got = to_numpy(layer.w_norm2).astype(np.float64)
        assert np.all(got >= n2) and np.all(got <= n2 * 1.004)          # an upper bound, and a tight one
    x = layer_x(layer, inp)
    logits = torch.empty((wl.T, wl.E), dtype=torch.float32, device=layer.device)
    layer.route(x, logits)
    torch.cuda.synchronize()
    assert np.array_equal(to_numpy(layer.expert_idx), idx_o)
    assert np.abs(to_numpy(layer.gate_w).astype(np.float64) - w_o).max() <= 2e-6
    assert np.abs(to_numpy(logits) - l_o).max() <= 1e-5 * max(1.0, np.abs(l_o).max())


def layer_x(layer, inp):
    from paper_2506_12417_amd.layer import to_device
    return to_device(inp["x"], layer.device)


def test_route_near_ties_take_the_exact_path(torch_gpu):
    # logits that differ only far below fp32 resolution of the accumulation, and exact ties:
    # the selection must still be the float64 one (ties to the lower index).
    torch = torch_gpu
    T, d, E, k = 128, 64, 8, 2
    r = np.random.default_rng(1)
    x = r.standard_normal((T, d)).astype(np.float32)
    Wg = r.standard_normal((d, E)).astype(np.float32) / 8
    Wg[:, 3] = Wg[:, 6]                        # experts 3 and 6 always tie exactly
    Wg[:, 5] = Wg[:, 1]
    Wg[0, 5] += np.float32(2.0 ** -20)         # expert 5 = expert 1 + x0 * 2^-20: tiny, sign follows x0
    wl = W.WORKLOADS["c1"].scaled(T=T, d=d, E=E, k=k)
    idx_o, w_o, _ = O.route_topk(x, Wg, None, k, 1)
    layer = make_layer(wl, {"W_g": Wg, "b": None})
    layer.route(torch.from_numpy(x).to(layer.device))
    torch.cuda.synchronize()
    assert np.array_equal(to_numpy(layer.expert_idx), idx_o)
    assert np.abs(to_numpy(layer.gate_w) - w_o).max() <= 2e-6


def test_route_near_ties_bf16_both_entry_points(torch_gpu):
    # the same planted ties in bf16, through the plain and the prepared-router entry points
    torch = torch_gpu
    T, d, E, k = 200, 128, 40, 3
    r = np.random.default_rng(2)
    x = W.f32_to_bf16_bits(r.standard_normal((T, d)).astype(np.float32))
    Wf = (r.standard_normal((d, E)) / 8).astype(np.float32)
    Wf[:, 7] = Wf[:, 30]                       # exact ties between experts 7 and 30
    Wf[:, 12] = Wf[:, 2]
    Wg = W.f32_to_bf16_bits(Wf)
    Wg[5, 12] ^= 1                             # one bf16 ulp in one coefficient: a gap far below the fp32 bound
    wl = W.WORKLOADS["c2"].scaled(T=T, d=d, E=E, k=k, renorm=1)
    idx_o, w_o, _ = O.route_topk(x, Wg, None, k, 1)
    from paper_2506_12417_amd.layer import to_device
    for packed in (False, True):
        layer = make_layer(wl, {})
        layer.load_router(Wg, None, packed=packed)
        assert layer.packed_router == packed
        layer.route(to_device(x, layer.device))
        torch.cuda.synchronize()
        assert np.array_equal(to_numpy(layer.expert_idx), idx_o), "packed=%s" % packed
        assert np.abs(to_numpy(layer.gate_w) - w_o).max() <= 2e-6


PERMUTE_CASES = [(1, 1, 1, 8), (256, 2, 8, 64), (1000, 1, 128, 32), (5000, 4, 60, 16), (3, 2, 256, 8),
                 (4097, 1, 7, 128), (16384, 1, 128, 768), (35000, 2, 200, 8)]   # the last: more than 64 blocks


@pytest.mark.parametrize("T,k,E,d", PERMUTE_CASES)
def test_permute(torch_gpu, T, k, E, d):
    torch = torch_gpu
    _note("permute T=%d k=%d E=%d d=%d" % (T, k, E, d))
    r = np.random.default_rng(T * 7 + k)
    p = 1.0 / np.arange(1, E + 1) ** 1.2
    idx = r.choice(E, size=(T, k), p=p / p.sum()).astype(np.int32)
    x = W.f32_to_bf16_bits(r.standard_normal((T, d)).astype(np.float32))
    ref = O.permute(idx, E)
    wl = W.WORKLOADS["c2"].scaled(T=T, k=k, E=E, d=d, F=64)
    layer = make_layer(wl, {})
    layer.expert_idx.copy_(torch.from_numpy(idx))
    from paper_2506_12417_amd.layer import to_device
    layer.perm.fill_(-1)
    layer.inv_perm.fill_(-1)
    layer.permute(to_device(x, layer.device))
    torch.cuda.synchronize()
    for n in ("counts", "offsets", "perm", "inv_perm"):
        assert np.array_equal(to_numpy(getattr(layer, n)), ref[n]), n
    assert np.array_equal(to_numpy(layer.x_perm), O.gather_rows(x, ref["perm"], k))


@pytest.mark.parametrize("T,k,E", [(1, 1, 1), (256, 2, 8), (1000, 1, 128), (5000, 4, 60), (3, 2, 256), (4097, 1, 7),
                                   (16384, 1, 128), (16384, 2, 200), (8192, 4, 60)])
def test_permute_plan_in_one_launch(torch_gpu, T, k, E):
    """moe_permute_plan: the sort and the schedule from one launch must be the oracle's counting sort
    and -- bit for bit -- the plan that moe_plan_tiles makes from its counts (all five policies)."""
    torch = torch_gpu
    from paper_2506_12417_amd import binding as B
    dev = torch.device("cuda:0")
    _note("permute_plan T=%d k=%d E=%d" % (T, k, E))
    r = np.random.default_rng(T * 11 + k)
    p = 1.0 / np.arange(1, E + 1) ** 1.1
    idx = r.choice(E, size=(T, k), p=p / p.sum()).astype(np.int32)
    ref = O.permute(idx, E)
    A, G, q, tile_m = T * k, 8, 50, 128
    cap = B.moe_plan_capacity(A, E, tile_m, G)
    idx_d = torch.from_numpy(idx).to(dev)
    for policy in range(5):
        out = {n: torch.full((m,), -3, dtype=torch.int32, device=dev) for n, m in (("counts", E), ("offsets", E + 1), ("perm", A), ("inv_perm", A))}
        tiles = torch.full((cap, 4), -1, dtype=torch.int32, device=dev)
        hdr = torch.full((B.MOE_PLAN_HDR_INTS,), -1, dtype=torch.int32, device=dev)
        sched = torch.full((E, G), -1, dtype=torch.int32, device=dev)
        B.moe_permute_plan(idx_d, T, E, k, out["counts"], out["offsets"], out["perm"], out["inv_perm"], tile_m, G, q, policy,
                           tiles, cap, hdr, sched)
        torch.cuda.synchronize()
        for n in out:
            assert np.array_equal(to_numpy(out[n]), ref[n]), (n, policy)
        tiles2 = torch.full((cap, 4), -1, dtype=torch.int32, device=dev)
        hdr2 = torch.full((B.MOE_PLAN_HDR_INTS,), -1, dtype=torch.int32, device=dev)
        sched2 = torch.full((E, G), -1, dtype=torch.int32, device=dev)
        B.moe_plan_tiles(out["counts"], out["offsets"], E, A, tile_m, G, q, policy, tiles2, cap, hdr2, sched2)
        torch.cuda.synchronize()
        assert torch.equal(tiles, tiles2) and torch.equal(hdr, hdr2) and torch.equal(sched, sched2), policy
    O.validate_tiles(to_numpy(tiles)[:int(to_numpy(hdr)[0])], to_numpy(hdr)[4:4 + G + 1], ref["counts"], ref["offsets"], tile_m, G)
    with pytest.raises(B.MoeError) as e:
        B.moe_permute_plan(idx_d, B.MOE_PERMUTE_PLAN_MAX + 1, E, 1, out["counts"], out["offsets"], out["perm"], out["inv_perm"],
                           tile_m, G, q, 1, tiles, 1 << 20, hdr, None)
    assert e.value.status == B.MOE_ERR_UNSUPPORTED


def test_permute_fp32_rows_and_empty_input(torch_gpu):
    torch = torch_gpu
    from paper_2506_12417_amd import binding as B
    r = np.random.default_rng(5)
    T, k, E, d = 130, 2, 8, 12
    idx = r.integers(0, E, size=(T, k)).astype(np.int32)
    x = r.standard_normal((T, d)).astype(np.float32)
    ref = O.permute(idx, E)
    wl = W.WORKLOADS["c1"].scaled(T=T, k=k, E=E, d=d, F=16)
    layer = make_layer(wl, {})
    layer.expert_idx.copy_(torch.from_numpy(idx))
    layer.permute(torch.from_numpy(x).to(layer.device))
    torch.cuda.synchronize()
    assert np.array_equal(to_numpy(layer.perm), ref["perm"])
    assert np.array_equal(to_numpy(layer.x_perm), O.gather_rows(x, ref["perm"], k))
    # T = 0: counts and offsets are written (all zero), nothing else is touched
    counts = torch.full((E,), 7, dtype=torch.int32, device=layer.device)
    offsets = torch.full((E + 1,), 7, dtype=torch.int32, device=layer.device)
    B.moe_permute(None, None, 0, d, E, k, B.MOE_F32, counts, offsets, None, None, None, layer.ws, layer.ws_bytes)
    torch.cuda.synchronize()
    assert to_numpy(counts).tolist() == [0] * E and to_numpy(offsets).tolist() == [0] * (E + 1)


def _plan_counts():
    r = np.random.default_rng(77)
    cases = []
    for name in ("c2", "c2u", "c3", "c4"):
        wl = W.WORKLOADS[name]
        inp = W.make_inputs(wl, weights=False)
        idx, _, _ = O.route_topk(inp["x"], inp["W_g"], inp["b"], wl.k, wl.renorm)
        cases.append((name, np.bincount(idx.reshape(-1), minlength=wl.E)))
    ids = W.routed_ids(W.WORKLOADS["c5"])
    cases.append(("c5", np.bincount(ids, minlength=32)))
    cases.append(("one-hot", np.array([0, 0, 4096, 0])))
    cases.append(("single", np.array([777])))
    cases.append(("empty", np.zeros(5, dtype=np.int64)))
    cases.append(("tiny", np.array([1, 2, 3, 4, 5, 6, 7, 8, 9])))
    cases.append(("rand256", (r.zipf(1.4, size=256) * 17 % 5000)))
    return cases


@pytest.mark.parametrize("policy", [0, 1, 2, 3, 4])
def test_plan_tiles_all_policies(torch_gpu, policy):
    torch = torch_gpu
    from paper_2506_12417_amd import binding as B
    dev = torch.device("cuda:0")
    for name, counts in _plan_counts():
        counts = np.asarray(counts, dtype=np.int64)
        E, A = len(counts), int(counts.sum())
        offsets = np.concatenate([[0], np.cumsum(counts)])
        for G, q, tile_m in ((8, 313, 128), (8, 1, 64), (3, 40, 16), (1, 5, 128), (16, 100, 128)):
            _note("plan %s policy=%d G=%d q=%d tile_m=%d" % (name, policy, G, q, tile_m))
            if policy == B.MOE_PLAN_BALANCED:
                S = O.schedule_balanced(counts, G, q, tile_m)
            elif policy == B.MOE_PLAN_HARMOENY:
                S = O.schedule_harmoeny(counts, G, q)
            elif policy == B.MOE_PLAN_STATIC:
                S = O.schedule_static(counts, G)
            elif policy == B.MOE_PLAN_EVEN_SPLIT:
                S = O.schedule_even_split(counts, G)
            else:
                S = O.schedule_round_robin(counts, G)
            tiles_o, bin_start_o = O.tiles_from_schedule(S, offsets, tile_m)
            cap = B.moe_plan_capacity(A, E, tile_m, G)
            assert len(tiles_o) <= cap
            c_d = torch.from_numpy(counts.astype(np.int32)).to(dev)
            o_d = torch.from_numpy(offsets.astype(np.int32)).to(dev)
            tiles = torch.full((cap, 4), -1, dtype=torch.int32, device=dev)
            hdr = torch.full((B.MOE_PLAN_HDR_INTS,), -1, dtype=torch.int32, device=dev)
            sched = torch.full((E, G), -1, dtype=torch.int32, device=dev)
            B.moe_plan_tiles(c_d, o_d, E, A, tile_m, G, q, policy, tiles, cap, hdr, sched)
            torch.cuda.synchronize()
            hdr_h, tiles_h = to_numpy(hdr), to_numpy(tiles)
            assert np.array_equal(to_numpy(sched), S)
            n = int(hdr_h[0])
            assert n == len(tiles_o) and hdr_h[1] == G
            assert np.array_equal(hdr_h[4:4 + G + 1], bin_start_o)
            assert np.array_equal(tiles_h[:n], tiles_o)
            O.validate_tiles(tiles_h[:n], hdr_h[4:4 + G + 1], counts, offsets, tile_m, G)
            if policy == B.MOE_PLAN_HARMOENY:
                _check_alg2_end_state(tiles_h[:n], counts, G, q, tile_m)


def _check_alg2_end_state(tiles, counts, G, q, tile_m):
    """What section 4.2 promises of the schedule, read off the GPU's tile table alone (one source,
    so a block is the rows of one expert on one bin).
    - The greedy loop has nothing left to do: no bin is above the floor average, or the largest
      block of the fullest bin is below q, or the emptiest bin cannot take q rows.
    - The balance that follows when it did not stop on a small block: every bin is within
      (G-1)(q-1) + (A mod G) rows of the average -- the slack q allows; with q = 1 the bins differ
      by the remainder only -- hence an expert with more rows than that bound is split over bins.
    - An expert with at least 2 tile_m rows is cut into at least two tiles."""
    E, A = len(counts), int(counts.sum())
    block = np.zeros((E, G), dtype=np.int64)
    n_tiles = np.zeros(E, dtype=np.int64)
    for e, _, rc, g in tiles:
        block[e, g] += rc
        n_tiles[e] += 1
    load = block.sum(axis=0)
    avg = A // G
    g_max, g_min = int(np.argmax(load)), int(np.argmin(load))
    balanced = load.max() <= avg
    small = block[:, g_max].max() < q
    no_room = g_min == g_max or load[g_min] + q > avg
    assert balanced or small or no_room, "a feasible move was left: loads %s" % load.tolist()
    if balanced or no_room:
        bound = avg + (G - 1) * (q - 1) + A % G
        assert load.max() <= bound
        for e in range(E):
            if counts[e] > bound:
                assert (block[e] > 0).sum() >= 2
    for e in range(E):
        if counts[e] >= 2 * tile_m:
            assert n_tiles[e] >= 2


PACK_CASES = [("f32", 1, 64, 128, False), ("bf16", 3, 768, 3072 // 4, False), ("bf16", 2, 96, 160, True),
              ("f32", 2, 40, 64, True), ("f32", 1, 50, 70, False), ("bf16", 1, 50, 96, False)]


def _bf16_row_order(mat):
    """Packed order of 16-bit weights: inside every block of 32 rows, row 16 h + j <- row 2 j + h."""
    n, rows, K = mat.shape
    blocks = mat.reshape(n, rows // 32, 16, 2, K)         # [.., j, h, :]
    return np.ascontiguousarray(np.swapaxes(blocks, 2, 3)).reshape(n, rows, K)


@pytest.mark.parametrize("dtype,n,K,N,inter", PACK_CASES)
def test_pack_weights(torch_gpu, dtype, n, K, N, inter):
    torch = torch_gpu
    from paper_2506_12417_amd import binding as B
    from paper_2506_12417_amd.layer import to_device
    dev = torch.device("cuda:0")
    r = np.random.default_rng(K + N)
    mk = (lambda: W.f32_to_bf16_bits(r.standard_normal((n, K, N)).astype(np.float32))) if dtype == "bf16" \
        else (lambda: r.standard_normal((n, K, N)).astype(np.float32))
    a = mk()
    b = mk() if inter else None
    dt = B.MOE_BF16 if dtype == "bf16" else B.MOE_F32
    rows = 2 * N if inter else N
    out = torch.zeros((n, rows, K), dtype=torch.bfloat16 if dtype == "bf16" else torch.float32, device=dev)
    B.moe_pack_weights(to_device(a, dev), None if b is None else to_device(b, dev), n, K, N, dt, out)
    torch.cuda.synchronize()
    at = np.transpose(a, (0, 2, 1))                      # output-major: row = output feature
    if inter:
        bt = np.transpose(b, (0, 2, 1))
        ref = np.empty((n, rows, K), dtype=a.dtype)
        for j in range(N // 32):
            ref[:, 64 * j:64 * j + 32] = at[:, 32 * j:32 * j + 32]
            ref[:, 64 * j + 32:64 * j + 64] = bt[:, 32 * j:32 * j + 32]
    else:
        ref = at
    if dtype == "bf16":
        ref = _bf16_row_order(ref)
    assert np.array_equal(to_numpy(out), ref)


@pytest.mark.parametrize("dtype,n,F,d", [("bf16", 2, 96, 160), ("bf16", 1, 50, 64), ("f32", 2, 40, 70)])
def test_pack_w_out(torch_gpu, dtype, n, F, d):
    """Output-major and in the row order of moe_pack_weights; bf16 values become the nearest IEEE
    half (exact in half's normal range, rounded on its subnormals, infinite beyond 65504)."""
    torch = torch_gpu
    from paper_2506_12417_amd import binding as B
    from paper_2506_12417_amd.layer import to_device
    dev = torch.device("cuda:0")
    r = np.random.default_rng(F + d)
    w32 = (r.standard_normal((n, F, d)) * np.exp2(r.integers(-30, 6, (n, F, d)))).astype(np.float32)
    w32[0, 0, :6] = [0.0, -0.0, 65504.0, 7e4, -1e30, 2.0 ** -24]
    if dtype == "bf16":
        w = W.f32_to_bf16_bits(w32)
        out = torch.zeros((n, d, F), dtype=torch.float16, device=dev)
        B.moe_pack_w_out(to_device(w, dev), n, F, d, B.MOE_BF16, out)
        torch.cuda.synchronize()
        with np.errstate(over="ignore"):
            ref = W.bf16_bits_to_f32(w).astype(np.float16)
        got = out.cpu().numpy()
        assert np.array_equal(got.view(np.uint16), _bf16_row_order(np.transpose(ref, (0, 2, 1)).view(np.uint16)))
        normal = (np.abs(ref) >= 2.0 ** -14) & np.isfinite(ref)
        assert normal.mean() > 0.3 and np.array_equal(ref[normal].astype(np.float32), W.bf16_bits_to_f32(w)[normal])
    else:
        out = torch.zeros((n, d, F), dtype=torch.float32, device=dev)
        B.moe_pack_w_out(to_device(w32, dev), n, F, d, B.MOE_F32, out)
        torch.cuda.synchronize()
        assert np.array_equal(to_numpy(out).view(np.uint32), np.transpose(w32, (0, 2, 1)).view(np.uint32))


def _stage_check(torch, wl, inp, tol_scale=1.0, flip_tol=1e-3, **layer_kw):
    """Runs route -> permute -> plan -> ffn -> combine on the GPU and checks every stage."""
    layer = make_layer(wl, inp, **layer_kw)
    x = layer_x(layer, inp)
    y = layer.forward(x)
    torch.cuda.synchronize()
    if layer.fold_combine or layer.fuse_gather:
        # forward() took a fused entry point (no x_perm and / or no y_perm); the separate calls
        # must give the same bits
        y_fused = y.clone()
        layer.permute(x)
        layer.ffn()
        if layer.shared_F:
            layer.shared_ffn(x)
        layer.combine(True)
        torch.cuda.synchronize()
        assert torch.equal(y_fused, layer.y)
    idx_o, w_o, _ = O.route_topk(inp["x"], inp["W_g"], inp["b"], wl.k, wl.renorm)
    assert np.array_equal(to_numpy(layer.expert_idx), idx_o)
    p = O.permute(idx_o, wl.E)
    for n in ("counts", "offsets", "perm", "inv_perm"):
        assert np.array_equal(to_numpy(getattr(layer, n)), p[n]), n
    xp = O.gather_rows(inp["x"], p["perm"], wl.k)
    assert np.array_equal(to_numpy(layer.x_perm), xp)
    hdr = to_numpy(layer.plan_hdr)
    O.validate_tiles(to_numpy(layer.tiles)[:hdr[0]], hdr[4:4 + layer.n_bins + 1], p["counts"], p["offsets"],
                     layer.tile_m, layer.n_bins)
    assert np.array_equal(to_numpy(layer.sched), O.schedule_harmoeny(p["counts"], layer.n_bins, layer.q_tokens))
    ew = expert_dict(wl, inp)
    yp_o = O.grouped_ffn(xp, p["offsets"], ew, wl.act)
    tol = TOL[wl.dtype] * tol_scale
    e_ffn = max_err_over_rms(to_numpy(layer.y_perm), yp_o)
    y_o = O.moe_layer(inp["x"], idx_o, w_o, ew, wl.act, shared=shared_dict(wl, inp))
    e_y = max_err_over_rms(to_numpy(y), y_o)
    print("   ffn err/rms %.3e   layer err/rms %.3e   (tol %.1e)" % (e_ffn, e_y, tol), flush=True)
    assert e_ffn <= tol and e_y <= tol
    if wl.dtype == "bf16":
        # against the oracle with half hidden activations only the rounding decisions that fall
        # differently (fp32 vs fp64 pre-activations) are left: a handful of one-ulp flips of h
        yp_m = O.grouped_ffn(xp, p["offsets"], ew, wl.act, h_round="f16")
        e_m = max_err_over_rms(to_numpy(layer.y_perm), yp_m)
        print("   ffn err/rms vs half-hidden oracle %.3e" % e_m, flush=True)
        assert e_m <= flip_tol
    return layer


LAYER_CASES = [
    ("c1", {}),
    ("c1", dict(T=77, d=24, F=40, E=3, k=1)),
    ("c1", dict(T=300, d=64, F=96, E=8, k=2, act="swiglu")),
    ("c2", dict(T=1500, d=128, F=256, E=16)),
    ("c2", dict(T=2048, d=768, F=3072, E=8)),
    ("c3", dict(T=700, d=256, F=192, E=12, shared_F=320)),
    ("c4", dict(T=900, d=512, F=1024, E=4)),
    # many tiny experts (most tiles hold a few rows, many stay empty), top-2, the on-demand hand-out at work
    ("c2", dict(T=1200, d=256, F=512, E=256, k=2)),
    # one token; a hot expert holding nearly everything (256-row tiles, fixed stride); top-1 with the folded combine
    ("c2", dict(T=1, d=64, F=512, E=4)),
    ("c4", dict(T=4200, d=256, F=512, E=2, k=1)),
    ("c2", dict(T=5000, d=192, F=1024, E=24)),
]


@pytest.mark.parametrize("name,over", LAYER_CASES)
def test_layer_stage_by_stage(torch_gpu, name, over):
    wl = W.WORKLOADS[name].scaled(**over)
    _note("layer %s %s" % (name, over))
    inp = W.make_inputs(wl)
    _stage_check(torch_gpu, wl, inp)


@pytest.mark.parametrize("act", ["relu", "swiglu"])
def test_hidden_activations_saturate_at_the_half_range(torch_gpu, act):
    """The bf16 path keeps the hidden activations in IEEE half.  A hidden activation beyond +-65504
    is stored as +-65504 (it does not become infinite): a few rows of x are scaled by 2^17, so
    their pre-activations reach about 1e5.  Those rows must come out finite and equal to the
    oracle's diagnostic mode (hidden activations rounded to half with saturation) within 1e-3 of
    the row's own RMS; every other row keeps the layer's tolerance against the exact oracle."""
    torch = torch_gpu
    from paper_2506_12417_amd.layer import to_device
    wl = W.WORKLOADS["c2"].scaled(T=700, d=256, F=512, E=6, k=1, act=act)
    _note("saturation %s" % act)
    inp = W.make_inputs(wl)
    big = np.array([3, 150, 699])
    x32 = W.bf16_bits_to_f32(inp["x"])
    x32[big] *= 2.0 ** 17                                   # exact in bf16
    x_bits = W.f32_to_bf16_bits(x32)
    assert np.array_equal(W.bf16_bits_to_f32(x_bits), x32)
    layer = make_layer(wl, inp)
    r = np.random.default_rng(3)
    idx = r.integers(0, wl.E, size=(wl.T, 1)).astype(np.int32)
    layer.expert_idx.copy_(torch.from_numpy(idx))
    layer.gate_w.fill_(1.0)
    y = to_numpy(layer.forward(to_device(x_bits, layer.device), routed=True))
    torch.cuda.synchronize()
    assert np.isfinite(y).all()
    ew, ones = expert_dict(wl, inp), np.ones((wl.T, 1))
    y_sat = O.moe_layer(x_bits, idx, ones, ew, act, tokens=big, h_round="f16")
    # the planted rows do saturate: without the clamp the same rounding gives infinities
    h_big = O.to_f64(x_bits[big[0]]) @ O.to_f64(ew["W1" if act == "relu" else "Wu"][idx[big[0], 0]])
    assert np.abs(h_big).max() > 65504
    for i, t in enumerate(big):
        row_rms = float(np.sqrt(np.mean(y_sat[i] ** 2)))
        assert np.abs(y[t] - y_sat[i]).max() <= 1e-3 * row_rms, (act, t)
    rest = np.setdiff1d(np.arange(wl.T), big)
    y_o = O.moe_layer(x_bits, idx, ones, ew, act, tokens=rest)
    assert max_err_over_rms(y[rest], y_o) <= TOL["bf16"]


STREAM_CASES = [
    # T, d, F, E, k, skew: the register-streaming kernels against the LDS-ring kernels
    (1500, 256, 512, 16, 1, "zipf"),        # few K-steps per item in the first product: fixed stride, rows fetched on the spot
    (3000, 768, 3072, 40, 1, "zipf"),       # c2's shapes: on-demand hand-out, gather and scatter folded in
    (2000, 512, 1024, 24, 2, "zipf"),       # top-2: plain second product, combine kernel
    (700, 64, 512, 5, 1, "hot"),            # one K-step per item in the first product
    (900, 192, 640, 300 // 20, 1, "uniform"),   # d and F not multiples of the item width
    (1, 128, 512, 4, 1, "uniform"),         # a single row
]


@pytest.mark.parametrize("T,d,F,E,k,skew", STREAM_CASES)
def test_streaming_kernels_give_the_bits_of_the_lds_ring_kernels(torch_gpu, T, d, F, E, k, skew):
    """moe_ffn_kernel_mode: the 128-row bf16 configuration run by the kernels that stream the
    weights into registers (mode 2) and by the LDS-ring kernels (mode 1) -- through the plain, the
    top-1 and the fused entry points -- must give identical hidden activations and outputs, and
    the layer must agree with the oracle."""
    torch = torch_gpu
    from paper_2506_12417_amd import binding as B
    wl = W.WORKLOADS["c2"].scaled(T=T, d=d, F=F, E=E, k=k, skew=skew)
    _note("stream vs ring T=%d d=%d F=%d E=%d k=%d %s" % (T, d, F, E, k, skew))
    inp = W.make_inputs(wl)
    layer = make_layer(wl, inp, tile_m=128)
    x = layer_x(layer, inp)
    before = B.moe_ffn_kernel_mode(-1)
    try:
        out = {}
        for mode in (1, 2):
            B.moe_ffn_kernel_mode(mode)
            assert B.moe_ffn_kernel_mode(-1) == mode
            layer.h.fill_(float("nan"))
            layer.y.fill_(float("nan"))
            layer.y_perm.fill_(float("nan"))
            y = layer.forward(x).clone()                     # the fused entry points where the layer uses them
            h_fused = layer.h.clone()
            layer.h.fill_(float("nan"))
            layer.y_perm.fill_(float("nan"))
            layer.permute(x)
            layer.ffn()                                       # the plain entry point
            torch.cuda.synchronize()
            out[mode] = (y, h_fused, layer.h.clone(), layer.y_perm.clone())
        for a, b_, name in zip(out[1], out[2], ("y", "H (fused call)", "H", "y_perm")):
            assert torch.equal(a.view(torch.int32) if a.dtype == torch.float32 else a.view(torch.int16),
                               b_.view(torch.int32) if b_.dtype == torch.float32 else b_.view(torch.int16)), name
    finally:
        B.moe_ffn_kernel_mode(before)
    idx_o, w_o, _ = O.route_topk(inp["x"], inp["W_g"], inp["b"], wl.k, wl.renorm)
    y_o = O.moe_layer(inp["x"], idx_o, w_o, expert_dict(wl, inp), wl.act)
    assert max_err_over_rms(to_numpy(out[2][0]), y_o) <= TOL["bf16"]


WIDE_CASES = [
    # T, d, F, E, k, act, skew, bins: the four-wavefront kernels for 256-row tiles against the LDS-ring kernels
    (3000, 256, 512, 4, 2, "swiglu", "hot", 8),       # full and ragged tiles, several column blocks
    (5000, 768, 3072, 6, 1, "relu", "zipf", 8),       # c5's shapes
    (2500, 512, 1408, 3, 2, "swiglu", "zipf", 8),     # F not a multiple of the column block: ragged last block in the first product
    (1100, 320, 704, 5, 1, "relu", "uniform", 8),     # d not a multiple of the column block: ragged last block in the second product
    (40, 256, 256, 2, 1, "swiglu", "uniform", 8),     # every tile a few rows: whole row blocks skipped
    (1, 256, 256, 1, 1, "relu", "uniform", 8),        # a single row
    (70000, 256, 512, 3, 1, "relu", "hot", 1),        # one bin: all 256 work-groups on one list, more items than work-groups
    (9000, 512, 512, 7, 2, "swiglu", "zipf", 3),      # three bins: work-groups dealt unevenly (86, 85, 85)
]


@pytest.mark.parametrize("T,d,F,E,k,act,skew,bins", WIDE_CASES)
def test_four_wavefront_kernels_give_the_bits_of_the_lds_ring_kernels(torch_gpu, T, d, F, E, k, act, skew, bins):
    """256-row tiles: the kernels of four wavefronts (the default, mode 0: the layer then folds the
    row gather into the first product and, for top-1, the combine into the second) and the LDS-ring
    kernels of eight (moe_ffn_kernel_mode 1: separate gather and combine) must give identical
    hidden activations and outputs, and the layer must agree with the oracle."""
    torch = torch_gpu
    from paper_2506_12417_amd import binding as B
    wl = W.WORKLOADS["c4"].scaled(T=T, d=d, F=F, E=E, k=k, act=act, skew=skew)
    _note("wide vs ring T=%d d=%d F=%d E=%d k=%d %s %s bins=%d" % (T, d, F, E, k, act, skew, bins))
    inp = W.make_inputs(wl)
    before = B.moe_ffn_kernel_mode(-1)
    try:
        out = {}
        for mode in (1, 0):
            B.moe_ffn_kernel_mode(mode)
            layer = make_layer(wl, inp, tile_m=256, n_bins=bins)   # (the layer asks the library which fusions it offers)
            assert layer.fuse_gather == (mode == 0 and d >= 256 and (k > 1 or F >= 512))
            x = layer_x(layer, inp)
            layer.h.fill_(float("nan"))
            layer.y.fill_(float("nan"))
            layer.y_perm.fill_(float("nan"))
            y = layer.forward(x).clone()
            torch.cuda.synchronize()
            out[mode] = (y, layer.h.clone()) + ((layer.y_perm.clone(),) if k > 1 else ())
            if mode == 0:                                     # the plain entry point with the same kernels
                layer.h.fill_(float("nan"))
                layer.y_perm.fill_(float("nan"))
                layer.permute(x)
                layer.plan()
                layer.ffn()
                layer.combine(True)
                torch.cuda.synchronize()
                out[2] = (layer.y.clone(), layer.h.clone()) + ((layer.y_perm.clone(),) if k > 1 else ())
        for other in (0, 2):
            for a, b_, name in zip(out[1], out[other], ("y", "H", "y_perm")):
                assert torch.equal(a.view(torch.int32) if a.dtype == torch.float32 else a.view(torch.int16),
                                   b_.view(torch.int32) if b_.dtype == torch.float32 else b_.view(torch.int16)), (name, other)
    finally:
        B.moe_ffn_kernel_mode(before)
    idx_o, w_o, _ = O.route_topk(inp["x"], inp["W_g"], inp["b"], wl.k, wl.renorm)
    y_o = O.moe_layer(inp["x"], idx_o, w_o, expert_dict(wl, inp), wl.act)
    assert max_err_over_rms(to_numpy(out[0][0]), y_o) <= TOL["bf16"]


@pytest.mark.parametrize("T", [300000, 400000])
def test_layer_with_very_many_tiles_in_a_bin(torch_gpu, T):
    """All rows on ONE bin in 128-row tiles.  400 000 rows: more than 3 100 tiles, beyond the per-bin
    block table the GEMM kernel keeps in LDS, so its items are taken in plain column-block-major
    order.  300 000 rows: the table is used, and the experts' runs of tiles exceed the 256 tiles a
    block may have, so they are cut."""
    wl = W.WORKLOADS["c2"].scaled(T=T, d=64, F=64, E=4)
    _note("layer, one bin, %d rows" % wl.T)
    inp = W.make_inputs(wl)
    # (F = 64: a single hidden activation whose half rounding falls the other way is a larger share
    # of an output than with the long contractions of the other cases, and the maximum is over
    # 25 million outputs: 1.2e-3 observed)
    layer = _stage_check(torch_gpu, wl, inp, flip_tol=2e-3, n_bins=1, tile_m=128)
    n_tiles = int(to_numpy(layer.plan_hdr)[0])
    assert (n_tiles > 3068) == (T == 400000) and int(to_numpy(layer.counts).max()) > 4 * 256 * 128


@pytest.mark.parametrize("name,over", [("c2", dict(T=3000, d=256, F=512, E=24)), ("c3", dict(T=700, d=256, F=192, E=12, shared_F=320)),
                                       ("c4", dict(T=4200, d=256, F=512, E=2, k=1)), ("c1", {})])
def test_forward_in_two_timed_halves_gives_the_same_output(torch_gpu, name, over):
    """forward(marks=...) runs the two grouped GEMMs through the *_phase entry points with events
    between them (what bench.py times); the output is that of the single call, bit for bit."""
    torch = torch_gpu
    wl = W.WORKLOADS[name].scaled(**over)
    inp = W.make_inputs(wl)
    layer = make_layer(wl, inp)
    x = layer_x(layer, inp)
    ref = layer.forward(x).clone()
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    layer.y.fill_(float("nan"))
    y = layer.forward(x, marks=marks)
    torch.cuda.synchronize()
    assert torch.equal(y, ref)
    assert marks[0].elapsed_time(marks[1]) > 0 and marks[1].elapsed_time(marks[2]) > 0


def test_combine_identity_and_error_paths(torch_gpu):
    torch = torch_gpu
    from paper_2506_12417_amd import binding as B
    dev = torch.device("cuda:0")
    r = np.random.default_rng(3)
    T, d, E = 500, 32, 6
    x = r.standard_normal((T, d)).astype(np.float32)
    idx = r.integers(0, E, size=(T, 1)).astype(np.int32)
    p = O.permute(idx, E)
    xp = torch.from_numpy(O.gather_rows(x, p["perm"], 1)).to(dev)
    y = torch.empty((T, d), dtype=torch.float32, device=dev)
    B.moe_unpermute_combine(xp, torch.from_numpy(p["inv_perm"]).to(dev), None, None, T, d, 1, y)
    torch.cuda.synchronize()
    assert np.array_equal(to_numpy(y), x)          # unpermute(permute(x)) = x, bit for bit
    with pytest.raises(B.MoeError) as e:
        B.moe_unpermute_combine(xp, None, None, None, T, d, 1, y)
    assert e.value.status == B.MOE_ERR_ARG
    with pytest.raises(B.MoeError) as e:
        B.moe_unpermute_combine(xp, xp, None, None, T, 30, 1, y)
    assert e.value.status == B.MOE_ERR_UNSUPPORTED


def _share(torch, wl, inp, n_local, n_slots, group=None):
    from paper_2506_12417_amd.layer import PreRoutedShare
    sh = PreRoutedShare(wl.T, wl.d, wl.F, wl.E, n_local, n_slots, act=wl.act, dtype=wl.dtype, group=group)
    for e in range(wl.E):
        sh.load_expert(e, {n: inp[n][e] for n in ("W1", "W2")})
    return sh


@pytest.mark.parametrize("n_slots,group,d,F", [(7, None, 128, 256), (3, None, 128, 256), (2, 1, 128, 256), (1, 1, 128, 256),
                                               (7, None, 256, 512), (2, None, 256, 512)])
def test_prefetch_overwrite_matches_all_resident(torch_gpu, n_slots, group, d, F):
    """The pre-routed share (rows arrive with their expert ids, some experts live in pinned host
    memory): with every expert resident, with a slot per host expert, and with fewer slots than
    host experts (slots are overwritten while later groups compute) the output must be the same
    bits, and equal to the oracle's per-row FFN within the bf16 tolerance.  Slots are poisoned
    first, so an expert used before its copy landed, or a slot overwritten too early, shows.
    (d = 256, F = 512: the groups run through moe_grouped_ffn_fused -- no gather before them, no
    combine after them; the output buffer is poisoned too, every row must be written.)"""
    torch = torch_gpu
    from paper_2506_12417_amd.layer import to_device
    wl = W.WORKLOADS["c5"].scaled(T=3000, d=d, F=F, E=12, n_local=5)
    _note("prefetch n_slots=%d group=%s d=%d F=%d" % (n_slots, group, d, F))
    inp = W.make_inputs(wl)
    ids = inp["ids"]
    x = to_device(inp["x"], "cuda:0")
    ids_d = torch.from_numpy(ids).to("cuda:0")
    ref_layer = _share(torch, wl, inp, n_local=wl.E, n_slots=1)           # everything resident
    y_res = to_numpy(ref_layer.forward(x, ids_d)).copy()
    torch.cuda.synchronize()
    ref_layer.close()
    y_o = O.moe_layer(inp["x"], ids.reshape(-1, 1), np.ones((wl.T, 1)), {n: inp[n] for n in ("W1", "W2")}, wl.act)
    assert max_err_over_rms(y_res, y_o) <= TOL["bf16"]
    sh = _share(torch, wl, inp, n_local=wl.n_local, n_slots=n_slots, group=group)
    counts = np.bincount(ids, minlength=wl.E)
    heavy_first = sorted(range(wl.n_local, wl.E), key=lambda e: (-counts[e], e))
    for order in (None, heavy_first, None):                                # three passes over the same engine
        assert sh.fused == (d >= 256)
        sh.slots.fill_(0x7f)
        sh.y_perm.fill_(float("nan"))
        sh.y.fill_(float("nan"))
        torch.cuda.synchronize()
        y = to_numpy(sh.forward(x, ids_d, fetch_order=order))
        torch.cuda.synchronize()
        assert np.array_equal(y, y_res), "order=%s" % (order,)
    assert sh.bytes_fetched == 3 * (wl.E - wl.n_local) * sh.bytes_each
    sh.close()


@pytest.mark.parametrize("n_slots,ahead,d,F", [(7, 3, 128, 256), (3, 2, 128, 256), (2, 1, 256, 512), (5, 5, 256, 512)])
def test_lookahead_prefetch_across_two_layers(torch_gpu, n_slots, ahead, d, F):
    """Two MoE layers (different weights, different rows and expert ids) share one expert cache.
    While a layer's last groups compute, the first host-resident experts of the NEXT layer are
    fetched into the slots it has released (section 1: the system looks ahead), also from the
    second layer to the first layer of the next batch.  Every layer's output must be the bits
    of the same layer with all experts resident, pass after pass; slots are poisoned first."""
    torch = torch_gpu
    from paper_2506_12417_amd.layer import ExpertCache, PreRoutedShare, to_device
    wl = W.WORKLOADS["c5"].scaled(T=2500, d=d, F=F, E=12, n_local=5)
    _note("look-ahead n_slots=%d ahead=%d d=%d F=%d" % (n_slots, ahead, d, F))
    layers_in = [W.make_inputs(wl), W.make_inputs(wl, seed=wl.seed() + 1)]
    assert not np.array_equal(layers_in[0]["ids"], layers_in[1]["ids"])
    xs = [to_device(inp["x"], "cuda:0") for inp in layers_in]
    ids = [torch.from_numpy(inp["ids"]).to("cuda:0") for inp in layers_in]
    y_res = []
    for inp, x, i in zip(layers_in, xs, ids):
        ref = _share(torch, wl, inp, n_local=wl.E, n_slots=1)
        y_res.append(to_numpy(ref.forward(x, i)).copy())
        torch.cuda.synchronize()
        ref.close()
    y_o = O.moe_layer(layers_in[1]["x"], layers_in[1]["ids"].reshape(-1, 1), np.ones((wl.T, 1)),
                      {n: layers_in[1][n] for n in ("W1", "W2")}, wl.act)
    assert max_err_over_rms(y_res[1], y_o) <= TOL["bf16"]
    cache = None
    shares = []
    for l, inp in enumerate(layers_in):
        sh = PreRoutedShare(wl.T, wl.d, wl.F, wl.E, wl.n_local, n_slots, act=wl.act, dtype=wl.dtype, cache=cache, layer_id=l)
        cache = sh.cache
        for e in range(wl.E):
            sh.load_expert(e, {n: inp[n][e] for n in ("W1", "W2")})
        shares.append(sh)
    assert isinstance(cache, ExpertCache) and shares[1].cache is shares[0].cache
    orders = []
    for inp in layers_in:
        cnt = np.bincount(inp["ids"], minlength=wl.E)
        orders.append(sorted(range(wl.n_local, wl.E), key=lambda e: (-cnt[e], e)))
    cache.slots.fill_(0x7f)
    torch.cuda.synchronize()
    passes = 3
    for p in range(passes):
        for l in (0, 1):
            nxt = 1 - l
            shares[l].y.fill_(float("nan"))
            shares[l].y_perm.fill_(float("nan"))
            # (the last layer of the last pass looks ahead as well: its fetches stay in the cache)
            y = to_numpy(shares[l].forward(xs[l], ids[l], fetch_order=orders[l], lookahead=(shares[nxt], orders[nxt][:ahead])))
            torch.cuda.synchronize()
            assert np.array_equal(y, y_res[l]), "pass %d layer %d" % (p, l)
            # what the look-ahead fetched for the next layer is in the cache now
            got = sorted(k - cache.key(nxt, 0) for k in cache.where if k // 4096 == nxt)
            assert got == sorted(orders[nxt][:min(ahead, n_slots)]), (p, l, got)
    n_for = wl.E - wl.n_local
    assert shares[1].bytes_fetched == passes * n_for * shares[1].bytes_each
    assert shares[0].bytes_fetched == (passes * n_for + min(ahead, n_slots)) * shares[0].bytes_each
    for k in list(cache.where):
        cache.release(k)
    shares[0].close()
    shares[1].close()
    cache.close()


def test_plan_subset_is_the_plan_of_the_masked_counts(torch_gpu):
    torch = torch_gpu
    from paper_2506_12417_amd import binding as B
    dev = torch.device("cuda:0")
    r = np.random.default_rng(9)
    E, G, q, tile_m = 40, 8, 100, 128
    counts = (r.zipf(1.3, size=E) * 37 % 3000).astype(np.int64)
    offsets = np.concatenate([[0], np.cumsum(counts)])
    A = int(counts.sum())
    keep = [3, 17, 17, 0, 39, 21, 8]
    masked = np.zeros_like(counts)
    masked[keep] = counts[keep]
    S = O.schedule_balanced(masked, G, q, tile_m)
    tiles_o, bin_start_o = O.tiles_from_schedule(S, offsets, tile_m)
    cap = B.moe_plan_capacity(A, E, tile_m, G)
    tiles = torch.full((cap, 4), -1, dtype=torch.int32, device=dev)
    hdr = torch.full((B.MOE_PLAN_HDR_INTS,), -1, dtype=torch.int32, device=dev)
    sched = torch.full((E, G), -1, dtype=torch.int32, device=dev)
    B.moe_plan_tiles_subset(torch.from_numpy(counts.astype(np.int32)).to(dev), torch.from_numpy(offsets.astype(np.int32)).to(dev),
                            E, A, tile_m, G, q, B.MOE_PLAN_BALANCED, keep, tiles, cap, hdr, sched)
    torch.cuda.synchronize()
    hdr_h = to_numpy(hdr)
    assert np.array_equal(to_numpy(sched), S)
    assert hdr_h[0] == len(tiles_o) and np.array_equal(hdr_h[4:4 + G + 1], bin_start_o)
    assert np.array_equal(to_numpy(tiles)[:hdr_h[0]], tiles_o)
    with pytest.raises(B.MoeError) as e:
        B.moe_plan_tiles_subset(tiles, tiles, E, A, tile_m, G, q, 0, [E], tiles, cap, hdr, None)
    assert e.value.status == B.MOE_ERR_ARG


FULL_SIZE = [("c2", 384), ("c2u", 256), ("c3", 192), ("c4", 64)]


@pytest.mark.parametrize("name,n_sample", FULL_SIZE)
def test_full_size_workloads_sampled(torch_gpu, name, n_sample):
    """The workloads at their full sizes, in the launch configuration bench.py times.  Integer
    stages (expert indices, counts, offsets, permutation, tile table) are checked in full; the
    layer output on a seeded sample of tokens that always holds the first and last row of every
    expert's group and every token of the two coldest experts (the oracle computes any token
    on its own, straight from the definition)."""
    torch = torch_gpu
    wl = W.WORKLOADS[name]
    _note("full size %s: drawing inputs" % name)
    inp = W.make_inputs(wl)
    layer = make_layer(wl, inp)
    x = layer_x(layer, inp)
    _note("full size %s: forward" % name)
    y = layer.forward(x)
    torch.cuda.synchronize()
    idx_o, w_o, _ = O.route_topk(inp["x"], inp["W_g"], inp["b"], wl.k, wl.renorm)
    assert np.array_equal(to_numpy(layer.expert_idx), idx_o)
    assert np.abs(to_numpy(layer.gate_w).astype(np.float64) - w_o).max() <= 2e-6
    flat = idx_o.reshape(-1)
    counts = np.bincount(flat, minlength=wl.E)
    perm_o = np.argsort(flat, kind="stable")            # the stable counting sort (pinned in the CPU tests)
    offsets = np.concatenate([[0], np.cumsum(counts)])
    assert np.array_equal(to_numpy(layer.counts), counts)
    assert np.array_equal(to_numpy(layer.offsets), offsets)
    assert np.array_equal(to_numpy(layer.perm), perm_o)
    inv = np.empty_like(perm_o)
    inv[perm_o] = np.arange(perm_o.size)
    assert np.array_equal(to_numpy(layer.inv_perm), inv)
    hdr = to_numpy(layer.plan_hdr)
    O.validate_tiles(to_numpy(layer.tiles)[:hdr[0]], hdr[4:4 + layer.n_bins + 1], counts, offsets, layer.tile_m, layer.n_bins)
    assert np.array_equal(to_numpy(layer.sched), O.schedule_harmoeny(counts, layer.n_bins, layer.q_tokens))
    # sampled tokens
    r = np.random.default_rng(123)
    tok = set(r.choice(wl.T, n_sample, replace=False).tolist())
    for e in range(wl.E):
        if counts[e]:
            tok.add(int(perm_o[offsets[e]]) // wl.k)
            tok.add(int(perm_o[offsets[e + 1] - 1]) // wl.k)
    cold = [e for e in np.argsort(counts, kind="stable") if counts[e] > 0][:2]
    for e in cold:
        if counts[e] <= 64:
            tok.update((perm_o[offsets[e]:offsets[e + 1]] // wl.k).tolist())
    tok = np.array(sorted(tok))
    _note("full size %s: oracle on %d tokens" % (name, tok.size))
    y_o = O.moe_layer(inp["x"], idx_o, w_o, expert_dict(wl, inp), wl.act, shared=shared_dict(wl, inp), tokens=tok)
    y_h = to_numpy(y)
    rms = float(np.sqrt(np.mean(y_o ** 2)))
    err = float(np.abs(y_h[tok].astype(np.float64) - y_o).max()) / rms
    print("   %s: %d tokens, max err / rms = %.3e (tol %.0e)" % (name, tok.size, err, TOL[wl.dtype]), flush=True)
    assert err <= TOL[wl.dtype]
    assert np.isfinite(y_h).all()


def test_full_size_prerouted_share_with_host_experts(torch_gpu):
    """c5 at its stated size (32768 rows, 16 resident + 16 host-resident experts, d = 768,
    F = 3072), in the launch configuration bench.py times: all experts resident, then the
    section 4.3 flow with a slot per host expert and with 4 slots (overwrite), by id and
    heaviest first.  Integer stages in full; the output bit-identical between the flows, and on a
    seeded sample of rows plus the first and last row of every expert's group against the
    oracle's per-row definition (weights 1: the gate is applied at the rows' source GPU)."""
    torch = torch_gpu
    from paper_2506_12417_amd.layer import to_device
    wl = W.WORKLOADS["c5"]
    _note("full size c5: drawing inputs")
    inp = W.make_inputs(wl)
    ids = inp["ids"]
    x = to_device(inp["x"], "cuda:0")
    ids_d = torch.from_numpy(ids).to("cuda:0")
    counts = np.bincount(ids, minlength=wl.E)
    offsets = np.concatenate([[0], np.cumsum(counts)])
    perm_o = np.argsort(ids, kind="stable")
    inv_o = np.empty_like(perm_o)
    inv_o[perm_o] = np.arange(perm_o.size)
    assert abs(counts[wl.n_local:].sum() / wl.T - 0.30) < 0.02          # the workload's stated foreign share

    _note("full size c5: all experts resident")
    ref_layer = _share(torch, wl, inp, n_local=wl.E, n_slots=1)
    ref_layer.y.fill_(float("nan"))
    y_res = to_numpy(ref_layer.forward(x, ids_d)).copy()
    torch.cuda.synchronize()
    for n, ref in (("counts", counts), ("offsets", offsets), ("perm", perm_o), ("inv_perm", inv_o)):
        assert np.array_equal(to_numpy(getattr(ref_layer, n)), ref), n
    tile_m = ref_layer.tile_m
    ref_layer.close()
    del ref_layer
    assert np.isfinite(y_res).all()

    r = np.random.default_rng(55)
    rows = set(r.choice(wl.T, 256, replace=False).tolist())
    for e in range(wl.E):
        if counts[e]:
            rows.add(int(perm_o[offsets[e]]))
            rows.add(int(perm_o[offsets[e + 1] - 1]))
            # the last row of every full tile and the row after it (tile seams)
            for b in range(tile_m, int(counts[e]), tile_m):
                if len(rows) < 700:
                    rows.update((int(perm_o[offsets[e] + b - 1]), int(perm_o[offsets[e] + b])))
    rows = np.array(sorted(rows))
    _note("full size c5: oracle on %d rows (tile_m %d)" % (rows.size, tile_m))
    y_o = O.moe_layer(inp["x"], ids.reshape(-1, 1), np.ones((wl.T, 1)), {n: inp[n] for n in ("W1", "W2")}, wl.act, tokens=rows)
    err = float(np.abs(y_res[rows].astype(np.float64) - y_o).max()) / float(np.sqrt(np.mean(y_o ** 2)))
    print("   c5: %d rows, max err / rms = %.3e (tol %.0e)" % (rows.size, err, TOL["bf16"]), flush=True)
    assert err <= TOL["bf16"]

    heavy_first = sorted(range(wl.n_local, wl.E), key=lambda e: (-counts[e], e))
    for n_slots in (16, 4):
        _note("full size c5: %d slots" % n_slots)
        sh = _share(torch, wl, inp, n_local=wl.n_local, n_slots=n_slots)
        assert sh.tile_m == tile_m
        for order in (None, heavy_first):
            sh.slots.fill_(0x7f)
            sh.y_perm.fill_(float("nan"))
            sh.y.fill_(float("nan"))
            torch.cuda.synchronize()
            y = to_numpy(sh.forward(x, ids_d, fetch_order=order))
            torch.cuda.synchronize()
            assert np.array_equal(y, y_res), "n_slots=%d order=%s" % (n_slots, "by id" if order is None else "heavy first")
        assert np.array_equal(to_numpy(sh.perm), perm_o) and np.array_equal(to_numpy(sh.counts), counts)
        assert sh.bytes_fetched == 2 * (wl.E - wl.n_local) * sh.bytes_each
        sh.close()
        del sh


@pytest.mark.parametrize("T,d,F,E,gate,skew,tile_m", [(1500, 128, 512, 16, True, "zipf", 128), (1500, 128, 512, 16, False, "zipf", 128),
                                                      (4096, 768, 3072, 128, True, "zipf", 128), (777, 192, 640, 5, True, "hot", 128),
                                                      (300, 64, 1024, 40, True, "uniform", 128),
                                                      (5000, 256, 512, 3, True, "hot", 256)])
def test_ffn_top1_is_ffn_then_combine(torch_gpu, T, d, F, E, gate, skew, tile_m):
    """moe_grouped_ffn_top1 writes what moe_grouped_ffn + moe_unpermute_combine write, bit for bit:
    ragged tiles, empty experts, with and without gate values, 256-row tiles, and twice in a row
    on one plan."""
    torch = torch_gpu
    from paper_2506_12417_amd import binding as B
    from paper_2506_12417_amd.layer import MoELayer
    dev = torch.device("cuda:0")
    r = np.random.default_rng(T + F)
    if skew == "zipf":
        p_e = 1.0 / np.arange(1, E + 1)
    elif skew == "hot":
        p_e = np.array([0.9] + [0.1 / (E - 1)] * (E - 1))
    else:
        p_e = np.ones(E)
    p_e[E // 2] = 0.0                                     # one expert stays empty
    ids = r.choice(E, size=T, p=p_e / p_e.sum()).astype(np.int32)
    L = MoELayer(T, d, F, E, 1, "relu", "bf16", 0, tile_m=tile_m)
    L.experts.w_in.normal_(0, d ** -0.5)
    B.moe_pack_w_out(torch.randn(E, F, d, device=dev).mul_(F ** -0.5).to(torch.bfloat16), E, F, d, B.MOE_BF16, L.experts.w_out)
    L.expert_idx.copy_(torch.from_numpy(ids).view(T, 1))
    L.gate_w.copy_(torch.rand(T, 1, device=dev) + 0.05)
    x = torch.randn(T, d, device=dev).to(torch.bfloat16)
    L.permute(x)
    L.plan()
    L.ffn()
    L.combine(gate)
    y_sep = L.y.clone()
    for rep in range(2):
        L.y.fill_(float("nan"))
        g = L.experts
        B.moe_grouped_ffn_top1(L.x_perm, T, d, F, E, L.act, L.dt, g.in_ptrs, g.out_ptrs, L.tiles, L.plan_hdr, L.tile_m,
                               L.h, L.perm, L.gate_w if gate else None, L.y)
        torch.cuda.synchronize()
        assert torch.equal(L.y, y_sep), rep
    assert int(L.plan_hdr[B.MOE_PLAN_HDR_CTR:].abs().sum()) == 0      # the work counters are back at zero


@pytest.mark.parametrize("T,d,F,E,k,act,skew", [(1500, 256, 512, 16, 1, "relu", "zipf"), (1500, 256, 512, 16, 2, "swiglu", "zipf"),
                                                 (4096, 768, 3072, 128, 1, "relu", "zipf"), (777, 320, 640, 5, 3, "relu", "hot"),
                                                 (300, 1024, 1024, 40, 1, "swiglu", "uniform"), (1, 256, 512, 4, 4, "relu", "uniform")])
def test_ffn_fused_is_gather_then_ffn(torch_gpu, T, d, F, E, k, act, skew):
    """moe_grouped_ffn_fused reads the rows moe_permute would have gathered and writes what the
    separate calls write, bit for bit (H, and y_perm or -- top-1 -- y): ragged tiles, empty
    experts, the shortest contraction it accepts, and twice in a row on one plan."""
    torch = torch_gpu
    from paper_2506_12417_amd import binding as B
    from paper_2506_12417_amd.layer import MoELayer
    dev = torch.device("cuda:0")
    r = np.random.default_rng(T + F + k)
    if skew == "zipf":
        p_e = 1.0 / np.arange(1, E + 1)
    elif skew == "hot":
        p_e = np.array([0.9] + [0.1 / (E - 1)] * (E - 1))
    else:
        p_e = np.ones(E)
    if E > k + 1:
        p_e[E // 2] = 0.0                                 # one expert stays empty
    ids = np.stack([r.choice(E, size=k, replace=False, p=p_e / p_e.sum()) for _ in range(T)]).astype(np.int32)
    L = MoELayer(T, d, F, E, k, act, "bf16", 0, tile_m=128, fuse_gather=False)
    L.experts.w_in.normal_(0, d ** -0.5)
    B.moe_pack_w_out(torch.randn(E, F, d, device=dev).mul_(F ** -0.5).to(torch.bfloat16), E, F, d, B.MOE_BF16, L.experts.w_out)
    L.expert_idx.copy_(torch.from_numpy(ids))
    L.gate_w.copy_(torch.rand(T, k, device=dev) + 0.05)
    x = torch.randn(T, d, device=dev).to(torch.bfloat16)
    L.permute(x)
    L.plan()
    L.ffn()
    L.combine(True)
    torch.cuda.synchronize()
    h_sep, yp_sep, y_sep = L.h.clone(), L.y_perm.clone(), L.y.clone()
    g = L.experts
    for rep in range(2):
        L.x_perm.fill_(float("nan"))                      # the fused call must not need it
        L.h.fill_(float("nan"))
        out = L.y if k == 1 else L.y_perm
        out.fill_(float("nan"))
        B.moe_grouped_ffn_fused(x, T, d, F, E, k, L.act, L.dt, g.in_ptrs, g.out_ptrs, L.tiles, L.plan_hdr, L.tile_m,
                                L.h, L.perm, L.gate_w, out)
        torch.cuda.synchronize()
        assert torch.equal(L.h.view(torch.int16), h_sep.view(torch.int16)), rep
        assert torch.equal(out, y_sep if k == 1 else yp_sep), rep
    assert int(L.plan_hdr[B.MOE_PLAN_HDR_CTR:].abs().sum()) == 0      # the work counters are back at zero


@pytest.mark.parametrize("name,over", [("c2", dict(T=2048, d=128, F=512, E=16)), ("c4", dict(T=900, d=256, F=512, E=4)),
                                       ("c1", {})])
def test_plan_policies_give_the_same_layer_output(torch_gpu, name, over):
    """The four schedules (section 5.3.2's comparison) run the same rows through the same kernels:
    only which work-group takes which tile differs, so the layer output is bit-identical."""
    torch = torch_gpu
    from paper_2506_12417_amd import binding as B
    wl = W.WORKLOADS[name].scaled(**over)
    inp = W.make_inputs(wl)
    layer = make_layer(wl, inp)
    x = layer_x(layer, inp)
    ref = layer.forward(x).clone()
    torch.cuda.synchronize()
    for pol in (B.MOE_PLAN_BALANCED, B.MOE_PLAN_STATIC, B.MOE_PLAN_EVEN_SPLIT, B.MOE_PLAN_ROUND_ROBIN):
        layer.policy = pol
        y = layer.forward(x)
        torch.cuda.synchronize()
        assert torch.equal(y, ref), pol


@pytest.mark.parametrize("alpha,n_hot", [(0.0, 1), (0.5, 1), (0.9, 10), (0.95, 1)])
def test_layer_with_sampled_ids_alpha_skew(torch_gpu, alpha, n_hot):
    """Section 5.1's synthetic router (ids sampled, the first n_hot experts share probability
    alpha): permute -> plan -> FFN -> combine on given ids against the oracle's layer."""
    torch = torch_gpu
    wl = W.WORKLOADS["c2"].scaled(T=3000, d=128, F=512, E=32)
    inp = W.make_inputs(wl)
    layer = make_layer(wl, inp)
    x = layer_x(layer, inp)
    ids = W.alpha_skew_ids(wl.T, wl.E, alpha, n_hot, 77)
    layer.expert_idx.copy_(torch.from_numpy(ids).view(wl.T, 1))
    layer.gate_w.fill_(1.0)
    y = layer.forward(x, routed=True)
    torch.cuda.synchronize()
    p = O.permute(ids.reshape(-1, 1), wl.E)
    assert np.array_equal(to_numpy(layer.counts), p["counts"]) and np.array_equal(to_numpy(layer.perm), p["perm"])
    y_o = O.moe_layer(inp["x"], ids.reshape(-1, 1), np.ones((wl.T, 1)), expert_dict(wl, inp), wl.act)
    assert max_err_over_rms(to_numpy(y), y_o) <= TOL[wl.dtype]


def test_rebalance_three_dimensional_schedule(torch_gpu):
    """moe_rebalance (Alg. 2 with S[g_from, e, g_to]) against the oracle's step-by-step loop:
    the paper's 15-token example with its thresholds, and random Zipf-like count matrices up to
    8 GPUs x 128 experts."""
    torch = torch_gpu
    from paper_2506_12417_amd import binding as B
    dev = torch.device("cuda:0")

    def run(S0, q):
        G_src, E, G = S0.shape
        s_in = torch.from_numpy(S0.astype(np.int32)).to(dev)
        s_out = torch.full_like(s_in, -1)
        info = torch.full((4 + B.MOE_MAX_BINS,), -1, dtype=torch.int32, device=dev)
        B.moe_rebalance(s_in, G_src, E, G, q, s_out, info)
        torch.cuda.synchronize()
        return to_numpy(s_out).astype(np.int64), to_numpy(info)

    m_all = np.array([[1, 1, 3], [1, 2, 2], [0, 1, 4]])                 # tests/golden/alg2_example.txt
    S0 = O.initial_assign(m_all, [0, 1, 2], 3)
    for q, loads in ((1, [5, 5, 5]), (3, [5, 4, 6]), (4, [2, 4, 9]), (5, [2, 4, 9])):
        S, info = run(S0, q)
        assert np.array_equal(S, O.rebalance(S0, q)) and S.sum(axis=(0, 1)).tolist() == loads
        assert info[1] == 5 and info[4:7].tolist() == loads
    r = np.random.default_rng(41)
    for trial in range(24):
        G = int(r.choice([1, 2, 3, 5, 8, 16]))
        G_src = G if trial % 3 else int(r.integers(1, 9))
        E = int(r.choice([G, 17, 60, 128, 256])) if trial % 2 else int(r.integers(G, 64))
        if G_src * E * G * 4 > 128 * 1024:
            E = 64
        q = int(r.choice([1, 7, 64, 300]))
        m = (r.zipf(1.4, size=(G_src, E)) * 11 % 900).astype(np.int64)
        m[r.random((G_src, E)) < 0.15] = 0
        home = [e * G // E for e in range(E)]
        S0 = O.initial_assign(m, home, G)
        _note("rebalance trial %d G_src=%d E=%d G=%d q=%d" % (trial, G_src, E, G, q))
        S, info = run(S0, q)
        ref = O.rebalance(S0, q)
        assert np.array_equal(S, ref), (trial, G_src, E, G, q)
        assert np.array_equal(info[4:4 + G], ref.sum(axis=(0, 1)))
        assert np.array_equal(S.sum(axis=2), m)                          # every token still goes to its expert
