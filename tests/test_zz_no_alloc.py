"""moe_permute_static: the sort of moe_permute for callers that cannot allocate (no workspace
argument; the block histograms live in an array inside the library's device image).  Its outputs
must equal moe_permute's bit for bit -- and the oracle's -- on two calls in a row, the second one
smaller than the first, since every call on a GPU shares that GPU's one array."""
import numpy as np
import pytest

import moe_workloads as W
from oracle import moe_oracle as O

pytestmark = pytest.mark.gpu


def _run_both(torch, B, T, k, E, d, seed, with_rows):
    dev = torch.device("cuda:0")
    r = np.random.default_rng(seed)
    p = 1.0 / np.arange(1, E + 1) ** 1.1
    idx = r.choice(E, size=(T, k), p=p / p.sum()).astype(np.int32)
    x_bits = W.f32_to_bf16_bits(r.standard_normal((T, d)).astype(np.float32))
    A = T * k
    idx_d = torch.from_numpy(idx).to(dev)
    x_d = torch.from_numpy(x_bits.view(np.int16)).to(dev).view(torch.bfloat16)
    ws_bytes = B.moe_workspace_bytes(B.MOE_OP_PERMUTE, T, d, 0, E, k, B.MOE_BF16)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)
    out = []
    for static in (False, True):
        counts = torch.full((E,), -7, dtype=torch.int32, device=dev)
        offsets = torch.full((E + 1,), -7, dtype=torch.int32, device=dev)
        perm = torch.full((A,), -7, dtype=torch.int32, device=dev)
        inv = torch.full((A,), -7, dtype=torch.int32, device=dev)
        xp = torch.zeros((A, d), dtype=torch.bfloat16, device=dev) if with_rows else None
        torch.cuda.synchronize()
        if static:
            B.moe_permute_static(x_d if with_rows else None, idx_d, T, d, E, k, B.MOE_BF16, counts, offsets, perm, inv, xp)
        else:
            B.moe_permute(x_d if with_rows else None, idx_d, T, d, E, k, B.MOE_BF16, counts, offsets, perm, inv, xp,
                          ws, ws_bytes)
        torch.cuda.synchronize()
        out.append([t.cpu().numpy() for t in (counts, offsets, perm, inv)]
                   + ([xp.view(torch.int16).cpu().numpy().view(np.uint16)] if with_rows else []))
    names = ["counts", "offsets", "perm", "inv_perm", "x_perm"]
    for n, a, b in zip(names, out[0], out[1]):
        assert np.array_equal(a, b), "moe_permute_static differs from moe_permute in " + n
    ref = O.permute(idx, E)
    for n, b in zip(names[:4], out[1]):
        assert np.array_equal(b, ref[n]), n
    if with_rows:
        assert np.array_equal(out[1][4], O.gather_rows(x_bits, ref["perm"], k))


def test_permute_static_matches_permute_twice_in_a_row():
    import torch
    from paper_2506_12417_amd import binding as B
    assert torch.cuda.is_available(), "this test needs the MI355X"
    print("[case] permute_static: 70000 x 2 over 100 experts (137 blocks, separate scan), then 3000 x 1 over 16", flush=True)
    _run_both(torch, B, 70000, 2, 100, 64, seed=1, with_rows=True)
    _run_both(torch, B, 3000, 1, 16, 32, seed=2, with_rows=True)       # smaller: the array keeps the first call's contents
    print("[case] permute_static: 16384 x 1 over 128 (fused scan), indices only, then a single assignment", flush=True)
    _run_both(torch, B, 16384, 1, 128, 768, seed=3, with_rows=False)
    _run_both(torch, B, 1, 1, 2, 8, seed=4, with_rows=False)
    # beyond the array: refused, nothing enqueued
    E = 256
    T = (B.MOE_PERMUTE_STATIC_BYTES // (4 * E)) * 1024 + 1
    with pytest.raises(B.MoeError) as e:
        B.moe_permute_static(None, 0x1000, T, 8, E, 1, B.MOE_BF16, 0x1000, 0x1000, 0x1000, 0x1000, None)
    assert e.value.status == B.MOE_ERR_CAPACITY
    # T = 0 through the same entry point: counts and offsets written, all zero
    dev = torch.device("cuda:0")
    counts = torch.full((8,), 7, dtype=torch.int32, device=dev)
    offsets = torch.full((9,), 7, dtype=torch.int32, device=dev)
    B.moe_permute_static(None, None, 0, 16, 8, 2, B.MOE_F32, counts, offsets, None, None, None)
    torch.cuda.synchronize()
    assert counts.cpu().tolist() == [0] * 8 and offsets.cpu().tolist() == [0] * 9
