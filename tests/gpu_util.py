"""Helpers of the GPU parity tests: build a layer from a workload, move data, error metrics."""
import numpy as np

import moe_workloads as W


def to_numpy(t):
    """device tensor -> numpy; bfloat16 comes back as uint16 bit patterns."""
    import torch
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def make_layer(wl: W.MoEWorkload, inp, **kw):
    from paper_2506_12417_amd.layer import MoELayer
    layer = MoELayer(wl.T, wl.d, wl.F, wl.E, wl.k, wl.act, wl.dtype, wl.renorm, shared_F=wl.shared_F, **kw)
    if "W_g" in inp:
        layer.load_router(inp["W_g"], inp["b"])
    names = ("W1", "W2") if wl.act == "relu" else ("Wg", "Wu", "Wd")
    if names[0] in inp:
        layer.load_experts({n: inp[n] for n in names})
    if wl.shared_F and "sWg" in inp:
        layer.load_shared({"Wg": inp["sWg"], "Wu": inp["sWu"], "Wd": inp["sWd"]})
    return layer


def expert_dict(wl, inp):
    names = ("W1", "W2") if wl.act == "relu" else ("Wg", "Wu", "Wd")
    return {n: inp[n] for n in names}


def shared_dict(wl, inp):
    return {"Wg": inp["sWg"], "Wu": inp["sWu"], "Wd": inp["sWd"]} if wl.shared_F else None


def max_err_over_rms(got, ref):
    """max |got - ref| / RMS(ref): the layer's stated output tolerance is in these units."""
    ref = np.asarray(ref, dtype=np.float64)
    rms = float(np.sqrt(np.mean(ref ** 2)))
    return float(np.abs(np.asarray(got, dtype=np.float64) - ref).max()) / max(rms, 1e-300)


TOL = {"f32": 1e-4, "bf16": 2e-2}
