#!/usr/bin/env python3
"""MoE-layer forward benchmark on one MI355X.

A step is one pass of the whole hot path -- route -> permute -> plan -> grouped FFN (+ shared
expert) -> combine -- over one batch of seeded synthetic input already resident in HBM.
Default workload: c2 (Switch-style layer, bf16, T=16384, d=768, F=3072, E=128, top-1,
first-choice loads ~ Zipf(1.0)).  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2|c3|c4|c5] [--no-cpu-baseline]

--workload c5 times one GPU's expert-parallel share with 16 of its 32 experts in pinned host
memory (asynchronous fetching, section 4.3 of the paper): the step is permute -> resident experts
-> fetched experts group by group -> combine, with 16 and with 4 device slots, next to the same
step with every expert resident and to the bare copies.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published


def ffn_flops(wl, A):
    per_row = (6 if wl.act == "swiglu" else 4) * wl.d * wl.F
    f = A * per_row
    if wl.shared_F:
        f += wl.T * 6 * wl.d * wl.shared_F
    return f


def g1_algorithmic(wl, A, active):
    """Algorithmic work of the first grouped GEMM (H = act(x_perm W_in)) of the routed experts:
    FLOPs = 2 * A * d * F' (F' = F, or 2F with gate and up); bytes = W_in of every expert that
    has rows, once + x_perm once + H written once."""
    s = 2 if wl.dtype == "bf16" else 4
    Fp = 2 * wl.F if wl.act == "swiglu" else wl.F
    flops = 2.0 * A * wl.d * Fp
    byts = active * wl.d * Fp * s + A * wl.d * s + A * wl.F * s
    return flops, byts


def measured_traffic(workload, tag="G1"):
    """HBM bytes per launch of one grouped GEMM from the committed rocprofv3 counter summary
    (FETCH_SIZE + WRITE_SIZE, each scaled by what the same counter reports for a plain copy of
    known size); None if there is no summary for this workload."""
    path = os.path.join(ROOT, "profiles", "bench_%s_hbm_traffic.txt" % workload)
    try:
        with open(path) as f:
            for line in f:
                p = line.split()
                if len(p) == 5 and p[0] == "traffic" and p[1] == workload and p[2] == tag:
                    return int(p[3].split("=")[1]) + int(p[4].split("=")[1])
    except OSError:
        pass
    return None


def bench_prerouted(args):
    """Workload c5: rows arrive routed; 16 resident + 16 host-resident experts."""
    import numpy as np
    import torch
    import moe_workloads as W
    from paper_2506_12417_amd import binding as B
    from paper_2506_12417_amd.layer import PreRoutedShare, to_device

    wl = W.WORKLOADS["c5"]
    inp = W.make_inputs(wl)
    ids = inp["ids"]
    counts = np.bincount(ids, minlength=wl.E)
    x = to_device(inp["x"], "cuda:0")
    ids_d = torch.from_numpy(ids).to("cuda:0")
    heavy_first = sorted(range(wl.n_local, wl.E), key=lambda e: (-counts[e], e))

    def make(n_local, n_slots):
        sh = PreRoutedShare(wl.T, wl.d, wl.F, wl.E, n_local, n_slots, act=wl.act, dtype=wl.dtype)
        for e in range(wl.E):
            sh.load_expert(e, {"W1": inp["W1"][e], "W2": inp["W2"][e]})
        return sh

    def timed(sh, order):
        for _ in range(args.warmup):
            sh.forward(x, ids_d, fetch_order=order)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        start, end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        start.record()
        for _ in range(args.steps):
            sh.forward(x, ids_d, fetch_order=order)
        end.record()
        torch.cuda.synchronize()
        return start.elapsed_time(end) / args.steps, (time.perf_counter() - t0) * 1e3 / args.steps

    res = make(wl.E, 1)
    ms_res, _ = timed(res, None)
    y_res = res.y.clone()
    res.close()
    del res
    out_slots = {}
    for n_slots in (16, 4):
        sh = make(wl.n_local, n_slots)
        ms, wall = timed(sh, heavy_first)
        same = bool(torch.equal(sh.y, y_res))
        out_slots[n_slots] = (ms, wall, same)
        if n_slots == 16:
            # the bare copies: all 16 host experts into their slots, nothing else on the GPU
            c, nb = sh.cache, sh.bytes_each
            keys = [c.key(sh.layer_id, e) for e in heavy_first]
            hw = [sh.host_ptr(e) for e in heavy_first]
            t_copy = []
            for _ in range(5):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                c.fetch(keys, hw)
                c.wait(keys)
                torch.cuda.synchronize()
                t_copy.append((time.perf_counter() - t0) * 1e3)
                for k in keys:
                    c.release(k)
            ms_copy = min(t_copy)
            copy_bytes = len(heavy_first) * nb
        sh.close()
        del sh
    # Two layers on one cache (16 slots): with look-ahead a layer's last groups run while the next
    # layer's first experts are already being fetched into the slots it has released, so the host
    # link does not idle across the layer boundary (section 1 of the paper: the system looks ahead).
    from paper_2506_12417_amd.layer import ExpertCache
    inp2 = W.make_inputs(wl, seed=wl.seed() + 1)
    x2 = to_device(inp2["x"], "cuda:0")
    ids2_d = torch.from_numpy(inp2["ids"]).to("cuda:0")
    cnt2 = np.bincount(inp2["ids"], minlength=wl.E)
    order2 = sorted(range(wl.n_local, wl.E), key=lambda e: (-cnt2[e], e))
    shares, cache = [], None
    for l, w_in in enumerate((inp, inp2)):
        sh = PreRoutedShare(wl.T, wl.d, wl.F, wl.E, wl.n_local, 16, act=wl.act, dtype=wl.dtype, cache=cache, layer_id=l)
        cache = sh.cache
        for e in range(wl.E):
            sh.load_expert(e, {"W1": w_in["W1"][e], "W2": w_in["W2"][e]})
        shares.append(sh)
    feed = [(x, ids_d, heavy_first), (x2, ids2_d, order2)]

    def two_layers(ahead, passes):
        for _ in range(passes):
            for l in (0, 1):
                xl, il, ol = feed[l]
                la = (shares[1 - l], feed[1 - l][2][:ahead]) if ahead else None
                shares[l].forward(xl, il, fetch_order=ol, lookahead=la)

    look = {}
    for ahead in (0, 4):
        two_layers(ahead, max(2, args.warmup // 2))
        torch.cuda.synchronize()
        s_ev, e_ev = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s_ev.record()
        two_layers(ahead, max(3, args.steps // 2))
        e_ev.record()
        torch.cuda.synchronize()
        look[ahead] = s_ev.elapsed_time(e_ev) / (2 * max(3, args.steps // 2))
        for k in list(cache.where):                      # what the last look-ahead left in the cache
            cache.release(k)
    same_la = bool(torch.equal(shares[0].y, y_res))
    for sh in shares:
        sh.close()
    cache.close()
    ms16, wall16, same16 = out_slots[16]
    ms4, wall4, same4 = out_slots[4]
    overlap = (ms_res + ms_copy - ms16) / min(ms_res, ms_copy)
    out = {
        "metric": "MoE-layer tokens/sec on 1 MI355X under Zipf skew; grouped-FFN % bf16 MFMA peak",
        "value": round(wl.T / (ms16 * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms16, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": "c5: T=%d d=%d F=%d, %d resident + %d host-resident experts, ids Zipf(%.1f), %d slots, heavy experts fetched first"
                               % (wl.T, wl.d, wl.F, wl.n_local, wl.E - wl.n_local, wl.zipf_s, 16),
                   "seed": wl.seed(), "rows_to_host_experts": int(counts[wl.n_local:].sum())},
        "host_link": {"bytes_per_step": copy_bytes, "copy_only_ms": round(ms_copy, 4),
                      "copy_only_GBs": round(copy_bytes / (ms_copy * 1e-3) / 1e9, 1),
                      "all_resident_ms": round(ms_res, 4), "with_16_slots_ms": round(ms16, 4), "with_4_slots_ms": round(ms4, 4),
                      "host_wall_ms_16_slots": round(wall16, 4), "host_wall_ms_4_slots": round(wall4, 4),
                      "exposed_ms_16_slots": round(ms16 - ms_res, 4), "overlap_efficiency_16_slots": round(overlap, 3),
                      "bit_identical_to_all_resident": same16 and same4 and same_la,
                      "two_layers_one_cache": {"slots": 16, "ms_per_layer_no_lookahead": round(look[0], 4),
                                               "ms_per_layer_lookahead_4": round(look[4], 4),
                                               "copy_only_ms_per_layer": round(ms_copy, 4)}},
        "roofline": {"kernel": "hipMemcpyAsync H2D (expert fetch)", "bound": "host-link", "achieved": round(copy_bytes / (ms16 * 1e-3) / 1e9, 1),
                     "peak": 64.0, "unit": "GB/s", "frac": round(copy_bytes / (ms16 * 1e-3) / 1e9 / 64.0, 4), "traffic": copy_bytes},
    }
    print(json.dumps(out))


def stage_bytes(wl, name, fused_gather):
    """Algorithmic HBM bytes of one launch of a stage (s = bytes per activation element):
    route:   x once + W_g + indices and gate values written
    permute: the indices twice (histogram, rank) + perm and inv_perm written; with the row gather
             also x read and x_perm written
    combine: y_perm, inv_perm and gate values read (+ the shared expert's output), y written"""
    s = 2 if wl.dtype == "bf16" else 4
    A = wl.T * wl.k
    if name == "route":
        return wl.T * wl.d * s + wl.d * wl.E * s + A * 8
    if name == "permute":
        b = 2 * A * 4 + A * 8
        return b if fused_gather else b + wl.T * wl.d * s + A * wl.d * s
    if name == "combine":
        return A * wl.d * 4 + A * 12 + wl.T * wl.d * 4 + (wl.T * wl.d * 4 if wl.shared_F else 0)
    return None


class Leg:
    """One workload on the device: inputs drawn, weights packed, the layer ready to step."""

    def __init__(self, name):
        import torch
        import moe_workloads as W
        from paper_2506_12417_amd.layer import MoELayer, to_device
        self.torch = torch
        self.wl = wl = W.WORKLOADS[name]
        t0 = time.time()
        self.inp = inp = W.make_inputs(wl)
        t_gen = time.time() - t0
        self.names = ("W1", "W2") if wl.act == "relu" else ("Wg", "Wu", "Wd")
        self.layer = layer = MoELayer(wl.T, wl.d, wl.F, wl.E, wl.k, wl.act, wl.dtype, wl.renorm, shared_F=wl.shared_F)
        layer.load_router(inp["W_g"], inp["b"])
        layer.load_experts({n: inp[n] for n in self.names})
        if wl.shared_F:
            layer.load_shared({"Wg": inp["sWg"], "Wu": inp["sWu"], "Wd": inp["sWd"]})
        self.x = to_device(inp["x"], layer.device)
        torch.cuda.synchronize()
        print("[bench] %s: inputs drawn in %.1fs, weights packed on device" % (wl.name, t_gen), file=sys.stderr, flush=True)

    def timed(self, steps, warmup, marks_on=True):
        """Mean step time over `steps` steps (HIP events on the launch stream around all of them)
        and, with marks_on, the mean launch times of the two grouped GEMMs."""
        torch, layer, x = self.torch, self.layer, self.x
        for _ in range(warmup):
            layer.forward(x)
        torch.cuda.synchronize()
        marks = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)] if marks_on else None
        start, end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        start.record()
        for i in range(steps):
            layer.forward(x, marks=marks[i] if marks_on else None)
        end.record()
        torch.cuda.synchronize()
        ms = start.elapsed_time(end) / steps
        g1 = g2 = None
        if marks_on:
            g1 = sum(m[0].elapsed_time(m[1]) for m in marks) / steps
            g2 = sum(m[1].elapsed_time(m[2]) for m in marks) / steps
        return ms, g1, g2

    def stage_times(self, steps):
        """Mean time of every stage, from events recorded after each stage of the same step
        sequence (so every stage finds its inputs as cold or warm as in a real step)."""
        torch, layer, x = self.torch, self.layer, self.x
        runs = []
        for _ in range(steps):
            st = []
            layer.forward(x, stages=st)
            runs.append(st)
        torch.cuda.synchronize()
        names = [n for n, _ in runs[0][1:]]
        return {n: sum(r[i][1].elapsed_time(r[i + 1][1]) for r in runs) / steps * 1e3 for i, n in enumerate(names)}

    def stage_hbm(self, steps):
        us = self.stage_times(steps)
        out = {}
        for n in ("route", "permute", "combine"):
            if n in us:
                b = stage_bytes(self.wl, n, self.layer.fuse_gather)
                gbs = b / (us[n] * 1e-6) / 1e9
                out[n] = {"us": round(us[n], 2), "algorithmic_bytes": int(b), "GBs": round(gbs, 1),
                          "frac_of_8TBs": round(gbs / HBM_PEAK_GBS, 4)}
        if "permute_plan" in us:
            # the sort and the plan in one launch (moe_permute_plan): no bytes to speak of, latency only
            out["permute_plan_us"] = round(us["permute_plan"], 2)
        else:
            out["plan_us"] = round(us["plan"], 2)
        if self.wl.k == 1 and "combine" not in us:
            out["combine"] = "folded into the second grouped GEMM (top-1): no kernel of its own"
        if self.layer.fuse_gather:
            out["permute_note"] = ("the sort and the plan are one launch (moe_permute_plan); the row gather is done by the "
                                   "first grouped GEMM's loads")
        return out

    def gemm_rates(self, g1_ms, g2_ms):
        """TFLOP/s of the routed experts' two grouped GEMMs from their mean launch times."""
        wl = self.wl
        A = wl.T * wl.k
        Fp = 2 * wl.F if wl.act == "swiglu" else wl.F
        f1, f2 = 2.0 * A * wl.d * Fp, 2.0 * A * wl.F * wl.d
        r = lambda f, ms: f / (ms * 1e-3) / 1e12
        return {"g1_ms": round(g1_ms, 4), "g2_ms": round(g2_ms, 4),
                "g1_tflops": round(r(f1, g1_ms), 1), "g2_tflops": round(r(f2, g2_ms), 1),
                "both_tflops": round(r(f1 + f2, g1_ms + g2_ms), 1),
                "g1_frac": round(r(f1, g1_ms) / MFMA_BF16_PEAK_TFLOPS, 4), "g2_frac": round(r(f2, g2_ms) / MFMA_BF16_PEAK_TFLOPS, 4),
                "both_frac": round(r(f1 + f2, g1_ms + g2_ms) / MFMA_BF16_PEAK_TFLOPS, 4)}

    def free(self):
        self.layer = self.x = self.inp = None
        self.torch.cuda.empty_cache()


def device_copy_rate():
    """A plain device-to-device copy of 256 MiB (moe_copy_bytes): what this chip's HBM delivers to
    the simplest streaming kernel, beside the nominal 8 TB/s.  GB/s of bytes read + bytes written."""
    import torch
    from paper_2506_12417_amd import binding as B
    n = 256 << 20
    src = torch.empty(n, dtype=torch.uint8, device="cuda:0").fill_(1)
    dst = torch.empty_like(src)
    for _ in range(3):
        B.moe_copy_bytes(src, dst, n)
    s_ev, e_ev = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    s_ev.record()
    for _ in range(10):
        B.moe_copy_bytes(src, dst, n)
    e_ev.record()
    torch.cuda.synchronize()
    ms = s_ev.elapsed_time(e_ev) / 10
    return {"kernel": "copy_bytes_kernel", "bytes_read_plus_written": 2 * n, "ms": round(ms, 4),
            "GBs": round(2 * n / (ms * 1e-3) / 1e9, 1), "frac_of_8TBs": round(2 * n / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c2", choices=["c2", "c3", "c4", "c5"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-uniform", action="store_true")
    ap.add_argument("--no-ablation", action="store_true", help="skip the plan-policy and alpha-skew legs")
    ap.add_argument("--no-mfma-leg", action="store_true",
                    help="skip the arithmetic-bound workloads (c4, c3) that the default run times after c2")
    ap.add_argument("--ffn-kernels", default="auto", choices=["auto", "ring", "stream"],
                    help="which 16-bit GEMM kernels run 128-row tiles (moe_ffn_kernel_mode): the default (the "
                         "LDS-ring kernels), the LDS-ring kernels, or the register-streaming kernels")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain device copy of 256 MiB a few times (reference for scaling "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import moe_workloads as W
    from paper_2506_12417_amd import binding as B

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    B.moe_ffn_kernel_mode({"auto": 0, "ring": 1, "stream": 2}[args.ffn_kernels])
    if args.workload == "c5":
        return bench_prerouted(args)
    leg = Leg(args.workload)
    wl, inp, layer, x, names, timed = leg.wl, leg.inp, leg.layer, leg.x, leg.names, leg.timed

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=layer.device).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            B.moe_copy_bytes(src, dst, 256 << 20)   # copy_bytes_kernel: reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    ms, g1_ms, g2_ms = timed(args.steps, args.warmup)
    counts = layer.counts.cpu().numpy()
    A = wl.T * wl.k
    active = int((counts > 0).sum())
    tokens_per_s = wl.T / (ms * 1e-3)
    flops = ffn_flops(wl, A)
    g1_flops, g1_bytes = g1_algorithmic(wl, A, active)
    g1_tflops = g1_flops / (g1_ms * 1e-3) / 1e12
    g1_gbs = g1_bytes / (g1_ms * 1e-3) / 1e9
    ffn_tflops = ffn_flops(wl.scaled(shared_F=0), A) / ((g1_ms + g2_ms) * 1e-3) / 1e12
    # the binding roof of the first grouped GEMM: weights stream from HBM when the experts hold
    # few rows each (c2), the matrix cores bind when rows per expert are many (c3, c4)
    t_hbm, t_mfma = g1_bytes / (HBM_PEAK_GBS * 1e9), g1_flops / (MFMA_BF16_PEAK_TFLOPS * 1e12)
    # (256-row tiles run on the four-wavefront kernels unless the LDS ring is asked for)
    g1_kernel = "gemm_wide_kernel<G1>" if layer.tile_m == 256 and args.ffn_kernels != "ring" else "gemm_bf16_kernel<G1>"
    if t_hbm >= t_mfma:
        roofline = {"kernel": g1_kernel, "bound": "hbm", "achieved": round(g1_gbs, 1), "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": round(g1_gbs / HBM_PEAK_GBS, 4), "traffic": None,
                    "mfma_frac": round(g1_tflops / MFMA_BF16_PEAK_TFLOPS, 4)}
    else:
        roofline = {"kernel": g1_kernel, "bound": "mfma", "achieved": round(g1_tflops, 1),
                    "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(g1_tflops / MFMA_BF16_PEAK_TFLOPS, 4),
                    "traffic": None, "hbm_frac": round(g1_gbs / HBM_PEAK_GBS, 4)}
    roofline["traffic"] = measured_traffic(args.workload)
    # (hardware counters cannot be read from inside this run: the figure is the committed summary's)
    roofline["traffic_source"] = (None if roofline["traffic"] is None else
                                  "profiles/bench_%s_hbm_traffic.txt: rocprofv3 FETCH_SIZE + WRITE_SIZE of an earlier "
                                  "run of this command, not measured in this run" % args.workload)
    roofline["algorithmic_bytes"] = int(g1_bytes)
    roofline["algorithmic_flops"] = int(g1_flops)
    roofline["avg_launch_ms"] = round(g1_ms, 4)
    roofline["g2_avg_launch_ms"] = round(g2_ms, 4)

    out = {
        "metric": "MoE-layer tokens/sec on 1 MI355X under Zipf skew; grouped-FFN % bf16 MFMA peak",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": "%s: T=%d d=%d F=%d E=%d top-%d %s%s, skew=%s" % (
            wl.name, wl.T, wl.d, wl.F, wl.E, wl.k, wl.act, (" + shared F=%d" % wl.shared_F) if wl.shared_F else "",
            wl.skew), "seed": wl.seed(), "n_bins": layer.n_bins, "q_tokens": layer.q_tokens,
            "hidden_activations": "f16" if wl.dtype == "bf16" else "f32", "ffn_kernels": args.ffn_kernels,
            "active_experts": active, "max_expert_rows": int(counts.max()), "min_expert_rows": int(counts.min())},
        "ffn_tflops": round(ffn_tflops, 1), "ffn_mfma_frac": round(ffn_tflops / MFMA_BF16_PEAK_TFLOPS, 4),
        "layer_tflops": round(flops / (ms * 1e-3) / 1e12, 1),
        "roofline": roofline,
    }

    out["gemms"] = leg.gemm_rates(g1_ms, g2_ms)
    out["stage_hbm"] = leg.stage_hbm(max(5, args.steps // 5))
    out["device_copy"] = device_copy_rate()

    if args.workload == "c2" and not args.no_uniform:
        layer.load_router(inp["W_g"], np.zeros(wl.E, dtype=np.float32))     # same data, router bias 0
        ms_u, _, _ = timed(args.steps, max(3, args.warmup // 2), marks_on=False)
        out["uniform_tokens_per_s"] = round(wl.T / (ms_u * 1e-3), 1)
        out["skew_over_uniform"] = round(ms_u / ms, 4)
        layer.load_router(inp["W_g"], inp["b"])

    if not args.no_ablation:
        # The scheduling policies of section 5.3.2 / Fig. "skewnew" as modes of the same plan kernel
        # (same rows, same kernels, bit-identical outputs; only the tile schedule differs).
        # (timed without the event records between the kernels, which cost a few microseconds a step)
        abl = {"alg2": round(timed(max(10, args.steps // 2), 3, marks_on=False)[0], 4)}   # the default: Alg. 2 as printed
        for name, pol in (("balanced_tiles", B.MOE_PLAN_BALANCED), ("static", B.MOE_PLAN_STATIC), ("round_robin", B.MOE_PLAN_ROUND_ROBIN),
                          ("even_split", B.MOE_PLAN_EVEN_SPLIT)):
            layer.policy = pol
            abl[name] = round(timed(max(10, args.steps // 2), 3, marks_on=False)[0], 4)
        layer.policy = B.MOE_PLAN_HARMOENY
        out["plan_ablation_ms_per_step"] = abl
        # Alg. 2 in its three-dimensional form for 8 GPUs (the paper's deployment): this step's
        # assignments as if they had arrived on 8 source GPUs (T/8 consecutive tokens each), experts
        # housed in contiguous blocks.  One kernel, no host loop.
        idx_h = layer.expert_idx.cpu().numpy().reshape(8, -1)
        m_all = np.stack([np.bincount(idx_h[g], minlength=wl.E) for g in range(8)]).astype(np.int32)
        S0 = np.zeros((8, wl.E, 8), dtype=np.int32)
        for e in range(wl.E):
            S0[:, e, e * 8 // wl.E] = m_all[:, e]
        s_in = torch.from_numpy(S0).to(layer.device)
        s_out, info = torch.empty_like(s_in), torch.zeros(4 + B.MOE_MAX_BINS, dtype=torch.int32, device=layer.device)
        for _ in range(3):
            B.moe_rebalance(s_in, 8, wl.E, 8, layer.q_tokens, s_out, info)
        s_ev, e_ev = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        s_ev.record()
        for _ in range(20):
            B.moe_rebalance(s_in, 8, wl.E, 8, layer.q_tokens, s_out, info)
        e_ev.record()
        torch.cuda.synchronize()
        info_h = info.cpu().numpy()
        out["alg2_8gpu_schedule"] = {"us_per_call": round(s_ev.elapsed_time(e_ev) / 20 * 1e3, 1), "moves": int(info_h[0]),
                                     "loads_before": S0.sum(axis=(0, 1)).tolist(), "loads_after": info_h[4:12].tolist(),
                                     "q_tokens": layer.q_tokens}
    if not args.no_ablation and wl.k == 1:
        # Section 5.1's synthetic router: the first n_hot experts share probability alpha, ids are
        # sampled per token; alpha changes from batch to batch (the dynamic-skew experiment).
        # The router product is not part of these steps (the ids are the router's output).
        rs = np.random.default_rng(wl.seed() + 7)
        layer.gate_w.fill_(1.0)
        batches = []
        for bi in range(12):
            alpha = float(rs.uniform(0.0, 0.95)) if bi >= 3 else (0.0, 0.5, 0.9)[bi]
            n_hot = 1 if bi != 2 else 10
            ids = W.alpha_skew_ids(wl.T, wl.E, alpha, n_hot, wl.seed() + 100 + bi)
            layer.expert_idx.copy_(torch.from_numpy(ids).view(wl.T, 1))
            for _ in range(3):
                layer.forward(x, routed=True)
            s_ev, e_ev = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            s_ev.record()
            for _ in range(10):
                layer.forward(x, routed=True)
            e_ev.record()
            torch.cuda.synchronize()
            batches.append({"alpha": round(alpha, 3), "n_hot": n_hot, "ms": round(s_ev.elapsed_time(e_ev) / 10, 4)})
        t = np.array([b["ms"] for b in batches])
        out["alpha_skew"] = {"note": "sampled ids (no router product), 12 batches, alpha in [0, 0.95]",
                             "tokens_per_s_mean": round(float(wl.T / (t.mean() * 1e-3)), 1),
                             "ms_min": round(float(t.min()), 4), "ms_max": round(float(t.max()), 4),
                             "ms_std": round(float(t.std()), 4), "batches": batches}

    if args.workload == "c2" and not args.no_mfma_leg:
        # The second half of the metric: the grouped FFN's fraction of the bf16 matrix-core peak on
        # the workloads that are bound by arithmetic (c2 is bound by its weights' bytes).  Same code
        # path, same launch configuration as `--workload c4` / `--workload c3`, fewer steps.
        leg.free()
        out["mfma_leg"] = {"peak_tflops": MFMA_BF16_PEAK_TFLOPS}
        for name in ("c4", "c3"):
            ml = Leg(name)
            steps = max(5, args.steps // 5)
            ms_m, g1_m, g2_m = ml.timed(steps, 3)
            r = ml.gemm_rates(g1_m, g2_m)
            r.update({"workload": "%s: T=%d d=%d F=%d E=%d top-%d %s%s" % (
                          name, ml.wl.T, ml.wl.d, ml.wl.F, ml.wl.E, ml.wl.k, ml.wl.act,
                          (" + shared F=%d" % ml.wl.shared_F) if ml.wl.shared_F else ""),
                      "tile_m": ml.layer.tile_m, "steps": steps, "ms_per_step": round(ms_m, 4),
                      "tokens_per_s": round(ml.wl.T / (ms_m * 1e-3), 1),
                      "layer_ffn_tflops": round(ffn_flops(ml.wl, ml.wl.T * ml.wl.k) / (ms_m * 1e-3) / 1e12, 1),
                      "stage_hbm": ml.stage_hbm(steps)})
            out["mfma_leg"][name] = r
            ml.free()
            del ml

    if not args.no_cpu_baseline:
        from oracle import moe_oracle as O       # the CPU oracle, timed as it stands
        ew = {n: inp[n] for n in names}
        sh = {"Wg": inp["sWg"], "Wu": inp["sWu"], "Wd": inp["sWd"]} if wl.shared_F else None
        # bounded sample: whole workload when it takes seconds (c2), else a seeded token subset
        n_tok = wl.T if args.workload == "c2" else 1024
        tok = None if n_tok == wl.T else np.sort(np.random.default_rng(1).choice(wl.T, n_tok, replace=False))
        passes, t_cpu = 0, 0.0
        while t_cpu < 12.0 and passes < 20:
            t1 = time.time()
            idx_o, w_o, _ = O.route_topk(inp["x"], inp["W_g"], inp["b"], wl.k, wl.renorm)
            O.permute(idx_o, wl.E)
            O.moe_layer(inp["x"], idx_o, w_o, ew, wl.act, shared=sh, tokens=tok)
            t_cpu += time.time() - t1
            passes += 1
        try:
            cores = len(os.sched_getaffinity(0))
        except AttributeError:
            cores = os.cpu_count()
        cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))
        out["cpu_baseline"] = {"value": round(n_tok * passes / t_cpu, 1), "unit": "tokens/s", "cores": cores,
                               "kind": "oracle",
                               "sample": "%d of %d tokens (routing over all tokens), %d passes, %.1f s" % (n_tok, wl.T, passes, t_cpu)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
