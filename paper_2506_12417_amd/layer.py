"""One MoE layer forward as a chain of libmoe calls (Alg. 1 on one GPU).

This class owns device buffers (torch tensors used as memory) and marshals arguments; every step
of the path -- routing, grouping, scheduling, the expert FFNs, the combine, weight packing --
runs in the library's kernels.  Nothing here touches a tensor's values."""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np
import torch

from . import binding as B

XCDS = 8   # accelerator complex dies of an MI355X; work-groups are dealt to them round-robin


def to_device(a: np.ndarray, device) -> torch.Tensor:
    """numpy -> device tensor; uint16 arrays are bfloat16 bit patterns."""
    if a.dtype == np.uint16:
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


def default_q_tokens(dt: int) -> int:
    """Eq. 4 with one XCD as the unit and the rates this library reaches on an MI355X: phi = its
    share of the sustained grouped-GEMM rate (about 1.0 PFLOP/s in bf16: the matrix cores run
    near 1.55 GHz under load; 100 TFLOP/s for the fp32 FMA kernel), beta = its share of the HBM
    streaming rate (about 6.0 TB/s), d_type = bytes per weight.  With the chip's nominal peaks
    (2.5 PFLOP/s, 8 TB/s) q would be 313 rows, which overstates what a cold expert costs here
    and leaves the bins with unequal numbers of tiles."""
    if dt == B.MOE_BF16:
        return B.moe_token_threshold(1.0e15 / XCDS, 2, 6.0e12 / XCDS)
    return B.moe_token_threshold(100e12 / XCDS, 4, 6.0e12 / XCDS)


class ExpertGroup:
    """Packed weights of a set of experts on the device, plus the pointer tables the FFN reads."""

    def __init__(self, E: int, d: int, F: int, act: int, dt: int, device):
        self.E, self.d, self.F, self.act, self.dt = E, d, F, act, dt
        tdt = torch.bfloat16 if dt == B.MOE_BF16 else torch.float32
        self.rows_in = 2 * F if act == B.MOE_SWIGLU else F
        self.w_in = torch.empty((E, self.rows_in, d), dtype=tdt, device=device)
        self.w_out = torch.empty((E, d, F), dtype=tdt, device=device)
        self.refresh_pointers()

    def refresh_pointers(self, in_ptrs=None, out_ptrs=None):
        es = self.w_in.element_size()
        ip = in_ptrs if in_ptrs is not None else [self.w_in.data_ptr() + e * self.rows_in * self.d * es for e in range(self.E)]
        op = out_ptrs if out_ptrs is not None else [self.w_out.data_ptr() + e * self.d * self.F * es for e in range(self.E)]
        self.in_ptrs = torch.tensor(ip, dtype=torch.int64).to(self.w_in.device)
        self.out_ptrs = torch.tensor(op, dtype=torch.int64).to(self.w_in.device)

    def load_expert(self, e: int, w: Dict[str, np.ndarray], stream=None):
        """w: one expert's matrices in the paper's orientation (W1/W2 or Wg/Wu/Wd)."""
        dev = self.w_in.device
        if self.act == B.MOE_SWIGLU:
            a, b2, o = to_device(w["Wg"], dev), to_device(w["Wu"], dev), to_device(w["Wd"], dev)
            B.moe_pack_weights(a, b2, 1, self.d, self.F, self.dt, self.w_in[e], stream)
        else:
            a, o = to_device(w["W1"], dev), to_device(w["W2"], dev)
            B.moe_pack_weights(a, None, 1, self.d, self.F, self.dt, self.w_in[e], stream)
        B.moe_pack_w_out(o, 1, self.F, self.d, self.dt, self.w_out[e], stream)
        torch.cuda.synchronize(dev)   # the staging tensors above may be freed now


class MoELayer:
    def __init__(self, T: int, d: int, F: int, E: int, k: int, act: str, dtype: str, renorm: int,
                 shared_F: int = 0, n_bins: int = XCDS, q_tokens: Optional[int] = None,
                 policy: int = B.MOE_PLAN_HARMOENY, tile_m: Optional[int] = None, device="cuda:0",
                 fuse_gather: Optional[bool] = None):
        self.T, self.d, self.F, self.E, self.k, self.renorm = T, d, F, E, k, renorm
        self.A = T * k
        self.act = B.MOE_SWIGLU if act == "swiglu" else B.MOE_RELU
        self.dt = B.MOE_BF16 if dtype == "bf16" else B.MOE_F32
        self.tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
        self.n_bins, self.policy = n_bins, policy
        self.q_tokens = q_tokens if q_tokens is not None else default_q_tokens(self.dt)
        self.tile_m = tile_m if tile_m is not None else B.moe_ffn_pick_tile_m(self.dt, self.A, E)
        self.device = torch.device(device)
        dev, A = self.device, self.A
        i32, f32 = torch.int32, torch.float32
        self.W_g = None
        self.bias = None
        self.packed_router = False
        self.experts = ExpertGroup(E, d, F, self.act, self.dt, dev)
        self.expert_idx = torch.empty((T, k), dtype=i32, device=dev)
        self.gate_w = torch.empty((T, k), dtype=f32, device=dev)
        self.counts = torch.empty(E, dtype=i32, device=dev)
        self.offsets = torch.empty(E + 1, dtype=i32, device=dev)
        self.perm = torch.empty(A, dtype=i32, device=dev)
        self.inv_perm = torch.empty(A, dtype=i32, device=dev)
        self.x_perm = torch.empty((A, d), dtype=self.tdt, device=dev)
        self.ws_bytes = B.moe_workspace_bytes(B.MOE_OP_PERMUTE, T, d, F, E, k, self.dt)
        self.ws = torch.empty(max(self.ws_bytes, 16), dtype=torch.uint8, device=dev)
        self.tile_capacity = B.moe_plan_capacity(A, E, self.tile_m, n_bins)
        self.tiles = torch.empty((self.tile_capacity, 4), dtype=i32, device=dev)
        self.plan_hdr = torch.empty(B.MOE_PLAN_HDR_INTS, dtype=i32, device=dev)
        self.sched = torch.empty((E, n_bins), dtype=i32, device=dev)
        self.h = torch.empty((A, F), dtype=self.tdt, device=dev)
        self.y_perm = torch.empty((A, d), dtype=f32, device=dev)
        self.y = torch.empty((T, d), dtype=f32, device=dev)
        self.shared_F = shared_F
        # 256-row tiles: the library folds the gather and the scatter into the products of its
        # four-wavefront kernels (its default); its eight-wavefront kernels have no gather at this height
        tall_ok = self.tile_m == 128 or (B.moe_ffn_kernel_mode(-1) != 1 and d >= 256 and F >= 256)
        # top-1 routing without a shared expert: step 6 is folded into the second GEMM
        self.fold_combine = (k == 1 and self.dt == B.MOE_BF16 and not shared_F and tall_ok and F >= 512)
        # the row gather inside the first product (moe_grouped_ffn_fused): where the library offers it
        can_fuse = (self.dt == B.MOE_BF16 and tall_ok and d >= 256 and d % 64 == 0 and F % 64 == 0
                    and T * d * 2 < 2 ** 32 and (k > 1 or self.fold_combine))
        self.fuse_gather = can_fuse if fuse_gather is None else (fuse_gather and can_fuse)
        if shared_F:
            # the always-on shared expert is one more group: E = 1, every token, rows in place
            self.shared = ExpertGroup(1, d, shared_F, B.MOE_SWIGLU, self.dt, dev)
            self.s_counts = torch.tensor([T], dtype=i32).to(dev)
            self.s_offsets = torch.tensor([0, T], dtype=i32).to(dev)
            self.s_tile_m = B.moe_ffn_pick_tile_m(self.dt, T, 1)
            self.s_capacity = B.moe_plan_capacity(T, 1, self.s_tile_m, n_bins)
            self.s_tiles = torch.empty((self.s_capacity, 4), dtype=i32, device=dev)
            self.s_hdr = torch.empty(B.MOE_PLAN_HDR_INTS, dtype=i32, device=dev)
            self.s_h = torch.empty((T, shared_F), dtype=self.tdt, device=dev)
            self.s_y = torch.empty((T, d), dtype=f32, device=dev)
            B.moe_plan_tiles(self.s_counts, self.s_offsets, 1, T, self.s_tile_m, n_bins, self.q_tokens,
                             B.MOE_PLAN_HARMOENY, self.s_tiles, self.s_capacity, self.s_hdr, None)

    # ------------------------------------------------------------------ parameters
    def load_router(self, W_g: np.ndarray, b: Optional[np.ndarray], packed: Optional[bool] = None):
        """packed: prepare the router once with moe_pack_router and route with
        moe_route_topk_packed (default: whenever that entry point supports the shape)."""
        self.W_g = to_device(W_g, self.device)
        self.bias = None if b is None else to_device(np.asarray(b, dtype=np.float32), self.device)
        can_pack = self.dt == B.MOE_BF16 and self.d % 64 == 0
        self.packed_router = can_pack if packed is None else (packed and can_pack)
        if self.packed_router:
            self.W_gt = torch.empty((self.E, self.d), dtype=self.tdt, device=self.device)
            self.w_norm2 = torch.empty(self.E, dtype=torch.float32, device=self.device)
            B.moe_pack_router(self.W_g, self.d, self.E, self.dt, self.W_gt, self.w_norm2)
            torch.cuda.synchronize(self.device)

    def load_experts(self, weights: Dict[str, np.ndarray]):
        """weights: stacked [E, ...] arrays in the paper's orientation."""
        for e in range(self.E):
            self.experts.load_expert(e, {n: a[e] for n, a in weights.items() if not n.startswith("s")})

    def load_shared(self, w: Dict[str, np.ndarray]):
        self.shared.load_expert(0, w)

    # ------------------------------------------------------------------ the path, step by step
    def route(self, x, logits_out=None, stream=None):
        if self.packed_router:
            B.moe_route_topk_packed(x, self.W_gt, self.w_norm2, self.bias, self.T, self.d, self.E, self.k,
                                    self.renorm, self.dt, self.expert_idx, self.gate_w, logits_out, stream)
            return
        B.moe_route_topk(x, self.W_g, self.bias, self.T, self.d, self.E, self.k, self.renorm, self.dt,
                         self.expert_idx, self.gate_w, logits_out, stream)

    def permute(self, x, stream=None):
        """x = None: only the sort (counts, offsets, perm, inv_perm); x_perm is left alone."""
        B.moe_permute(x, self.expert_idx, self.T, self.d, self.E, self.k, self.dt, self.counts, self.offsets,
                      self.perm, self.inv_perm, None if x is None else self.x_perm, self.ws, self.ws_bytes, stream)

    def permute_plan(self, stream=None):
        """The sort (no row gather) and the plan: one launch where the library offers it."""
        if 1 <= self.A <= B.MOE_PERMUTE_PLAN_MAX:
            B.moe_permute_plan(self.expert_idx, self.T, self.E, self.k, self.counts, self.offsets, self.perm, self.inv_perm,
                               self.tile_m, self.n_bins, self.q_tokens, self.policy, self.tiles, self.tile_capacity,
                               self.plan_hdr, self.sched, stream)
        else:
            self.permute(None, stream)
            self.plan(stream)

    def plan(self, stream=None):
        B.moe_plan_tiles(self.counts, self.offsets, self.E, self.A, self.tile_m, self.n_bins, self.q_tokens,
                         self.policy, self.tiles, self.tile_capacity, self.plan_hdr, self.sched, stream)

    def ffn(self, stream=None):
        g = self.experts
        B.moe_grouped_ffn(self.x_perm, self.A, self.d, self.F, self.E, self.act, self.dt, g.in_ptrs, g.out_ptrs,
                          self.tiles, self.plan_hdr, self.tile_m, self.h, self.y_perm, stream)

    def ffn_phase(self, phase: int, stream=None):
        g = self.experts
        B.moe_grouped_ffn_phase(phase, self.x_perm, self.A, self.d, self.F, self.E, self.act, self.dt, g.in_ptrs,
                                g.out_ptrs, self.tiles, self.plan_hdr, self.tile_m, self.h, self.y_perm, stream)

    def shared_ffn(self, x, stream=None):
        g = self.shared
        B.moe_grouped_ffn(x, self.T, self.d, self.shared_F, 1, B.MOE_SWIGLU, self.dt, g.in_ptrs, g.out_ptrs,
                          self.s_tiles, self.s_hdr, self.s_tile_m, self.s_h, self.s_y, stream)

    def combine(self, use_gate: bool = True, stream=None):
        B.moe_unpermute_combine(self.y_perm, self.inv_perm, self.gate_w if use_gate else None,
                                self.s_y if self.shared_F else None, self.T, self.d, self.k, self.y, stream)

    def forward(self, x: torch.Tensor, stream=None, marks=None, routed: bool = False, stages=None) -> torch.Tensor:
        """Enqueues the whole layer on the current (or given) stream; returns the output buffer.
        marks: optional list of 3 torch.cuda.Event recorded before / between / after the two
        grouped GEMMs (for per-kernel timing).  routed: expert_idx and gate_w are already set
        (a router that samples ids, section 5.1's synthetic skew): step 1 is skipped.
        stages: optional list that receives (name, event) after every stage of the path, starting
        with ("start", event) (per-stage timing; the events are recorded on the current stream)."""
        if stages is not None:
            return self._forward_staged(x, stages, routed)
        if not routed:
            self.route(x, None, stream)
        if self.fuse_gather:
            # the first product gathers its rows from x itself (no x_perm); for top-1 the second one
            # also writes y directly
            self.permute_plan(stream)
            g = self.experts
            args = (x, self.T, self.d, self.F, self.E, self.k, self.act, self.dt, g.in_ptrs, g.out_ptrs, self.tiles,
                    self.plan_hdr, self.tile_m, self.h, self.perm, self.gate_w, self.y if self.k == 1 else self.y_perm,
                    stream)
            if marks is None:
                B.moe_grouped_ffn_fused(*args)
            else:
                marks[0].record()
                B.moe_grouped_ffn_fused_phase(1, *args)
                marks[1].record()
                B.moe_grouped_ffn_fused_phase(2, *args)
                marks[2].record()
            if self.k == 1:
                return self.y
            if self.shared_F:
                self.shared_ffn(x, stream)
            self.combine(True, stream)
            return self.y
        self.permute(x, stream)
        self.plan(stream)
        if self.fold_combine:
            # top-1: the second product writes y directly (no y_perm round trip, no combine kernel)
            g = self.experts
            args = (self.x_perm, self.T, self.d, self.F, self.E, self.act, self.dt, g.in_ptrs, g.out_ptrs, self.tiles,
                    self.plan_hdr, self.tile_m, self.h, self.perm, self.gate_w, self.y, stream)
            if marks is None:
                B.moe_grouped_ffn_top1(*args)
            else:
                marks[0].record()
                B.moe_grouped_ffn_top1_phase(1, *args)
                marks[1].record()
                B.moe_grouped_ffn_top1_phase(2, *args)
                marks[2].record()
            return self.y
        if marks is None:
            self.ffn(stream)
        else:
            marks[0].record()
            self.ffn_phase(1, stream)
            marks[1].record()
            self.ffn_phase(2, stream)
            marks[2].record()
        if self.shared_F:
            self.shared_ffn(x, stream)
        self.combine(True, stream)
        return self.y


    def _forward_staged(self, x: torch.Tensor, stages: list, routed: bool) -> torch.Tensor:
        """forward() with an event after every stage: the same calls in the same order."""
        def mark(name):
            ev = torch.cuda.Event(enable_timing=True)
            ev.record()
            stages.append((name, ev))

        g = self.experts
        mark("start")
        if not routed:
            self.route(x, None, None)
            mark("route")
        if self.fuse_gather:
            self.permute_plan(None)
            mark("permute_plan")
        else:
            self.permute(x, None)
            mark("permute")
            self.plan(None)
            mark("plan")
        if self.fuse_gather:
            args = (x, self.T, self.d, self.F, self.E, self.k, self.act, self.dt, g.in_ptrs, g.out_ptrs, self.tiles,
                    self.plan_hdr, self.tile_m, self.h, self.perm, self.gate_w, self.y if self.k == 1 else self.y_perm, None)
            B.moe_grouped_ffn_fused_phase(1, *args)
            mark("g1")
            B.moe_grouped_ffn_fused_phase(2, *args)
            mark("g2")
            if self.k == 1:
                return self.y
        elif self.fold_combine:
            args = (self.x_perm, self.T, self.d, self.F, self.E, self.act, self.dt, g.in_ptrs, g.out_ptrs, self.tiles,
                    self.plan_hdr, self.tile_m, self.h, self.perm, self.gate_w, self.y, None)
            B.moe_grouped_ffn_top1_phase(1, *args)
            mark("g1")
            B.moe_grouped_ffn_top1_phase(2, *args)
            mark("g2")
            return self.y
        else:
            self.ffn_phase(1, None)
            mark("g1")
            self.ffn_phase(2, None)
            mark("g2")
        if self.shared_F:
            self.shared_ffn(x, None)
            mark("shared")
        self.combine(True, None)
        mark("combine")
        return self.y


class ExpertCache:
    """The device slots that hold host-resident experts while they are needed, and the engine that
    fills them (section 4.3: asynchronous fetching, a finished expert's slot is overwritten).  One
    cache can serve several MoE layers of a model: an expert is named by (layer, expert id), so a
    layer can fetch the first experts of the NEXT layer into the slots it has released (section 1:
    the system looks ahead so that the right experts are in GPU memory when they are needed).
    The library alone decides which slot an expert goes to; this class only remembers the answer."""

    def __init__(self, n_slots: int, bytes_each: int, device="cuda:0"):
        assert n_slots >= 1
        self.n_slots, self.bytes_each = n_slots, bytes_each
        self.device = torch.device(device)
        self.slots = torch.empty((n_slots, bytes_each), dtype=torch.uint8, device=self.device)
        self.engine = B.moe_prefetch_create(n_slots, bytes_each, self.slots)
        self.where = {}          # key -> (slot address, sequence number) of experts fetched and not released
        self.seq = 0
        self.bytes_fetched = 0

    @staticmethod
    def key(layer: int, e: int) -> int:
        return layer * 4096 + e              # the engine takes any non-negative id

    def free_slots(self) -> int:
        return self.n_slots - len(self.where)

    def fetch(self, keys, host_ptrs):
        """Enqueues the copies (in this order) on the engine's stream."""
        if not keys:
            return
        got = B.moe_prefetch_experts(self.engine, keys, host_ptrs, self.bytes_each)
        for k, p in zip(keys, got):
            self.seq += 1
            self.where[k] = (p, self.seq)
        self.bytes_fetched += len(keys) * self.bytes_each

    def wait(self, keys, stream=None):
        """Makes the stream wait until all of these experts' copies have landed: copies complete in
        the order they were enqueued, so one wait for the one enqueued last covers the others
        (a chain of event waits on the compute stream costs far more than one)."""
        last = max(keys, key=lambda k: self.where[k][1])
        B.moe_prefetch_wait(self.engine, last, stream)

    def release(self, key, stream=None):
        B.moe_prefetch_release(self.engine, key, stream)
        del self.where[key]

    def close(self):
        if self.engine:
            torch.cuda.synchronize(self.device)
            B.moe_prefetch_destroy(self.engine)
            self.engine = 0


class PreRoutedShare:
    """One GPU's share of an expert-parallel MoE layer after the scatter (Alg. 1 steps 4-5): T rows
    that arrive already routed (one expert id each), E experts of which the first n_local are
    resident on the device and the others live in pinned host memory and are fetched into
    n_slots device slots while the resident ones compute (section 4.3: asynchronous fetching,
    a finished expert's slot is overwritten).  The output is the experts' result in the rows'
    original order (the gate is applied later, at the rows' source GPU: weights are 1 here).

    Experts run in groups: the resident ones first, then the fetched ones `group` at a time, in
    fetch order; each group is one moe_plan_tiles_subset + moe_grouped_ffn (or its fused form) over
    the same rows.

    cache / layer_id: several layers of a model can share one ExpertCache; forward(lookahead=...)
    then fetches the next layer's first experts into the slots this layer has released."""

    def __init__(self, T: int, d: int, F: int, E: int, n_local: int, n_slots: int, act: str = "relu",
                 dtype: str = "bf16", n_bins: int = XCDS, q_tokens: Optional[int] = None, group: Optional[int] = None,
                 device="cuda:0", cache: Optional[ExpertCache] = None, layer_id: int = 0):
        assert 0 <= n_local <= E and n_slots >= 1
        self.T, self.d, self.F, self.E, self.n_local = T, d, F, E, n_local
        self.n_foreign = E - n_local
        self.act = B.MOE_SWIGLU if act == "swiglu" else B.MOE_RELU
        self.dt = B.MOE_BF16 if dtype == "bf16" else B.MOE_F32
        self.tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
        self.device = torch.device(device)
        self.n_bins = n_bins
        self.q_tokens = q_tokens if q_tokens is not None else default_q_tokens(self.dt)
        self.tile_m = B.moe_ffn_pick_tile_m(self.dt, T, E)
        # one row per expert (k = 1): where the library offers it, the first product gathers its rows
        # from x and the second one writes every row to its place in y (moe_grouped_ffn_fused), so
        # that no gather precedes the groups and no combine follows the last one
        self.fused = (self.dt == B.MOE_BF16 and (self.tile_m == 128 or B.moe_ffn_kernel_mode(-1) != 1)
                      and d >= 256 and d % 64 == 0 and F >= 512 and F % 64 == 0 and T * d * 4 < 2 ** 31)
        dev, i32, f32 = self.device, torch.int32, torch.float32
        es = 2 if dtype == "bf16" else 4
        self.rows_in = 2 * F if self.act == B.MOE_SWIGLU else F
        self.in_bytes, self.out_bytes = self.rows_in * d * es, d * F * es
        self.bytes_each = self.in_bytes + self.out_bytes
        self.owns_cache = cache is None
        self.cache = cache if cache is not None else ExpertCache(n_slots, self.bytes_each, dev)
        assert self.cache.bytes_each >= self.bytes_each
        self.layer_id = layer_id
        self.n_slots = self.cache.n_slots
        # a group of fetched experts runs while the next group's copies are in flight
        self.group = group if group is not None else max(1, min(4, self.n_slots // 2))
        self.local = ExpertGroup(max(n_local, 1), d, F, self.act, self.dt, dev)
        self.host_w = torch.empty((max(self.n_foreign, 1), self.bytes_each), dtype=torch.uint8, pin_memory=True)
        self._stage = ExpertGroup(1, d, F, self.act, self.dt, dev)       # packing area for host-resident experts
        # where every expert's two matrices are: the resident block, or the slot the library chose
        ip, op = self._local_ptrs()
        tab = torch.zeros((2, E), dtype=torch.int64)
        tab[0, :n_local] = torch.tensor(ip, dtype=torch.int64)
        tab[1, :n_local] = torch.tensor(op, dtype=torch.int64)
        self.ptr_dev = tab.to(dev)
        self.expert_idx = torch.empty((T, 1), dtype=i32, device=dev)
        self.counts = torch.empty(E, dtype=i32, device=dev)
        self.offsets = torch.empty(E + 1, dtype=i32, device=dev)
        self.perm = torch.empty(T, dtype=i32, device=dev)
        self.inv_perm = torch.empty(T, dtype=i32, device=dev)
        self.x_perm = torch.empty((T, d), dtype=self.tdt, device=dev)
        self.ws_bytes = B.moe_workspace_bytes(B.MOE_OP_PERMUTE, T, d, F, E, 1, self.dt)
        self.ws = torch.empty(max(self.ws_bytes, 16), dtype=torch.uint8, device=dev)
        self.tile_capacity = B.moe_plan_capacity(T, E, self.tile_m, n_bins)
        self.tiles = torch.empty((self.tile_capacity, 4), dtype=i32, device=dev)
        self.plan_hdr = torch.empty(B.MOE_PLAN_HDR_INTS, dtype=i32, device=dev)
        self.h = torch.empty((T, F), dtype=self.tdt, device=dev)
        self.y_perm = torch.zeros((T, d), dtype=f32, device=dev)
        self.y = torch.empty((T, d), dtype=f32, device=dev)
        self.bytes_fetched = 0
        self._done = None

    @property
    def slots(self):
        return self.cache.slots

    def close(self):
        if self.owns_cache:
            self.cache.close()
        else:
            torch.cuda.synchronize(self.device)

    def load_expert(self, e: int, w: Dict[str, np.ndarray]):
        """w: one expert's matrices in the paper's orientation.  Resident experts are packed in
        place; host-resident ones are packed on the device once and parked in pinned memory, so
        that a fetch is a straight copy."""
        if e < self.n_local:
            self.local.load_expert(e, w)
            return
        self._stage.load_expert(0, w)
        j = e - self.n_local
        self.host_w[j, :self.in_bytes].copy_(self._stage.w_in.view(torch.uint8).reshape(-1))
        self.host_w[j, self.in_bytes:].copy_(self._stage.w_out.view(torch.uint8).reshape(-1))
        torch.cuda.synchronize(self.device)

    def _local_ptrs(self):
        g, es = self.local, self.local.w_in.element_size()
        ip = [g.w_in.data_ptr() + e * self.rows_in * self.d * es for e in range(self.n_local)]
        op = [g.w_out.data_ptr() + e * self.d * self.F * es for e in range(self.n_local)]
        return ip, op

    def host_ptr(self, e: int) -> int:
        return self.host_w[e - self.n_local].data_ptr()

    def forward(self, x: torch.Tensor, ids: torch.Tensor, fetch_order=None, stream=None, lookahead=None) -> torch.Tensor:
        """ids: [T] int32 on the device.  fetch_order: the host-resident experts' ids in the order
        they are to be fetched and run (default: by id); the host may know the rows per expert
        from the metadata exchange of Alg. 1 step 2 and put heavy experts first.
        lookahead: (next_share, expert ids) -- another layer on the same cache and the
        host-resident experts it will want first: once all of this layer's own fetches are
        enqueued, those are fetched into the slots this layer releases, so the host link does not
        idle between the two layers."""
        T, E, c, L = self.T, self.E, self.cache, self.layer_id
        # The host drives this flow group by group and does not run more than one pass ahead of the
        # GPU: copies that wait on "slot free" events of a pass still being enqueued were measured to
        # stall in the runtime (3.1 ms per pass with this wait, 3.4-4.3 ms without it).
        if self._done is not None:
            self._done.synchronize()
        order = list(range(self.n_local, E)) if fetch_order is None else [int(e) for e in fetch_order]
        assert sorted(order) == list(range(self.n_local, E))
        # experts that an earlier layer's look-ahead has already fetched run first: they hold slots
        order = [e for e in order if c.key(L, e) in c.where] + [e for e in order if c.key(L, e) not in c.where]
        pending = [(self, e) for e in order if c.key(L, e) not in c.where]
        if lookahead is not None:
            nxt_share, nxt_ids = lookahead
            assert nxt_share.cache is c and nxt_share.layer_id != L
            pending += [(nxt_share, int(e)) for e in nxt_ids if c.key(nxt_share.layer_id, int(e)) not in c.where]

        def fetch_more(n):
            take = pending[:max(0, min(n, c.free_slots()))]
            del pending[:len(take)]
            c.fetch([c.key(sh.layer_id, e) for sh, e in take], [sh.host_ptr(e) for sh, e in take])
            for sh, e in take:
                sh.bytes_fetched += sh.bytes_each

        def upload(group_ids):
            # the slots the library chose for this group's experts -> the device pointer table,
            # enqueued ahead of the group's kernels
            fetched = [e for e in group_ids if e >= self.n_local]
            B.moe_set_expert_pointers(self.ptr_dev[0], self.ptr_dev[1], E, fetched,
                                      [c.where[c.key(L, e)][0] for e in fetched], self.in_bytes, stream)

        self.expert_idx.view(-1).copy_(ids)
        B.moe_permute(None if self.fused else x, self.expert_idx, T, self.d, E, 1, self.dt, self.counts, self.offsets,
                      self.perm, self.inv_perm, None if self.fused else self.x_perm, self.ws, self.ws_bytes, stream)

        def run(group_ids):
            upload(group_ids)
            B.moe_plan_tiles_subset(self.counts, self.offsets, E, T, self.tile_m, self.n_bins, self.q_tokens,
                                    B.MOE_PLAN_HARMOENY, group_ids, self.tiles, self.tile_capacity, self.plan_hdr,
                                    None, stream)
            if self.fused:
                B.moe_grouped_ffn_fused(x, T, self.d, self.F, E, 1, self.act, self.dt, self.ptr_dev[0], self.ptr_dev[1],
                                        self.tiles, self.plan_hdr, self.tile_m, self.h, self.perm, None, self.y, stream)
            else:
                B.moe_grouped_ffn(self.x_perm, T, self.d, self.F, E, self.act, self.dt, self.ptr_dev[0],
                                  self.ptr_dev[1], self.tiles, self.plan_hdr, self.tile_m, self.h, self.y_perm, stream)

        fetch_more(c.n_slots)                           # fills every free slot; copies run while the resident experts compute
        if self.n_local:
            run(list(range(self.n_local)))
        done = 0
        while done < len(order):
            # the last expert runs as a group of its own: what follows the last copy -- and nothing
            # hides it -- is then one expert's work, not a whole group's
            left = len(order) - done
            take = self.group if left > self.group or self.group == 1 else max(1, left - 1)
            grp = []
            for e in order[done:done + take]:              # (as many as have a slot: fetches follow `order`)
                if c.key(L, e) not in c.where:
                    break
                grp.append(e)
            assert grp, "no slot holds the next expert and none is free"
            c.wait([c.key(L, e) for e in grp], stream)
            run(grp)
            for e in grp:
                c.release(c.key(L, e), stream)
            done += len(grp)
            fetch_more(len(grp))                        # into the slots just released
        if not self.fused:
            B.moe_unpermute_combine(self.y_perm, self.inv_perm, None, None, T, self.d, 1, self.y, stream)
        if self._done is None:
            self._done = torch.cuda.Event()
        self._done.record()
        return self.y
