"""ctypes binding of libmoe.so -- one Python function per entry point of include/moe.h, same
name, same argument order.  Tensors are torch tensors used as typed device pointers (torch is
plumbing here: device memory and streams); nothing is computed on this side.

Every function raises MoeError when the library returns a status other than MOE_OK."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch  # noqa: F401  (loads the HIP runtime the library links against)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoe.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(
        "libmoe.so is not built: run `python -m paper_2506_12417_amd.build` "
        "(or __graft_entry__.build()).  There is no fallback path.")
lib = C.CDLL(LIB_PATH)

MOE_OK, MOE_ERR_ARG, MOE_ERR_UNSUPPORTED, MOE_ERR_WORKSPACE, MOE_ERR_CAPACITY, MOE_ERR_HIP = 0, -1, -2, -3, -4, -5
MOE_F32, MOE_BF16 = 0, 1
MOE_RELU, MOE_SWIGLU = 0, 1
MOE_PLAN_BALANCED, MOE_PLAN_HARMOENY, MOE_PLAN_STATIC, MOE_PLAN_EVEN_SPLIT, MOE_PLAN_ROUND_ROBIN = 0, 1, 2, 3, 4
MOE_MAX_EXPERTS, MOE_MAX_TOPK, MOE_MAX_BINS = 256, 8, 16
MOE_PLAN_HDR_CTR = 4 + 2 * (MOE_MAX_BINS + 1)
MOE_PLAN_HDR_INTS = MOE_PLAN_HDR_CTR + MOE_MAX_BINS + 1
MOE_OP_PERMUTE = 1
MOE_PERMUTE_STATIC_BYTES = 1 << 20
MOE_PERMUTE_PLAN_MAX = 32768

EXPORTS = [
    "moe_route_topk", "moe_pack_router", "moe_route_topk_packed", "moe_permute", "moe_permute_static", "moe_plan_capacity", "moe_plan_tiles", "moe_permute_plan", "moe_plan_tiles_subset", "moe_rebalance", "moe_pack_weights", "moe_pack_w_out",
    "moe_ffn_tile_m", "moe_ffn_pick_tile_m", "moe_ffn_kernel_mode", "moe_grouped_ffn", "moe_grouped_ffn_phase", "moe_grouped_ffn_top1", "moe_grouped_ffn_top1_phase", "moe_grouped_ffn_fused", "moe_grouped_ffn_fused_phase", "moe_unpermute_combine", "moe_prefetch_create",
    "moe_prefetch_experts", "moe_set_expert_pointers", "moe_prefetch_wait", "moe_prefetch_release", "moe_prefetch_reset", "moe_prefetch_destroy",
    "moe_token_threshold", "moe_workspace_bytes", "moe_copy_bytes", "moe_last_error", "moe_version",
]

_vp, _i, _sz = C.c_void_p, C.c_int, C.c_size_t
lib.moe_route_topk.argtypes = [_vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp]
lib.moe_pack_router.argtypes = [_vp, _i, _i, _i, _vp, _vp, _vp]
lib.moe_route_topk_packed.argtypes = [_vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp]
lib.moe_permute.argtypes = [_vp, _vp, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
lib.moe_permute_static.argtypes = [_vp, _vp, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp]
lib.moe_plan_capacity.argtypes = [_i, _i, _i, _i]
lib.moe_plan_tiles.argtypes = [_vp, _vp, _i, _i, _i, _i, _i, _i, _vp, _i, _vp, _vp, _vp]
lib.moe_permute_plan.argtypes = [_vp, _i, _i, _i, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _vp, _i, _vp, _vp, _vp]
lib.moe_plan_tiles_subset.argtypes = [_vp, _vp, _i, _i, _i, _i, _i, _i, C.POINTER(C.c_int32), _i, _vp, _i, _vp, _vp, _vp]
lib.moe_rebalance.argtypes = [_vp, _i, _i, _i, _i, _vp, _vp, _vp]
lib.moe_pack_weights.argtypes = [_vp, _vp, _i, _i, _i, _i, _vp, _vp]
lib.moe_pack_w_out.argtypes = [_vp, _i, _i, _i, _i, _vp, _vp]
lib.moe_ffn_tile_m.argtypes = [_i]
lib.moe_ffn_pick_tile_m.argtypes = [_i, _i, _i]
lib.moe_ffn_kernel_mode.argtypes = [_i]
lib.moe_grouped_ffn.argtypes = [_vp, _i, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _i, _vp, _vp, _vp]
lib.moe_grouped_ffn_phase.argtypes = [_i, _vp, _i, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _i, _vp, _vp, _vp]
lib.moe_grouped_ffn_top1.argtypes = [_vp, _i, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _i, _vp, _vp, _vp, _vp, _vp]
lib.moe_grouped_ffn_top1_phase.argtypes = [_i, _vp, _i, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _i, _vp, _vp, _vp, _vp, _vp]
lib.moe_grouped_ffn_fused.argtypes = [_vp, _i, _i, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _i, _vp, _vp, _vp, _vp, _vp]
lib.moe_grouped_ffn_fused_phase.argtypes = [_i, _vp, _i, _i, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _i, _vp, _vp, _vp, _vp, _vp]
lib.moe_unpermute_combine.argtypes = [_vp, _vp, _vp, _vp, _i, _i, _i, _vp, _vp]
lib.moe_prefetch_create.argtypes = [C.POINTER(_vp), _i, _sz, _vp]
lib.moe_prefetch_experts.argtypes = [_vp, C.POINTER(C.c_int32), _i, C.POINTER(_vp), _sz, C.POINTER(_vp)]
lib.moe_set_expert_pointers.argtypes = [_vp, _vp, _i, C.POINTER(C.c_int32), _i, C.POINTER(_vp), _sz, _vp]
lib.moe_prefetch_wait.argtypes = [_vp, _i, _vp]
lib.moe_prefetch_release.argtypes = [_vp, _i, _vp]
lib.moe_prefetch_reset.argtypes = [_vp]
lib.moe_prefetch_destroy.argtypes = [_vp]
lib.moe_token_threshold.argtypes = [C.c_double, _i, C.c_double]
lib.moe_workspace_bytes.argtypes = [_i, _i, _i, _i, _i, _i, _i]
lib.moe_workspace_bytes.restype = _sz
lib.moe_copy_bytes.argtypes = [_vp, _vp, _sz, _vp]
lib.moe_last_error.restype = C.c_char_p
lib.moe_version.restype = C.c_char_p


class MoeError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__("libmoe status %d: %s" % (status, text))
        self.status = status


def _check(status: int) -> None:
    if status != MOE_OK:
        raise MoeError(status, lib.moe_last_error().decode())


def _p(t) -> Optional[int]:
    """Device (or host) address of a tensor; None stays NULL; ints pass through."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return MOE_F32
    if t.dtype == torch.bfloat16:
        return MOE_BF16
    raise MoeError(MOE_ERR_UNSUPPORTED, "dtype %s" % t.dtype)


def moe_version() -> str:
    return lib.moe_version().decode()


def moe_last_error() -> str:
    return lib.moe_last_error().decode()


def moe_workspace_bytes(op: int, T: int, d: int, F: int, E: int, k: int, dt: int) -> int:
    return int(lib.moe_workspace_bytes(op, T, d, F, E, k, dt))


def moe_token_threshold(phi: float, d_type: int, beta: float) -> int:
    return int(lib.moe_token_threshold(phi, d_type, beta))


def moe_plan_capacity(A: int, E: int, tile_m: int, n_bins: int) -> int:
    return int(lib.moe_plan_capacity(A, E, tile_m, n_bins))


def moe_ffn_tile_m(dt: int) -> int:
    return int(lib.moe_ffn_tile_m(dt))


def moe_ffn_pick_tile_m(dt: int, A: int, E: int) -> int:
    return int(lib.moe_ffn_pick_tile_m(dt, A, E))


def moe_route_topk(x, w_gate, bias, T, d, E, k, renorm, dt, expert_idx, gate_w, logits_out=None, stream=None):
    _check(lib.moe_route_topk(_p(x), _p(w_gate), _p(bias), T, d, E, k, renorm, dt, _p(expert_idx), _p(gate_w),
                              _p(logits_out), _stream(stream)))


def moe_pack_router(w_gate, d, E, dt, w_gate_t, w_norm2, stream=None):
    _check(lib.moe_pack_router(_p(w_gate), d, E, dt, _p(w_gate_t), _p(w_norm2), _stream(stream)))


def moe_route_topk_packed(x, w_gate_t, w_norm2, bias, T, d, E, k, renorm, dt, expert_idx, gate_w, logits_out=None,
                          stream=None):
    _check(lib.moe_route_topk_packed(_p(x), _p(w_gate_t), _p(w_norm2), _p(bias), T, d, E, k, renorm, dt,
                                     _p(expert_idx), _p(gate_w), _p(logits_out), _stream(stream)))


def moe_permute(x, expert_idx, T, d, E, k, dt, counts, offsets, perm, inv_perm, x_perm, ws, ws_bytes, stream=None):
    _check(lib.moe_permute(_p(x), _p(expert_idx), T, d, E, k, dt, _p(counts), _p(offsets), _p(perm), _p(inv_perm),
                           _p(x_perm), _p(ws), ws_bytes, _stream(stream)))


def moe_ffn_kernel_mode(mode: int) -> int:
    r = int(lib.moe_ffn_kernel_mode(mode))
    if r < 0:
        _check(r)
    return r


def moe_permute_static(x, expert_idx, T, d, E, k, dt, counts, offsets, perm, inv_perm, x_perm, stream=None):
    _check(lib.moe_permute_static(_p(x), _p(expert_idx), T, d, E, k, dt, _p(counts), _p(offsets), _p(perm),
                                  _p(inv_perm), _p(x_perm), _stream(stream)))


def moe_plan_tiles(counts, offsets, E, A, tile_m, n_bins, q_tokens, policy, tiles, tile_capacity, plan_hdr,
                   sched=None, stream=None):
    _check(lib.moe_plan_tiles(_p(counts), _p(offsets), E, A, tile_m, n_bins, q_tokens, policy, _p(tiles),
                              tile_capacity, _p(plan_hdr), _p(sched), _stream(stream)))


def moe_permute_plan(expert_idx, T, E, k, counts, offsets, perm, inv_perm, tile_m, n_bins, q_tokens, policy, tiles,
                     tile_capacity, plan_hdr, sched=None, stream=None):
    _check(lib.moe_permute_plan(_p(expert_idx), T, E, k, _p(counts), _p(offsets), _p(perm), _p(inv_perm), tile_m, n_bins,
                                q_tokens, policy, _p(tiles), tile_capacity, _p(plan_hdr), _p(sched), _stream(stream)))


def moe_plan_tiles_subset(counts, offsets, E, A, tile_m, n_bins, q_tokens, policy, expert_ids, tiles, tile_capacity,
                          plan_hdr, sched=None, stream=None):
    """expert_ids: a Python sequence of the expert ids that take part (host side)."""
    n = len(expert_ids)
    ids = (C.c_int32 * max(n, 1))(*expert_ids)
    _check(lib.moe_plan_tiles_subset(_p(counts), _p(offsets), E, A, tile_m, n_bins, q_tokens, policy, ids, n, _p(tiles),
                                     tile_capacity, _p(plan_hdr), _p(sched), _stream(stream)))


def moe_rebalance(s_initial, G_src, E, G, q_tokens, s_out, info=None, stream=None):
    _check(lib.moe_rebalance(_p(s_initial), G_src, E, G, q_tokens, _p(s_out), _p(info), _stream(stream)))


def moe_pack_weights(w_a, w_b, n, K, N, dt, out, stream=None):
    _check(lib.moe_pack_weights(_p(w_a), _p(w_b), n, K, N, dt, _p(out), _stream(stream)))


def moe_pack_w_out(w, n, F, d, dt, out, stream=None):
    _check(lib.moe_pack_w_out(_p(w), n, F, d, dt, _p(out), _stream(stream)))


def moe_grouped_ffn(x_perm, A, d, F, E, act, dt, w_in, w_out, tiles, plan_hdr, tile_m, h_scratch, y_perm,
                    stream=None):
    _check(lib.moe_grouped_ffn(_p(x_perm), A, d, F, E, act, dt, _p(w_in), _p(w_out), _p(tiles), _p(plan_hdr),
                               tile_m, _p(h_scratch), _p(y_perm), _stream(stream)))


def moe_grouped_ffn_top1(x_perm, T, d, F, E, act, dt, w_in, w_out, tiles, plan_hdr, tile_m, h_scratch, perm, gate_w, y,
                         stream=None):
    _check(lib.moe_grouped_ffn_top1(_p(x_perm), T, d, F, E, act, dt, _p(w_in), _p(w_out), _p(tiles), _p(plan_hdr),
                                    tile_m, _p(h_scratch), _p(perm), _p(gate_w), _p(y), _stream(stream)))


def moe_grouped_ffn_top1_phase(phase, x_perm, T, d, F, E, act, dt, w_in, w_out, tiles, plan_hdr, tile_m, h_scratch, perm,
                               gate_w, y, stream=None):
    _check(lib.moe_grouped_ffn_top1_phase(phase, _p(x_perm), T, d, F, E, act, dt, _p(w_in), _p(w_out), _p(tiles),
                                          _p(plan_hdr), tile_m, _p(h_scratch), _p(perm), _p(gate_w), _p(y), _stream(stream)))


def moe_grouped_ffn_fused(x, T, d, F, E, k, act, dt, w_in, w_out, tiles, plan_hdr, tile_m, h_scratch, perm, gate_w, y_out,
                          stream=None):
    _check(lib.moe_grouped_ffn_fused(_p(x), T, d, F, E, k, act, dt, _p(w_in), _p(w_out), _p(tiles), _p(plan_hdr),
                                     tile_m, _p(h_scratch), _p(perm), _p(gate_w), _p(y_out), _stream(stream)))


def moe_grouped_ffn_fused_phase(phase, x, T, d, F, E, k, act, dt, w_in, w_out, tiles, plan_hdr, tile_m, h_scratch, perm,
                                gate_w, y_out, stream=None):
    _check(lib.moe_grouped_ffn_fused_phase(phase, _p(x), T, d, F, E, k, act, dt, _p(w_in), _p(w_out), _p(tiles),
                                           _p(plan_hdr), tile_m, _p(h_scratch), _p(perm), _p(gate_w), _p(y_out),
                                           _stream(stream)))


def moe_grouped_ffn_phase(phase, x_perm, A, d, F, E, act, dt, w_in, w_out, tiles, plan_hdr, tile_m, h_scratch,
                          y_perm, stream=None):
    _check(lib.moe_grouped_ffn_phase(phase, _p(x_perm), A, d, F, E, act, dt, _p(w_in), _p(w_out), _p(tiles),
                                     _p(plan_hdr), tile_m, _p(h_scratch), _p(y_perm), _stream(stream)))


def moe_unpermute_combine(y_perm, inv_perm, gate_w, shared, T, d, k, y, stream=None):
    _check(lib.moe_unpermute_combine(_p(y_perm), _p(inv_perm), _p(gate_w), _p(shared), T, d, k, _p(y),
                                     _stream(stream)))


def moe_copy_bytes(src, dst, nbytes: int, stream=None):
    _check(lib.moe_copy_bytes(_p(src), _p(dst), nbytes, _stream(stream)))


def moe_prefetch_create(n_slots: int, slot_bytes: int, slot_base) -> int:
    h = _vp()
    _check(lib.moe_prefetch_create(C.byref(h), n_slots, slot_bytes, _p(slot_base)))
    return h.value


def moe_prefetch_experts(h: int, expert_ids: Sequence[int], host_w: Sequence[int], bytes_each: int):
    """host_w: addresses of pinned host buffers.  Returns the slot device address of each expert."""
    n = len(expert_ids)
    ids = (C.c_int32 * max(n, 1))(*expert_ids)
    hw = (_vp * max(n, 1))(*host_w)
    out = (_vp * max(n, 1))()
    _check(lib.moe_prefetch_experts(h, ids, n, hw, bytes_each, out))
    return [out[i] for i in range(n)]


def moe_set_expert_pointers(w_in, w_out, E: int, expert_ids: Sequence[int], ptrs: Sequence[int], out_offset: int, stream=None):
    n = len(expert_ids)
    ids = (C.c_int32 * max(n, 1))(*expert_ids)
    pp = (_vp * max(n, 1))(*ptrs)
    _check(lib.moe_set_expert_pointers(_p(w_in), _p(w_out), E, ids, n, pp, out_offset, _stream(stream)))


def moe_prefetch_wait(h: int, expert_id: int, stream=None):
    _check(lib.moe_prefetch_wait(h, expert_id, _stream(stream)))


def moe_prefetch_release(h: int, expert_id: int, stream=None):
    _check(lib.moe_prefetch_release(h, expert_id, _stream(stream)))


def moe_prefetch_reset(h: int):
    _check(lib.moe_prefetch_reset(h))


def moe_prefetch_destroy(h: int):
    _check(lib.moe_prefetch_destroy(h))
