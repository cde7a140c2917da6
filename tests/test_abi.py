"""The C ABI without a GPU: libmoe.so loads, exports every function include/moe.h declares, and
every argument error is reported by status code before anything is enqueued (so these calls
touch no device and run on a CPU-only machine).  Host-only helpers (Eq. 4, capacities,
workspace sizes) are checked against their closed forms."""
import ctypes as C
import math
import os
import re

import pytest

from paper_2506_12417_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x1000      # a non-null "pointer" that must never be dereferenced on these paths


def declared_functions():
    text = open(os.path.join(ROOT, "include", "moe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return re.findall(r"MOE_API\s+[A-Za-z_][A-Za-z_0-9\s\*]*?\b(moe_[a-z_0-9]+)\s*\(", text)


def test_library_exports_every_declared_function():
    names = declared_functions()
    assert len(names) >= 20 and len(set(names)) == len(names)
    for n in names:
        assert hasattr(B.lib, n), "libmoe.so does not export %s" % n
    assert sorted(names) == sorted(B.EXPORTS), "binding.EXPORTS and include/moe.h disagree"
    assert "gfx950" in B.moe_version()


def status(fn, *args):
    try:
        fn(*args)
    except B.MoeError as e:
        assert str(e) and B.moe_last_error()
        return e.status
    return B.MOE_OK


def test_route_argument_errors():
    r = B.moe_route_topk
    ok = dict(x=FAKE, w=FAKE, b=None, T=4, d=64, E=8, k=2, renorm=1, dt=B.MOE_BF16, idx=FAKE, gw=FAKE)

    def call(**kw):
        a = dict(ok, **kw)
        return status(r, a["x"], a["w"], a["b"], a["T"], a["d"], a["E"], a["k"], a["renorm"], a["dt"], a["idx"], a["gw"], None, 0)

    assert call(k=9, E=8) == B.MOE_ERR_ARG                 # k > E
    assert call(k=0) == B.MOE_ERR_ARG
    assert call(E=0) == B.MOE_ERR_ARG
    assert call(T=-1) == B.MOE_ERR_ARG
    assert call(dt=7) == B.MOE_ERR_UNSUPPORTED
    assert call(d=20) == B.MOE_ERR_UNSUPPORTED             # d % 8
    assert call(E=B.MOE_MAX_EXPERTS + 1) == B.MOE_ERR_UNSUPPORTED
    assert call(E=32, k=B.MOE_MAX_TOPK + 1) == B.MOE_ERR_UNSUPPORTED
    assert call(x=None) == B.MOE_ERR_ARG
    assert call(idx=None) == B.MOE_ERR_ARG
    assert call(T=0, x=None, w=None, idx=None, gw=None) == B.MOE_OK      # T = 0 is a no-op


def test_permute_argument_errors():
    def call(x=FAKE, idx=FAKE, T=8, d=64, E=4, k=2, dt=B.MOE_BF16, counts=FAKE, offsets=FAKE, perm=FAKE, inv=FAKE,
             xp=FAKE, ws=FAKE, ws_bytes=1 << 20):
        return status(B.moe_permute, x, idx, T, d, E, k, dt, counts, offsets, perm, inv, xp, ws, ws_bytes, 0)

    assert call(E=0) == B.MOE_ERR_ARG
    assert call(k=0) == B.MOE_ERR_ARG
    assert call(E=B.MOE_MAX_EXPERTS + 1) == B.MOE_ERR_UNSUPPORTED
    assert call(dt=5) == B.MOE_ERR_UNSUPPORTED
    assert call(d=12) == B.MOE_ERR_UNSUPPORTED             # 24-byte rows
    assert call(x=None) == B.MOE_ERR_ARG                   # x without x_perm
    assert call(counts=None) == B.MOE_ERR_ARG
    assert call(perm=None) == B.MOE_ERR_ARG
    assert call(ws_bytes=8) == B.MOE_ERR_WORKSPACE
    assert call(T=1 << 29, k=4) == B.MOE_ERR_UNSUPPORTED


def test_permute_static_argument_errors():
    def call(x=FAKE, idx=FAKE, T=8, d=64, E=4, k=2, dt=B.MOE_BF16, counts=FAKE, offsets=FAKE, perm=FAKE, inv=FAKE, xp=FAKE):
        return status(B.moe_permute_static, x, idx, T, d, E, k, dt, counts, offsets, perm, inv, xp, 0)

    assert call(E=0) == B.MOE_ERR_ARG
    assert call(dt=5) == B.MOE_ERR_UNSUPPORTED
    assert call(x=None) == B.MOE_ERR_ARG
    assert call(counts=None) == B.MOE_ERR_ARG
    # the built-in array holds 1 MiB of block histograms: ceil(T*k / 1024) * E * 4 bytes must fit
    fits = (B.MOE_PERMUTE_STATIC_BYTES // (4 * 128)) * 1024
    assert B.moe_workspace_bytes(B.MOE_OP_PERMUTE, fits, 64, 0, 128, 1, B.MOE_BF16) == B.MOE_PERMUTE_STATIC_BYTES
    assert call(T=fits + 1, k=1, E=128) == B.MOE_ERR_CAPACITY
    assert "moe_permute" in B.moe_last_error()


def test_permute_plan_argument_errors():
    def call(idx=FAKE, T=64, E=8, k=2, counts=FAKE, perm=FAKE, tile_m=128, G=8, q=10, policy=1, tiles=FAKE, cap=10000, hdr=FAKE):
        return status(B.moe_permute_plan, idx, T, E, k, counts, FAKE, perm, FAKE, tile_m, G, q, policy, tiles, cap, hdr, None, 0)

    assert call(T=0) == B.MOE_ERR_ARG
    assert call(E=B.MOE_MAX_EXPERTS + 1) == B.MOE_ERR_UNSUPPORTED
    assert call(T=B.MOE_PERMUTE_PLAN_MAX // 2 + 1) == B.MOE_ERR_UNSUPPORTED      # times k = 2
    assert call(G=0) == B.MOE_ERR_ARG and call(q=0) == B.MOE_ERR_ARG and call(policy=9) == B.MOE_ERR_ARG
    assert call(idx=None) == B.MOE_ERR_ARG and call(perm=None) == B.MOE_ERR_ARG and call(hdr=None) == B.MOE_ERR_ARG
    assert call(cap=3) == B.MOE_ERR_CAPACITY


def test_workspace_and_capacity_closed_forms():
    # one histogram of E int32 counters per block of 1024 assignments
    for T, k, E in ((1, 1, 1), (1024, 1, 8), (1025, 1, 8), (16384, 4, 60), (0, 2, 5)):
        A = T * k
        assert B.moe_workspace_bytes(B.MOE_OP_PERMUTE, T, 64, 0, E, k, B.MOE_BF16) == max(1, math.ceil(A / 1024)) * E * 4
    assert B.moe_workspace_bytes(99, 1, 1, 1, 1, 1, 0) == 0
    # every (expert, bin) block can end with one ragged tile
    for A, E, tm, G in ((0, 5, 128, 8), (16384, 128, 128, 8), (777, 1, 64, 3), (32768, 32, 256, 16)):
        cap = B.moe_plan_capacity(A, E, tm, G)
        assert cap >= math.ceil(A / tm) + E and cap <= A // tm + E * G + G
    assert B.moe_ffn_tile_m(B.MOE_BF16) == 128 and B.moe_ffn_tile_m(B.MOE_F32) == 64
    assert B.moe_ffn_pick_tile_m(B.MOE_BF16, 16384, 128) == 128
    assert B.moe_ffn_pick_tile_m(B.MOE_BF16, 16384, 8) == 256
    assert B.moe_ffn_pick_tile_m(B.MOE_BF16, 32768, 60) == 128
    assert B.moe_ffn_pick_tile_m(B.MOE_F32, 16384, 8) == 64


def test_token_threshold_is_eq4():
    # q = ceil(phi * d_type / (2 * beta)), section 4.4 Eq. 4
    for phi, dtb, beta in ((2.5e15, 2, 64e9), (2.5e15 / 8, 2, 1e12), (14e12, 4, 12e9), (1.0, 1, 1e30)):
        want = max(1, math.ceil(phi * dtb / (2 * beta)))
        assert B.moe_token_threshold(phi, dtb, beta) == min(want, 10 ** 9)
    assert B.moe_token_threshold(2.5e15 / 8, 2, 1e12) == 313
    assert B.moe_token_threshold(-1.0, 2, 1.0) == 1 and B.moe_token_threshold(1.0, 0, 1.0) == 1


def test_plan_argument_errors():
    def call(counts=FAKE, offsets=FAKE, E=8, A=1000, tile_m=128, G=8, q=10, policy=0, tiles=FAKE, cap=10000, hdr=FAKE):
        return status(B.moe_plan_tiles, counts, offsets, E, A, tile_m, G, q, policy, tiles, cap, hdr, None, 0)

    assert call(E=0) == B.MOE_ERR_ARG
    assert call(A=-1) == B.MOE_ERR_ARG
    assert call(G=0) == B.MOE_ERR_ARG and call(G=B.MOE_MAX_BINS + 1) == B.MOE_ERR_ARG
    assert call(tile_m=0) == B.MOE_ERR_ARG
    assert call(q=0) == B.MOE_ERR_ARG                      # Alg. 2 needs a threshold of at least one token
    assert call(policy=5) == B.MOE_ERR_ARG and call(policy=-1) == B.MOE_ERR_ARG
    assert call(E=B.MOE_MAX_EXPERTS + 1) == B.MOE_ERR_UNSUPPORTED
    assert call(A=1 << 26) == B.MOE_ERR_UNSUPPORTED
    assert call(counts=None) == B.MOE_ERR_ARG and call(hdr=None) == B.MOE_ERR_ARG
    assert call(cap=3) == B.MOE_ERR_CAPACITY


def test_ffn_argument_errors():
    def call(x=FAKE, A=256, d=128, F=256, E=4, act=B.MOE_RELU, dt=B.MOE_BF16, w_in=FAKE, w_out=FAKE, tiles=FAKE,
             hdr=FAKE, tile_m=128, h=FAKE, y=FAKE):
        return status(B.moe_grouped_ffn, x, A, d, F, E, act, dt, w_in, w_out, tiles, hdr, tile_m, h, y, 0)

    assert call(dt=3) == B.MOE_ERR_UNSUPPORTED
    assert call(act=2) == B.MOE_ERR_UNSUPPORTED
    assert call(E=0) == B.MOE_ERR_ARG
    assert call(tile_m=64) == B.MOE_ERR_UNSUPPORTED        # bf16 tiles are 128 or 256 rows
    assert call(d=96) == B.MOE_ERR_UNSUPPORTED             # bf16 needs multiples of 64
    assert call(dt=B.MOE_F32, tile_m=128) == B.MOE_ERR_UNSUPPORTED
    assert call(dt=B.MOE_F32, tile_m=64, d=30) == B.MOE_ERR_UNSUPPORTED
    assert call(tiles=None) == B.MOE_ERR_ARG
    assert call(x=None) == B.MOE_ERR_ARG and call(w_out=None) == B.MOE_ERR_ARG
    assert call(A=0, x=None, tiles=None, hdr=None, h=None, y=None) == B.MOE_OK
    assert status(B.moe_grouped_ffn_phase, 3, FAKE, 256, 128, 256, 4, 0, 1, FAKE, FAKE, FAKE, FAKE, 128, FAKE, FAKE, 0) == B.MOE_ERR_ARG


def test_pack_combine_copy_argument_errors():
    assert status(B.moe_pack_weights, FAKE, None, 1, 0, 8, B.MOE_F32, FAKE, 0) == B.MOE_ERR_ARG
    assert status(B.moe_pack_weights, FAKE, FAKE, 1, 8, 48, B.MOE_F32, FAKE, 0) == B.MOE_ERR_UNSUPPORTED   # N % 32
    assert status(B.moe_pack_weights, FAKE, None, 1, 8, 48, B.MOE_BF16, FAKE, 0) == B.MOE_ERR_UNSUPPORTED  # N % 32, 16-bit
    assert status(B.moe_pack_w_out, FAKE, 1, 8, 48, B.MOE_BF16, FAKE, 0) == B.MOE_ERR_UNSUPPORTED
    assert status(B.moe_pack_weights, None, None, 1, 8, 8, B.MOE_F32, FAKE, 0) == B.MOE_ERR_ARG
    assert status(B.moe_pack_weights, None, None, 0, 8, 8, B.MOE_F32, None, 0) == B.MOE_OK
    reb = lambda s_in=FAKE, Gs=8, E=128, G=8, q=1, s_out=FAKE: status(B.moe_rebalance, s_in, Gs, E, G, q, s_out, None, 0)
    assert reb(Gs=0) == B.MOE_ERR_ARG and reb(G=17) == B.MOE_ERR_ARG and reb(q=0) == B.MOE_ERR_ARG
    assert reb(E=257) == B.MOE_ERR_UNSUPPORTED and reb(Gs=16, E=256, G=16) == B.MOE_ERR_UNSUPPORTED
    assert reb(s_in=None) == B.MOE_ERR_ARG and reb(s_out=None) == B.MOE_ERR_ARG
    assert status(B.moe_pack_w_out, FAKE, 1, 0, 8, B.MOE_BF16, FAKE, 0) == B.MOE_ERR_ARG
    top1 = lambda dt, F, perm, y: status(B.moe_grouped_ffn_top1, FAKE, 8, 64, F, 2, B.MOE_RELU, dt, FAKE, FAKE, FAKE, FAKE,
                                         128, FAKE, perm, None, y, 0)
    assert top1(B.MOE_F32, 512, FAKE, FAKE) == B.MOE_ERR_UNSUPPORTED
    assert top1(B.MOE_BF16, 448, FAKE, FAKE) == B.MOE_ERR_UNSUPPORTED
    assert top1(B.MOE_BF16, 512, None, FAKE) == B.MOE_ERR_ARG
    assert top1(B.MOE_BF16, 512, FAKE, None) == B.MOE_ERR_ARG
    assert status(B.moe_grouped_ffn_top1_phase, 3, FAKE, 8, 64, 512, 2, B.MOE_RELU, B.MOE_BF16, FAKE, FAKE, FAKE, FAKE,
                  128, FAKE, FAKE, None, FAKE, 0) == B.MOE_ERR_ARG
    fused = lambda dt=B.MOE_BF16, T=8, d=256, F=512, k=1, tile_m=128, perm=FAKE, y=FAKE: status(
        B.moe_grouped_ffn_fused, FAKE, T, d, F, 2, k, B.MOE_RELU, dt, FAKE, FAKE, FAKE, FAKE, tile_m, FAKE, perm, None, y, 0)
    assert fused(dt=B.MOE_F32) == B.MOE_ERR_UNSUPPORTED and fused(tile_m=64) == B.MOE_ERR_UNSUPPORTED
    before = B.moe_ffn_kernel_mode(1)        # 256-row tiles: only the four-wavefront kernels gather
    try:
        assert fused(tile_m=256) == B.MOE_ERR_UNSUPPORTED
    finally:
        B.moe_ffn_kernel_mode(before)
    assert fused(d=192) == B.MOE_ERR_UNSUPPORTED and fused(F=448) == B.MOE_ERR_UNSUPPORTED       # top-1 needs F >= 512
    assert fused(T=2 ** 24, d=256) == B.MOE_ERR_UNSUPPORTED                                        # x of 8 GiB
    assert fused(k=0) == B.MOE_ERR_ARG and fused(perm=None) == B.MOE_ERR_ARG and fused(y=None) == B.MOE_ERR_ARG
    assert fused(T=0, perm=None, y=None) == B.MOE_OK
    assert status(B.moe_grouped_ffn_fused_phase, 0, FAKE, 8, 256, 512, 2, 1, B.MOE_RELU, B.MOE_BF16, FAKE, FAKE, FAKE, FAKE,
                  128, FAKE, FAKE, None, FAKE, 0) == B.MOE_ERR_ARG
    assert status(B.moe_pack_w_out, None, 1, 8, 32, B.MOE_BF16, FAKE, 0) == B.MOE_ERR_ARG
    assert status(B.moe_pack_w_out, FAKE, 1, 8, 8, 7, FAKE, 0) == B.MOE_ERR_UNSUPPORTED
    assert status(B.moe_pack_w_out, None, 0, 8, 8, B.MOE_BF16, None, 0) == B.MOE_OK
    assert status(B.moe_unpermute_combine, FAKE, FAKE, None, None, 4, 30, 1, FAKE, 0) == B.MOE_ERR_UNSUPPORTED
    assert status(B.moe_unpermute_combine, FAKE, None, None, None, 4, 32, 1, FAKE, 0) == B.MOE_ERR_ARG
    assert status(B.moe_unpermute_combine, FAKE, FAKE, None, None, 4, 32, 0, FAKE, 0) == B.MOE_ERR_ARG
    assert status(B.moe_unpermute_combine, None, None, None, None, 0, 32, 1, None, 0) == B.MOE_OK
    assert status(B.moe_copy_bytes, FAKE, FAKE + 0x1000, 24, 0) == B.MOE_ERR_UNSUPPORTED
    assert status(B.moe_copy_bytes, None, FAKE, 32, 0) == B.MOE_ERR_ARG
    assert status(B.moe_copy_bytes, FAKE + 4, FAKE + 0x1000, 32, 0) == B.MOE_ERR_UNSUPPORTED
    assert status(B.moe_copy_bytes, None, None, 0, 0) == B.MOE_OK


def test_prefetch_argument_errors_before_any_device_work():
    h = C.c_void_p()
    assert B.lib.moe_prefetch_create(C.byref(h), 0, 16, FAKE) == B.MOE_ERR_ARG
    assert B.lib.moe_prefetch_create(C.byref(h), 2, 0, FAKE) == B.MOE_ERR_ARG
    assert B.lib.moe_prefetch_create(C.byref(h), 2, 16, None) == B.MOE_ERR_ARG
    assert B.lib.moe_prefetch_create(None, 2, 16, FAKE) == B.MOE_ERR_ARG
    ids, ptrs = (C.c_int32 * 2)(1, 9), (C.c_void_p * 2)(FAKE, FAKE)
    assert B.lib.moe_set_expert_pointers(FAKE, FAKE, 8, ids, 2, ptrs, 64, None) == B.MOE_ERR_ARG        # id 9 outside [0, 8)
    assert B.lib.moe_set_expert_pointers(None, FAKE, 16, ids, 2, ptrs, 64, None) == B.MOE_ERR_ARG
    assert B.lib.moe_set_expert_pointers(FAKE, FAKE, 16, ids, 2, (C.c_void_p * 2)(FAKE, None), 64, None) == B.MOE_ERR_ARG
    assert B.lib.moe_set_expert_pointers(FAKE, FAKE, 16, ids, 0, ptrs, 64, None) == B.MOE_OK            # nothing to write
    assert B.lib.moe_prefetch_wait(None, 0, None) == B.MOE_ERR_ARG
    assert B.lib.moe_prefetch_release(None, 0, None) == B.MOE_ERR_ARG
    assert B.lib.moe_prefetch_reset(None) == B.MOE_ERR_ARG
    assert B.lib.moe_prefetch_destroy(None) == B.MOE_OK


def test_plan_subset_and_packed_router_argument_errors():
    ids = (C.c_int32 * 2)(1, 9)
    st = B.lib.moe_plan_tiles_subset(FAKE, FAKE, 8, 100, 128, 8, 10, 0, ids, 2, FAKE, 10000, FAKE, None, None)
    assert st == B.MOE_ERR_ARG                                  # expert id 9 outside [0, 8)
    st = B.lib.moe_plan_tiles_subset(FAKE, FAKE, 8, 100, 128, 8, 10, 0, None, 2, FAKE, 10000, FAKE, None, None)
    assert st == B.MOE_ERR_ARG
    st = B.lib.moe_plan_tiles_subset(FAKE, FAKE, 8, 100, 128, 8, 0, 0, ids, 1, FAKE, 10000, FAKE, None, None)
    assert st == B.MOE_ERR_ARG                                  # q = 0
    assert status(B.moe_pack_router, None, 64, 8, B.MOE_BF16, FAKE, FAKE, 0) == B.MOE_ERR_ARG
    assert status(B.moe_pack_router, FAKE, 64, 0, B.MOE_BF16, FAKE, FAKE, 0) == B.MOE_ERR_ARG
    assert status(B.moe_pack_router, FAKE, 64, 8, 9, FAKE, FAKE, 0) == B.MOE_ERR_UNSUPPORTED

    def rp(x=FAKE, wt=FAKE, n2=FAKE, T=4, d=64, E=8, k=2, dt=B.MOE_BF16, idx=FAKE, gw=FAKE):
        return status(B.moe_route_topk_packed, x, wt, n2, None, T, d, E, k, 1, dt, idx, gw, None, 0)

    assert rp(dt=B.MOE_F32) == B.MOE_ERR_UNSUPPORTED            # the prepared-router path is bf16 only
    assert rp(d=72) == B.MOE_ERR_UNSUPPORTED                    # d % 64
    assert rp(k=9) == B.MOE_ERR_ARG and rp(E=300) == B.MOE_ERR_UNSUPPORTED
    assert rp(n2=None) == B.MOE_ERR_ARG and rp(wt=None) == B.MOE_ERR_ARG
    assert rp(T=0, x=None, wt=None, n2=None, idx=None, gw=None) == B.MOE_OK


def test_ticket_register_check():
    """The build refuses GEMM kernels in which the compiler touches the register that receives
    the work-counter's answer behind its back; the check itself, on hand-made assembly."""
    from paper_2506_12417_amd import build as b
    r = b.TICKET_REG
    ok = ("_Z1av:\n\tglobal_atomic_add v%d, v1, v2, s[4:5] sc0\n\tv_add_u32_e32 v3, v4, v5\n"
          "\tv_readfirstlane_b32 s3, v%d\n" % (r, r))
    # another kernel may use the register freely as long as it has no ticket instructions
    free = "_Z1bv:\n\tv_mfma_f32_32x32x16_bf16 v[240:255], v[0:3], v[4:7], v[240:255]\n\tv_mov_b32_e32 v%d, 0\n" % r
    assert b.check_ticket_register(ok + free) == []
    for line in ("v_mov_b32_e32 v3, v%d" % r, "scratch_store_dword off, v%d, off" % r,
                 "ds_read_b128 v[%d:%d], v31" % (r - 2, r + 1), "v_writelane_b32 v%d, s2, 0" % r):
        bad = b.check_ticket_register(ok + "\t" + line + "\n" + free)
        assert bad == [("_Z1av", line)], line
    asm = os.path.join(os.path.dirname(b.LIB), "_build", "ffn_bf16.s")
    if os.path.exists(asm):          # the assembly of the library that is loaded here
        text = open(asm).read()
        assert "global_atomic_add v%d," % r in text
        assert b.check_ticket_register(text) == []


def test_build_checks_the_registers_of_the_streamed_weight_loads():
    """build.check_stream_registers: in the kernels that load weights with hand-written
    buffer_load_dwordx4, a register that holds (or awaits) such a load's data may be read by the
    matrix instruction's B operand only, on every path through the kernel."""
    from paper_2506_12417_amd import build as b
    head = "_ZN1x18gemm_stream_kernelILi0EEEvv: ; @k\n"
    tail = "\ts_endpgm\n.Lfunc_end0:\n"
    load = "\tbuffer_load_dwordx4 v[20:23], v1, s[4:7], s9 offen offset:64\n"
    mfma = "\tv_mfma_f32_16x16x32_bf16 v[40:43], v[8:11], v[20:23], v[40:43]\n"
    loop = (head + "\tv_mov_b32_e32 v20, 0\n\tv_add_u32_e32 v2, v20, v20\n"      # before any load: free to use
            + load + ".LBB0_1:\n\ts_waitcnt vmcnt(0)\n" + mfma
            + "\tv_lshlrev_b32_e32 v21, 2, v0\n\tds_read_b32 v22, v21\n"          # consumed, overwritten, reused
            + load + "\ts_cbranch_scc1 .LBB0_1\n" + tail)
    assert b.check_stream_registers(loop) == []
    # a copy right after the load, a spill, the A operand of the matrix instruction, a read at the
    # top of the loop (reached from the load at its bottom), an accumulator in a loaded register
    for line in ("v_mov_b32_e32 v3, v21", "scratch_store_dword off, v23, off",
                 "v_mfma_f32_16x16x32_bf16 v[40:43], v[20:23], v[8:11], v[40:43]", "v_fmac_f32_e32 v20, v1, v2"):
        text = loop.replace(load + ".LBB0_1:", load + "\t" + line + "\n.LBB0_1:", 1)
        assert [c for _, c in b.check_stream_registers(text)] == [line], line
    text = loop.replace(".LBB0_1:\n", ".LBB0_1:\n\tv_add_u32_e32 v5, v22, v22\n", 1)
    assert [c for _, c in b.check_stream_registers(text)] == ["v_add_u32_e32 v5, v22, v22"]
    assert b.check_stream_registers("_Z1av:\n\ts_endpgm\n.Lfunc_end0:\n")          # no such kernel at all: reported
    asm = os.path.join(os.path.dirname(b.LIB), "_build", "ffn_stream.s")
    if os.path.exists(asm):          # the assembly of the library that is loaded here
        text = open(asm).read()
        assert text.count("buffer_load_dwordx4") > 32
        assert b.check_stream_registers(text) == [] and b.check_ticket_register(text) == []


def test_build_refuses_gemm_kernels_with_state_behind_generic_pointers():
    """build.check_no_flat_access: a GEMM kernel whose device assembly holds a flat access keeps
    part of its state in scratch memory (slow, but correct: no parity test would notice)."""
    from paper_2506_12417_amd import build as b
    ok = "_ZN1x16gemm_wide_kernelILi0EEEvv:\n\tbuffer_load_dwordx4 v1, s[0:3], 0 offen lds\n\tds_read_b128 v[0:3], v4\n\ts_endpgm\n.Lfunc_end0:\n"
    assert b.check_no_flat_access(ok) == []
    for line in ("flat_load_dword v2, v[2:3]", "flat_store_dwordx2 v[2:3], v[4:5]", "flat_atomic_add v1, v[2:3], v4"):
        text = ok.replace("\ts_endpgm", "\t" + line + "\n\ts_endpgm")
        assert [c for _, c in b.check_no_flat_access(text)] == [line]
    # other kernels may use flat accesses
    assert b.check_no_flat_access("_Z11plan_kernelv:\n\tflat_load_dword v2, v[2:3]\n\ts_endpgm\n.Lfunc_end0:\n") == []
    for name in ("ffn_bf16.s", "ffn_stream.s", "ffn_wide.s"):
        asm = os.path.join(os.path.dirname(b.LIB), "_build", name)
        if os.path.exists(asm):      # the assembly of the library that is loaded here
            text = open(asm).read()
            assert "gemm_" in text and b.check_no_flat_access(text) == []
