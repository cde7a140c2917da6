"""Builds libmoe.so (gfx950) in-tree with hipcc.  `python -m paper_2506_12417_amd.build`."""
from __future__ import annotations

import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmoe.so")
SOURCES = ["common.hip", "route.hip", "route_mfma.hip", "permute.hip", "plan.hip", "ffn.hip", "ffn_bf16.hip", "ffn_stream.hip", "ffn_wide.hip", "combine.hip", "pack.hip", "prefetch.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    # no packed-fp32 instructions (v_pk_*_f32) in generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


TICKET_REG = 250          # MOE_TICKET_REG of ffn_bf16.hip


def _vgprs(token: str):
    m = re.fullmatch(r"v(\d+)", token)
    if m:
        return range(int(m.group(1)), int(m.group(1)) + 1)
    m = re.fullmatch(r"v\[(\d+):(\d+)\]", token)
    return range(int(m.group(1)), int(m.group(2)) + 1) if m else range(0)


def check_ticket_register(asm_text: str, reg: int = TICKET_REG):
    """The GEMM kernels that hand out work dynamically receive the answer of an atomic in a fixed
    VGPR behind the compiler's back (take_ticket / read_ticket in ffn_bf16.hip).  That is sound
    only if the compiler's own code never touches that register in those kernels.  Returns a
    list of (kernel, instruction) violations found in the device assembly."""
    bad = []
    kernel, uses, ticket = None, [], 0

    def close():
        if kernel and ticket:
            bad.extend((kernel, u) for u in uses)

    for line in asm_text.split("\n"):
        m = re.match(r"^(_Z\w+):", line)
        if m:
            close()
            kernel, uses, ticket = m.group(1), [], 0
            continue
        code = line.split(";")[0].strip()
        if not code or kernel is None:
            continue
        if any(reg in _vgprs(t) for t in re.findall(r"v\[\d+:\d+\]|v\d+", code)):
            if re.fullmatch(r"global_atomic_add v%d, v\d+, v\d+, s\[\d+:\d+\] sc0" % reg, code) or \
                    re.fullmatch(r"v_readfirstlane_b32 s\d+, v%d" % reg, code):
                ticket += 1
            else:
                uses.append(code)
    close()
    return bad


_VREG = re.compile(r"v\[\d+:\d+\]|v\d+")
_STREAM_LOAD = re.compile(r"buffer_load_dwordx4 (v\[\d+:\d+\]), v\d+, s\[\d+:\d+\], s\d+ offen(?: offset:\d+)?$")
# instructions whose first vector operand is not a destination (everything is read)
_NO_DST = ("buffer_store", "global_store", "scratch_store", "flat_store", "ds_write", "ds_store", "v_cmp", "v_cmpx",
           "v_readfirstlane", "v_readlane", "buffer_atomic", "s_", "global_atomic_add v", "buffer_wbl2", "buffer_inv")
# instructions that read their destination as well
_RMW = ("v_fmac", "v_mac", "v_writelane", "v_movrel", "v_swap", "v_pk_fmac", "v_dot2c", "v_dot4c", "v_dot8c")


def _reads_writes(code: str):
    """(VGPRs read, VGPRs written) of one instruction -- a small model of the ISA's operand roles:
    the first vector operand is the destination unless the instruction is a store / compare /
    lane read; a few instructions also read their destination."""
    op = code.split(None, 1)[0]
    rest = code[len(op):]
    ops = [o.strip() for o in rest.split(",")]
    regs = [[r for t in _VREG.findall(o) for r in _vgprs(t)] for o in ops]
    if any(code.startswith(p) for p in _NO_DST) or "lds" in ops[-1].split():
        return {r for rs in regs for r in rs}, set()
    if op.startswith("global_atomic") or op.startswith("flat_atomic"):
        # with a returned value (sc0) the first operand is written
        if "sc0" in rest and regs and regs[0]:
            return {r for rs in regs[1:] for r in rs}, set(regs[0])
        return {r for rs in regs for r in rs}, set()
    written = set(regs[0]) if regs else set()
    read = {r for rs in regs[1:] for r in rs}
    if any(op.startswith(p) for p in _RMW):
        read |= written
    return read, written


def check_stream_registers(asm_text: str):
    """The kernels of ffn_stream.hip load their weights with buffer_load_dwordx4 written as
    assembly: the compiler neither tracks nor waits for these loads (the kernel waits itself), it
    only knows that the instruction defines a value.  That is sound only if nothing but a matrix
    instruction ever READS a register while it holds (or awaits) such a load's data: a copy or a
    spill placed by the compiler could see the register before its data has arrived.

    A forward data-flow pass over each kernel's control-flow graph: a register is LOADED from a
    weight load until another instruction overwrites it; reading a register that may be LOADED is
    allowed to v_mfma_f32_16x16x32 through its B operand only.  Returns (kernel, instruction)
    violations."""
    bad = []
    kernels = list(re.finditer(r"^(_Z\w*gemm_stream_kernel\w*):[^\n]*\n(.*?)\.Lfunc_end", asm_text, flags=re.S | re.M))
    if not kernels:
        return [("(none)", "no gemm_stream_kernel found in the assembly")]
    for m in kernels:
        kernel, body = m.group(1), m.group(2)
        # basic blocks: a label starts one, a branch ends one
        blocks, cur, label_of = [], {"label": None, "code": []}, {}
        for raw in body.split("\n"):
            line = raw.split(";")[0].strip()
            if not line:
                continue
            lm = re.fullmatch(r"(\.LBB\w+):", line)
            if lm:
                if cur["code"] or cur["label"]:
                    blocks.append(cur)
                cur = {"label": lm.group(1), "code": []}
                continue
            if line.startswith("."):
                continue
            cur["code"].append(line)
            if line.startswith("s_branch") or line.startswith("s_cbranch") or line.startswith("s_endpgm") or line.startswith("s_setpc"):
                blocks.append(cur)
                cur = {"label": None, "code": []}
        if cur["code"] or cur["label"]:
            blocks.append(cur)
        for i, b in enumerate(blocks):
            if b["label"]:
                label_of[b["label"]] = i
        succ = []
        for i, b in enumerate(blocks):
            s_ = []
            last = b["code"][-1] if b["code"] else ""
            if last.startswith("s_branch"):
                s_.append(label_of[last.split()[1]])
            elif last.startswith("s_cbranch"):
                s_.append(label_of[last.split()[1]])
                if i + 1 < len(blocks):
                    s_.append(i + 1)
            elif last.startswith("s_endpgm") or last.startswith("s_setpc"):
                pass
            elif i + 1 < len(blocks):
                s_.append(i + 1)
            succ.append(s_)
        n_loads = sum(1 for b in blocks for c in b["code"] if _STREAM_LOAD.fullmatch(c))
        if n_loads == 0:
            bad.append((kernel, "no weight load found"))
            continue

        def transfer(state, code, report):
            lm = _STREAM_LOAD.fullmatch(code)
            if lm:
                return state | set(_vgprs(lm.group(1)))
            read, written = _reads_writes(code)
            hot = read & state
            if hot:
                ops = [o.strip() for o in code.split(None, 1)[1].split(",")]
                ok = code.startswith("v_mfma_f32_16x16x32") and len(ops) >= 4 and not (
                    {r for o in (ops[1], ops[3]) for t in _VREG.findall(o) for r in _vgprs(t)} & state)
                if not ok and report is not None:
                    report.append((kernel, code))
            return state - written

        entry = [set() for _ in blocks]
        work = [0]
        while work:
            i = work.pop()
            st = set(entry[i])
            for c in blocks[i]["code"]:
                st = transfer(st, c, None)
            for j in succ[i]:
                if not st <= entry[j]:
                    entry[j] |= st
                    work.append(j)
        seen = set()
        for i, b in enumerate(blocks):
            st = set(entry[i])
            for c in b["code"]:
                rep = []
                st = transfer(st, c, rep)
                for r in rep:
                    if r not in seen:
                        seen.add(r)
                        bad.append(r)
    return bad


def check_no_flat_access(asm_text: str):
    """The GEMM kernels keep their whole state in registers and reach memory through buffer
    descriptors and LDS instructions only.  A flat_load / flat_store in one of them means that
    the compiler has left part of that state (a closure, a descriptor, an index table) in
    scratch memory behind generic pointers: every such access waits for all loads in flight,
    and the kernel runs several times slower with correct results -- a failure no parity test
    sees.  Returns a list of (kernel, instruction) found in the device assembly."""
    bad = []
    kernel = None
    for line in asm_text.split("\n"):
        m = re.match(r"^(_Z\w+):", line)
        if m:
            kernel = m.group(1)
            continue
        if line.startswith(".Lfunc_end"):
            kernel = None
            continue
        code = line.split(";")[0].strip()
        if kernel and "gemm_" in kernel and re.match(r"flat_(load|store|atomic)", code):
            bad.append((kernel, code))
    return bad


def build(verbose: bool = True, jobs: int = 8) -> str:
    """Compiles every source (always; no staleness check) and links libmoe.so."""
    obj_dir = os.path.join(HERE, "_build")
    os.makedirs(obj_dir, exist_ok=True)
    procs = []
    objs = []
    # the device assembly of the GEMM kernels, for check_ticket_register (same flags, same code)
    asm_paths = []
    for src in ("ffn_bf16.hip", "ffn_stream.hip", "ffn_wide.hip"):
        asm_path = os.path.join(obj_dir, src.replace(".hip", ".s"))
        asm_paths.append(asm_path)
        asm_cmd = [HIPCC, *FLAGS, "-S", "--cuda-device-only", os.path.join(CSRC, src), "-o", asm_path]
        procs.append((src + " (assembly)", asm_cmd,
                      subprocess.Popen(asm_cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for src in SOURCES:
        obj = os.path.join(obj_dir, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        while sum(p.poll() is None for _, _, p in procs) >= jobs:
            for _, _, p in procs:
                if p.poll() is None:
                    p.wait()
                    break
    failed = False
    for src, cmd, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
        if p.returncode != 0:
            failed = True
            sys.stderr.write("FAILED: %s\n%s\n" % (" ".join(cmd), out))
        elif verbose and out.strip():
            sys.stderr.write("[%s]\n%s\n" % (src, out))
    if failed:
        raise RuntimeError("hipcc failed")
    for asm_path in asm_paths:
        bad = check_ticket_register(open(asm_path).read())
        if bad:
            raise RuntimeError("%s: v%d is not private to the ticket instructions:\n%s"
                               % (os.path.basename(asm_path), TICKET_REG, "\n".join("  %s: %s" % b for b in bad[:20])))
        bad = check_no_flat_access(open(asm_path).read())
        if bad:
            raise RuntimeError("%s: kernel state behind generic pointers (flat accesses):\n%s"
                               % (os.path.basename(asm_path), "\n".join("  %s: %s" % b for b in bad[:20])))
    bad = check_stream_registers(open(asm_paths[1]).read())
    if bad:
        raise RuntimeError("ffn_stream.hip: registers of the weight loads are touched by other code:\n%s"
                           % "\n".join("  %s: %s" % b for b in bad[:20]))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()
