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
SOURCES = ["common.hip", "route.hip", "route_mfma.hip", "permute.hip", "plan.hip", "ffn.hip", "ffn_bf16.hip", "combine.hip", "pack.hip", "prefetch.hip"]

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


def build(verbose: bool = True, jobs: int = 8) -> str:
    """Compiles every source (always; no staleness check) and links libmoe.so."""
    obj_dir = os.path.join(HERE, "_build")
    os.makedirs(obj_dir, exist_ok=True)
    procs = []
    objs = []
    # the device assembly of the GEMM kernels, for check_ticket_register (same flags, same code)
    asm_path = os.path.join(obj_dir, "ffn_bf16.s")
    asm_cmd = [HIPCC, *FLAGS, "-S", "--cuda-device-only", os.path.join(CSRC, "ffn_bf16.hip"), "-o", asm_path]
    procs.append(("ffn_bf16.hip (assembly)", asm_cmd,
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
    bad = check_ticket_register(open(asm_path).read())
    if bad:
        raise RuntimeError("ffn_bf16.hip: v%d is not private to the ticket instructions:\n%s"
                           % (TICKET_REG, "\n".join("  %s: %s" % b for b in bad[:20])))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()
