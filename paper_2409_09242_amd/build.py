"""Build libdw.so (the C-ABI library) from csrc/*.hip for gfx950, in-tree.

Usage:  python -m paper_2409_09242_amd.build
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libdw.so")
STAMP = os.path.join(HERE, "libdw.sources.sha256")      # digest of the sources the library was built from

FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    # packed fp32 instructions are kept out of every kernel
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
]


def _hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.basename(src) + ".o")
    cmd = [_hipcc(), *FLAGS, "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, r.stdout, r.stderr))
    noise = "packed-fp32-ops' is not a recognized feature"
    warn = "\n".join(l for l in r.stderr.splitlines() if l.strip() and noise not in l)
    if "warning:" in warn:
        sys.stderr.write(warn + "\n")
    return obj


# The data-gradient kernel of dw_gemm_bf16_dma.hip issues its LDS transpose reads from inline assembly, so the
# compiler does not know that their results arrive late; the source keeps every use behind an explicit wait.  A copy
# that the compiler places on such a register between the read and the wait would move a stale value.  The check
# below reads the kernels' own assembly and reports every instruction that touches the destination of a
# ds_read_b64_tr_b16 before the next s_waitcnt lgkmcnt(0).
ASM_CHECKED = "dw_gemm_bf16_dma.hip"


def premature_uses_of_transposed_reads(asm_text: str):
    """[(function, line number, instruction)] for the assembly of ASM_CHECKED; empty when the code is sound.
    Also returns the number of transpose reads seen, so that a caller can tell the check looked at something."""
    import re
    found, n_reads = [], 0
    parts = re.split(r"\n(_ZN2dw4b16d18dual_gemm_bf16_dma\w+): ", asm_text)
    for idx in range(1, len(parts), 2):
        name, lines = parts[idx], parts[idx + 1].split("\n")
        end = next((i for i, l in enumerate(lines) if "s_endpgm" in l), len(lines))
        pending = set()
        for i, l in enumerate(lines[:end]):
            ins = l.split(";")[0].strip()
            if not ins or ins.startswith("."):
                continue
            if ins.startswith("ds_read_b64_tr_b16"):
                n_reads += 1
                m = re.search(r"v\[(\d+):(\d+)\]", ins)
                pending.update(range(int(m.group(1)), int(m.group(2)) + 1))
                continue
            if ins.startswith("s_waitcnt"):
                if "lgkmcnt(0)" in ins:
                    pending = set()
                continue
            regs = set()
            for m in re.finditer(r"v\[(\d+):(\d+)\]", ins):
                regs.update(range(int(m.group(1)), int(m.group(2)) + 1))
            for m in re.finditer(r"\bv(\d+)\b", ins):
                regs.add(int(m.group(1)))
            if regs & pending:
                found.append((name, i, ins))
    return found, n_reads


def check_transposed_reads() -> str:
    """Compile ASM_CHECKED to assembly (device side) and run the check; raises when it finds something."""
    os.makedirs(OBJ, exist_ok=True)
    out = os.path.join(OBJ, ASM_CHECKED + ".s")
    cmd = [_hipcc(), *FLAGS, "-S", "--cuda-device-only", os.path.join(CSRC, ASM_CHECKED), "-o", out]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc -S failed for %s:\n%s\n%s" % (ASM_CHECKED, r.stdout, r.stderr))
    found, n_reads = premature_uses_of_transposed_reads(open(out).read())
    if n_reads == 0:
        raise RuntimeError("no ds_read_b64_tr_b16 found in %s: the check no longer sees the kernels" % out)
    if found:
        raise RuntimeError("registers of LDS transpose reads are touched before the wait for LDS:\n" +
                           "\n".join("%s line %d: %s" % f for f in found[:10]))
    return out


def _source_digest() -> str:
    import hashlib
    h = hashlib.sha256()
    files = sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hip", ".h")))
    files.append(os.path.join(ROOT, "include", "dw.h"))
    for f in files:
        h.update(os.path.basename(f).encode() + b"\0")
        h.update(open(f, "rb").read())
    h.update(" ".join(f for f in FLAGS if not os.path.isabs(f)).encode())      # (the tree may sit anywhere)
    return h.hexdigest()


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    digest = _source_digest()
    srcs = sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))
    with ThreadPoolExecutor(max_workers=min(8, len(srcs) + 1)) as ex:
        check = ex.submit(check_transposed_reads)
        objs = list(ex.map(_compile, srcs))
        check.result()
    cmd = [_hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (r.stdout, r.stderr))
    with open(STAMP, "w") as f:
        f.write(digest + "\n")
    if verbose:
        print("built", LIB)
    return LIB


def ensure_built() -> str:
    """Build the library when none is there, or when the sources have changed since the one that is there was built
    (its digest file says so; a library without a digest file is taken as it is).  Tests, the smoke check and the
    benchmark call this.  The binding itself does not: without a library it raises."""
    if not os.path.exists(LIB):
        return build(verbose=True)
    if os.path.exists(STAMP) and open(STAMP).read().strip() != _source_digest():
        sys.stderr.write("libdw.so is older than its sources: building again\n")
        return build(verbose=True)
    return LIB


if __name__ == "__main__":
    build()
