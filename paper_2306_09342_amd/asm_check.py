"""Static check of the device assembly for one hazard of hand-issued loads.

Some kernels issue LDS reads and global loads as inline assembly and wait for them later with an explicit
``s_waitcnt`` (the fragment reads of the GEMMs, the owned-row loads of the one-workgroup attention backward).  The
compiler does not know that the destination registers of such a load are not valid until that wait: if it moves,
copies or spills one of them in between, the kernel computes with stale register contents, silently.  This module
compiles a source file to assembly (``hipcc -S``, device side only) and walks every kernel: it keeps the queue of
outstanding LDS and vector-memory operations, retires them at each ``s_waitcnt`` the way the hardware counters do
(in order, "at most n outstanding"), and reports every instruction that touches the destination registers of an
inline-assembly load that is still outstanding.  Loads the compiler issued itself are counted (they share the
counters) but not checked: the compiler inserts their waits.

The walk is linear (it does not follow branches), which is exact for the straight-line loop bodies these kernels
use between a load and its wait.

    python -m paper_2306_09342_amd.asm_check            # all sources that contain hand-issued loads
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
import tempfile

from . import build as _b

SOURCES = ("gemm_nt_dma.hip", "gemm_wgrad_dma.hip", "attention_mfma.hip")

_REG = re.compile(r"\b([va])(?:(\d+)|\[(\d+):(\d+)\])")
_VM_LOAD = ("global_load", "buffer_load", "scratch_load", "flat_load")
_VM_OTHER = ("global_store", "buffer_store", "scratch_store", "flat_store", "global_atomic", "buffer_atomic")


def _regs(text: str) -> set:
    out = set()
    for m in _REG.finditer(text):
        if m.group(2) is not None:
            out.add((m.group(1), int(m.group(2))))
        else:
            out.update((m.group(1), i) for i in range(int(m.group(3)), int(m.group(4)) + 1))
    return out


def assemble(src: str, out: str) -> None:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    subprocess.run([hipcc] + _b.FLAGS + ["--cuda-device-only", "-S", os.path.join(_b.CSRC, src), "-o", out],
                   check=True, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)


def check_assembly(path: str) -> list:
    """Returns a list of (kernel, line number, instruction, registers) findings."""
    findings = []
    kernel = None
    lgkm, vm = [], []          # outstanding operations, oldest first: (destination registers, issued by inline asm)
    in_asm = False

    def live(queue):
        s = set()
        for regs, from_asm in queue:
            if from_asm:
                s |= regs
        return s

    with open(path) as f:
        for ln, line in enumerate(f, 1):
            if "#ASMSTART" in line:
                in_asm = True
                continue
            if "#ASMEND" in line:
                in_asm = False
                continue
            s = line.split(";")[0].strip()
            if not s:
                continue
            m = re.match(r"^(_Z\w+):$", s)
            if m:
                kernel, lgkm, vm = m.group(1), [], []
                continue
            if kernel is None or s.startswith(".") or s.endswith(":"):
                continue
            op = s.split()[0]
            rest = s[len(op):]
            if op == "s_endpgm":
                lgkm, vm = [], []
                continue
            if op == "s_waitcnt":
                for name, queue in (("lgkmcnt", lgkm), ("vmcnt", vm)):
                    mm = re.search(name + r"\((\d+)\)", rest)
                    if mm:
                        n = int(mm.group(1))
                        del queue[: max(0, len(queue) - n)]
                continue
            used = _regs(rest)
            hit = used & (live(lgkm) | live(vm))
            is_lds = op.startswith("ds_")
            is_vm_load = op.startswith(_VM_LOAD)
            if hit:
                findings.append((kernel, ln, s, sorted(hit)))
            if is_lds:
                dest = _regs(rest.split(",")[0]) if op.startswith(("ds_read", "ds_load")) else set()
                lgkm.append((dest, in_asm))
            elif op.startswith(("s_load", "s_buffer_load")):
                lgkm.append((set(), False))
            elif is_vm_load:
                dest = set() if "lds" in op else _regs(rest.split(",")[0])
                vm.append((dest, in_asm))
            elif op.startswith(_VM_OTHER):
                vm.append((set(), False))
    return findings


def check_sources(sources=SOURCES, verbose: bool = True) -> list:
    found = []
    with tempfile.TemporaryDirectory() as tmp:
        for src in sources:
            out = os.path.join(tmp, src.replace(".hip", ".s"))
            assemble(src, out)
            got = check_assembly(out)
            if verbose:
                print(f"{src}: {len(got)} use(s) of a hand-issued load's registers before its wait", flush=True)
            found += [(src,) + g for g in got]
    return found


if __name__ == "__main__":
    bad = check_sources()
    for item in bad[:20]:
        print(item)
    sys.exit(1 if bad else 0)
