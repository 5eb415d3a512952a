"""Host-side check of the compiled packed-operand contraction kernel (gemm_pk_k).

Its weight fragments are loaded by inline-assembly buffer loads whose data arrive later; the wait that makes a
fragment valid is another inline-assembly statement, placed by hand in front of the fragment's first product.  The
compiler takes the registers for defined from the load on, so when registers are short it may copy them (into
accumulator registers, to scratch) between load and wait, and the copy holds what had not arrived.  This script
reads the gfx950 assembly of gemm.hip and reports every instruction that reads the destination registers of such a
load before the first MFMA that consumes them (or a wait for all loads).  Used by the CPU test suite.
"""
from __future__ import annotations

import os
import re
import subprocess
import tempfile

from .build import CSRC, FLAGS

_KERNEL = re.compile(r"^(_ZN4hift12_GLOBAL__N_19gemm_pk_k\w+):")


def _regs(tok: str) -> set:
    m = re.match(r"v\[(\d+):(\d+)\]", tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.match(r"v(\d+)$", tok)
    return {int(m.group(1))} if m else set()


def device_assembly(source: str = "gemm.hip") -> str:
    """gfx950 assembly text of one source of the library, compiled with the library's flags."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    with tempfile.TemporaryDirectory() as d:
        out = os.path.join(d, "dev.s")
        subprocess.run([hipcc, *FLAGS, "--cuda-device-only", "-S", os.path.join(CSRC, source), "-o", out], check=True,
                       stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
        with open(out) as f:
            return f.read()


def early_reads_of_async_loads(asm: str) -> dict:
    """{kernel symbol: (asynchronous fragment loads found, [(load, offending instruction), ...])}."""
    lines = asm.split("\n")
    result = {}
    starts = [(i, _KERNEL.match(l).group(1)) for i, l in enumerate(lines) if _KERNEL.match(l)]
    for i, name in starts:
        end = next(x for x in range(i, len(lines)) if lines[x].startswith(".Lfunc_end"))
        body = [l.strip() for l in lines[i:end]]
        loads, bad = 0, []
        for x, l in enumerate(body):
            if not (l.startswith("buffer_load_dwordx4") and " lds" not in l and "offen" in l):
                continue
            dst = _regs(l[len("buffer_load_dwordx4"):].split(",")[0].strip())
            if len(dst) != 4:
                continue
            loads += 1
            for m in body[x + 1:x + 1500]:
                if not m or m[0] in ";." or m.endswith(":"):
                    continue
                parts = m.split(None, 1)
                if len(parts) < 2:
                    continue
                op, toks = parts[0], [t.strip() for t in parts[1].split(",")]
                if op == "s_waitcnt" and "vmcnt(0)" in m:
                    break
                if op.startswith(("s_cbranch", "s_branch")) or op == "s_endpgm":
                    break
                stores = op.startswith(("buffer_store", "global_store", "scratch_store", "ds_write", "ds_store"))
                srcs = set()
                for t in (toks if stores else toks[1:]):
                    if t:
                        srcs |= _regs(t.split()[0])
                if op.startswith("v_mfma"):
                    if srcs & dst:
                        break  # consumed by its product, behind the hand-placed wait
                    continue
                if srcs & dst:
                    bad.append((l, m))
                    break
                if toks and toks[0] and _regs(toks[0].split()[0]) & dst and not op.startswith("s_"):
                    break  # overwritten
        result[name] = (loads, bad)
    return result
