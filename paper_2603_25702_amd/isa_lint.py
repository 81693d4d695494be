"""Build-time check of the compiled gfx950 code: no matrix instruction under a narrowed execution mask.

`v_mfma_*` ignores EXEC.  A source-level `if (cond) acc = mfma(...)` whose condition lives in a vector
register is compiled to an execution-mask region (`s_and_saveexec_b64` ... `s_or_b64 exec`); the compiler
normally jumps over the region when no lane is left (`s_cbranch_execz`), but drops that jump when the region is
short and holds nothing it considers unsafe to run with an empty mask, and MFMA is not on that list.  The
region's MFMAs then run although the condition is false for the whole wavefront.  The kernels avoid this by
deriving every condition that guards an MFMA from scalars (`__builtin_amdgcn_readfirstlane` of the wavefront
index), which gives scalar branches; this module checks the result on the emitted assembly.

    python -m paper_2603_25702_amd.isa_lint          # compiles csrc/*.hip to assembly and scans it
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor
from typing import List, Tuple

from .build import CSRC, FLAGS, SOURCES, _hipcc

_NARROW = re.compile(r"^s_(and|andn2|or|xor|nand|nor|xnor|orn2)_saveexec_b64\b")
_EXEC_WRITE = re.compile(r"^s_(and|andn2|xor|mov)_b64\s+exec\b")
_EXEC_RESTORE = re.compile(r"^s_or_b64\s+exec\b")
_KERNEL = re.compile(r"^(_Z\w+):")


def scan_asm(text: str) -> List[Tuple[str, int, str]]:
    """Returns (kernel, line number, instruction) for every MFMA that follows a narrowing of EXEC with no
    `s_cbranch_execz` in between, up to the point where EXEC is widened again or control leaves the block."""
    kernel, narrowed, guarded = "?", False, False
    found = []
    for no, raw in enumerate(text.splitlines(), 1):
        m = _KERNEL.match(raw)
        if m:
            kernel, narrowed = m.group(1), False
        ins = raw.split(";")[0].strip()
        if not ins or ins.startswith("."):
            continue
        if _NARROW.match(ins) or _EXEC_WRITE.match(ins):
            narrowed, guarded = True, False
        elif _EXEC_RESTORE.match(ins) or ins.startswith(("s_branch", "s_endpgm")):
            narrowed = False
        elif ins.startswith("s_cbranch_execz") and narrowed:
            guarded = True
        elif ins.startswith(("v_mfma", "v_smfmac")) and narrowed and not guarded:
            found.append((kernel, no, ins))
    return found


def compile_to_asm(src: str, out_dir: str) -> str:
    out = os.path.join(out_dir, src.replace(".hip", ".s"))
    flags = [f for f in FLAGS if f != "-fPIC"]
    cmd = [_hipcc(), *flags, "--cuda-device-only", "-S", os.path.join(CSRC, src), "-o", out]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc -S failed on {src}:\n{r.stderr}")
    return out


def lint_sources(sources=None, jobs: int = 6) -> List[Tuple[str, str, int, str]]:
    sources = [s for s in (sources or SOURCES)
               if "mfma" in open(os.path.join(CSRC, s)).read() or s in ("attention.hip", "attention_wide.hip")]
    with tempfile.TemporaryDirectory() as tmp:
        with ThreadPoolExecutor(max_workers=jobs) as ex:
            paths = list(ex.map(lambda s: compile_to_asm(s, tmp), sources))
        found = []
        for src, path in zip(sources, paths):
            found += [(src, k, no, ins) for k, no, ins in scan_asm(open(path).read())]
    return found


if __name__ == "__main__":
    bad = lint_sources()
    for src, k, no, ins in bad:
        print(f"{src}: {k}: line {no}: {ins}")
    print(f"{len(bad)} matrix instruction(s) under a narrowed execution mask without a skip branch")
    sys.exit(1 if bad else 0)
