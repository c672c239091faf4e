"""A check of the compiler's output for one code-generation fault that wrong results were traced to.

When a kernel needs more vector registers than its launch bounds allow, hipcc spills some to scratch
memory.  A spill store is a vector store like any other: it writes only the lanes that the exec mask
enables.  In one build of the scan kernel the compiler put the store of a value that every lane
needs later (the target side's scale factor) into a stretch of code that runs with the mask narrowed
to a few lanes (between an `s_and_saveexec_b64` and the `s_or_b64 exec, exec, ...` that ends it, with
no branch around it, so the stretch is on every wavefront's path).  The other lanes later reloaded
whatever their scratch slot happened to hold, and the target-side argmin of about half the rows
came out wrong; the parity tests caught it.  That build was avoided by giving the variant more
registers, but nothing keeps the compiler from doing the same elsewhere after an unrelated change,
so the generated assembly of every kernel is searched for the pattern:

    a spill store (`scratch_store_* ... Folded Spill`) that is reached, within its straight-line
    stretch of code, after an instruction that narrows exec and before one that widens it again,
    for a register that is not written between the narrowing and the store.

A register written after the narrowing holds a value made by the enabled lanes for themselves, which
is fine; one written before it may be needed by lanes that the store then misses.

`python -m paper_2506_05632_amd.audit` compiles the device side of every source to assembly (about
15 s per file, no GPU needed) and lists what it finds; `tests/test_build_audit.py` runs the same.
"""
import os
import re
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

from .build import CSRC, FLAGS, SOURCES, _hipcc

_LABEL = re.compile(r"^(\.LBB\d+_\d+|_Z\w+|\w+):")
_NARROW = re.compile(r"^(s_\w+_saveexec_b64\b|s_mov_b64 exec,|s_and_b64 exec,|s_andn2_b64 exec,)")
_WIDEN = re.compile(r"^s_or_b64 exec, exec,")
_SPILL = re.compile(r"^scratch_store_\w+\s+off, (v\[(\d+):(\d+)\]|v(\d+)), .*Folded Spill")
_WRITES = re.compile(r"^(?:v_\w+|ds_read\w*|ds_bpermute\w*|global_load\w*|scratch_load\w*|buffer_load\w*|flat_load\w*)\s+"
                     r"(?:v\[(\d+):(\d+)\]|v(\d+))")


def _span(lo, hi, single):
    if single is not None:
        return set([int(single)])
    return set(range(int(lo), int(hi) + 1))


def spill_stores_under_narrowed_exec(asm: str):
    """[(kernel, line number, the narrowing instruction, the store)] for every match of the pattern."""
    found = []
    lines = asm.split("\n")
    kernel = ""
    for i, raw in enumerate(lines):
        m = re.match(r"^(_Z\w+):", raw)
        if m:
            kernel = m.group(1)
        t = raw.strip()
        s = _SPILL.match(t)
        if not s:
            continue
        regs = _span(s.group(2), s.group(3), s.group(4))
        written = False
        for k in range(i - 1, -1, -1):
            u = lines[k].strip()
            if _LABEL.match(u) or _WIDEN.match(u):
                break  # another stretch, or the mask is whole again before the store
            if _NARROW.match(u):
                if not written:
                    found.append((kernel, i + 1, u, t))
                break
            w = _WRITES.match(u)
            if w and regs & _span(w.group(1), w.group(2), w.group(3)):
                written = True
    return found


def device_assembly(source: str, out_dir: str) -> str:
    """Compile the device side of csrc/<source> to assembly with the build's flags; returns the text."""
    out = os.path.join(out_dir, source.replace(".hip", ".s"))
    cmd = [_hipcc(), *[f for f in FLAGS if f not in ("-fPIC", "-Wall")], "--cuda-device-only", "-S",
           os.path.join(CSRC, source), "-o", out]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + r.stderr)
    with open(out) as fh:
        return fh.read()


def audit(sources=tuple(SOURCES) + ("probe.hip",), workers: int = 6):
    """{source: findings} over the sources of both libraries (only those with findings)."""
    with tempfile.TemporaryDirectory() as tmp:
        def one(src):
            return src, spill_stores_under_narrowed_exec(device_assembly(src, tmp))
        with ThreadPoolExecutor(max_workers=workers) as ex:
            return {src: f for src, f in ex.map(one, sources) if f}


if __name__ == "__main__":
    bad = audit()
    for src, findings in bad.items():
        for kernel, line, narrowing, store in findings:
            print(f"{src}: {kernel} line {line}: after `{narrowing}`: {store}")
    print("no spill store under a narrowed exec mask" if not bad else f"{sum(map(len, bad.values()))} finding(s)")
    sys.exit(1 if bad else 0)
