"""Static check of the split attention kernels' machine code (developer tool; nothing at run time uses it).

attn_mfma_kernel issues its query loads from inline assembly (csrc/decode_mfma.hip), so the compiler takes the
destination registers for valid at once although the data lands later.  That is safe only while the compiled
code never copies such a register (to an AGPR, another VGPR or scratch) between the load and the kernel's first
MFMA, i.e. before the loop's first wait.  This script compiles csrc/decode_mfma.hip to assembly for gfx950 and
lists every instantiation in which it finds such a copy.

    python -m paper_2503_01586_amd.check_inflight_registers            # compile (about three minutes) and scan
    python -m paper_2503_01586_amd.check_inflight_registers file.s     # scan an existing assembly file

Copies to AGPRs and scratch are reported as errors (exit status 1).  Plain VGPR moves are listed as notes: the
scan follows the text, not the control flow, and the block that finishes the newest token's cache row (fused
decode step, executed before the query is requested) lies behind the other path's query loads in the text and
moves its own temporaries.
"""
from __future__ import annotations

import collections
import os
import re
import subprocess
import sys
import tempfile

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
HARD = ("v_accvgpr_write", "v_accvgpr_mov", "scratch_store")
SOFT = ("v_mov_b32", "v_mov_b64", "v_pk_mov")


def _regs(tok: str) -> set:
    tok = re.sub(r"\s.*", "", tok.strip())
    m = re.match(r"v\[(\d+):(\d+)\]", tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.match(r"v(\d+)$", tok)
    return {int(m.group(1))} if m else set()


def scan(path: str):
    kernels, cur = collections.OrderedDict(), None
    for ln in open(path):
        m = re.match(r"^(_ZN3ekv16attn_mfma_kernel\S+):", ln)
        if m:
            cur = m.group(1)
            kernels[cur] = []
        elif cur is not None:
            if ln.startswith(".Lfunc_end"):
                cur = None
            else:
                kernels[cur].append(ln.rstrip("\n"))
    errors, notes = [], []
    for name, lines in kernels.items():
        first_mfma = next((i for i, ln in enumerate(lines) if ln.strip().startswith("v_mfma")), len(lines))
        live = set()
        for ln in lines[:first_mfma]:
            s = ln.strip()
            if not s or s[0] in ";.":
                continue
            op = s.split()[0]
            ops = s[len(op):].split(",")
            if op == "global_load_dwordx4":          # the hand-issued query loads (tile loads are global_load_lds_*)
                live |= _regs(ops[0])
            elif op.startswith(HARD) or op.startswith(SOFT):
                src = set().union(*[_regs(t) for t in (ops if op.startswith("scratch_store") else ops[1:])])
                if src & live:
                    (errors if op.startswith(HARD) else notes).append((name, s))
    return kernels, errors, notes


def main(argv):
    if len(argv) > 1:
        asm = argv[1]
    else:
        spec_path = os.path.join(PKG_DIR, "build.py")
        import importlib.util
        spec = importlib.util.spec_from_file_location("_elitekv_build", spec_path)
        build = importlib.util.module_from_spec(spec)
        spec.loader.exec_module(build)
        asm = os.path.join(tempfile.mkdtemp(prefix="ekv_isa_"), "decode_mfma.s")
        cmd = [build.HIPCC, *build.FLAGS, "--cuda-device-only", "-S", os.path.join(build.CSRC, "decode_mfma.hip"), "-o", asm]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            sys.stderr.write(res.stderr)
            return 2
    kernels, errors, notes = scan(asm)
    short = lambda n: n.replace("_ZN3ekv16attn_mfma_kernelI", "<").replace("EEEvNS_14AttnMfmaParamsE", ">")
    by = collections.Counter(n for n, _ in errors)
    for n, c in by.items():
        print("ERROR %s: %d copies of registers of in-flight loads, e.g. %s" % (short(n), c, next(s for m, s in errors if m == n)))
    for n, c in collections.Counter(n for n, _ in notes).items():
        print("note  %s: %d VGPR moves to look at, e.g. %s" % (short(n), c, next(s for m, s in notes if m == n)))
    print("%d instantiations scanned, %d with copies to AGPRs or scratch" % (len(kernels), len(by)))
    return 1 if errors else 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
