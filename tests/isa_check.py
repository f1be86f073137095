"""Check of the compiled kernels for one hazard the compiler has been seen to miss.

A matrix instruction writes its result several cycles after it issues: a `v_mfma_f32_32x32x16_bf16`
(8 passes) needs 11 wait states before another kind of instruction may read its destination.  The
compiler pads straight-line code with `s_nop` accordingly, but on the taken edge of a branch that
sits between the matrix instruction and the first reader it has emitted too few (seen with a
wave-uniform `if` per score element in the decode kernel: 3 wait states, wrong scores).  This
script compiles the matrix-core kernels to assembly and walks every path of up to a dozen
instructions behind each matrix instruction, through branches and their targets; a reader reached
across a branch in fewer than 11 wait states is reported.  Matrix instructions whose result tile
lies in VGPRs are the kernels' own inline assembly, which the compiler does not pad at all: for
them a reader in fewer than 11 wait states is reported on straight-line paths as well.

A following matrix instruction counts as a reader through any of its operands: SrcA, SrcB, and
SrcC or a destination that overlaps the tile, unless it is the accumulation form (destination and
SrcC both exactly the tile), which the hardware interlocks.  A path that is still inside the hazard
window when the branch-depth limit is reached is reported too, never dropped silently.

Test and build infrastructure, not part of the product package: `__graft_entry__.build()` runs
check_all() after compiling and fails on any finding; `tests/test_isa_check.py` does the same.

    python -m tests.isa_check        # prints findings, exit status 1 if any
"""
import os
import re
import subprocess
import sys
import tempfile

from paper_2603_17484_amd.build import CSRC, FLAGS, HIPCC

KERNEL_SOURCES = ["attn_fwd_bf16.hip", "attn_bwd_dq_bf16.hip", "attn_bwd_dkdv_bf16.hip", "attn_decode_bf16.hip"]
WAIT_STATES = 11      # 8-pass matrix instruction -> read of its result by another unit
MAX_BRANCH_DEPTH = 6
DEPTH_LIMIT = "<branch depth limit reached inside the hazard window>"


def _regs(tok):
    m = re.match(r"([va])\[(\d+):(\d+)\]$", tok)
    if m:
        return {(m.group(1), i) for i in range(int(m.group(2)), int(m.group(3)) + 1)}
    m = re.match(r"([va])(\d+)$", tok)
    return {(m.group(1), int(m.group(2)))} if m else set()


def _instructions(text):
    ins = []
    for line in text.splitlines():
        s = line.split(";")[0].strip()
        if not s or (s.startswith(".") and not re.match(r"^\.LBB\d+_\d+:", s)):
            continue
        ins.append(s)
    return ins


def scan(text):
    """[(matrix instruction, reader, wait states)] for readers reached too early: across a branch, or
    anywhere behind a matrix instruction with a VGPR destination (inline assembly)."""
    ins = _instructions(text)
    label = {}
    for i, s in enumerate(ins):
        m = re.match(r"^(\.LBB\d+_\d+):", s)
        if m:
            label[m.group(1)] = i
    found = {}

    def walk(j, ws, dst, crossed, depth, origin):
        if depth >= MAX_BRANCH_DEPTH and ws < WAIT_STATES and j < len(ins):
            found.setdefault(origin, (ins[origin], DEPTH_LIMIT, ws))
            return
        while j < len(ins) and ws < WAIT_STATES:
            t = ins[j]
            if t.startswith(".LBB"):
                j += 1
                continue
            parts = t.split()
            op = parts[0]
            toks = [x.rstrip(",") for x in parts[1:]]
            if op == "s_nop":
                ws += int(toks[0]) + 1
            elif op == "s_endpgm":
                return
            elif op == "s_branch":
                j, crossed, ws = label.get(toks[0], len(ins)), True, ws + 1
                continue
            elif op.startswith("s_cbranch"):
                if toks[0] in label:
                    walk(label[toks[0]], ws + 1, dst, True, depth + 1, origin)
                ws += 1
            else:
                if op.startswith("v_mfma"):
                    d2, c2 = _regs(toks[0]), (_regs(toks[3]) if len(toks) > 3 else set())
                    if d2 == dst and c2 == dst:
                        return                      # accumulating into the same tile is interlocked
                    srcs = set().union(*[_regs(x) for x in toks[1:3]]) | c2 | d2
                else:
                    stores = op.startswith(("ds_write", "global_store", "scratch_store", "buffer_store"))
                    srcs = set().union(*[_regs(x) for k, x in enumerate(toks) if k > 0 or stores] or [set()])
                if srcs & dst:
                    if crossed or any(r[0] == "v" for r in dst):
                        found.setdefault(origin, (ins[origin], t, ws))
                    return
                if toks and _regs(toks[0]) & dst and op.startswith("v_") and not op.startswith("v_mfma"):
                    return                          # overwritten before it is read
                ws += 1
            j += 1

    for i, s in enumerate(ins):
        if s.startswith("v_mfma"):
            walk(i + 1, 0, _regs(s.split()[1].rstrip(",")), False, 0, i)
    return list(found.values())


def assembly(src):
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "k.s")
        cmd = [HIPCC] + FLAGS + ["--cuda-device-only", "-S", os.path.join(CSRC, src), "-o", out]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{r.stderr[-2000:]}")
        return open(out).read()


def check_all():
    return {src: scan(assembly(src)) for src in KERNEL_SOURCES}


if __name__ == "__main__":
    bad = 0
    for src, hits in check_all().items():
        print(src, "ok" if not hits else f"{len(hits)} reader(s) too early")
        for mfma, reader, ws in hits:
            print(f"    {mfma[:70]}\n      -> {reader[:70]}   after {ws} wait states")
        bad += len(hits)
    sys.exit(1 if bad else 0)
