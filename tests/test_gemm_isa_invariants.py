"""The grouped GEMM copies its token tile global memory -> LDS with an instruction
the compiler does not see (inline assembly) and waits for it with a counted
s_waitcnt: "at most N memory operations still in flight".  Memory operations
retire in order, so this is only a proof that the copies have landed if at least
N memory instructions are issued between the last copy and the wait.  This test
compiles the kernel to assembly (no GPU needed) and checks, for every K loop,
that the body is one straight-line block, that the memory instructions on the
path from the last copy to the wait (within one trip, or over the back edge when
the copies follow the wait) are exactly N, and that a wait for everything
precedes the loop (the copies issued before the loop are waited for there)."""
import os
import re
import shutil
import subprocess
import tempfile

import pytest

from paper_2603_19172_amd import build as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2603_19172_amd", "csrc", "ffn_gemm.hip")

VMEM = re.compile(r"^\s*(global_|buffer_|flat_|scratch_)(load|store|atomic)")


def _assembly():
    if shutil.which("hipcc") is None:
        pytest.skip("hipcc not found")
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "ffn_gemm.s")
        # the flags the library is built with
        cmd = ["hipcc", *B.COMMON, *B.PER_FILE.get("ffn_gemm.hip", []), "-S", "--cuda-device-only", SRC, "-o", out]
        subprocess.run(cmd, check=True, capture_output=True)
        with open(out) as f:
            return f.read().split("\n")


def _blocks(lines):
    """inline-assembly blocks: (first line, last line, text)"""
    blocks = []
    i = 0
    while i < len(lines):
        if "#ASMSTART" in lines[i]:
            j = i
            while "#ASMEND" not in lines[j]:
                j += 1
            blocks.append((i, j, " ".join(l.strip() for l in lines[i + 1:j])))
            i = j
        i += 1
    return blocks


def _vmem_between(lines, first, last, asm_lines):
    """compiler-issued memory instructions on lines [first, last], which must be straight-line code"""
    n = 0
    for k in range(first, last + 1):
        if k in asm_lines:
            continue
        text = lines[k].strip()
        assert not re.match(r"^\.LBB\d+_\d+:", text), "label inside the loop body (line %d)" % k
        assert not text.startswith("s_cbranch") and not text.startswith("s_branch"), \
            "branch inside the loop body (line %d)" % k
        if VMEM.match(text):
            n += 1
    return n


def test_counted_waits_cover_the_tile_copies():
    lines = _assembly()
    blocks = _blocks(lines)
    asm_lines = set()
    for b in blocks:
        asm_lines.update(range(b[0], b[1] + 1))
    copies = [b for b in blocks if "global_load_lds_dwordx4" in b[2]]
    waits = [(b, int(re.search(r"s_waitcnt vmcnt\((\d+)\)", b[2]).group(1)))
             for b in blocks if re.search(r"s_waitcnt vmcnt\((\d+)\)", b[2])]
    assert copies and waits
    labels = {}
    for i, l in enumerate(lines):
        m = re.match(r"^(\.LBB\d+_\d+):", l)
        if m:
            labels[m.group(1)] = i
    checked = 0
    seen = set()
    for i, l in enumerate(lines):
        m = re.search(r"s_cbranch_\w+\s+(\.LBB\d+_\d+)", l)
        if not m or m.group(1) not in labels or labels[m.group(1)] > i:
            continue
        head, tail = labels[m.group(1)], i             # a loop: head label .. backward branch
        if any(head < v < tail for v in labels.values()):
            continue                                   # not an innermost loop (code layout of the dispatch)
        in_copies = [c for c in copies if head < c[0] < tail]
        in_waits = [w for w in waits if head < w[0][0] < tail]
        if not in_copies:
            continue
        assert len(in_waits) == 1, "K loop at line %d: expected one counted wait" % head
        (w, n) = in_waits[0]
        assert n > 0
        last_copy = max(in_copies, key=lambda c: c[1])
        if all(c[1] < w[0] for c in in_copies):
            # copies first, wait later in the same trip
            issued = _vmem_between(lines, last_copy[1] + 1, w[0] - 1, asm_lines)
        else:
            # all copies of the body come after the wait; their wait is the next trip's
            assert all(c[0] > w[1] for c in in_copies), "K loop at line %d: copies on both sides of the wait" % head
            issued = (_vmem_between(lines, last_copy[1] + 1, tail - 1, asm_lines)
                      + _vmem_between(lines, head + 1, w[0] - 1, asm_lines))
        _vmem_between(lines, head + 1, tail - 1, asm_lines)      # the whole body is straight-line code
        assert issued >= n, ("K loop at line %d: the wait allows %d operations in flight but only %d are "
                             "issued between the last copy and the wait" % (head, n, issued))
        assert issued == n, "K loop at line %d: wait stricter than needed (%d issued, %d allowed)" % (head, issued, n)
        # entering the loop: the nearest wait before the head waits for everything
        before = [x for x in waits if x[0][1] < head]
        assert before and max(before, key=lambda x: x[0][1])[1] == 0, \
            "K loop at line %d is entered without a wait for the copies issued before it" % head
        checked += 1
        seen.update(c[0] for c in in_copies)
    # copies outside the K loops (the first two tiles): a wait for everything
    # stands between them and the next workgroup barrier
    for c in copies:
        if c[0] in seen:
            continue
        k = c[1] + 1
        waited = False
        while "s_barrier" not in lines[k]:
            if k in asm_lines and "s_waitcnt vmcnt(0)" in lines[k]:
                waited = True
            k += 1
        assert waited, "copy at line %d reaches a barrier without a wait for everything" % c[0]
    assert checked >= 32         # 4 precisions x 4 fragment counts x 2 projections
