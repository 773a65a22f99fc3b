"""The grouped GEMM copies its token tile global memory -> LDS with an instruction
the compiler does not see (inline assembly) and waits for it with a counted
s_waitcnt: "at most N memory operations still in flight".  Memory operations
retire in order, so this is only a proof that the copies have landed if at least
N memory instructions are issued between the last copy and the wait, on a
straight-line path.  This test compiles the kernel to assembly (no GPU needed)
and checks exactly that for every such wait."""
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


def test_counted_waits_cover_the_tile_copies():
    lines = _assembly()
    # inline-assembly blocks: (first line, last line, text)
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
    copies = [b for b in blocks if "global_load_lds_dwordx4" in b[2]]
    waits = [b for b in blocks if re.search(r"s_waitcnt vmcnt\((\d+)\)", b[2])]
    assert copies and waits
    counted = 0
    for w in waits:
        n = int(re.search(r"vmcnt\((\d+)\)", w[2]).group(1))
        if n == 0:
            continue            # waits for everything: nothing to prove
        counted += 1
        prev = [c for c in copies if c[1] < w[0]]
        assert prev, "a counted wait with no tile copy before it"
        last_copy = max(prev, key=lambda c: c[1])
        issued = 0
        for k in range(last_copy[1] + 1, w[0]):
            text = lines[k].strip()
            assert not re.match(r"^\.LBB\d+_\d+:", text), "label between a tile copy and its wait (line %d)" % k
            assert not text.startswith("s_cbranch") and not text.startswith("s_branch"), \
                "branch between a tile copy and its wait (line %d)" % k
            if VMEM.match(text):
                issued += 1
        assert issued >= n, ("wait at line %d allows %d operations in flight but only %d were issued "
                             "after the last tile copy" % (w[0], n, issued))
        assert issued == n, "wait at line %d is stricter than needed (%d issued, %d allowed)" % (w[0], issued, n)
    assert counted >= 9          # 3 precisions x fragment counts x 2 projections
