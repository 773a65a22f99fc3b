"""Host-side checks of libdymoe.so that need no GPU: the library loads, exports
every symbol the header declares, validates arguments before touching the
device, and its host-side depth schedule agrees with the paper's closed forms."""
import ctypes as C
import os
import re

import pytest

from oracle import dymoe_oracle as O
from paper_2603_19172_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
P = 0x10000  # a non-null, 64 KiB aligned dummy "pointer"; never dereferenced by validation


def test_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "dymoe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(dymoe_[a-z0-9_]+)\s*\(", text))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(B.lib, name), name


def test_strerror_and_workspace():
    assert B.strerror(0) == "success"
    for code in (-1, -2, -3, -4, -5):
        assert B.strerror(code) and "unknown" not in B.strerror(code)
    assert "unknown" in B.strerror(-99)
    assert B.workspace_bytes(0, 0, 0, 0, 0) == 0
    assert B.workspace_bytes(4, 256, 512, 8, 9) == 0
    small = B.workspace_bytes(16, 256, 512, 8, 2)
    big = B.workspace_bytes(512, 4096, 14336, 8, 2)
    assert 0 < small < big and big % 256 == 0
    # holds the fp32 intermediate of every (token, expert) pair
    assert big >= 512 * 2 * 14336 * 4


def test_depth_schedule_matches_golden_and_oracle():
    for line in open(os.path.join(ROOT, "tests", "golden", "schedule_tables.txt")):
        if line.startswith("#") or not line.strip():
            continue
        f = line.split()
        L, M, lam = int(f[0]), int(f[1]), float(f[2])
        assert [B.depth_schedule(l, L, lam, M) for l in range(L)] == [int(v) for v in f[3:]]
    for L in (1, 2, 7, 32, 48):
        for M in (8, 60, 128):
            for lam in (0.0, 0.3, 0.5, 0.75, 0.8, 1.0):
                for l in range(L):
                    assert B.depth_schedule(l, L, lam, M) == O.depth_schedule(l, L, lam, M)
    assert B.depth_schedule(4, 4, 0.5, 8) == B.EINVAL
    assert B.depth_schedule(0, 4, -0.1, 8) == B.EINVAL
    assert B.depth_schedule(0, 0, 0.5, 8) == B.EINVAL
    assert B.depth_schedule(0, 4, 0.5, 0) == B.EINVAL
    # mean retained fraction over the stack is (1 + lambda)/2 up to the ceilings
    L, M = 32, 128
    mean = sum(B.depth_schedule(l, L, 0.5, M) for l in range(L)) / (L * M)
    assert 0.75 <= mean < 0.75 + 1.0 / M


def test_argument_validation_happens_before_any_device_work():
    lib = B.lib
    # route: valid arguments but no context -> ENOCTX; bad ones -> EINVAL / ENOTSUP first
    assert lib.dymoe_route_topk(None, P, P, None, 4, 256, 8, 2, 1, P, P, P, None) == B.ENOCTX
    assert lib.dymoe_route_topk(None, None, P, None, 4, 256, 8, 2, 1, P, P, P, None) == B.EINVAL
    assert lib.dymoe_route_topk(None, P, P, None, 4, 256, 8, 9, 1, P, P, P, None) == B.EINVAL
    assert lib.dymoe_route_topk(None, P, P, None, 4, 252, 8, 2, 1, P, P, P, None) == B.EINVAL
    assert lib.dymoe_route_topk(None, P + 2, P, None, 4, 256, 8, 2, 1, P, P, P, None) == B.EINVAL
    assert lib.dymoe_route_topk(None, P, P, None, 4, 256, 2048, 2, 1, P, P, P, None) == B.ENOTSUP
    assert lib.dymoe_token_score_norm(None, P, 4, 256, P, None) == B.ENOCTX
    assert lib.dymoe_token_score_norm(None, P, 4, 250, P, None) == B.EINVAL
    # importance
    assert lib.dymoe_expert_importance(None, 0, P, None, P, 16, 8, 2, 3, P, P, None) == B.ENOCTX
    assert lib.dymoe_expert_importance(None, 0, P, None, None, 16, 8, 2, 3, P, P, None) == B.EINVAL
    assert lib.dymoe_expert_importance(None, 0, P, None, P, 16, 8, 2, 17, P, P, None) == B.EINVAL
    assert lib.dymoe_expert_importance(None, 1, P, None, None, 1, 8, 2, 0, P, P, None) == B.EINVAL
    assert lib.dymoe_expert_importance(None, 7, P, P, P, 1, 8, 2, 0, P, P, None) == B.EINVAL
    # assignment: host tier tables are read during validation
    tc = (C.c_int32 * 3)(2, 3, 3)
    tb = (C.c_uint8 * 3)(16, 4, 2)
    tcp, tbp = C.cast(tc, C.c_void_p), C.cast(tb, C.c_void_p)
    assert lib.dymoe_assign_precision(None, 0, P, P, 8, 3, tcp, tbp, 0, P, P, None) == B.ENOCTX
    assert lib.dymoe_assign_precision(None, 0, P, P, 9, 3, tcp, tbp, 0, P, P, None) == B.EINVAL
    assert lib.dymoe_assign_precision(None, 0, P, P, 8, 3, tcp, tbp, 3, P, P, None) == B.EINVAL
    bad = (C.c_uint8 * 3)(16, 5, 2)
    assert lib.dymoe_assign_precision(None, 0, P, P, 8, 3, tcp, C.cast(bad, C.c_void_p), 0, P, P, None) == B.EINVAL
    assert lib.dymoe_assign_precision(None, 0, P, P, 8, 9, tcp, tbp, 0, P, P, None) == B.EINVAL
    # quantize
    assert lib.dymoe_quantize_pack(None, P, 8, 256, 4, 64, P, P, P, None) == B.ENOCTX
    assert lib.dymoe_quantize_pack(None, P, 8, 256, 8, 64, P, P, P, None) == B.ENOCTX
    assert lib.dymoe_quantize_pack(None, P, 8, 256, 3, 64, P, P, P, None) == B.EINVAL
    assert lib.dymoe_quantize_pack(None, P, 8, 200, 4, 64, P, P, P, None) == B.EINVAL
    assert lib.dymoe_quantize_pack(None, P, 8, 256, 4, 32, P, P, P, None) == B.ENOTSUP
    assert lib.dymoe_quantize_pack(None, P + 8, 8, 256, 4, 64, P, P, P, None) == B.EINVAL
    assert lib.dymoe_quantize_experts(None, P, P, None, 8, 256, 512, 64, 0, None) == B.ENOCTX
    assert lib.dymoe_quantize_experts(None, P, P, None, 8, 256, 512, 64, 1, None) == B.ENOCTX
    assert lib.dymoe_quantize_experts(None, P, P, None, 8, 250, 512, 64, 0, None) == B.EINVAL
    assert lib.dymoe_quantize_experts(None, P, P, None, 8, 256, 512, 64, 2, None) == B.EINVAL
    assert lib.dymoe_quantize_experts(None, P, P, None, 8, 192, 512, 64, 1, None) == B.EINVAL   # tiles need multiples of 128
    assert lib.dymoe_pack_tiles(None, P, 64, 256, 2 * P, None) == B.ENOCTX
    assert lib.dymoe_pack_tiles(None, P, 48, 256, 2 * P, None) == B.EINVAL
    assert lib.dymoe_pack_tiles(None, P, 64, 192, 2 * P, None) == B.EINVAL
    assert lib.dymoe_pack_tiles(None, P, 64, 256, P, None) == B.EINVAL                          # in place
    pc = lib.dymoe_pack_code_tiles
    assert pc(None, P, P, P, 64, 256, 4, 2 * P, 2 * P, 2 * P, None) == B.ENOCTX
    assert pc(None, P, P, P, 48, 256, 4, 2 * P, 2 * P, 2 * P, None) == B.EINVAL
    assert pc(None, P, P, P, 64, 192, 4, 2 * P, 2 * P, 2 * P, None) == B.EINVAL
    assert pc(None, P, P, P, 64, 256, 3, 2 * P, 2 * P, 2 * P, None) == B.EINVAL
    assert pc(None, P, P, P, 64, 256, 4, P, 2 * P, 2 * P, None) == B.EINVAL                     # in place
    # fused decode front end
    df = lib.dymoe_decode_front
    assert df(None, P, P, None, 1, 256, 8, 2, 1, 3, tcp, tbp, 0, P, P, P, P, P, P, P, None) == B.ENOCTX
    assert df(None, P, P, None, 0, 256, 8, 2, 1, 3, tcp, tbp, 0, P, P, P, P, P, P, P, None) == B.EINVAL
    assert df(None, P, P, None, B.FRONT_MAX_TOKENS + 1, 256, 8, 2, 1, 3, tcp, tbp, 0, P, P, P, P, P, P, P, None) == B.EINVAL
    assert df(None, P, P, None, 1, 256, 9, 2, 1, 3, tcp, tbp, 0, P, P, P, P, P, P, P, None) == B.EINVAL   # tiers sum to 8
    assert df(None, P, P, None, 1, 256, 8, 2, 1, 3, tcp, tbp, 3, P, P, P, P, P, P, P, None) == B.EINVAL
    assert df(None, P, P, None, 1, 256, 8, 2, 1, 3, tcp, tbp, 0, P, P, None, P, P, P, None, None) == B.ENOCTX  # probs, rank optional
    assert df(None, P, P, None, 1, 256, 8, 2, 1, 3, tcp, tbp, 0, P, P, P, None, P, P, P, None) == B.EINVAL
    # attention-derived token score
    ta = lib.dymoe_token_score_attention
    aw = int(lib.dymoe_attention_workspace_bytes(77, 8))
    assert aw >= 77 * 8 * 12 and aw % 256 == 0 and lib.dymoe_attention_workspace_bytes(0, 8) == 0
    assert ta(None, P, P, 77, 8, 2, 128, 0.0, 1, P, P, aw, None) == B.ENOCTX
    assert ta(None, P, P, 77, 8, 2, 128, 0.0, 1, P, P, aw - 1, None) == B.ENOSPC
    assert ta(None, P, P, 77, 8, 3, 128, 0.0, 1, P, P, aw, None) == B.EINVAL          # heads not a multiple of kv heads
    assert ta(None, P, P, 77, 8, 2, 96, 0.0, 1, P, P, aw, None) == B.ENOTSUP
    assert ta(None, P, P, 77, 8, 2, 100, 0.0, 1, P, P, aw, None) == B.EINVAL
    assert ta(None, P, P, 77, 8, 2, 128, -1.0, 1, P, P, aw, None) == B.EINVAL
    assert ta(None, P, P, 77, 8, 2, 128, 0.0, 2, P, P, aw, None) == B.EINVAL
    assert ta(None, P + 2, P, 77, 8, 2, 128, 0.0, 1, P, P, aw, None) == B.EINVAL
    assert ta(None, P, P, 77, 8, 2, 128, 0.0, 1, None, P, aw, None) == B.EINVAL
    assert ta(None, None, None, 0, 8, 2, 128, 0.0, 1, None, None, 0, None) == B.ENOCTX   # T = 0 needs only a context
    # error-compensated quantizer
    gq = lib.dymoe_gptq_quantize_pack
    gw = int(lib.dymoe_gptq_workspace_bytes(100, 256))
    assert gw >= 100 * 256 * 4 + 64 * 128 * 4 and gw % 256 == 0 and lib.dymoe_gptq_workspace_bytes(0, 256) == 0
    assert gq(None, P, P, 100, 256, 4, 64, P, P, P, P, gw, None) == B.ENOCTX
    assert gq(None, P, P, 100, 256, 4, 64, P, P, P, P, gw - 1, None) == B.ENOSPC
    assert gq(None, P, P, 100, 256, 3, 64, P, P, P, P, gw, None) == B.EINVAL
    assert gq(None, P, P, 100, 250, 4, 64, P, P, P, P, gw, None) == B.EINVAL
    assert gq(None, P, P, 100, 256, 4, 32, P, P, P, P, gw, None) == B.EINVAL
    assert gq(None, P, None, 100, 256, 4, 64, P, P, P, P, gw, None) == B.EINVAL
    assert gq(None, P, P + 4, 100, 256, 4, 64, P, P, P, P, gw, None) == B.EINVAL
    assert gq(None, P, P, 100, 256, 4, 64, P, P, P, P + 16, gw, None) == B.EINVAL     # workspace alignment
    gh = lib.dymoe_gptq_hessian
    assert gh(None, P, 300, 256, 0, P, None) == B.ENOCTX
    assert gh(None, P, 300, 250, 0, P, None) == B.EINVAL
    assert gh(None, P, 0, 256, 0, P, None) == B.EINVAL
    assert gh(None, P, 300, 256, 2, P, None) == B.EINVAL
    assert gh(None, P, 300, 256, 0, None, None) == B.EINVAL
    gf = lib.dymoe_gptq_factor
    fw = int(lib.dymoe_gptq_factor_workspace_bytes(256))
    assert fw >= 2 * 256 * 256 * 4 + 64 * 256 * 4 and lib.dymoe_gptq_factor_workspace_bytes(0) == 0
    assert gf(None, P, 256, 0.01, 2 * P, P, fw, None) == B.ENOCTX
    assert gf(None, P, 256, 0.01, 2 * P, P, fw - 1, None) == B.ENOSPC
    assert gf(None, P, 200, 0.01, 2 * P, P, fw, None) == B.EINVAL
    assert gf(None, P, 256, -1.0, 2 * P, P, fw, None) == B.EINVAL
    assert gf(None, P, 256, 0.01, P, P, fw, None) == B.EINVAL                           # in place
    # stream copy
    assert lib.dymoe_stream_copy(None, P, 2 * P, 1024, None) == B.ENOCTX
    assert lib.dymoe_stream_copy(None, P, 2 * P, 1000, None) == B.EINVAL
    assert lib.dymoe_stream_copy(None, P + 4, 2 * P, 1024, None) == B.EINVAL
    assert lib.dymoe_stream_copy(None, None, 2 * P, 1024, None) == B.EINVAL
    assert lib.dymoe_stream_copy(None, None, None, 0, None) == B.OK
    # ffn
    ws = B.workspace_bytes(16, 256, 512, 8, 2)
    ffn = lib.dymoe_moe_ffn_mixed
    assert ffn(None, P, P, P, P, P, 16, 256, 512, 8, 2, 64, 0, 0, P, P, ws, None) == B.ENOCTX
    assert ffn(None, P, P, P, P, P, 16, 256, 512, 8, 2, 64, 0, 0, P, P, ws - 1, None) == B.ENOSPC
    assert ffn(None, P, P, P, P, P, 16, 256, 512, 8, 2, 64, 5, 0, P, P, ws, None) == B.EINVAL
    assert ffn(None, P, P, P, P, P, 16, 256, 512, 8, 2, 64, 0, 7, P, P, ws, None) == B.EINVAL
    assert ffn(None, P, P, P, P, None, 16, 256, 512, 8, 2, 64, 0, 0, P, P, ws, None) == B.EINVAL
    assert ffn(None, P, P, P, P, P, 16, 256, 500, 8, 2, 64, 0, 0, P, P, ws, None) == B.EINVAL
    # shapes the MFMA path cannot take when it is asked for explicitly
    ws2 = B.workspace_bytes(16, 192, 512, 8, 2)
    assert ffn(None, P, P, P, P, P, 16, 192, 512, 8, 2, 64, 0, 2, P, P, ws2, None) == B.ENOTSUP
    assert ffn(None, P, P, P, P, P, 16, 192, 512, 8, 2, 64, 0, 0, P, P, ws2, None) == B.ENOCTX
    # more tiles than a grid's y dimension holds: refused before anything is launched (H = F = 128, 2 M tokens x 4)
    big = B.workspace_bytes(1 << 21, 128, 128, 8, 4)
    assert ffn(None, P, P, P, P, P, 1 << 21, 128, 128, 8, 4, 64, 0, 2, P, P, big, None) == B.ENOTSUP
    # the form with the static scratch: same checks, and a fixed capacity instead of a workspace size
    ffn_na = lib.dymoe_moe_ffn_mixed_noalloc
    assert ffn_na(None, P, P, P, P, P, 16, 256, 512, 8, 2, 64, 0, 0, P, None) == B.ENOCTX
    assert ffn_na(None, P, P, P, P, P, 16, 256, 512, 8, 2, 64, 5, 0, P, None) == B.EINVAL
    assert ffn_na(None, P, P, P, None, P, 16, 256, 512, 8, 2, 64, 0, 0, P, None) == B.EINVAL
    assert B.workspace_bytes(16, 4096, 14336, 8, 2) <= B.STATIC_SCRATCH_BYTES < B.workspace_bytes(512, 4096, 14336, 8, 2)
    assert ffn_na(None, P, P, P, P, P, 16, 4096, 14336, 8, 2, 64, 0, 0, P, None) == B.ENOCTX
    assert ffn_na(None, P, P, P, P, P, 512, 4096, 14336, 8, 2, 64, 0, 0, P, None) == B.ENOSPC


def test_format_presence_test_the_kernels_apply_to_a_table_entry():
    """The kernels run an expert at b bits only if its table entry holds every pointer of that format (the bit
    widths are chosen on the device, so a NULL must never be read through).  The same inline test, on the host:
    a format is present exactly when all of its pointers for the three matrices are set; any one NULL removes it,
    other formats' pointers never matter, and the optional tile copy of the bf16 weights is not required."""
    fields = {16: ("w",), 8: ("q8", "s8", "z8"), 4: ("q4", "s4", "z4"), 2: ("q2", "s2", "z2")}
    empty = B.ExpertFmt()
    for b in (16, 8, 4, 2, 0, 3, 1, 32, -4):
        assert not B.format_present(empty, b)
    assert B.lib.dymoe_format_present(None, 16) == 0
    for b, names in fields.items():
        full = B.ExpertFmt()
        for n in names:
            for m in range(3):
                getattr(full, n)[m] = 0x1000 * (m + 1)
        assert B.format_present(full, b)
        for other in fields:
            if other != b:
                assert not B.format_present(full, other)        # only this format was filled in
        for n in names:                                          # any single pointer missing: absent
            for m in range(3):
                one = B.ExpertFmt.from_buffer_copy(bytes(full))
                getattr(one, n)[m] = None
                assert not B.format_present(one, b), (b, n, m)
        assert not B.format_present(full, 0) and not B.format_present(full, 5)
    # everything set: every width present
    allset = B.ExpertFmt()
    for n, _ in B.ExpertFmt._fields_:
        for m in range(3):
            getattr(allset, n)[m] = 0x40
    assert all(B.format_present(allset, b) for b in (16, 8, 4, 2))
    for m in range(3):
        allset.wt[m] = None
    assert B.format_present(allset, 16)
    u = C.c_uint(7)
    assert B.lib.dymoe_device_flags(None, C.byref(u), None) == B.ENOCTX
    assert B.lib.dymoe_device_flags(None, None, None) == B.EINVAL


def test_create_without_gpu_reports_error():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    h = C.c_void_p()
    assert B.lib.dymoe_create(C.byref(h), 0) == B.EHIP and not h.value
    with pytest.raises(B.DymoeError):
        B.Context(0)


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""
