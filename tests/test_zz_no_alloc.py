"""dymoe_moe_ffn_mixed_noalloc (scratch in a static device array, nothing allocated) against
dymoe_moe_ffn_mixed on the same inputs: the two share their kernels and every sum is taken in a
fixed order, so the outputs have to be the same bits.  Two calls in a row, the second smaller, so
that the array still holds the first call's contents when the second runs; then the oracle."""
import numpy as np
import pytest
import torch

from oracle import dymoe_oracle as O
from paper_2603_19172_amd import binding as B
from paper_2603_19172_amd import synth
from gpu_helpers import DEV, oracle_quantize_expert, rel_err_per_token, tiles_from_rowmajor, to_bf16, upload_q

pytestmark = pytest.mark.gpu


def _case(ctx, T, H, F, E, k, seed, path, out_dtype):
    rng = np.random.default_rng(seed)
    cfg = synth.scaled(synth.CONFIGS["tiny"], T=T, H=H, F=F, E=E, k=k, config_id=900 + seed)
    x, _ = synth.activations(cfg)
    mats = [synth.expert_weights(cfg, e) for e in range(E)]
    bits = np.array([(16, 4, 2, 8)[e % 4] for e in range(E)], np.uint8)
    idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    g = rng.random((T, k)) + 0.1
    g /= g.sum(1, keepdims=True)
    host_q = {e: oracle_quantize_expert(mats[e], int(bits[e])) for e in range(E) if bits[e] != 16}
    experts = []
    for e in range(E):
        d = {"w": [to_bf16(m) for m in mats[e]], "wt": None}
        if bits[e] != 16:
            # the GEMV path reads the codes row by row, the grouped GEMM in 32 x 128 tiles
            trip = host_q[e] if path == B.PATH_GEMV else [tiles_from_rowmajor(cd, sc, zr, int(bits[e])) for cd, sc, zr in host_q[e]]
            d["q%d" % bits[e]] = upload_q(trip)
        experts.append(d)
    table, keep = B.make_expert_table(experts, DEV)
    xd = to_bf16(x)
    idx_d = torch.from_numpy(idx).to(DEV)
    g_d = torch.from_numpy(g.astype(np.float32)).to(DEV)
    bits_d = torch.from_numpy(bits).to(DEV)
    dt = torch.float32 if out_dtype == B.OUT_F32 else torch.bfloat16
    y_ws = torch.empty((T, H), dtype=dt, device=DEV)
    y_st = torch.full((T, H), float("nan"), dtype=dt, device=DEV)
    nbytes = B.workspace_bytes(T, H, F, E, k)
    assert nbytes <= B.STATIC_SCRATCH_BYTES
    ws = torch.empty((nbytes,), dtype=torch.uint8, device=DEV)
    st = B._stream(None)
    B._check(B.lib.dymoe_moe_ffn_mixed(ctx._h, xd.data_ptr(), idx_d.data_ptr(), g_d.data_ptr(), bits_d.data_ptr(),
                                       table.data_ptr(), T, H, F, E, k, 64, out_dtype, path, y_ws.data_ptr(),
                                       ws.data_ptr(), nbytes, st), "dymoe_moe_ffn_mixed")
    B._check(B.lib.dymoe_moe_ffn_mixed_noalloc(ctx._h, xd.data_ptr(), idx_d.data_ptr(), g_d.data_ptr(),
                                               bits_d.data_ptr(), table.data_ptr(), T, H, F, E, k, 64, out_dtype,
                                               path, y_st.data_ptr(), st), "dymoe_moe_ffn_mixed_noalloc")
    torch.cuda.synchronize()
    assert torch.equal(y_ws.view(torch.int16 if dt == torch.bfloat16 else torch.int32),
                       y_st.view(torch.int16 if dt == torch.bfloat16 else torch.int32))
    ob = [{"w": mats[e]} if bits[e] == 16 else {"q": host_q[e]} for e in range(E)]
    ref = O.moe_ffn_mixed(x, idx, g.astype(np.float32).astype(np.float64), bits, ob)
    err = rel_err_per_token(y_st.float().cpu().numpy().astype(np.float64), ref)
    assert err <= 2e-2, err
    return keep


def test_noalloc_entry_point_matches_the_workspace_one_on_two_calls_in_a_row():
    ctx = B.Context(0)
    # first a 16-token step of ragged width on the GEMV path, then a smaller one: what the first left in the
    # array must not reach the second's result
    _case(ctx, T=16, H=320, F=704, E=8, k=2, seed=1, path=B.PATH_GEMV, out_dtype=B.OUT_F32)
    _case(ctx, T=3, H=256, F=512, E=8, k=2, seed=2, path=B.PATH_GEMV, out_dtype=B.OUT_BF16)
    # the grouped-GEMM path inside the same limit, larger first
    _case(ctx, T=40, H=256, F=512, E=8, k=2, seed=3, path=B.PATH_GEMM, out_dtype=B.OUT_F32)
    _case(ctx, T=9, H=128, F=256, E=4, k=2, seed=4, path=B.PATH_GEMM, out_dtype=B.OUT_BF16)
    ctx.close()


def test_noalloc_entry_point_rejects_what_does_not_fit():
    ctx = B.Context(0)
    cfg = synth.CONFIGS["mixtral_prefill"]
    assert B.workspace_bytes(cfg.T, cfg.H, cfg.F, cfg.E, cfg.k) > B.STATIC_SCRATCH_BYTES
    one = torch.zeros((256,), dtype=torch.uint8, device=DEV)
    rc = B.lib.dymoe_moe_ffn_mixed_noalloc(ctx._h, one.data_ptr(), one.data_ptr(), one.data_ptr(), one.data_ptr(),
                                           one.data_ptr(), cfg.T, cfg.H, cfg.F, cfg.E, cfg.k, 64, B.OUT_BF16,
                                           B.PATH_AUTO, one.data_ptr(), B._stream(None))
    assert rc == B.ENOSPC
    ctx.close()
