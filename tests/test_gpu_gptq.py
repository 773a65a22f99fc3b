"""GPU parity of the error-compensated quantizer (paper Sec. 5: GPTQ as the base
quantizer) against the CPU oracle: the column sweep bit for bit, given the same
inverse-Hessian factor."""
import numpy as np
import pytest
import torch

from oracle import dymoe_oracle as O
from paper_2603_19172_amd import binding as B
from paper_2603_19172_amd import synth
from gpu_helpers import DEV, bits_of, to_bf16

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = B.Context(0)
    yield c
    c.close()


def _case(cid, N, K, n=None):
    xb = synth.calibration_inputs(cid, n or max(256, 2 * K), K)
    wb = synth.normal_bf16(cid, 77, (N, K), 0.02)
    U = O.gptq_factor(O.gptq_hessian(xb)).astype(np.float32)
    return xb, wb, U


def _same(got, want):
    codes, scale, zero = got
    torch.cuda.synchronize()
    return (np.array_equal(codes.cpu().numpy(), want[0]) and np.array_equal(bits_of(scale), want[1])
            and np.array_equal(bits_of(zero), want[2]))


# rows: fewer than a workgroup's 64, a ragged tail, several workgroups; columns: one group (no
# trailing update), a ragged 128-column trail tile, many steps
@pytest.mark.parametrize("N,K", [(24, 64), (24, 192), (130, 320), (64, 1024), (257, 2048)])
@pytest.mark.parametrize("bits", [2, 4, 8])
def test_gptq_sweep_is_bit_exact(ctx, N, K, bits):
    if K == 2048 and bits != 4:
        pytest.skip("the largest case runs once")
    _, wb, U = _case(700 + N, N, K)
    want = O.gptq_quantize_pack(wb, U, bits)
    got = ctx.gptq_quantize_pack(to_bf16(wb), torch.from_numpy(U).to(DEV), bits)
    torch.cuda.synchronize()
    codes = got[0].cpu().numpy()
    print("N=%d K=%d bits=%d: code bytes equal %.6f" % (N, K, bits, (codes == want[0]).mean()))
    assert _same(got, want)
    # and it is not the plain quantizer's answer
    plain = O.quantize_pack(wb, bits)
    assert K == 64 or not np.array_equal(want[0], plain[0])


def test_gptq_identity_factor_gives_the_plain_quantizer(ctx):
    _, wb, _ = _case(720, 100, 256)
    w = to_bf16(wb)
    eye = torch.eye(256, dtype=torch.float32, device=DEV)
    for bits in (2, 4, 8):
        a = ctx.gptq_quantize_pack(w, eye, bits)
        b = ctx.quantize_pack(w, bits)
        torch.cuda.synchronize()
        assert all(torch.equal(x, y) for x, y in zip(a, b))


def test_gptq_reuses_a_dirty_workspace_and_lowers_the_output_error(ctx):
    xb, wb, U = _case(730, 96, 512, n=1024)
    w, u = to_bf16(wb), torch.from_numpy(U).to(DEV)
    need = int(B.lib.dymoe_gptq_workspace_bytes(96, 512))
    ws = torch.full((need + 512,), 0xFF, dtype=torch.uint8, device=DEV)
    first = ctx.gptq_quantize_pack(w, u, 4, workspace=ws)
    second = ctx.gptq_quantize_pack(w, u, 4, workspace=ws)
    torch.cuda.synchronize()
    assert all(torch.equal(x, y) for x, y in zip(first, second))
    assert _same(first, O.gptq_quantize_pack(wb, U, 4))
    H = O.gptq_hessian(xb)
    wf = synth.bf16_bits_to_f32(wb).astype(np.float64)
    deq = O.dequantize(first[0].cpu().numpy(), bits_of(first[1]), bits_of(first[2]), 4)
    plain = O.dequantize(*O.quantize_pack(wb, 4), 4)
    assert O.output_error(wf, deq, H) < 0.5 * O.output_error(wf, plain, H)


# samples: fewer than a step's 64, ragged, several steps; columns: one tile, a ragged last tile, several tiles
@pytest.mark.parametrize("n,K", [(9, 64), (300, 320), (1000, 512), (64, 1024)])
def test_gptq_hessian_matches_the_oracle(ctx, n, K):
    xb = synth.calibration_inputs(740 + K, n, K)
    want = O.gptq_hessian(xb)
    x = to_bf16(xb)
    got = ctx.gptq_hessian(x)
    torch.cuda.synchronize()
    g = got.cpu().numpy().astype(np.float64)
    scale = np.sqrt(np.outer(np.diag(want), np.diag(want)))
    err = np.abs(g - want) / scale
    print("n=%d K=%d: max |dH| / sqrt(Hii Hjj) = %.2e" % (n, K, err.max()))
    assert err.max() < 1e-5 and np.array_equal(g, g.T)
    # a second batch added on top
    both = ctx.gptq_hessian(x, out=got, accumulate=True)
    torch.cuda.synchronize()
    assert np.abs(both.cpu().numpy() - 2.0 * want).max() <= 2e-5 * scale.max()


@pytest.mark.parametrize("K", [64, 192, 1024])
def test_gptq_factor_matches_the_oracle(ctx, K):
    xb = synth.calibration_inputs(760 + K, 2 * K, K)
    H = O.gptq_hessian(xb)
    H[:, 5] = 0.0                      # a column no input reached
    H[5, :] = 0.0
    want = O.gptq_factor(H, damp=0.01)
    got = ctx.gptq_factor(torch.from_numpy(H.astype(np.float32)).to(DEV), damp=0.01)
    torch.cuda.synchronize()
    U = got.cpu().numpy().astype(np.float64)
    assert np.isfinite(U).all() and np.array_equal(U, np.triu(U)) and (np.diag(U) > 0).all()
    rel = np.abs(U - want).max(axis=1) / np.abs(want).max(axis=1)
    Hd = O.gptq_damped(H, 0.01)
    resid = np.abs(U.T @ U @ Hd - np.eye(K)).max()
    print("K=%d: max row-relative error %.2e, |U^T U Hd - I| = %.2e" % (K, rel.max(), resid))
    assert rel.max() < 2e-4 and resid < 2e-3


def test_gptq_chain_on_the_device(ctx):
    """Hessian, factor and sweep all on the device; the result is as good as the oracle's own chain (the
    factors differ in the last fp32 digits, so a code may differ here and there)."""
    N, K = 128, 512
    xb = synth.calibration_inputs(780, 1024, K)
    wb = synth.normal_bf16(780, 77, (N, K), 0.02)
    H = O.gptq_hessian(xb)
    want = O.gptq_quantize_pack(wb, O.gptq_factor(H), 4)
    hess = ctx.gptq_hessian(to_bf16(xb))
    u = ctx.gptq_factor(hess)
    got = ctx.gptq_quantize_pack(to_bf16(wb), u, 4)
    torch.cuda.synchronize()
    wf = synth.bf16_bits_to_f32(wb).astype(np.float64)
    d_got = O.dequantize(got[0].cpu().numpy(), bits_of(got[1]), bits_of(got[2]), 4)
    d_want = O.dequantize(*want, 4)
    e_got, e_want = O.output_error(wf, d_got, H), O.output_error(wf, d_want, H)
    e_plain = O.output_error(wf, O.dequantize(*O.quantize_pack(wb, 4), 4), H)
    same = (d_got == d_want).mean()
    print("same dequantised values %.4f; output error device %.4e oracle %.4e plain %.4e" % (same, e_got, e_want, e_plain))
    assert same > 0.98 and abs(e_got - e_want) <= 0.02 * e_want and e_got < 0.5 * e_plain


def test_gptq_mixtral_sized_matrix(ctx):
    """The first expert matrix of the Mixtral-shaped layer at full size (14336 x 4096), 1024 calibration
    tokens.  Rows are independent in the sweep, so the oracle checks a seeded sample of them bit for bit;
    the factor is compared in full."""
    N, K, n = 14336, 4096, 1024
    cfg = synth.CONFIGS["mixtral_decode"]
    wb = synth.expert_matrix(cfg, 0, 0)
    assert wb.shape == (N, K)
    xb = synth.calibration_inputs(790, n, K)
    H = O.gptq_hessian(xb)
    U = O.gptq_factor(H)
    x = to_bf16(xb)
    hess = ctx.gptq_hessian(x)
    u_dev = ctx.gptq_factor(hess)
    torch.cuda.synchronize()
    Ud = u_dev.cpu().numpy().astype(np.float64)
    rel = np.abs(Ud - U).max(axis=1) / np.abs(U).max(axis=1)
    print("factor K=%d: max row-relative error %.2e" % (K, rel.max()))
    assert np.isfinite(Ud).all() and rel.max() < 5e-4
    del Ud
    # the sweep with the oracle's own factor, so that the comparison is bit for bit
    U32 = U.astype(np.float32)
    got = ctx.gptq_quantize_pack(to_bf16(wb), torch.from_numpy(U32).to(DEV), 4)
    torch.cuda.synchronize()
    rows = np.sort(np.random.default_rng(790).choice(N, size=24, replace=False))
    rows[0], rows[-1] = 0, N - 1
    want = O.gptq_quantize_pack(wb[rows], U32, 4)
    assert np.array_equal(got[0].cpu().numpy()[rows], want[0])
    assert np.array_equal(bits_of(got[1])[rows], want[1]) and np.array_equal(bits_of(got[2])[rows], want[2])
    # the sampled rows' output error against the plain quantizer's
    wf = synth.bf16_bits_to_f32(wb[rows]).astype(np.float64)
    e_comp = O.output_error(wf, O.dequantize(*want, 4), H)
    e_plain = O.output_error(wf, O.dequantize(*O.quantize_pack(wb[rows], 4), 4), H)
    print("output error on 24 rows: compensated %.4e, plain %.4e" % (e_comp, e_plain))
    assert e_comp < 0.7 * e_plain


def test_gptq_experts_feed_the_mixed_ffn(ctx):
    """The compensated quantizer writes the plain quantizer's formats: the FFN reads its experts unchanged.
    Two experts (int4 and int2) quantised on the device with calibration inputs for [F,H] and [H,F]; the
    FFN's output against the oracle's FFN over the oracle's own compensated codes."""
    cfg = synth.scaled(synth.CONFIGS["tiny"], T=3, H=256, F=512, E=2, k=2, config_id=83)
    x, _ = synth.activations(cfg)
    hw = {e: synth.expert_weights(cfg, e) for e in range(cfg.E)}
    cal = {cfg.H: synth.calibration_inputs(83, 1024, cfg.H), cfg.F: synth.calibration_inputs(84, 1024, cfg.F)}
    U = {K: O.gptq_factor(O.gptq_hessian(cal[K])).astype(np.float32) for K in cal}
    Ud = {K: torch.from_numpy(U[K]).to(DEV) for K in U}
    bits_np = np.array([4, 2], dtype=np.uint8)
    experts_dev, experts_ref = [], []
    for e in range(cfg.E):
        b = int(bits_np[e])
        experts_dev.append({"q%d" % b: [ctx.gptq_quantize_pack(to_bf16(m), Ud[m.shape[1]], b) for m in hw[e]]})
        experts_ref.append({"q": [O.gptq_quantize_pack(m, U[m.shape[1]], b) for m in hw[e]]})
    table, keep = B.make_expert_table(experts_dev, DEV)
    idx_np = np.array([[0, 1], [1, 0], [0, 1]], dtype=np.int32)
    w_np = np.array([[0.6, 0.4], [0.3, 0.7], [0.5, 0.5]], dtype=np.float32)
    y = ctx.moe_ffn_mixed(to_bf16(x), torch.from_numpy(idx_np).to(DEV), torch.from_numpy(w_np).to(DEV),
                          torch.from_numpy(bits_np).to(DEV), table, cfg.F, out_dtype=B.OUT_F32)
    torch.cuda.synchronize()
    ref = O.moe_ffn_mixed(x, idx_np, w_np.astype(np.float64), bits_np, experts_ref)
    rms = np.sqrt((ref ** 2).mean(axis=1, keepdims=True))
    err = float((np.abs(y.cpu().numpy() - ref) / rms).max())
    print("FFN over compensated experts: max err / rms = %.2e" % err)
    assert err <= 2e-2


def test_code_tiles_from_rowmajor_equal_the_quantizers_own_tiles(ctx):
    """dymoe_pack_code_tiles is the permutation between the two layouts the plain quantizer can write."""
    from paper_2603_19172_amd.layer import ExpertStore
    cfg = synth.scaled(synth.CONFIGS["tiny"], H=384, F=256, E=3, k=2, config_id=85)
    hw = {e: synth.expert_weights(cfg, e) for e in range(cfg.E)}
    store = ExpertStore([[to_bf16(m) for m in hw[e]] for e in range(cfg.E)], cfg.H, cfg.F, DEV, formats=(8, 4, 2))
    bits = torch.tensor([8, 4, 2], dtype=torch.uint8, device=DEV)
    ones = torch.ones((cfg.E,), dtype=torch.int32, device=DEV)
    ctx.quantize_experts(store.table, bits, ones, cfg.E, cfg.H, cfg.F, layout=B.LAYOUT_TILE)
    for e, b in enumerate((8, 4, 2)):
        for i in range(3):
            tiles = ctx.pack_code_tiles(ctx.quantize_pack(store.w[e][i], b), b)
            torch.cuda.synchronize()
            # scale and zero of a tile are 64 fp16 in lane order: compare as flat arrays
            assert torch.equal(tiles[0].flatten(), store.q[b][e][i][0].flatten())
            assert torch.equal(tiles[1].flatten(), store.q[b][e][i][1].flatten())
            assert torch.equal(tiles[2].flatten(), store.q[b][e][i][2].flatten())


def test_gptq_experts_feed_the_grouped_gemm(ctx):
    """Compensated experts, re-packed into tiles, through the MFMA path (8 tokens) against the oracle's FFN."""
    cfg = synth.scaled(synth.CONFIGS["tiny"], T=8, H=256, F=512, E=2, k=2, config_id=86)
    x, _ = synth.activations(cfg)
    hw = {e: synth.expert_weights(cfg, e) for e in range(cfg.E)}
    cal = {cfg.H: synth.calibration_inputs(86, 1024, cfg.H), cfg.F: synth.calibration_inputs(87, 1024, cfg.F)}
    U = {K: O.gptq_factor(O.gptq_hessian(cal[K])).astype(np.float32) for K in cal}
    Ud = {K: torch.from_numpy(U[K]).to(DEV) for K in U}
    bits_np = np.array([4, 2], dtype=np.uint8)
    experts_dev, experts_ref = [], []
    for e in range(cfg.E):
        b = int(bits_np[e])
        rm = [ctx.gptq_quantize_pack(to_bf16(m), Ud[m.shape[1]], b) for m in hw[e]]
        experts_dev.append({"q%d" % b: [ctx.pack_code_tiles(t, b) for t in rm]})
        experts_ref.append({"q": [O.gptq_quantize_pack(m, U[m.shape[1]], b) for m in hw[e]]})
    table, keep = B.make_expert_table(experts_dev, DEV)
    rng = np.random.default_rng(86)
    idx_np = np.stack([rng.permutation(2) for _ in range(cfg.T)]).astype(np.int32)
    w_np = rng.uniform(0.2, 0.8, size=(cfg.T, 1)).astype(np.float32)
    w_np = np.concatenate([w_np, 1.0 - w_np], axis=1)
    y = ctx.moe_ffn_mixed(to_bf16(x), torch.from_numpy(idx_np).to(DEV), torch.from_numpy(w_np).to(DEV),
                          torch.from_numpy(bits_np).to(DEV), table, cfg.F, out_dtype=B.OUT_F32, path=B.PATH_GEMM)
    torch.cuda.synchronize()
    ref = O.moe_ffn_mixed(x, idx_np, w_np.astype(np.float64), bits_np, experts_ref)
    rms = np.sqrt((ref ** 2).mean(axis=1, keepdims=True))
    err = float((np.abs(y.cpu().numpy() - ref) / rms).max())
    print("grouped GEMM over compensated experts: max err / rms = %.2e" % err)
    assert err <= 2e-2


def test_gptq_factor_with_fewer_samples_than_columns(ctx):
    """64 calibration tokens for 512 columns: the Hessian has rank 64 and only the damping keeps it
    positive definite (condition number about 1e4), the case fp32 Cholesky has least room for."""
    K = 512
    H = O.gptq_hessian(synth.calibration_inputs(864, 64, K))
    want = O.gptq_factor(H)
    got = ctx.gptq_factor(torch.from_numpy(H.astype(np.float32)).to(DEV))
    torch.cuda.synchronize()
    U = got.cpu().numpy().astype(np.float64)
    rel = np.abs(U - want).max(axis=1) / np.abs(want).max(axis=1)
    print("rank-deficient Hessian: max row-relative error %.2e" % rel.max())
    assert np.isfinite(U).all() and rel.max() < 5e-4


def test_gptq_sweep_edge_rows(ctx):
    """One row; a group of equal weights (scale 0: every code 0, the whole value becomes error and is passed
    on); a group of zeros; values at the top of the bf16 range the plain quantizer accepts."""
    K = 256
    _, wb, U = _case(741, 4, K)
    w = synth.bf16_bits_to_f32(wb).copy()
    w[1, 64:128] = 0.01953125          # one bf16 value through a whole group
    w[2, 0:64] = 0.0
    w[3, 128:192] *= 1.0e6             # ~2e4: near the fp16 range of scale and zero
    wb = synth.f32_to_bf16_bits(w)
    for rows in (slice(0, 1), slice(0, 4)):
        for bits in (2, 4, 8):
            want = O.gptq_quantize_pack(wb[rows], U, bits)
            got = ctx.gptq_quantize_pack(to_bf16(wb[rows]), torch.from_numpy(U).to(DEV), bits)
            assert _same(got, want)
    # one calibration token
    xb = synth.calibration_inputs(742, 1, 128)
    h = ctx.gptq_hessian(to_bf16(xb))
    torch.cuda.synchronize()
    assert np.allclose(h.cpu().numpy(), O.gptq_hessian(xb), rtol=1e-6, atol=0)
