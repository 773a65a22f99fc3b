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
