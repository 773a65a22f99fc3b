"""Pins for the CPU oracle: closed forms, invariants, brute force and special
cases that reduce to a numpy routine.  None of these re-types the oracle's own
formula; each is chosen so that a dropped term, a wrong sign or index, or a
transposed operand in the oracle fails at least one of them."""
import itertools
import os
from decimal import Decimal, getcontext

import numpy as np
import pytest

from oracle import dymoe_oracle as O
from paper_2603_19172_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bf16(a):
    return synth.f32_to_bf16_bits(np.asarray(a, np.float32))


def widen(b):
    return synth.bf16_bits_to_f32(b).astype(np.float64)


# --------------------------------------------------------------------- formats

def test_fp16_conversion_matches_numpy():
    rng = np.random.default_rng(1)
    vals = np.concatenate([
        rng.standard_normal(4000).astype(np.float32) * np.float32(0.02),
        rng.standard_normal(2000).astype(np.float32) * np.float32(1e-6),   # fp16 subnormals
        rng.standard_normal(2000).astype(np.float32) * np.float32(3e4),    # near overflow
        np.array([0.0, -0.0, 65504.0, 65519.99, 65520.0, 1e9, -1e9, 2.0 ** -24, 2.0 ** -25,
                  1.5 * 2.0 ** -25, 2.0 ** -14, 2.0 ** -14 - 2.0 ** -26, 1.0 + 2.0 ** -11,
                  1.0 + 3 * 2.0 ** -11, 1e-45], np.float32),
    ])
    with np.errstate(over="ignore"):
        ref = vals.astype(np.float16).view(np.uint16)
    got = np.array([O.f32_to_f16(v) for v in vals], np.uint16)
    assert np.array_equal(ref, got)
    # and back, over every finite fp16 bit pattern
    allh = np.arange(0, 0x10000, dtype=np.uint32).astype(np.uint16)
    fin = np.isfinite(allh.view(np.float16))
    back = np.array([O.f16_to_f32(int(h)) for h in allh[fin]], np.float32)
    assert np.array_equal(back.view(np.uint32), allh[fin].view(np.float16).astype(np.float32).view(np.uint32))


def test_bf16_widening():
    assert O.bf16_to_f32(0x3F80) == 1.0
    assert O.bf16_to_f32(0xC000) == -2.0
    assert O.bf16_to_f32(0x3C00) == 2.0 ** -7


# --------------------------------------------------------------------- routing

def _route_inputs(T, H, E, seed, bias=False):
    rng = np.random.default_rng(seed)
    x = bf16(rng.standard_normal((T, H)))
    wg = bf16(rng.standard_normal((E, H)) * 0.1)
    b = rng.standard_normal(E).astype(np.float32) if bias else None
    return x, wg, b


def test_route_hand_example():
    # x = (1, 2); experts (1,0), (0,1), (1,1), (0,0): logits 1, 2, 3, 0
    x = bf16([[1.0, 2.0]])
    wg = bf16([[1, 0], [0, 1], [1, 1], [0, 0]])
    idx, w, p, lg = O.route_topk(x, wg, None, k=2, renorm=True)
    assert lg.tolist() == [[1.0, 2.0, 3.0, 0.0]]
    den = np.e ** 1 + np.e ** 2 + np.e ** 3 + 1.0
    assert np.allclose(p[0], np.array([np.e, np.e ** 2, np.e ** 3, 1.0]) / den, rtol=1e-14)
    assert idx.tolist() == [[2, 1]]
    # renormalised over the two chosen: e^3/(e^3+e^2) = 1/(1+1/e)
    assert np.allclose(w[0], [1 / (1 + np.e ** -1), 1 / (1 + np.e)], rtol=1e-14)
    _, w2, _, _ = O.route_topk(x, wg, None, k=2, renorm=False)
    assert np.allclose(w2[0], p[0][[2, 1]], rtol=1e-15)


def test_route_against_numpy_sort_and_brute_force():
    for seed, (T, H, E, k, bias) in enumerate([(5, 32, 8, 2, False), (7, 64, 6, 3, True),
                                               (3, 16, 40, 8, True)]):
        x, wg, b = _route_inputs(T, H, E, seed, bias)
        idx, w, p, lg = O.route_topk(x, wg, b, k=k, renorm=True)
        ref_l = widen(x) @ widen(wg).T + (b.astype(np.float64) if b is not None else 0.0)
        assert np.allclose(lg, ref_l, rtol=1e-12, atol=1e-12)
        assert np.allclose(p.sum(1), 1.0, rtol=1e-13)
        assert np.allclose(w.sum(1), 1.0, rtol=1e-13)
        order = np.argsort(-lg, axis=1, kind="stable")[:, :k]
        assert np.array_equal(order, idx)
        # softmax is monotone in the logit and shift invariant
        assert np.allclose(np.log(p) - np.log(p[:, :1]), lg - lg[:, :1], atol=1e-11)
        if E <= 8:  # brute force: the chosen set maximises the total probability
            for t in range(T):
                best = max(itertools.combinations(range(E), k), key=lambda s: p[t, list(s)].sum())
                assert set(best) == set(idx[t].tolist())


def test_route_ties_and_permutation():
    # two identical experts: the lower index comes first
    x = bf16([[1.0, -1.0, 0.5, 2.0]])
    row = [0.5, 0.25, 1.0, 0.125]          # logit 1; the zero row has logit 0
    wg = bf16([row, [0, 0, 0, 0], row])
    idx, w, p, _ = O.route_topk(x, wg, None, k=2)
    assert idx.tolist() == [[0, 2]]
    assert w[0, 0] == w[0, 1] == 0.5
    idx, _, _, _ = O.route_topk(x, bf16([[0, 0, 0, 0], row, row, [0, 0, 0, 0]]), None, k=3)
    assert idx.tolist() == [[1, 2, 0]]
    # permuting the experts permutes the indices
    x, wg, b = _route_inputs(6, 48, 8, 11, True)
    idx, w, p, lg = O.route_topk(x, wg, b, k=3)
    perm = np.random.default_rng(3).permutation(8)
    idx2, w2, p2, _ = O.route_topk(x, wg[perm], b[perm], k=3)
    assert np.array_equal(perm[idx2], idx)
    assert np.allclose(w2, w, rtol=1e-13)
    assert np.allclose(p2, p[:, perm], rtol=1e-13)


# ------------------------------------------------------------------ importance

def test_importance_hand_example():
    # 4 tokens, 3 experts, top-2 routing; scores make tokens 2 and 0 the heavy hitters
    idx = np.array([[0, 1], [1, 2], [2, 0], [1, 0]], np.int32)
    score = np.array([5.0, 1.0, 9.0, 2.0])
    imp, load, heavy = O.expert_importance_prefill(idx, score, E=3, k_hh=2)
    assert heavy.tolist() == [1, 0, 1, 0]
    assert imp.tolist() == [2, 1, 1]      # token0 -> {0,1}, token2 -> {2,0}
    assert load.tolist() == [3, 3, 2]
    # score ties go to the lower token index
    imp, _, heavy = O.expert_importance_prefill(idx, np.array([1.0, 1.0, 1.0, 1.0]), E=3, k_hh=1)
    assert heavy.tolist() == [1, 0, 0, 0] and imp.tolist() == [1, 1, 0]


def test_importance_invariants_and_bincount():
    rng = np.random.default_rng(5)
    T, E, k, k_hh = 200, 16, 4, 17
    idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    score = rng.standard_normal(T) ** 2
    imp, load, heavy = O.expert_importance_prefill(idx, score, E=E, k_hh=k_hh)
    assert imp.sum() == k * k_hh and load.sum() == k * T and heavy.sum() == k_hh
    assert np.array_equal(load, np.bincount(idx.ravel(), minlength=E))
    top = np.argsort(-score, kind="stable")[:k_hh]
    assert set(np.nonzero(heavy)[0].tolist()) == set(top.tolist())
    assert np.array_equal(imp, np.bincount(idx[top].ravel(), minlength=E))
    # every token heavy: importance is the token-frequency count (total load)
    imp_all, load_all, _ = O.expert_importance_prefill(idx, score, E=E, k_hh=T)
    assert np.array_equal(imp_all, load_all)
    imp0, _, _ = O.expert_importance_prefill(idx, score, E=E, k_hh=0)
    assert imp0.sum() == 0


def test_importance_decode_is_gate_score():
    p = np.array([[0.1, 0.6, 0.3]])
    assert np.array_equal(O.expert_importance_decode(p), p[0])
    p2 = np.array([[0.1, 0.6, 0.3], [0.5, 0.2, 0.3]])
    assert np.allclose(O.expert_importance_decode(p2), [0.3, 0.4, 0.3], rtol=1e-15)


def test_token_score_norm():
    rng = np.random.default_rng(2)
    x = bf16(rng.standard_normal((9, 130)) * 3)
    assert np.allclose(O.token_score_norm(x), np.linalg.norm(widen(x), axis=1), rtol=1e-14)


# -------------------------------------------------------------------- schedule

def _dec_cos(x: Decimal) -> Decimal:
    # Taylor series at 60 digits; independent of libm
    getcontext().prec = 60
    term, s, n = Decimal(1), Decimal(1), 0
    while abs(term) > Decimal(10) ** -55:
        n += 2
        term = -term * x * x / (n * (n - 1))
        s += term
    return s


PI = Decimal("3.14159265358979323846264338327950288419716939937510582097494")


def test_schedule_golden_tables():
    for line in open(os.path.join(GOLDEN, "schedule_tables.txt")):
        if line.startswith("#") or not line.strip():
            continue
        f = line.split()
        L, M, lam = int(f[0]), int(f[1]), float(f[2])
        want = [int(v) for v in f[3:]]
        assert [O.depth_schedule(l, L, lam, M) for l in range(L)] == want, line


def test_schedule_closed_forms():
    for L in (2, 5, 32, 48):
        for lam in (0.0, 0.25, 0.5, 0.8, 1.0):
            r = [O.retention_ratio(l, L, lam) for l in range(L)]
            assert r[0] == 1.0 and abs(r[-1] - lam) < 1e-15
            assert all(r[i] >= r[i + 1] - 1e-15 for i in range(L - 1))
            assert abs(sum(r) / L - (1 + lam) / 2) < 1e-13   # cosine term is odd about the middle
    assert O.retention_ratio(0, 1, 0.3) == 1.0
    # slow start: the first quarter of a 32-layer stack keeps > 92% at lambda = 0.5
    assert O.retention_ratio(8, 32, 0.5) > 0.92


def test_schedule_against_high_precision_ceiling():
    getcontext().prec = 60
    for L in (4, 7, 13, 32, 61):
        for M in (8, 60, 128):
            for lam_s in ("0.5", "0.8", "0.25", "0.9"):
                lam = Decimal(lam_s)
                for l in range(L):
                    c = _dec_cos(PI * l / (L - 1))
                    v = ((1 - lam) * (c + 1) / 2 + lam) * M
                    near = v.quantize(Decimal(1))
                    exact = int(near) if abs(v - near) < Decimal("1e-40") else int(v.to_integral_value(rounding="ROUND_CEILING"))
                    exact = min(max(exact, 1), M)
                    assert O.depth_schedule(l, L, float(lam), M) == exact, (L, M, lam_s, l)


def test_schedule_rejects_bad_arguments():
    assert O.depth_schedule(4, 4, 0.5, 8) < 0
    assert O.depth_schedule(0, 4, 1.5, 8) < 0
    assert O.depth_schedule(0, 4, 0.5, 0) < 0


# ------------------------------------------------------------------ assignment

def test_assign_hand_example():
    imp = [3, 7, 3, 0, 7, 1]
    load = [10, 2, 12, 5, 9, 5]
    bits, rank = O.assign_precision(imp, load, tier_count=[1, 2, 3], tier_bits=[16, 4, 2])
    # order: e4 (7, load 9), e1 (7, load 2), e2 (3, load 12), e0 (3, load 10), e5, e3
    assert rank.tolist() == [3, 1, 2, 5, 0, 4]
    assert bits.tolist() == [2, 4, 4, 2, 16, 2]
    bits, _ = O.assign_precision(imp, load, [1, 2, 3], [16, 4, 2], floor_bits=4)
    assert bits.tolist() == [4, 4, 4, 4, 16, 4]
    # full ties fall back to the expert index
    bits, rank = O.assign_precision([1, 1, 1], [2, 2, 2], [1, 1, 1], [16, 4, 0])
    assert rank.tolist() == [0, 1, 2] and bits.tolist() == [16, 4, 0]
    with pytest.raises(ValueError):
        O.assign_precision(imp, load, [1, 2, 2], [16, 4, 2])


def test_assign_invariants():
    rng = np.random.default_rng(8)
    E = 128
    imp = rng.integers(0, 6, E)
    load = rng.integers(0, 50, E)
    tc, tb = [13, 39, 76], [16, 4, 2]
    bits, rank = O.assign_precision(imp, load, tc, tb)
    assert sorted(rank.tolist()) == list(range(E))
    assert [(bits == b).sum() for b in tb] == tc
    # monotone: strictly more important never gets fewer bits
    for a in range(E):
        for b in range(E):
            if imp[a] > imp[b]:
                assert bits[a] >= bits[b]
    # reference ordering by lexsort (last key is primary)
    order = np.lexsort((np.arange(E), -load, -imp))
    assert np.array_equal(np.argsort(rank), order)
    # permutation equivariance (keys made distinct so that the index tie-break is idle)
    imp_d = imp * 1000 + rng.permutation(E)
    bits_d, _ = O.assign_precision(imp_d, load, tc, tb)
    perm = rng.permutation(E)
    bits_p, _ = O.assign_precision(imp_d[perm], load[perm], tc, tb)
    assert np.array_equal(bits_p, bits_d[perm])
    # paper mode: two tiers, t_l critical experts
    t = O.depth_schedule(20, 32, 0.5, E)
    b2, _ = O.assign_precision(imp_d, load, [t, E - t], [4, 2])
    assert (b2 == 4).sum() == t and set(np.argsort(-imp_d)[:t].tolist()) == set(np.nonzero(b2 == 4)[0].tolist())


# ---------------------------------------------------------------- quantization

def _unpack(codes, bits):
    """Brute-force bit unpacking, one code at a time."""
    N, B = codes.shape
    per = 8 // bits
    out = np.zeros((N, B * per), np.int64)
    for n in range(N):
        for j in range(B):
            byte = int(codes[n, j])
            for i in range(per):
                out[n, j * per + i] = (byte >> (bits * i)) & ((1 << bits) - 1)
    return out


def f16(bits_arr):
    return np.asarray(bits_arr, np.uint16).view(np.float16).astype(np.float64)


def test_pack_hand_bytes():
    # one group, scale 1, zero 0 -> codes are the values themselves
    row4 = np.array([[1, 2, 3, 4] + [0] * 59 + [15]], np.float32)
    codes, sc, zr = O.quantize_pack(bf16(row4), 4)
    assert f16(sc)[0, 0] == 1.0 and f16(zr)[0, 0] == 0.0
    assert codes[0, :2].tolist() == [0x21, 0x43] and codes[0, 31] == 0xF0
    row2 = np.array([[1, 2, 3, 0] + [0] * 59 + [3]], np.float32)
    codes, sc, zr = O.quantize_pack(bf16(row2), 2)
    assert f16(sc)[0, 0] == 1.0 and f16(zr)[0, 0] == 0.0
    assert codes[0, 0] == 0x39 and codes[0, 15] == 0xC0
    # 8 bits: one code per byte, in column order (0..255 are exact in bf16)
    row8 = np.array([[1, 2, 3, 200] + [0] * 59 + [255]], np.float32)
    codes, sc, zr = O.quantize_pack(bf16(row8), 8)
    assert codes.shape == (1, 64)
    assert f16(sc)[0, 0] == 1.0 and f16(zr)[0, 0] == 0.0
    assert codes[0, :5].tolist() == [1, 2, 3, 200, 0] and codes[0, 63] == 255
    assert np.array_equal(O.dequantize(codes, sc, zr, 8), row8.astype(np.float64))


def test_quantize_exact_cases():
    g = np.tile(np.arange(16, dtype=np.float32), 4)[None, :]
    codes, sc, zr = O.quantize_pack(bf16(g), 4)
    assert f16(sc)[0, 0] == 1.0 and f16(zr)[0, 0] == 0.0
    assert np.array_equal(_unpack(codes, 4)[0], g[0].astype(np.int64))
    assert np.array_equal(O.dequantize(codes, sc, zr, 4), g.astype(np.float64))
    codes, sc, zr = O.quantize_pack(bf16(g), 2)
    assert f16(sc)[0, 0] == 5.0
    assert _unpack(codes, 2)[0, :16].tolist() == [0, 0, 0, 1, 1, 1, 1, 1, 2, 2, 2, 2, 2, 3, 3, 3]
    # shifted and negative: zero = group minimum
    g2 = g * 0.5 - 3.0
    codes, sc, zr = O.quantize_pack(bf16(g2), 4)
    assert f16(sc)[0, 0] == 0.5 and f16(zr)[0, 0] == -3.0
    assert np.array_equal(O.dequantize(codes, sc, zr, 4), g2.astype(np.float64))
    # constant and all-zero groups: scale 0, codes 0, decode exact
    for v in (0.0, 0.75, -1.5):
        c = np.full((2, 128), v, np.float32)
        for b in (2, 4, 8):
            codes, sc, zr = O.quantize_pack(bf16(c), b)
            assert not codes.any() and not sc.any()
            assert np.array_equal(O.dequantize(codes, sc, zr, b), c.astype(np.float64))
    # ties round to even: values 0, .5, 1.5, 2.5 with scale 1 (max 15)
    t = np.zeros((1, 64), np.float32)
    t[0, :5] = [0.5, 1.5, 2.5, 3.5, 15.0]
    codes, sc, zr = O.quantize_pack(bf16(t), 4)
    assert _unpack(codes, 4)[0, :5].tolist() == [0, 2, 2, 4, 15]


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_quantize_round_trip_bound_and_independent_codes(bits):
    cfg = synth.CONFIGS["tiny"]
    w = synth.expert_weights(cfg, 0)[0]                    # [512,256] ~ N(0, 0.02)
    qmax = (1 << bits) - 1
    codes, sc, zr = O.quantize_pack(w, bits)
    q = _unpack(codes, bits)
    wf = widen(w)
    N, K = wf.shape
    G = K // 64
    s = np.repeat(f16(sc), 64, axis=1)
    m = np.repeat(f16(zr), 64, axis=1)
    grp = wf.reshape(N, G, 64)
    # stored zero is the group minimum (bf16 values of this size are fp16-exact)
    assert np.array_equal(f16(zr), grp.min(2))
    # stored scale is fp16((max-min)/qmax): numpy's own rounding of the exact quotient
    assert np.array_equal(f16(sc), ((grp.max(2) - grp.min(2)) / qmax).astype(np.float32).astype(np.float16).astype(np.float64))
    # dequantised values come from s*q + m
    deq = O.dequantize(codes, sc, zr, bits)
    assert np.array_equal(deq, s * q + m)
    # round-to-nearest error bound, min -> 0, max -> qmax.  The code is rint((w - m) * inv) with inv = fl(1/s) and
    # the product rounded once more: two binary32 roundings, so the computed quotient is within qmax * 2^-23 of the
    # exact one and a value that close to a tie may round either way, which lengthens the half step by the factor
    # 1 + qmax * 2^-22 at most: 3.6e-6 at 4 bits (inside the 2^-18 this test has always allowed), 6.1e-5 at 8 bits
    # (tested with twice that).
    slack = 2.0 ** -18 if bits <= 4 else qmax * 2.0 ** -21
    assert np.all(np.abs(wf - deq) <= 0.5 * s * (1 + slack))
    assert np.all(q.reshape(N, G, 64)[np.arange(N)[:, None], np.arange(G)[None, :], grp.argmin(2)] == 0)
    assert np.all(q.reshape(N, G, 64)[np.arange(N)[:, None], np.arange(G)[None, :], grp.argmax(2)] == qmax)
    # codes equal the fp64 rounding except close to a .5 tie
    exact = (wf - m) / s
    clear = np.abs(exact - np.floor(exact) - 0.5) > (1e-5 if bits <= 4 else 1e-4)      # several times qmax * 2^-23
    assert clear.mean() > 0.99
    assert np.array_equal(q[clear], np.clip(np.rint(exact), 0, qmax).astype(np.int64)[clear])


def test_quantize_subnormal_scale_and_ragged_group_rejection():
    # range so small that the fp16 scale is subnormal
    w = np.zeros((1, 64), np.float32)
    w[0, 1] = 2.0 ** -20
    codes, sc, zr = O.quantize_pack(bf16(w), 4)
    s = f16(sc)[0, 0]
    assert 0 < s < 2.0 ** -14
    # 2^-20 / 15 lies between 1 and 2 fp16 subnormal units and rounds to 1 unit, so the
    # largest element (16 units) saturates at code 15; the upper clamp is what keeps it legal
    assert s == 2.0 ** -24
    q = _unpack(codes, 4)[0]
    assert q[1] == 15 and q.sum() == 15
    assert O.dequantize(codes, sc, zr, 4)[0, 1] == 15 * 2.0 ** -24
    with pytest.raises(ValueError):
        O.quantize_pack(bf16(np.zeros((1, 96), np.float32)), 4, group=64)


# ------------------------------------------------------------------------- FFN

def _silu(a):
    return a / (1.0 + np.exp(-a))


def _tiny_layer(E=4, T=5, H=64, F=128, k=2, seed=0):
    rng = np.random.default_rng(seed)
    x = bf16(rng.standard_normal((T, H)))
    ws = [[bf16(rng.standard_normal(s) * 0.05) for s in ((F, H), (F, H), (H, F))] for _ in range(E)]
    idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    g = rng.random((T, k)) + 0.1
    g /= g.sum(1, keepdims=True)
    return x, ws, idx, g


def _numpy_moe(x, mats64, idx, g, skip=()):
    """MoE with fp64 weight matrices through numpy matmul."""
    xf = widen(x)
    T, H = xf.shape
    y = np.zeros((T, H))
    for t in range(T):
        for s in range(idx.shape[1]):
            e = int(idx[t, s])
            if e in skip:
                continue
            w1, w3, w2 = mats64[e]
            y[t] += g[t, s] * (w2 @ (_silu(w1 @ xf[t]) * (w3 @ xf[t])))
    return y


def test_ffn_all_bf16_is_plain_moe_and_dense_mlp():
    x, ws, idx, g = _tiny_layer()
    E = len(ws)
    y = O.moe_ffn_mixed(x, idx, g, np.full(E, 16, np.uint8), [{"w": w} for w in ws])
    ref = _numpy_moe(x, [[widen(m) for m in w] for w in ws], idx, g)
    assert np.allclose(y, ref, rtol=1e-11, atol=1e-13)
    # one expert, k = 1, weight 1: a dense SwiGLU MLP
    idx1 = np.zeros((x.shape[0], 1), np.int32)
    y1 = O.moe_ffn_mixed(x, idx1, np.ones((x.shape[0], 1)), np.array([16], np.uint8), [{"w": ws[0]}])
    w1, w3, w2 = [widen(m) for m in ws[0]]
    xf = widen(x)
    assert np.allclose(y1, (_silu(xf @ w1.T) * (xf @ w3.T)) @ w2.T, rtol=1e-11, atol=1e-13)


def test_ffn_mixed_precisions_use_dequantised_weights():
    x, ws, idx, g = _tiny_layer(E=4, seed=3)
    bits = np.array([16, 4, 2, 4], np.uint8)
    experts, mats = [], []
    for e, w in enumerate(ws):
        if bits[e] == 16:
            experts.append({"w": w})
            mats.append([widen(m) for m in w])
        else:
            q = [O.quantize_pack(m, int(bits[e])) for m in w]
            experts.append({"q": q})
            # weights rebuilt from brute-force unpacked codes, not from the oracle's dequantiser
            mats.append([np.repeat(f16(sc), 64, 1) * _unpack(cd, int(bits[e])) + np.repeat(f16(zr), 64, 1)
                         for cd, sc, zr in q])
    y = O.moe_ffn_mixed(x, idx, g, bits, experts)
    ref = _numpy_moe(x, mats, idx, g)
    assert np.allclose(y, ref, rtol=1e-11, atol=1e-13)
    # int2 is visibly different from bf16, so the precision switch is live
    y16 = O.moe_ffn_mixed(x, idx, g, np.full(4, 16, np.uint8), [{"w": w} for w in ws])
    assert np.abs(y - y16).max() > 1e-3 * np.abs(y16).max()


def test_ffn_zero_bit_skip_linearity_and_zero_gate():
    x, ws, idx, g = _tiny_layer(E=4, seed=5)
    experts = [{"w": w} for w in ws]
    mats = [[widen(m) for m in w] for w in ws]
    bits = np.array([16, 0, 16, 16], np.uint8)
    y = O.moe_ffn_mixed(x, idx, g, bits, experts)
    assert np.allclose(y, _numpy_moe(x, mats, idx, g, skip={1}), rtol=1e-11, atol=1e-13)
    # linear in the gate weights
    all16 = np.full(4, 16, np.uint8)
    ya = O.moe_ffn_mixed(x, idx, g, all16, experts)
    yb = O.moe_ffn_mixed(x, idx, 3.0 * g, all16, experts)
    assert np.allclose(yb, 3.0 * ya, rtol=1e-12)
    # W1 = 0 -> silu(0) = 0 -> y = 0
    zeroed = [{"w": [np.zeros_like(w[0]), w[1], w[2]]} for w in ws]
    assert not O.moe_ffn_mixed(x, idx, g, all16, zeroed).any()


def test_synth_configs_shapes():
    cfg = synth.CONFIGS["tiny"]
    x, heavy = synth.activations(cfg)
    assert x.shape == (16, 256) and x.dtype == np.uint16 and heavy.size == 0
    c3 = synth.scaled(synth.CONFIGS["mixtral_prefill"], H=128, F=256)
    x3, heavy3 = synth.activations(c3)
    n = np.linalg.norm(widen(x3), axis=1)
    assert heavy3.size == 26 and set(np.argsort(-n)[:26].tolist()) == set(heavy3.tolist())
    wg, bias = synth.router(synth.CONFIGS["fine_grained"])
    assert wg.shape == (128, 2048) and bias.shape == (128,) and bias.max() == 0.0
    assert abs(widen(wg).std() - 0.02) < 1e-3
    # same key, same bytes
    assert np.array_equal(synth.expert_weights(cfg, 3)[2], synth.expert_weights(cfg, 3)[2])
    assert sum(synth.CONFIGS["fine_grained"].tier_count) == 128


# ------------------------------------------------------------------ stack glue (not from the paper)

def test_bf16_rounding_of_the_stack_glue():
    # ties go to the even mantissa; the next representable value is 2^-7 above 1
    assert O.f64_to_bf16(1.0) == 0x3F80
    assert O.f64_to_bf16(1.0 + 2.0 ** -8) == 0x3F80          # tie -> even (down)
    assert O.f64_to_bf16(1.0 + 3 * 2.0 ** -8) == 0x3F82      # tie -> even (up)
    assert O.f64_to_bf16(1.0 + 2.0 ** -8 + 2.0 ** -20) == 0x3F81
    assert O.f64_to_bf16(-2.5) == 0xC020
    assert O.f64_to_bf16(0.0) == 0


def test_residual_rmsnorm_closed_forms():
    # (1, 2, -2, 0) has RMS 1.5 -> (2/3, 4/3, -4/3, 0), written here as bf16 bit patterns
    h = np.array([[0x3F80, 0x4000, 0xC000, 0x0000]], dtype=np.uint16)
    out = O.residual_rmsnorm(h, np.zeros((1, 4)), 1.0)
    assert out.tolist() == [[0x3F2B, 0x3FAB, 0xBFAB, 0x0000]]
    # y enters scaled by alpha: h = 0, y = (4, 0, 0, 0), alpha = 0.5 -> v = (2, 0, 0, 0), RMS 1 -> (2, 0, 0, 0)
    z = np.zeros((1, 4), dtype=np.uint16)
    assert O.residual_rmsnorm(z, np.array([[4.0, 0, 0, 0]]), 0.5).tolist() == [[0x4000, 0, 0, 0]]
    # scale invariance: multiplying h and y by 4 changes nothing; a zero row stays zero
    rng = np.random.default_rng(5)
    hb = synth.f32_to_bf16_bits(rng.standard_normal((3, 64)).astype(np.float32))
    y = rng.standard_normal((3, 64))
    hb[2] = 0
    y[2] = 0.0
    a = O.residual_rmsnorm(hb, y, 0.25)
    h4 = synth.f32_to_bf16_bits(4.0 * synth.bf16_bits_to_f32(hb))
    assert np.array_equal(a, O.residual_rmsnorm(h4, 4.0 * y, 0.25))
    assert (a[2] == 0).all()
    rms = np.sqrt((synth.bf16_bits_to_f32(a[:2]).astype(np.float64) ** 2).mean(axis=1))
    assert np.allclose(rms, 1.0, atol=2e-3)


def test_predicted_frequency_counts_and_cut():
    """Eq. 7: the counts are a histogram of the predicted top-k sets (sum = T k); the list is the t
    largest counts, lower index first among equals, and never names an expert nobody asked for."""
    cfg = synth.scaled(synth.CONFIGS["tiny"], T=12, config_id=31)
    x, _ = synth.activations(cfg)
    wg, _ = synth.router(cfg)
    c, pred, lg = O.predicted_frequency(x, wg, 2, 3)
    assert c.sum() == 12 * 2 and lg.shape == (12, 8)
    top2 = np.argsort(-lg, axis=1, kind="stable")[:, :2]
    assert np.array_equal(c, np.bincount(top2.ravel(), minlength=8))
    assert pred == sorted(range(8), key=lambda e: (-c[e], e))[:3]
    # one token, k = 2, t = 5: only the two experts it asks for
    c1, pred1, lg1 = O.predicted_frequency(x[:1], wg, 2, 5)
    assert sorted(pred1) == sorted(top2[0].tolist()) and c1.sum() == 2
    # the first layer of the prefill composition: k_hh = T makes Eq. 2's importance the load itself
    mats = synth.expert_weights(cfg, 0)
    h, log, preds = O.prefill_stack(x, [wg, wg], lambda l, e: mats, 2, 12, (8,), (16,), None, 0.25, predict_t=3)
    idx, bits, _, imp, load = log[0]
    assert np.array_equal(imp, load) and load.sum() == 24 and (bits == 16).all()
    assert preds[0][1] == pred and np.array_equal(preds[0][0], c)      # same router, same input
    # identical experts, all 16-bit: the layer is a dense SwiGLU MLP with gate weights summing to one
    y = O.moe_ffn_mixed(x, idx, np.full(idx.shape, 0.5), np.full(8, 16, np.uint8), [{"w": mats}] * 8)
    assert np.array_equal(O.residual_rmsnorm(x, y, 0.25), O.prefill_stack(x, [wg], lambda l, e: mats, 2, 12, (8,), (16,), None, 0.25)[0])


# ------------------------------------------------- the one-token stack of layers (Sec. 4.1 steps 1-6)

def _np_bf16_rne(v):
    """float64 array -> bf16 bit patterns, nearest, ties to the even mantissa (directly, no detour through
    binary32's own rounding: the two candidates are compared in fp64)."""
    v = np.asarray(v, np.float64)
    lo = (np.abs(v).astype(np.float32).view(np.uint32) >> 16).astype(np.uint32)   # a neighbour at or next to |v|
    out = np.zeros(v.shape, np.uint16)
    for i in np.ndindex(v.shape):
        a = abs(float(v[i]))
        c = int(lo[i])
        cands = [c - 1, c, c + 1] if c > 0 else [c, c + 1]
        val = lambda bits: float(np.array([bits << 16], np.uint32).view(np.float32)[0])
        best = min(cands, key=lambda bts: (abs(val(bts) - a), bts & 1))
        out[i] = best | (0x8000 if np.signbit(v[i]) else 0)
    return out


def _np_decode_stack(h_bits, routers, mats_fn, k, tier_count, tier_bits, floors, alpha, run_bits=None):
    """The one-token stack written out with numpy only (matmul, exp, sorted): softmax gate, top-k, decode
    importance = gate probability, tiers by rank with the layer's floor, dequantised weights rebuilt from
    brute-force unpacked codes, SwiGLU, residual + RMS normalisation.  Returns the final hidden state, the
    per-layer (selected experts, their assigned bits) and the per-layer inputs."""
    h = np.array(h_bits, np.uint16, copy=True)
    trace, inputs = [], []
    for l, wg in enumerate(routers):
        inputs.append(h.copy())
        hf = widen(h)[0]
        E = wg.shape[0]
        logits = widen(wg) @ hf
        sel = sorted(range(E), key=lambda e: (-logits[e], e))[:k]
        p = np.exp(logits - logits.max())
        p /= p.sum()
        g = p[sel] / p[sel].sum()
        order = sorted(range(E), key=lambda e: (-p[e], -(1 if e in sel else 0), e))
        bits = np.zeros(E, np.int64)
        pos = 0
        for n, b in zip(tier_count, tier_bits):
            for e in order[pos:pos + n]:
                bits[e] = max(b, floors[l] if floors else 0)
            pos += n
        y = np.zeros_like(hf)
        for e, ge in zip(sel, g):
            b = int(bits[e])
            if b == 0:
                continue
            if run_bits is not None:
                b = int(run_bits[l].get(e, b))
            ws = mats_fn(l, e)
            if b == 16:
                w1, w3, w2 = [widen(m) for m in ws]
            else:
                w1, w3, w2 = [np.repeat(f16(sc), 64, 1) * _unpack(cd, b) + np.repeat(f16(zr), 64, 1)
                              for cd, sc, zr in (O.quantize_pack(m, b) for m in ws)]
            y += ge * (w2 @ (_silu(w1 @ hf) * (w3 @ hf)))
        v = hf + alpha * y
        h = _np_bf16_rne(v / np.sqrt((v * v).mean()))[None, :]
        trace.append((sel, [int(bits[e]) for e in sel]))
    return h, trace, inputs


def _stack_case(L=3, E=4, H=64, F=128, seed=11):
    rng = np.random.default_rng(seed)
    h0 = bf16(rng.standard_normal((1, H)))
    routers = [bf16(rng.standard_normal((E, H)) * 0.2) for _ in range(L)]
    ws = {(l, e): [bf16(rng.standard_normal(s) * 0.08) for s in ((F, H), (F, H), (H, F))]
          for l in range(L) for e in range(E)}
    return h0, routers, (lambda l, e: ws[(l, e)])


def _same_hidden(a, b):
    """bf16 rows equal up to the last place on a few elements (the two sides add their fp64 terms in a different order)."""
    fa, fb = widen(a), widen(b)
    return (a == b).mean() >= 0.97 and np.all(np.abs(fa - fb) <= 2.0 ** -7 * np.maximum(np.abs(fa), 2.0 ** -6))


def test_decode_stack_against_a_numpy_composition():
    """Three layers, tiers 1/1/2 at 16/4/2 bits, a floor that differs from layer to layer: every routing and precision
    decision and the hidden state agree with the stack written out in numpy; the floor lands on its own layer."""
    h0, routers, mats = _stack_case()
    tiers, tbits, floors = (1, 1, 2), (16, 4, 2), [4, 2, 16]
    h, log, preds = O.decode_stack(h0, routers, mats, 2, tiers, tbits, floors, 0.5, predict_t=2)
    ref_h, trace, inputs = _np_decode_stack(h0, routers, mats, 2, tiers, tbits, floors, 0.5)
    assert len(log) == 3
    for l in range(3):
        idx, bits_of_idx, logits, imp = log[l]
        assert idx[0].tolist() == trace[l][0] and bits_of_idx.tolist() == trace[l][1]
        assert np.allclose(logits[0], widen(routers[l]) @ widen(inputs[l])[0], rtol=1e-12, atol=1e-12)
        assert np.allclose(imp.sum(), 1.0) and np.argmax(imp) == idx[0][0]          # Eq. 3: importance is the gate score
    # rank 0 gets bf16, rank 1 int4 (tiers 1/1/2); floors: layer 0 lifts nothing (both already >= 4), layer 2 lifts int4 -> 16
    assert [t[1] for t in trace] == [[16, 4], [16, 4], [16, 16]]
    assert _same_hidden(h, ref_h)
    # a floor of 4 on every layer changes nothing here (the two active experts never drop below 4), one of 16 on
    # layer 1 alone changes that layer's second expert and nothing before it
    h_b, log_b, _ = O.decode_stack(h0, routers, mats, 2, tiers, tbits, [4, 16, 16], 0.5)
    assert log_b[0][1].tolist() == [16, 4] and log_b[1][1].tolist() == [16, 16]
    assert np.array_equal(log_b[0][0], log[0][0]) and np.array_equal(log_b[0][2], log[0][2])
    assert not np.array_equal(h_b, h)
    # Eq. 6 / Eq. 8: the prediction made at layer l is the top-t of the NEXT router on layer l's input; the last
    # layer predicts nothing
    assert len(preds) == 2
    for l in range(2):
        nxt = widen(routers[l + 1]) @ widen(inputs[l])[0]
        assert preds[l] == sorted(range(4), key=lambda e: (-nxt[e], e))[:2]
    assert O.decode_stack(h0, routers, mats, 2, tiers, tbits, floors, 0.5)[2] == []


def test_decode_stack_single_layer_run_bits_and_dense_special_case():
    h0, routers, mats = _stack_case(L=2, seed=23)
    tiers, tbits = (1, 1, 2), (16, 4, 2)
    # L = 1 is the single-layer chain of the pinned functions
    h1, log1, _ = O.decode_stack(h0, routers[:1], mats, 2, tiers, tbits, None, 0.25)
    idx, w, probs, _ = O.route_topk(h0, routers[0], None, 2)
    bits, _ = O.assign_precision(O.expert_importance_decode(probs), np.bincount(idx.ravel(), minlength=4), tiers, tbits)
    ex = [({"w": mats(0, e)} if bits[e] == 16 else {"q": [O.quantize_pack(m, int(bits[e])) for m in mats(0, e)]})
          if e in idx[0] else {} for e in range(4)]
    use = np.array([bits[e] if e in idx[0] else 0 for e in range(4)], np.uint8)
    assert np.array_equal(h1, O.residual_rmsnorm(h0, O.moe_ffn_mixed(h0, idx, w, use, ex), 0.25))
    assert log1[0][1].tolist() == [16, 4]
    # run_bits (Conservative Reuse: a resident higher precision is run instead of the assigned one): naming the
    # int4 expert of layer 0 at 16 bits changes the arithmetic of that expert only: the decisions logged for layer 0
    # stay, the result equals the numpy stack told the same, and naming an expert that is not active changes nothing
    e4 = int(idx[0][1])
    idle = [e for e in range(4) if e not in idx[0]][0]
    base = O.decode_stack(h0, routers, mats, 2, tiers, tbits, None, 0.25)
    over = O.decode_stack(h0, routers, mats, 2, tiers, tbits, None, 0.25, run_bits=[{e4: 16}, {}])
    same = O.decode_stack(h0, routers, mats, 2, tiers, tbits, None, 0.25, run_bits=[{idle: 16}, {}])
    assert over[1][0][1].tolist() == [16, 4] and np.array_equal(over[1][0][0], base[1][0][0])
    assert np.array_equal(same[0], base[0]) and not np.array_equal(over[0], base[0])
    ref_over, _, _ = _np_decode_stack(h0, routers, mats, 2, tiers, tbits, None, 0.25, run_bits=[{e4: 16}, {}])
    ref_base, _, _ = _np_decode_stack(h0, routers, mats, 2, tiers, tbits, None, 0.25)
    assert _same_hidden(over[0], ref_over) and _same_hidden(base[0], ref_base)
    # all experts identical and 16-bit: every layer is the dense SwiGLU MLP of that one expert (gate weights sum to 1)
    one = mats(0, 0)
    w1, w3, w2 = [widen(m) for m in one]
    hd = O.decode_stack(h0, routers, lambda l, e: one, 2, (4,), (16,), None, 0.5)[0]
    ref = np.array(h0, copy=True)
    for _ in range(2):
        hf = widen(ref)[0]
        v = hf + 0.5 * (w2 @ (_silu(w1 @ hf) * (w3 @ hf)))
        ref = _np_bf16_rne(v / np.sqrt((v * v).mean()))[None, :]
    assert _same_hidden(hd, ref)


# ---------------------------------------------------------------- attention-derived token score

def _harmonic(n):
    return sum(1.0 / j for j in range(1, n + 1))


def test_attention_score_closed_forms():
    rng = np.random.default_rng(5)
    T, Hh, Hkv, d = 9, 4, 2, 16
    k = bf16(rng.standard_normal((T, Hkv, d)))
    zero_q = bf16(np.zeros((T, Hh, d)))
    # all logits equal: every query spreads its unit of attention evenly over the keys it sees
    s = O.token_score_attention(zero_q, k, Hh, Hkv, causal=False)
    assert np.allclose(s, 1.0 / T, rtol=0, atol=1e-15)
    s = O.token_score_attention(zero_q, k, Hh, Hkv, causal=True)
    want = [(_harmonic(T) - _harmonic(i)) / T for i in range(T)]      # key i is seen by queries i..T-1, 1/(q+1) each
    assert np.allclose(s, want, rtol=0, atol=1e-15)
    # one key dominates: keys = 0 but key 3 = 40 e_0, queries = e_0; exp(-10) mass elsewhere
    kk = np.zeros((T, 1, d), np.float32)
    kk[3, 0, 0] = 40.0
    qq = np.zeros((T, 2, d), np.float32)
    qq[:, :, 0] = 1.0
    s = O.token_score_attention(bf16(qq), bf16(kk), 2, 1, causal=False)       # scale 1/4: logit 10 at key 3
    p3 = np.exp(10.0) / (np.exp(10.0) + (T - 1))
    assert np.isclose(s[3], p3, rtol=1e-14) and np.allclose(np.delete(s, 3), (1 - p3) / (T - 1), rtol=1e-12)
    # causal: queries before token 3 do not see it
    s = O.token_score_attention(bf16(qq), bf16(kk), 2, 1, causal=True)
    want3 = sum(np.exp(10.0) / (np.exp(10.0) + q) for q in range(3, T)) / T
    assert np.isclose(s[3], want3, rtol=1e-14)


def test_attention_score_invariants_and_brute_force():
    rng = np.random.default_rng(6)
    T, Hh, Hkv, d = 7, 4, 2, 8
    q = bf16(rng.standard_normal((T, Hh, d)))
    k = bf16(rng.standard_normal((T, Hkv, d)))
    for causal in (False, True):
        s = O.token_score_attention(q, k, Hh, Hkv, causal=causal)
        assert np.isclose(s.sum(), 1.0, rtol=1e-14)                        # every query hands out one unit
        # brute force, one probability at a time
        qf, kf = widen(q), widen(k)
        ref = np.zeros(T)
        for h in range(Hh):
            for i in range(T):
                keys = range(i + 1) if causal else range(T)
                lg = {j: float(np.dot(qf[i, h], kf[j, h // 2])) / np.sqrt(d) for j in keys}
                z = sum(np.exp(v) for v in lg.values())
                for j, v in lg.items():
                    ref[j] += np.exp(v) / z / (Hh * T)
        assert np.allclose(s, ref, rtol=1e-12)
    # without a mask the score follows the keys when the tokens are permuted (queries are averaged over)
    perm = rng.permutation(T)
    s0 = O.token_score_attention(q, k, Hh, Hkv, causal=False)
    s1 = O.token_score_attention(q[perm], k[perm], Hh, Hkv, causal=False)
    assert np.allclose(s1, s0[perm], rtol=1e-13)
    # a common shift of all keys of a head changes every logit of a row alike: softmax unchanged
    s2 = O.token_score_attention(q, bf16(widen(k) * 2.0), Hh, Hkv, causal=True, scale=0.5 / np.sqrt(d))
    assert np.allclose(s2, O.token_score_attention(q, k, Hh, Hkv, causal=True), rtol=1e-13)


def test_attention_inputs_make_the_heavy_hitters_score_highest():
    cfg = synth.scaled(synth.CONFIGS["mixtral_prefill"], T=256, k_hh=13, config_id=41)
    q, k, heavy = synth.attention_inputs(cfg, 8, 2, 64, boost=1.5)
    assert heavy.size == 13
    s = O.token_score_attention(q, k, 8, 2, causal=False)
    assert set(np.argsort(-s)[:13].tolist()) == set(heavy.tolist())


# ------------------------------------------------- error-compensated quantizer (Sec. 5: GPTQ)

def _calib_case(cid, N, K, n=384, sigma=0.02):
    xb = synth.calibration_inputs(cid, n, K)
    wb = synth.normal_bf16(cid, 77, (N, K), sigma)
    return xb, wb, widen(wb)


def test_gptq_hessian_brute_force():
    xb = synth.calibration_inputs(911, 9, 6, rank=2)
    x = widen(xb)
    want = np.zeros((6, 6))
    for s in range(9):
        for i in range(6):
            for j in range(6):
                want[i, j] += x[s, i] * x[s, j]
    got = O.gptq_hessian(xb)
    assert np.allclose(got, want, rtol=1e-13, atol=0) and np.array_equal(got, got.T)


def test_gptq_factor_closed_forms_and_definition():
    # 2 x 2 without damping: H^-1 = [[c, -b], [-b, a]] / det  =>  U = [[sqrt(c/det), -b/sqrt(c det)], [0, 1/sqrt(c)]]
    a, b, c = 5.0, 1.5, 2.0
    det = a * c - b * b
    U = O.gptq_factor(np.array([[a, b], [b, c]]), damp=0.0)
    assert np.allclose(U, [[np.sqrt(c / det), -b / np.sqrt(c * det)], [0.0, 1.0 / np.sqrt(c)]], rtol=1e-13)
    # diagonal H with damping: U = diag(1 / sqrt(h + damp mean h)); a dead column counts as h = 1
    h = np.array([4.0, 0.0, 9.0, 1.0])
    hd = np.array([4.0, 1.0, 9.0, 1.0])
    U = O.gptq_factor(np.diag(h), damp=0.1)
    assert np.allclose(U, np.diag(1.0 / np.sqrt(hd + 0.1 * hd.mean())), rtol=1e-13)
    # general: upper triangular, positive diagonal, U^T U (H + damping) = I
    xb, _, _ = _calib_case(912, 1, 192)
    H = O.gptq_hessian(xb)
    U = O.gptq_factor(H, damp=0.01)
    assert np.array_equal(U, np.triu(U)) and (np.diag(U) > 0).all()
    Hd = H + 0.01 * np.mean(np.diag(H)) * np.eye(192)
    assert np.abs(U.T @ U @ Hd - np.eye(192)).max() < 1e-8


def test_gptq_sweep_hand_example():
    """One group of 4 columns, 2 bits: lo = 0, hi = 3, scale 1, zero 0.  Column 1 holds 0.375 -> code 0,
    error 0.375, divided by U[1,1] = 0.5 -> e = 0.75; U[1,2] = -1 moves column 2 from 1.0 to 1.75 -> code 2
    (plain rounding gives 1).  A flipped sign gives 0.25 -> 0, a transposed U or a dropped update gives 1,
    a dropped division gives 1.375 -> 1."""
    w = bf16(np.array([[0.0, 0.375, 1.0, 3.0]]))
    U = np.eye(4)
    U[1, 1] = 0.5
    U[1, 2] = -1.0
    codes, scale, zero = O.gptq_quantize_pack(w, U, 2, group=4)
    assert O.f16_to_f32(int(scale[0, 0])) == 1.0 and O.f16_to_f32(int(zero[0, 0])) == 0.0
    assert codes[0, 0] == (0 | 0 << 2 | 2 << 4 | 3 << 6)
    plain, _, _ = O.quantize_pack(w, 2, group=4)
    assert plain[0, 0] == (0 | 0 << 2 | 1 << 4 | 3 << 6)
    # the same through the fp64 twin and the one-column-at-a-time form (H^-1 = U^T U)
    q, _ = O.gptq_sweep_f64(widen(w), U, 2, group=4)
    assert q.tolist() == [[0, 0, 2, 3]]
    q, _ = O.gptq_sweep_textbook(widen(w), np.linalg.inv(U.T @ U), 2, group=4)
    assert q.tolist() == [[0, 0, 2, 3]]


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_gptq_identity_factor_is_the_plain_quantizer(bits):
    _, wb, _ = _calib_case(913, 24, 192)
    got = O.gptq_quantize_pack(wb, np.eye(192), bits)
    want = O.quantize_pack(wb, bits)
    for g, r in zip(got, want):
        assert np.array_equal(g, r)
    # and a factor scaled by a power of two changes nothing (e / U[c,c] * U[c,j] is scale free)
    xb, _, _ = _calib_case(913, 1, 192)
    U = O.gptq_factor(O.gptq_hessian(xb)).astype(np.float32)
    a = O.gptq_quantize_pack(wb, U, bits)
    b = O.gptq_quantize_pack(wb, U * np.float32(4.0), bits)
    for g, r in zip(a, b):
        assert np.array_equal(g, r)


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_gptq_factor_rows_equal_the_column_by_column_definition(bits):
    """The sweep with rows of U is the textbook procedure (quantise a column, correct the rest with the
    current inverse Hessian, eliminate the column): same codes, same corrected weights."""
    xb, wb, w = _calib_case(914 + bits, 12, 192)
    H = O.gptq_hessian(xb)
    Hd = O.gptq_damped(H)
    U = O.gptq_factor(H)
    q1, d1 = O.gptq_sweep_f64(w, U, bits)
    q2, d2 = O.gptq_sweep_textbook(w, Hd, bits)
    assert np.array_equal(q1, q2) and np.abs(d1 - d2).max() < 1e-9
    # binary32 sweep against the fp64 twin: a near-tie may flip a code here and there, nothing more
    codes, sc, ze = O.gptq_quantize_pack(wb, U, bits)
    d3 = O.dequantize(codes, sc, ze, bits)
    assert (d3 == d1).mean() > 0.995
    e1, e3 = O.output_error(w, d1, H), O.output_error(w, d3, H)
    assert abs(e3 - e1) <= 0.02 * e1


@pytest.mark.parametrize("bits", [2, 4])
def test_gptq_lowers_the_output_error_on_correlated_inputs(bits):
    xb, wb, w = _calib_case(920, 32, 256, n=512)
    H = O.gptq_hessian(xb)
    U = O.gptq_factor(H)
    codes, sc, ze = O.gptq_quantize_pack(wb, U, bits)
    plain = O.quantize_pack(wb, bits)
    e_comp = O.output_error(w, O.dequantize(codes, sc, ze, bits), H)
    e_plain = O.output_error(w, O.dequantize(*plain, bits), H)
    # measured directly on the inputs, not through H: || (W - What) X^T ||^2
    x = widen(xb)
    direct = float((((w - O.dequantize(codes, sc, ze, bits)) @ x.T) ** 2).sum())
    assert abs(direct - e_comp) <= 1e-9 * e_comp
    assert e_comp < 0.5 * e_plain
