"""numpy-facing wrapper of the C oracle (oracle/dymoe_oracle.c).

Test infrastructure only.  Every function takes and returns numpy arrays;
bf16 / fp16 tensors travel as uint16 bit patterns.  The arithmetic lives in
the C file; this module only marshals arguments.
"""
import ctypes as C

import numpy as np

from . import build as _build

_lib = C.CDLL(_build.build())

_u16p = C.POINTER(C.c_uint16)
_u8p = C.POINTER(C.c_uint8)
_i32p = C.POINTER(C.c_int32)
_f64p = C.POINTER(C.c_double)
_f32p = C.POINTER(C.c_float)


def _ptr(a, typ):
    return a.ctypes.data_as(typ) if a is not None else typ()


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


_lib.oracle_f32_to_f16.restype = C.c_uint16
_lib.oracle_f32_to_f16.argtypes = [C.c_float]
_lib.oracle_f16_to_f32.restype = C.c_float
_lib.oracle_f16_to_f32.argtypes = [C.c_uint16]
_lib.oracle_bf16_to_f32.restype = C.c_float
_lib.oracle_bf16_to_f32.argtypes = [C.c_uint16]
_lib.oracle_retention_ratio.restype = C.c_double
_lib.oracle_retention_ratio.argtypes = [C.c_int, C.c_int, C.c_double]
_lib.oracle_depth_schedule.restype = C.c_int
_lib.oracle_depth_schedule.argtypes = [C.c_int, C.c_int, C.c_double, C.c_int]
_lib.oracle_route_topk.restype = C.c_int
_lib.oracle_route_topk.argtypes = [_u16p, _u16p, _f32p, C.c_int, C.c_int, C.c_int, C.c_int,
                                   C.c_int, _i32p, _f64p, _f64p, _f64p]
_lib.oracle_token_score_norm.restype = None
_lib.oracle_token_score_norm.argtypes = [_u16p, C.c_int, C.c_int, _f64p]
_lib.oracle_expert_importance_prefill.restype = C.c_int
_lib.oracle_expert_importance_prefill.argtypes = [_i32p, _f64p, C.c_int, C.c_int, C.c_int,
                                                  C.c_int, _i32p, _i32p, _u8p]
_lib.oracle_expert_importance_decode.restype = None
_lib.oracle_expert_importance_decode.argtypes = [_f64p, C.c_int, C.c_int, _f64p]
_lib.oracle_assign_precision.restype = C.c_int
_lib.oracle_assign_precision.argtypes = [_f64p, _i32p, C.c_int, C.c_int, _i32p, _u8p, C.c_int,
                                         _u8p, _i32p]
_lib.oracle_quantize_pack.restype = C.c_int
_lib.oracle_quantize_pack.argtypes = [_u16p, C.c_long, C.c_long, C.c_int, C.c_int, _u8p, _u16p,
                                      _u16p]
_lib.oracle_dequantize.restype = None
_lib.oracle_dequantize.argtypes = [_u8p, _u16p, _u16p, C.c_long, C.c_long, C.c_int, C.c_int,
                                   _f64p]
_pp = C.POINTER(C.c_void_p)
_lib.oracle_moe_ffn_mixed.restype = C.c_int
_lib.oracle_moe_ffn_mixed.argtypes = [_u16p, _i32p, _f64p, _u8p, _pp, _pp, _pp, _pp, C.c_int,
                                      C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _f64p]


def f32_to_f16(v: float) -> int:
    return int(_lib.oracle_f32_to_f16(float(v)))


def f16_to_f32(bits: int) -> float:
    return float(_lib.oracle_f16_to_f32(int(bits)))


def bf16_to_f32(bits: int) -> float:
    return float(_lib.oracle_bf16_to_f32(int(bits)))


def retention_ratio(layer, n_layers, lam):
    return float(_lib.oracle_retention_ratio(layer, n_layers, lam))


def depth_schedule(layer, n_layers, lam, M):
    return int(_lib.oracle_depth_schedule(layer, n_layers, lam, M))


def route_topk(x_bits, wg_bits, bias, k, renorm=True):
    """x [T,H], wg [E,H] as bf16 bit patterns (uint16); bias [E] float32 or None.
    Returns idx [T,k] int32, w [T,k] f64, probs [T,E] f64, logits [T,E] f64."""
    x = _c(x_bits, np.uint16)
    wg = _c(wg_bits, np.uint16)
    T, H = x.shape
    E = wg.shape[0]
    assert wg.shape[1] == H
    b = _c(bias, np.float32) if bias is not None else None
    idx = np.zeros((T, k), np.int32)
    w = np.zeros((T, k), np.float64)
    probs = np.zeros((T, E), np.float64)
    logits = np.zeros((T, E), np.float64)
    rc = _lib.oracle_route_topk(_ptr(x, _u16p), _ptr(wg, _u16p), _ptr(b, _f32p), T, H, E, k,
                                1 if renorm else 0, _ptr(idx, _i32p), _ptr(w, _f64p),
                                _ptr(probs, _f64p), _ptr(logits, _f64p))
    if rc != 0:
        raise ValueError("oracle_route_topk rc=%d" % rc)
    return idx, w, probs, logits


def token_score_norm(x_bits):
    x = _c(x_bits, np.uint16)
    T, H = x.shape
    s = np.zeros(T, np.float64)
    _lib.oracle_token_score_norm(_ptr(x, _u16p), T, H, _ptr(s, _f64p))
    return s


def expert_importance_prefill(idx, score, E, k_hh):
    """Returns importance [E] int32, load [E] int32, heavy [T] uint8."""
    idx = _c(idx, np.int32)
    T, k = idx.shape
    score = _c(score, np.float64)
    assert score.shape == (T,)
    imp = np.zeros(E, np.int32)
    load = np.zeros(E, np.int32)
    heavy = np.zeros(max(T, 1), np.uint8)
    rc = _lib.oracle_expert_importance_prefill(_ptr(idx, _i32p), _ptr(score, _f64p), T, E, k,
                                               k_hh, _ptr(imp, _i32p), _ptr(load, _i32p),
                                               _ptr(heavy, _u8p))
    if rc != 0:
        raise ValueError("oracle_expert_importance_prefill rc=%d" % rc)
    return imp, load, heavy[:T]


def expert_importance_decode(probs):
    probs = _c(probs, np.float64)
    T, E = probs.shape
    imp = np.zeros(E, np.float64)
    _lib.oracle_expert_importance_decode(_ptr(probs, _f64p), T, E, _ptr(imp, _f64p))
    return imp


def assign_precision(importance, load, tier_count, tier_bits, floor_bits=0):
    """Returns bits [E] uint8, rank [E] int32."""
    imp = _c(importance, np.float64)
    E = imp.shape[0]
    ld = _c(load, np.int32) if load is not None else None
    tc = _c(tier_count, np.int32)
    tb = _c(tier_bits, np.uint8)
    bits = np.zeros(E, np.uint8)
    rank = np.zeros(E, np.int32)
    rc = _lib.oracle_assign_precision(_ptr(imp, _f64p), _ptr(ld, _i32p), E, len(tc),
                                      _ptr(tc, _i32p), _ptr(tb, _u8p), floor_bits,
                                      _ptr(bits, _u8p), _ptr(rank, _i32p))
    if rc != 0:
        raise ValueError("oracle_assign_precision rc=%d" % rc)
    return bits, rank


def quantize_pack(w_bits, bits, group=64):
    """w [N,K] bf16 bit patterns.  Returns codes [N,K*bits/8] uint8,
    scale [N,K/group] and zero [N,K/group] as fp16 bit patterns (uint16)."""
    w = _c(w_bits, np.uint16)
    N, K = w.shape
    codes = np.zeros((N, K * bits // 8), np.uint8)
    scale = np.zeros((N, K // group), np.uint16)
    zero = np.zeros((N, K // group), np.uint16)
    rc = _lib.oracle_quantize_pack(_ptr(w, _u16p), N, K, bits, group, _ptr(codes, _u8p),
                                   _ptr(scale, _u16p), _ptr(zero, _u16p))
    if rc != 0:
        raise ValueError("oracle_quantize_pack rc=%d" % rc)
    return codes, scale, zero


def dequantize(codes, scale, zero, bits, group=64):
    codes = _c(codes, np.uint8)
    scale = _c(scale, np.uint16)
    zero = _c(zero, np.uint16)
    N = codes.shape[0]
    K = codes.shape[1] * 8 // bits
    out = np.zeros((N, K), np.float64)
    _lib.oracle_dequantize(_ptr(codes, _u8p), _ptr(scale, _u16p), _ptr(zero, _u16p), N, K, bits,
                           group, _ptr(out, _f64p))
    return out


def moe_ffn_mixed(x_bits, idx, w, bits, experts, group=64):
    """experts: list of E dicts; expert e holds, for the precision bits[e],
    either 'w' = (W1,W3,W2) bf16 bit arrays, or 'q' = three (codes, scale, zero)
    triples as produced by quantize_pack.  Returns y [T,H] f64."""
    x = _c(x_bits, np.uint16)
    idx = _c(idx, np.int32)
    w = _c(w, np.float64)
    bits = _c(bits, np.uint8)
    T, H = x.shape
    k = idx.shape[1]
    E = len(experts)
    keep = []
    tabs = [(C.c_void_p * (3 * E))() for _ in range(4)]
    F = None
    for e, ex in enumerate(experts):
        b = int(bits[e])
        if b == 16:
            mats = [_c(m, np.uint16) for m in ex["w"]]
            keep.append(mats)
            F = mats[0].shape[0]
            assert mats[0].shape == (F, H) and mats[1].shape == (F, H) and mats[2].shape == (H, F)
            for i in range(3):
                tabs[0][3 * e + i] = mats[i].ctypes.data
        elif b in (8, 4, 2):
            for i in range(3):
                cd, sc, zr = ex["q"][i] if "q" in ex else ex["q%d" % b][i]
                cd, sc, zr = _c(cd, np.uint8), _c(sc, np.uint16), _c(zr, np.uint16)
                keep.append((cd, sc, zr))
                tabs[1][3 * e + i] = cd.ctypes.data
                tabs[2][3 * e + i] = sc.ctypes.data
                tabs[3][3 * e + i] = zr.ctypes.data
                if i == 0:
                    F = cd.shape[0]
        elif b != 0:
            raise ValueError("bits[%d]=%d" % (e, b))
    if F is None:
        raise ValueError("no expert with a non-zero precision")
    y = np.zeros((T, H), np.float64)
    rc = _lib.oracle_moe_ffn_mixed(_ptr(x, _u16p), _ptr(idx, _i32p), _ptr(w, _f64p),
                                   _ptr(bits, _u8p), tabs[0], tabs[1], tabs[2], tabs[3], T, H, F,
                                   E, k, group, _ptr(y, _f64p))
    if rc != 0:
        raise ValueError("oracle_moe_ffn_mixed rc=%d" % rc)
    return y


_lib.oracle_f64_to_bf16.restype = C.c_uint16
_lib.oracle_f64_to_bf16.argtypes = [C.c_double]
_lib.oracle_residual_rmsnorm.restype = None
_lib.oracle_residual_rmsnorm.argtypes = [_u16p, _f64p, C.c_double, C.c_int, C.c_int, _u16p]


def f64_to_bf16(v: float) -> int:
    return int(_lib.oracle_f64_to_bf16(float(v)))


def residual_rmsnorm(h_bits, y, alpha=1.0):
    """h [T,H] bf16 bits, y [T,H] f64 -> bf16 bits of (h + alpha*y) / rms(h + alpha*y)."""
    h = _c(h_bits, np.uint16)
    y = _c(y, np.float64)
    T, H = h.shape
    out = np.zeros((T, H), np.uint16)
    _lib.oracle_residual_rmsnorm(_ptr(h, _u16p), _ptr(y, _f64p), float(alpha), T, H, _ptr(out, _u16p))
    return out


def decode_stack(h0_bits, routers, expert_matrices, k, tier_count, tier_bits, floor_bits, alpha,
                 predict_t=0, run_bits=None):
    """A stack of expert layers on one token (composition of the functions above,
    no arithmetic of its own): per layer gating, decode importance, assignment
    (with the layer's floor), quantisation of the active experts to their
    assigned width, FFN, residual + normalisation.
    routers: list of wg [E,H] bf16 bits; expert_matrices(layer, e) -> (W1, W3, W2) bf16 bits.
    run_bits: None, or per layer a dict {expert: bits} naming the precision an active expert is
    actually run at (a cache may hold, and then reuse, a higher precision than the assigned one).
    Returns (final h bits, per-layer list of (idx, bits of idx, logits, importance),
    per-layer predicted top-t experts of the NEXT layer from this layer's input)."""
    h = _c(h0_bits, np.uint16)
    log, preds = [], []
    for l, wg in enumerate(routers):
        E = wg.shape[0]
        idx, w, probs, logits = route_topk(h, wg, None, k)
        if predict_t and l + 1 < len(routers):
            pidx, _, _, _ = route_topk(h, routers[l + 1], None, predict_t)
            preds.append([int(v) for v in pidx[0]])
        imp = expert_importance_decode(probs)
        load = np.bincount(idx.ravel(), minlength=E).astype(np.int32)
        bits, _ = assign_precision(imp, load, tier_count, tier_bits, floor_bits[l] if floor_bits else 0)
        experts = []
        use_bits = np.zeros(E, np.uint8)
        for e in range(E):
            b = int(bits[e])
            if e not in idx[0] or b == 0:
                experts.append({})
                continue
            if run_bits is not None:
                b = int(run_bits[l].get(e, b))
            use_bits[e] = b
            mats = expert_matrices(l, e)
            experts.append({"w": mats} if b == 16 else {"q": [quantize_pack(m, b) for m in mats]})
        if use_bits.any():
            y = moe_ffn_mixed(h, idx, w, use_bits, experts)
        else:
            y = np.zeros(h.shape, np.float64)
        log.append((idx.copy(), bits[idx[0]].copy(), logits.copy(), imp.copy()))
        h = residual_rmsnorm(h, y, alpha)
    return h, log, preds



def predicted_frequency(h_bits, wg_next, k, t):
    """Sec. 4.4.1 Eq. 6 + Eq. 7: the next layer's router on the current hidden
    states; c[e] = number of tokens whose predicted top-k holds expert e; the
    t experts of highest c (ties: lower index; experts nobody asks for are left out).
    Returns (c [E] int32, list of predicted experts, the predicted logits [T,E])."""
    pidx, _, _, plogits = route_topk(h_bits, wg_next, None, k)
    E = wg_next.shape[0]
    c = np.bincount(pidx.ravel(), minlength=E).astype(np.int32)
    order = sorted(range(E), key=lambda e: (-int(c[e]), e))
    return c, [e for e in order[:t] if c[e] > 0], plogits


def prefill_stack(h0_bits, routers, expert_matrices, k, k_hh, tier_count, tier_bits, floor_bits, alpha,
                  predict_t=0, run_bits=None, token_score=None):
    """A stack of expert layers on a batch of T tokens (composition of the
    functions above): per layer gating, heavy-hitter importance (Eq. 2) with
    one score per token for the whole stack (given, or the row norms of the
    stack's input), assignment, quantisation of the loaded experts to their
    assigned width, FFN, residual + normalisation; with predict_t, the experts
    Eq. 7 would fetch ahead for the next layer.
    tier_count: one tuple, or one per layer.  run_bits as in decode_stack.
    Returns (final h bits, per-layer (idx, bits [E], logits, importance, load), per-layer predictions)."""
    h = _c(h0_bits, np.uint16)
    score = token_score_norm(h) if token_score is None else np.asarray(token_score, np.float64)
    per_layer = isinstance(tier_count[0], (tuple, list))
    log, preds = [], []
    for l, wg in enumerate(routers):
        E = wg.shape[0]
        idx, w, probs, logits = route_topk(h, wg, None, k)
        if predict_t and l + 1 < len(routers):
            preds.append(predicted_frequency(h, routers[l + 1], k, predict_t))
        imp, load, _ = expert_importance_prefill(idx, score, E, k_hh)
        bits, _ = assign_precision(imp, load, tier_count[l] if per_layer else tier_count, tier_bits,
                                   floor_bits[l] if floor_bits else 0)
        experts = []
        use_bits = np.zeros(E, np.uint8)
        for e in range(E):
            b = int(bits[e])
            if load[e] == 0 or b == 0:
                experts.append({})
                continue
            if run_bits is not None:
                b = int(run_bits[l].get(e, b))
            use_bits[e] = b
            mats = expert_matrices(l, e)
            experts.append({"w": mats} if b == 16 else {"q": [quantize_pack(m, b) for m in mats]})
        y = moe_ffn_mixed(h, idx, w, use_bits, experts) if use_bits.any() else np.zeros(h.shape, np.float64)
        log.append((idx.copy(), bits.copy(), logits.copy(), imp.copy(), load.copy()))
        h = residual_rmsnorm(h, y, alpha)
    return h, log, preds


def _widen_bf16(bits):
    """bf16 bit patterns -> the float32 values they denote (exact)."""
    return (np.ascontiguousarray(bits, np.uint16).astype(np.uint32) << 16).view(np.float32)


def token_score_attention(q_bits, k_bits, n_heads, n_kv_heads, causal=True, scale=None):
    """Sec. 4.2.1, first equation: s_i = (1/Hh) sum_h a_i^(h), read as the attention
    token i RECEIVES in head h averaged over the T queries: a_i^(h) = (1/T) sum_q P^(h)[q, i],
    P^(h) = softmax over keys of q_q . k_i * scale (causal: keys after the query masked out).
    q [T, n_heads, d], k [T, n_kv_heads, d] as bf16 bits; query head h reads key head
    h // (n_heads / n_kv_heads).  fp64 throughout; returns s [T] (sums to 1)."""
    q = _widen_bf16(q_bits).astype(np.float64)
    k = _widen_bf16(k_bits).astype(np.float64)
    T, Hh, d = q.shape
    assert Hh == n_heads and k.shape == (T, n_kv_heads, d) and n_heads % n_kv_heads == 0
    group = n_heads // n_kv_heads
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    s = np.zeros(T, np.float64)
    visible = np.tril(np.ones((T, T), bool)) if causal else np.ones((T, T), bool)
    for h in range(n_heads):
        logits = (q[:, h, :] @ k[:, h // group, :].T) * scale          # [query, key]
        logits = np.where(visible, logits, -np.inf)
        p = np.exp(logits - logits.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        s += p.sum(axis=0)
    return s / (n_heads * T)


# ---------------------------------------------------------------------------
# Error-compensated quantizer (paper Sec. 5: GPTQ is the base quantizer of the
# paper's implementation).  Hessian and its factor in fp64 with numpy's linear
# algebra as library steps; the column sweep is the C function (binary32, the
# sequence the GPU must reproduce), with an fp64 twin and the textbook
# one-column-at-a-time form beside it for the pins.

_lib.oracle_gptq_quantize_pack.restype = C.c_int
_lib.oracle_gptq_quantize_pack.argtypes = [_u16p, C.c_long, C.c_long, C.c_int, C.c_int, _f32p, _u8p, _u16p, _u16p]


def gptq_hessian(x_bits):
    """H = X^T X over the calibration rows x [n, K] (bf16 bit patterns), fp64."""
    x = _widen_bf16(x_bits).astype(np.float64)
    return x.T @ x


def gptq_damped(hess, damp=0.01):
    """H + damp * mean(diag H) * I; a column that never saw an input (H[c,c] = 0) gets H[c,c] = 1 first."""
    h = np.array(hess, dtype=np.float64, copy=True)
    d = np.diagonal(h).copy()
    d[d == 0.0] = 1.0
    np.fill_diagonal(h, d)
    h[np.diag_indices_from(h)] += damp * d.mean()
    return h


def gptq_factor(hess, damp=0.01):
    """Upper triangular U with (damped H)^-1 = U^T U, positive diagonal."""
    return np.linalg.cholesky(np.linalg.inv(gptq_damped(hess, damp))).T.copy()


def gptq_quantize_pack(w_bits, u, bits, group=64):
    """The binary32 sweep.  u [K,K] (rounded to fp32 here if it is not).  Returns codes, scale, zero."""
    w = _c(w_bits, np.uint16)
    N, K = w.shape
    uf = _c(u, np.float32)
    assert uf.shape == (K, K)
    codes = np.zeros((N, K * bits // 8), np.uint8)
    scale = np.zeros((N, K // group), np.uint16)
    zero = np.zeros((N, K // group), np.uint16)
    rc = _lib.oracle_gptq_quantize_pack(_ptr(w, _u16p), N, K, bits, group, _ptr(uf, _f32p), _ptr(codes, _u8p),
                                        _ptr(scale, _u16p), _ptr(zero, _u16p))
    if rc != 0:
        raise ValueError("oracle_gptq_quantize_pack rc=%d" % rc)
    return codes, scale, zero


def _grid_f64(lo, hi, qmax):
    """Scale and zero of a group as the quantizer stores them (fp16), as fp64 numbers."""
    m = np.array([f16_to_f32(f32_to_f16(float(np.float32(v)))) for v in lo])
    step = (np.float32(hi) - np.float32(lo)) / np.float32(qmax)
    s = np.array([f16_to_f32(f32_to_f16(float(v))) for v in step])
    return s, m


def gptq_sweep_f64(w, u, bits, group=64):
    """The same sweep in fp64 (group grids rounded to fp16 as stored).  Returns integer codes [N,K] and
    the dequantised matrix."""
    v = np.array(w, dtype=np.float64, copy=True)
    N, K = v.shape
    qmax = (1 << bits) - 1
    q = np.zeros((N, K), np.int64)
    deq = np.zeros((N, K))
    for c in range(K):
        if c % group == 0:
            blk = v[:, c:c + group]
            s, m = _grid_f64(blk.min(axis=1), blk.max(axis=1), qmax)
            inv = np.where(s > 0, 1.0 / np.where(s > 0, s, 1.0), 0.0)
        q[:, c] = np.clip(np.rint((v[:, c] - m) * inv), 0, qmax)
        deq[:, c] = q[:, c] * s + m
        e = (v[:, c] - deq[:, c]) / u[c, c]
        v[:, c + 1:] -= np.outer(e, u[c, c + 1:])
    return q, deq


def gptq_sweep_textbook(w, hess_damped, bits, group=64):
    """One column at a time, from the definition: quantise column c, move every remaining weight by
    -(w_c - dq_c) / [H^-1]_cc * H^-1[c, :] (the minimiser of the output error with w_c pinned), then drop
    column c from the problem (H^-1 of the remaining columns by eliminating row and column c)."""
    v = np.array(w, dtype=np.float64, copy=True)
    N, K = v.shape
    qmax = (1 << bits) - 1
    hinv = np.linalg.inv(hess_damped)
    q = np.zeros((N, K), np.int64)
    deq = np.zeros((N, K))
    for c in range(K):
        if c % group == 0:
            blk = v[:, c:c + group]
            s, m = _grid_f64(blk.min(axis=1), blk.max(axis=1), qmax)
            inv = np.where(s > 0, 1.0 / np.where(s > 0, s, 1.0), 0.0)
        q[:, c] = np.clip(np.rint((v[:, c] - m) * inv), 0, qmax)
        deq[:, c] = q[:, c] * s + m
        err = (v[:, c] - deq[:, c]) / hinv[c, c]
        v[:, c + 1:] -= np.outer(err, hinv[c, c + 1:])
        hinv = hinv - np.outer(hinv[:, c], hinv[c, :]) / hinv[c, c]
        hinv[c, :] = 0.0
        hinv[:, c] = 0.0
        hinv[c, c] = 1.0                         # keeps the slot harmless; column c is never read again
    return q, deq


def output_error(w, deq, hess):
    """sum over rows of (w - deq) H (w - deq)^T = || (W - What) X^T ||_F^2 on the calibration inputs."""
    d = np.asarray(w, np.float64) - deq
    return float(np.einsum("nk,kj,nj->", d, hess, d))
