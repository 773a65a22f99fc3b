"""Thin ctypes binding of libdymoe.so (see include/dymoe.h for the contract).

Argument marshalling only: every step of the MoE layer runs in the HIP
library.  Device buffers are torch tensors (torch is used for device memory
and streams only); each function takes tensors, checks dtype / contiguity and
passes raw device pointers and sizes through the C ABI.  There is no fallback:
if the shared library is missing, importing this module raises.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdymoe.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "libdymoe.so is not built: run `python -m paper_2603_19172_amd.build` "
        "(there is no CPU or PyTorch fallback for the DyMoE kernels)")

lib = C.CDLL(LIB_PATH)

OK, EINVAL, ENOSPC, EHIP, ENOTSUP, ENOCTX = 0, -1, -2, -3, -4, -5
PHASE_PREFILL, PHASE_DECODE = 0, 1
FRONT_MAX_TOKENS = 16
FLAG_FORMAT_MISSING = 1
OUT_BF16, OUT_F32 = 0, 1
PATH_AUTO, PATH_GEMV, PATH_GEMM = 0, 1, 2
LAYOUT_ROWMAJOR, LAYOUT_TILE = 0, 1

# every symbol include/dymoe.h declares
EXPORTS = [
    "dymoe_create", "dymoe_destroy", "dymoe_strerror", "dymoe_workspace_bytes", "dymoe_ffn_plan_offset",
    "dymoe_route_topk", "dymoe_token_score_norm", "dymoe_attention_workspace_bytes",
    "dymoe_token_score_attention", "dymoe_expert_importance",
    "dymoe_depth_schedule", "dymoe_assign_precision", "dymoe_quantize_pack",
    "dymoe_gptq_workspace_bytes", "dymoe_gptq_quantize_pack", "dymoe_gptq_hessian",
    "dymoe_gptq_factor_workspace_bytes", "dymoe_gptq_factor",
    "dymoe_quantize_experts", "dymoe_pack_tiles", "dymoe_pack_code_tiles", "dymoe_moe_ffn_mixed", "dymoe_moe_ffn_mixed_noalloc",
    "dymoe_stream_copy", "dymoe_mfma_peak", "dymoe_device_flags", "dymoe_format_present",
    "dymoe_decode_front", "dymoe_decode_step", "dymoe_prefetch_submit", "dymoe_prefetch_wait", "dymoe_prefetch_done",
    "dymoe_prefetch_release", "dymoe_residual_rmsnorm",
    "dymoe_cache_create", "dymoe_cache_create_pools", "dymoe_cache_destroy", "dymoe_cache_request", "dymoe_cache_request_at",
    "dymoe_cache_set_cyclic", "dymoe_cache_lookup",
    "dymoe_cache_block_bytes", "dymoe_cache_bytes_resident",
    "dymoe_timing_enable", "dymoe_timing_read", "dymoe_kernel_name",
]

KERNELS = ["route", "token_norm", "importance", "assign", "quantize", "gemv_phase1",
           "gemv_phase2", "gemv_combine", "plan", "gemm1", "gemm2", "gemm_combine", "stream_copy", "decode_front",
           "attn_stats", "attn_colsum", "gptq_group", "gptq_trail", "gptq_hessian", "gptq_factor", "mfma_peak", "route_select"]


class ExpertFmt(C.Structure):
    """Mirror of dymoe_expert_fmt."""
    _fields_ = [("w", C.c_void_p * 3), ("wt", C.c_void_p * 3), ("q4", C.c_void_p * 3), ("s4", C.c_void_p * 3),
                ("z4", C.c_void_p * 3), ("q2", C.c_void_p * 3), ("s2", C.c_void_p * 3),
                ("z2", C.c_void_p * 3), ("q8", C.c_void_p * 3), ("s8", C.c_void_p * 3),
                ("z8", C.c_void_p * 3)]


CACHE_MAX_FORMATS, CACHE_MAX_EVICT = 4, 16
CACHE_HIT, CACHE_MISS, CACHE_PROMOTE = 0, 1, 2


class CacheAction(C.Structure):
    """Mirror of dymoe_cache_action."""
    _fields_ = [("kind", C.c_int32), ("use_bits", C.c_int32), ("load_bits", C.c_int32), ("n_evicted", C.c_int32),
                ("offset", C.c_int64), ("dropped_offset", C.c_int64), ("evicted", C.c_int64 * CACHE_MAX_EVICT)]


_vp, _i, _l, _sz, _d = C.c_void_p, C.c_int, C.c_long, C.c_size_t, C.c_double
lib.dymoe_cache_create.restype = _i
lib.dymoe_cache_create.argtypes = [C.POINTER(_vp), _sz, _i, _vp, _vp]
lib.dymoe_cache_set_cyclic.restype = _i
lib.dymoe_cache_set_cyclic.argtypes = [_vp, _i]
lib.dymoe_cache_request_at.restype = _i
lib.dymoe_cache_request_at.argtypes = [_vp, C.c_int64, _i, _vp, _i, _i, C.POINTER(CacheAction)]
lib.dymoe_cache_create_pools.restype = _i
lib.dymoe_cache_create_pools.argtypes = [C.POINTER(_vp), _i, _vp, _vp, _vp]
lib.dymoe_cache_destroy.restype = None
lib.dymoe_cache_destroy.argtypes = [_vp]
lib.dymoe_cache_request.restype = _i
lib.dymoe_cache_request.argtypes = [_vp, C.c_int64, _i, _vp, _i, C.POINTER(CacheAction)]
lib.dymoe_cache_lookup.restype = _i
lib.dymoe_cache_lookup.argtypes = [_vp, C.c_int64, C.POINTER(C.c_int32), C.POINTER(C.c_int64)]
lib.dymoe_cache_block_bytes.restype = _sz
lib.dymoe_cache_block_bytes.argtypes = [_vp]
lib.dymoe_cache_bytes_resident.restype = _sz
lib.dymoe_cache_bytes_resident.argtypes = [_vp]
lib.dymoe_create.restype = _i
lib.dymoe_create.argtypes = [C.POINTER(_vp), _i]
lib.dymoe_destroy.restype = None
lib.dymoe_destroy.argtypes = [_vp]
lib.dymoe_strerror.restype = C.c_char_p
lib.dymoe_strerror.argtypes = [_i]
lib.dymoe_workspace_bytes.restype = _sz
lib.dymoe_workspace_bytes.argtypes = [_i] * 5
lib.dymoe_ffn_plan_offset.restype = _sz
lib.dymoe_ffn_plan_offset.argtypes = [_i] * 5
lib.dymoe_decode_front.restype = _i
lib.dymoe_decode_front.argtypes = [_vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _vp, _vp, _i,
                                   _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
lib.dymoe_decode_step.restype = _i
lib.dymoe_decode_step.argtypes = [_vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _i, _vp, _vp, _i, _vp, _i, _i,
                                  _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
lib.dymoe_prefetch_submit.restype = _i
lib.dymoe_prefetch_submit.argtypes = [_vp, _vp, _vp, _sz, _vp, C.POINTER(_vp)]
lib.dymoe_prefetch_wait.restype = _i
lib.dymoe_prefetch_wait.argtypes = [_vp, _vp, _vp]
lib.dymoe_prefetch_done.restype = _i
lib.dymoe_prefetch_done.argtypes = [_vp, _vp]
lib.dymoe_prefetch_release.restype = _i
lib.dymoe_prefetch_release.argtypes = [_vp, _vp]
lib.dymoe_residual_rmsnorm.restype = _i
lib.dymoe_residual_rmsnorm.argtypes = [_vp, _vp, _vp, _i, C.c_float, _i, _i, _vp, _vp]
lib.dymoe_attention_workspace_bytes.restype = _sz
lib.dymoe_attention_workspace_bytes.argtypes = [_i, _i]
lib.dymoe_token_score_attention.restype = _i
lib.dymoe_token_score_attention.argtypes = [_vp, _vp, _vp, _i, _i, _i, _i, C.c_float, _i, _vp, _vp, _sz, _vp]
lib.dymoe_device_flags.restype = _i
lib.dymoe_device_flags.argtypes = [_vp, C.POINTER(C.c_uint), _vp]
lib.dymoe_format_present.restype = _i
lib.dymoe_format_present.argtypes = [_vp, _i]
lib.dymoe_mfma_peak.restype = _i
lib.dymoe_mfma_peak.argtypes = [_vp, _i, _i, _vp, _sz, C.POINTER(_d), _vp]
lib.dymoe_stream_copy.restype = _i
lib.dymoe_stream_copy.argtypes = [_vp, _vp, _vp, _sz, _vp]
lib.dymoe_route_topk.restype = _i
lib.dymoe_route_topk.argtypes = [_vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp]
lib.dymoe_token_score_norm.restype = _i
lib.dymoe_token_score_norm.argtypes = [_vp, _vp, _i, _i, _vp, _vp]
lib.dymoe_expert_importance.restype = _i
lib.dymoe_expert_importance.argtypes = [_vp, _i, _vp, _vp, _vp, _i, _i, _i, _i, _vp, _vp, _vp]
lib.dymoe_depth_schedule.restype = _i
lib.dymoe_depth_schedule.argtypes = [_i, _i, _d, _i]
lib.dymoe_assign_precision.restype = _i
lib.dymoe_assign_precision.argtypes = [_vp, _i, _vp, _vp, _i, _i, _vp, _vp, _i, _vp, _vp, _vp]
lib.dymoe_quantize_pack.restype = _i
lib.dymoe_quantize_pack.argtypes = [_vp, _vp, _l, _l, _i, _i, _vp, _vp, _vp, _vp]
lib.dymoe_gptq_workspace_bytes.restype = _sz
lib.dymoe_gptq_workspace_bytes.argtypes = [_l, _l]
lib.dymoe_gptq_hessian.restype = _i
lib.dymoe_gptq_hessian.argtypes = [_vp, _vp, _l, _l, _i, _vp, _vp]
lib.dymoe_gptq_factor_workspace_bytes.restype = _sz
lib.dymoe_gptq_factor_workspace_bytes.argtypes = [_l]
lib.dymoe_gptq_factor.restype = _i
lib.dymoe_gptq_factor.argtypes = [_vp, _vp, _l, C.c_float, _vp, _vp, _sz, _vp]
lib.dymoe_gptq_quantize_pack.restype = _i
lib.dymoe_gptq_quantize_pack.argtypes = [_vp, _vp, _vp, _l, _l, _i, _i, _vp, _vp, _vp, _vp, _sz, _vp]
lib.dymoe_quantize_experts.restype = _i
lib.dymoe_quantize_experts.argtypes = [_vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _vp]
lib.dymoe_pack_code_tiles.restype = _i
lib.dymoe_pack_code_tiles.argtypes = [_vp, _vp, _vp, _vp, _l, _l, _i, _vp, _vp, _vp, _vp]
lib.dymoe_pack_tiles.restype = _i
lib.dymoe_pack_tiles.argtypes = [_vp, _vp, _l, _l, _vp, _vp]
lib.dymoe_moe_ffn_mixed.restype = _i
lib.dymoe_moe_ffn_mixed.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _i, _i,
                                    _vp, _vp, _sz, _vp]
STATIC_SCRATCH_BYTES = 8 << 20
lib.dymoe_moe_ffn_mixed_noalloc.restype = _i
lib.dymoe_moe_ffn_mixed_noalloc.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _i, _i, _vp, _vp]


lib.dymoe_timing_enable.restype = _i
lib.dymoe_timing_enable.argtypes = [_vp, C.c_uint]
lib.dymoe_timing_read.restype = _i
lib.dymoe_timing_read.argtypes = [_vp, _i, C.POINTER(_d), C.POINTER(_i)]
lib.dymoe_kernel_name.restype = C.c_char_p
lib.dymoe_kernel_name.argtypes = [_i]


class DymoeError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__("%s failed: %s (%d)" % (where, strerror(code), code))


def strerror(code: int) -> str:
    return lib.dymoe_strerror(int(code)).decode()


def _check(rc, where):
    if rc != 0:
        raise DymoeError(rc, where)


def _ptr(t, dtype=None):
    """Device pointer of a tensor (None -> NULL); ints pass through."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if dtype is not None and t.dtype != dtype:
        raise TypeError("expected %s, got %s" % (dtype, t.dtype))
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def workspace_bytes(T, H, F, E, k) -> int:
    return int(lib.dymoe_workspace_bytes(T, H, F, E, k))


def format_present(entry, bits) -> bool:
    """Whether a host ExpertFmt holds every pointer that running its expert at `bits` reads (the kernels' own test)."""
    return bool(lib.dymoe_format_present(C.byref(entry), int(bits)))


def read_ffn_plan(ws, T, H, F, E, k):
    """The token grouping a GEMM-path call left in workspace `ws` (uint8 tensor): (counts [E], offsets [E+1],
    perm [T*k]) as host int32 arrays; perm[offsets[e] + i] is the i-th (token * k + slot) pair of expert e."""
    off = int(lib.dymoe_ffn_plan_offset(T, H, F, E, k))
    n = 3 * E + 1 + 8 + T * k
    ints = ws[off:off + 4 * n].view(torch.int32).cpu().numpy()
    return ints[:E].copy(), ints[E:2 * E + 1].copy(), ints[3 * E + 9:3 * E + 9 + T * k].copy()


def depth_schedule(layer, n_layers, lam, M) -> int:
    return int(lib.dymoe_depth_schedule(layer, n_layers, float(lam), M))


class Context:
    """Owns a dymoe_ctx.  All methods enqueue on `stream` (default: torch's current)."""

    def __init__(self, device: int = 0):
        h = _vp()
        _check(lib.dymoe_create(C.byref(h), device), "dymoe_create")
        self._h = h
        self.device = device

    def close(self):
        # at interpreter shutdown the module globals may already be gone
        if getattr(self, "_h", None) and lib is not None:
            lib.dymoe_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()

    def timing_enable(self, kernels=()):
        mask = 0
        for name in kernels:
            mask |= 1 << KERNELS.index(name)
        _check(lib.dymoe_timing_enable(self._h, mask), "dymoe_timing_enable")

    def timing_read(self, kernel):
        ms, n = _d(0.0), _i(0)
        _check(lib.dymoe_timing_read(self._h, KERNELS.index(kernel), C.byref(ms), C.byref(n)),
               "dymoe_timing_read")
        return ms.value, n.value

    # -- S1
    def route_topk(self, x, wg, bias, k, renorm=True, probs=True, stream=None):
        T, H = x.shape
        E = wg.shape[0]
        dev = x.device
        idx = torch.empty((T, k), dtype=torch.int32, device=dev)
        w = torch.empty((T, k), dtype=torch.float32, device=dev)
        p = torch.empty((T, E), dtype=torch.float32, device=dev) if probs else None
        _check(lib.dymoe_route_topk(self._h, _ptr(x, torch.bfloat16), _ptr(wg, torch.bfloat16),
                                    _ptr(bias, torch.float32), T, H, E, k, 1 if renorm else 0,
                                    _ptr(idx), _ptr(w), _ptr(p), _stream(stream)),
               "dymoe_route_topk")
        return idx, w, p

    def token_score_norm(self, x, stream=None):
        T, H = x.shape
        s = torch.empty((T,), dtype=torch.float32, device=x.device)
        _check(lib.dymoe_token_score_norm(self._h, _ptr(x, torch.bfloat16), T, H, _ptr(s),
                                          _stream(stream)), "dymoe_token_score_norm")
        return s

    # -- S2
    def expert_importance(self, phase, idx, E, probs=None, token_score=None, k_hh=0, stream=None):
        T, k = idx.shape
        dev = idx.device
        imp = torch.empty((E,), dtype=torch.int32 if phase == PHASE_PREFILL else torch.float32,
                          device=dev)
        load = torch.empty((E,), dtype=torch.int32, device=dev)
        _check(lib.dymoe_expert_importance(self._h, phase, _ptr(idx, torch.int32),
                                           _ptr(probs, torch.float32),
                                           _ptr(token_score, torch.float32), T, E, k, k_hh,
                                           _ptr(imp), _ptr(load), _stream(stream)),
               "dymoe_expert_importance")
        return imp, load

    # -- S3
    def assign_precision(self, phase, importance, load, tier_count, tier_bits, floor_bits=0,
                         stream=None):
        E = importance.shape[0]
        dev = importance.device
        n = len(tier_count)
        tc = (C.c_int32 * n)(*[int(v) for v in tier_count])
        tb = (C.c_uint8 * n)(*[int(v) for v in tier_bits])
        bits = torch.empty((E,), dtype=torch.uint8, device=dev)
        rank = torch.empty((E,), dtype=torch.int32, device=dev)
        want = torch.int32 if phase == PHASE_PREFILL else torch.float32
        _check(lib.dymoe_assign_precision(self._h, phase, _ptr(importance, want),
                                          _ptr(load, torch.int32), E, n,
                                          C.cast(tc, _vp), C.cast(tb, _vp), floor_bits,
                                          _ptr(bits), _ptr(rank), _stream(stream)),
               "dymoe_assign_precision")
        return bits, rank

    # -- S1 + S2 + S3 of a decode step in one launch
    def decode_front(self, x, wg, bias, k, tier_count, tier_bits, floor_bits=0, renorm=True,
                     stream=None):
        T, H = x.shape
        E = wg.shape[0]
        dev = x.device
        n = len(tier_count)
        tc = (C.c_int32 * n)(*[int(v) for v in tier_count])
        tb = (C.c_uint8 * n)(*[int(v) for v in tier_bits])
        idx = torch.empty((T, k), dtype=torch.int32, device=dev)
        w = torch.empty((T, k), dtype=torch.float32, device=dev)
        probs = torch.empty((T, E), dtype=torch.float32, device=dev)
        imp = torch.empty((E,), dtype=torch.float32, device=dev)
        load = torch.empty((E,), dtype=torch.int32, device=dev)
        bits = torch.empty((E,), dtype=torch.uint8, device=dev)
        rank = torch.empty((E,), dtype=torch.int32, device=dev)
        _check(lib.dymoe_decode_front(self._h, _ptr(x, torch.bfloat16), _ptr(wg, torch.bfloat16),
                                      _ptr(bias, torch.float32), T, H, E, k, 1 if renorm else 0, n,
                                      C.cast(tc, _vp), C.cast(tb, _vp), floor_bits, _ptr(idx), _ptr(w),
                                      _ptr(probs), _ptr(imp), _ptr(load), _ptr(bits), _ptr(rank),
                                      _stream(stream)), "dymoe_decode_front")
        return idx, w, probs, imp, load, bits, rank

    # -- S4
    def quantize_pack(self, w, bits, group=64, out=None, stream=None):
        N, K = w.shape
        dev = w.device
        if out is None:
            codes = torch.empty((N, K * bits // 8), dtype=torch.uint8, device=dev)
            scale = torch.empty((N, K // group), dtype=torch.float16, device=dev)
            zero = torch.empty((N, K // group), dtype=torch.float16, device=dev)
        else:
            codes, scale, zero = out
        _check(lib.dymoe_quantize_pack(self._h, _ptr(w, torch.bfloat16), N, K, bits, group,
                                       _ptr(codes, torch.uint8), _ptr(scale, torch.float16),
                                       _ptr(zero, torch.float16), _stream(stream)),
               "dymoe_quantize_pack")
        return codes, scale, zero

    def gptq_hessian(self, x, out=None, accumulate=False, stream=None):
        """hess (+)= X^T X for calibration inputs x [n, K] bf16; returns hess [K, K] fp32."""
        n, K = x.shape
        if out is None:
            out = torch.empty((K, K), dtype=torch.float32, device=x.device)
        _check(lib.dymoe_gptq_hessian(self._h, _ptr(x, torch.bfloat16), n, K, int(bool(accumulate)),
                                      _ptr(out, torch.float32), _stream(stream)), "dymoe_gptq_hessian")
        return out

    def gptq_factor(self, hess, damp=0.01, out=None, workspace=None, stream=None):
        """The upper triangular U with (H + damp mean(diag H) I)^-1 = U^T U."""
        K = hess.shape[0]
        if out is None:
            out = torch.empty((K, K), dtype=torch.float32, device=hess.device)
        if workspace is None:
            workspace = torch.empty((int(lib.dymoe_gptq_factor_workspace_bytes(K)),), dtype=torch.uint8,
                                    device=hess.device)
        _check(lib.dymoe_gptq_factor(self._h, _ptr(hess, torch.float32), K, float(damp), _ptr(out, torch.float32),
                                     _ptr(workspace, torch.uint8), workspace.numel(), _stream(stream)),
               "dymoe_gptq_factor")
        return out

    def gptq_quantize_pack(self, w, u, bits, group=64, out=None, workspace=None, stream=None):
        """Error-compensated quantize-and-pack of w [N,K] bf16 with the factor u [K,K] fp32."""
        N, K = w.shape
        dev = w.device
        if out is None:
            codes = torch.empty((N, K * bits // 8), dtype=torch.uint8, device=dev)
            scale = torch.empty((N, K // group), dtype=torch.float16, device=dev)
            zero = torch.empty((N, K // group), dtype=torch.float16, device=dev)
        else:
            codes, scale, zero = out
        need = int(lib.dymoe_gptq_workspace_bytes(N, K))
        if workspace is None:
            workspace = torch.empty((need,), dtype=torch.uint8, device=dev)
        _check(lib.dymoe_gptq_quantize_pack(self._h, _ptr(w, torch.bfloat16), _ptr(u, torch.float32), N, K, bits,
                                            group, _ptr(codes, torch.uint8), _ptr(scale, torch.float16),
                                            _ptr(zero, torch.float16), _ptr(workspace, torch.uint8),
                                            workspace.numel(), _stream(stream)), "dymoe_gptq_quantize_pack")
        return codes, scale, zero

    def quantize_experts(self, table, bits, load, E, H, F, group=64, layout=LAYOUT_ROWMAJOR,
                         stream=None):
        _check(lib.dymoe_quantize_experts(self._h, _ptr(table), _ptr(bits, torch.uint8),
                                          _ptr(load, torch.int32), E, H, F, group, layout,
                                          _stream(stream)), "dymoe_quantize_experts")

    def pack_code_tiles(self, trip, bits, stream=None):
        """(codes, scale, zero) row-major -> the same in the tile layout (new tensors)."""
        codes, scale, zero = trip
        N = codes.shape[0]
        K = codes.shape[1] * 8 // bits
        out = (torch.empty_like(codes), torch.empty_like(scale), torch.empty_like(zero))
        _check(lib.dymoe_pack_code_tiles(self._h, _ptr(codes, torch.uint8), _ptr(scale, torch.float16),
                                         _ptr(zero, torch.float16), N, K, bits, _ptr(out[0], torch.uint8),
                                         _ptr(out[1], torch.float16), _ptr(out[2], torch.float16), _stream(stream)),
               "dymoe_pack_code_tiles")
        return out

    def pack_tiles(self, w, stream=None):
        N, K = w.shape
        out = torch.empty_like(w)
        _check(lib.dymoe_pack_tiles(self._h, _ptr(w, torch.bfloat16), N, K, _ptr(out),
                                    _stream(stream)), "dymoe_pack_tiles")
        return out

    # -- host-resident experts
    def prefetch_submit(self, host_ptr, dev_ptr, nbytes, side_stream):
        ev = _vp()
        _check(lib.dymoe_prefetch_submit(self._h, host_ptr, dev_ptr, nbytes, side_stream, C.byref(ev)),
               "dymoe_prefetch_submit")
        return ev

    def prefetch_wait(self, ev, compute_stream):
        _check(lib.dymoe_prefetch_wait(self._h, ev, compute_stream), "dymoe_prefetch_wait")

    def prefetch_done(self, ev):
        r = lib.dymoe_prefetch_done(self._h, ev)
        if r < 0:
            _check(r, "dymoe_prefetch_done")
        return bool(r)

    def prefetch_release(self, ev):
        _check(lib.dymoe_prefetch_release(self._h, ev), "dymoe_prefetch_release")

    def residual_rmsnorm(self, h, y, alpha=1.0, out=None, stream=None):
        T, H = h.shape
        if out is None:
            out = torch.empty_like(h)
        yd = OUT_BF16 if y.dtype == torch.bfloat16 else OUT_F32
        _check(lib.dymoe_residual_rmsnorm(self._h, _ptr(h, torch.bfloat16), _ptr(y), yd, float(alpha), T, H,
                                          _ptr(out, torch.bfloat16), _stream(stream)), "dymoe_residual_rmsnorm")
        return out

    def token_score_attention(self, q, k, causal=True, scale=0.0, out=None, workspace=None, stream=None):
        """q [T, n_heads, d], k [T, n_kv_heads, d] bf16 -> score [T] fp32."""
        T, n_heads, d = q.shape
        n_kv = k.shape[1]
        if out is None:
            out = torch.empty((T,), dtype=torch.float32, device=q.device)
        nb = int(lib.dymoe_attention_workspace_bytes(T, n_heads))
        if workspace is None:
            workspace = torch.empty((max(nb, 256),), dtype=torch.uint8, device=q.device)
        _check(lib.dymoe_token_score_attention(self._h, _ptr(q, torch.bfloat16), _ptr(k, torch.bfloat16), T, n_heads,
                                               n_kv, d, float(scale), 1 if causal else 0, _ptr(out, torch.float32),
                                               _ptr(workspace, torch.uint8), workspace.numel(), _stream(stream)),
               "dymoe_token_score_attention")
        return out

    def stream_copy(self, src, dst, stream=None):
        """Plain copy of src's bytes into dst (same byte count): a measurement aid."""
        n = src.numel() * src.element_size()
        if n != dst.numel() * dst.element_size():
            raise ValueError("stream_copy: byte counts differ")
        _check(lib.dymoe_stream_copy(self._h, _ptr(src), _ptr(dst), n, _stream(stream)), "dymoe_stream_copy")
        return dst

    def device_flags(self, stream=None) -> int:
        """Conditions the kernels met and went on from since the last read (FLAG_*); waits for the stream, clears."""
        v = C.c_uint(0)
        _check(lib.dymoe_device_flags(self._h, C.byref(v), _stream(stream)), "dymoe_device_flags")
        return int(v.value)

    def mfma_peak(self, iters, waves_per_simd, sink, stream=None):
        """Register-only bf16 MFMA loop (measurement aid); returns the floating-point operations of the launch."""
        fl = _d(0.0)
        _check(lib.dymoe_mfma_peak(self._h, int(iters), int(waves_per_simd), _ptr(sink, torch.float32), sink.numel(),
                                   C.byref(fl), _stream(stream)), "dymoe_mfma_peak")
        return fl.value

    # -- S5
    def moe_ffn_mixed(self, x, idx, w, bits, table, F, out_dtype=OUT_BF16, path=PATH_AUTO,
                      group=64, y=None, workspace=None, stream=None):
        T, H = x.shape
        k = idx.shape[1]
        E = bits.shape[0]
        dev = x.device
        if y is None:
            y = torch.empty((T, H), dtype=torch.bfloat16 if out_dtype == OUT_BF16 else torch.float32,
                            device=dev)
        if workspace is None:
            workspace = torch.empty((workspace_bytes(T, H, F, E, k),), dtype=torch.uint8, device=dev)
        _check(lib.dymoe_moe_ffn_mixed(self._h, _ptr(x, torch.bfloat16), _ptr(idx, torch.int32),
                                       _ptr(w, torch.float32), _ptr(bits, torch.uint8), _ptr(table),
                                       T, H, F, E, k, group, out_dtype, path, _ptr(y),
                                       _ptr(workspace, torch.uint8), workspace.numel(),
                                       _stream(stream)), "dymoe_moe_ffn_mixed")
        return y


def make_expert_table(experts, device):
    """Build the device-resident dymoe_expert_fmt[E] from per-expert dicts of
    tensors: 'w' = [W1,W3,W2] bf16 and/or 'q8' / 'q4' / 'q2' = three (codes, scale,
    zero) triples.  Returns (table tensor, keepalive list); the caller keeps
    both alive while the table is in use."""
    E = len(experts)
    arr = (ExpertFmt * E)()
    keep = []
    for e, ex in enumerate(experts):
        if ex.get("w") is not None:
            for i in range(3):
                arr[e].w[i] = _ptr(ex["w"][i], torch.bfloat16)
            keep.append(ex["w"])
        if ex.get("wt") is not None:
            for i in range(3):
                arr[e].wt[i] = _ptr(ex["wt"][i], torch.bfloat16)
            keep.append(ex["wt"])
        for b in (8, 4, 2):
            trip = ex.get("q%d" % b)
            if trip is None:
                continue
            for i in range(3):
                cd, sc, zr = trip[i]
                getattr(arr[e], "q%d" % b)[i] = _ptr(cd, torch.uint8)
                getattr(arr[e], "s%d" % b)[i] = _ptr(sc, torch.float16)
                getattr(arr[e], "z%d" % b)[i] = _ptr(zr, torch.float16)
            keep.append(trip)
    raw = bytes(arr)
    host = torch.frombuffer(bytearray(raw), dtype=torch.uint8)
    table = host.to(device)
    return table, keep
