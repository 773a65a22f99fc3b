"""One MoE layer with every buffer pre-allocated, so that a step is nothing but
the five libdymoe calls enqueued back to back on one stream (no allocation, no
host read-back): route -> importance -> precision -> quantize -> FFN.

Argument marshalling only; all arithmetic is in libdymoe.so.
"""
import ctypes as C

import torch

from . import binding as B


class ExpertStore:
    """Device-resident weights of a layer's experts: the bf16 originals plus
    output buffers for the quantised formats (int4 and int2; int8 when asked
    for), and the dymoe_expert_fmt table that points at them."""

    def __init__(self, w_bf16, H, F, device, group=64, ctx=None, w_tiles=None, formats=(4, 2)):
        # w_bf16: list over experts of [W1 [F,H], W3 [F,H], W2 [H,F]] bf16 tensors on `device`.
        # With a context, a tile-layout copy of the bf16 weights is made for the GEMM path.
        self.E = len(w_bf16)
        self.H, self.F = H, F
        self.w = w_bf16
        self.wt = w_tiles
        if self.wt is None and ctx is not None and H % 128 == 0 and F % 128 == 0:
            self.wt = [[ctx.pack_tiles(m) for m in ex] for ex in w_bf16]
        self.formats = tuple(formats)
        self.q = {}
        for b in self.formats:
            self.q[b] = [[(torch.empty((n, k * b // 8), dtype=torch.uint8, device=device),
                           torch.empty((n, k // group), dtype=torch.float16, device=device),
                           torch.empty((n, k // group), dtype=torch.float16, device=device))
                          for n, k in ((F, H), (F, H), (H, F))] for _ in range(self.E)]
        experts = [dict({"w": self.w[e], "wt": self.wt[e] if self.wt is not None else None},
                        **{"q%d" % b: self.q[b][e] for b in self.formats}) for e in range(self.E)]
        self.table, self._keep = B.make_expert_table(experts, device)

    def clone(self):
        wt = [[m.clone() for m in ex] for ex in self.wt] if self.wt is not None else None
        return ExpertStore([[m.clone() for m in ex] for ex in self.w], self.H, self.F,
                           self.table.device, w_tiles=wt, formats=self.formats)


class MoELayer:
    def __init__(self, ctx, T, H, F, E, k, phase, tier_count, tier_bits, k_hh=0, floor_bits=0,
                 out_dtype=B.OUT_BF16, path=B.PATH_AUTO, device="cuda:0", group=64):
        self.ctx, self.T, self.H, self.F, self.E, self.k = ctx, T, H, F, E, k
        self.phase = B.PHASE_PREFILL if phase == "prefill" else B.PHASE_DECODE
        self.k_hh, self.floor_bits, self.out_dtype, self.path, self.group = k_hh, floor_bits, out_dtype, path, group
        n = len(tier_count)
        self._tc = (C.c_int32 * n)(*[int(v) for v in tier_count])
        self._tb = (C.c_uint8 * n)(*[int(v) for v in tier_bits])
        self._nt = n
        dev = device
        self.idx = torch.empty((T, k), dtype=torch.int32, device=dev)
        self.gate = torch.empty((T, k), dtype=torch.float32, device=dev)
        self.probs = torch.empty((T, E), dtype=torch.float32, device=dev)
        self.score = torch.empty((T,), dtype=torch.float32, device=dev)
        self.imp = torch.empty((E,), dtype=torch.int32 if self.phase == B.PHASE_PREFILL else torch.float32, device=dev)
        self.load = torch.empty((E,), dtype=torch.int32, device=dev)
        self.bits = torch.empty((E,), dtype=torch.uint8, device=dev)
        self.rank = torch.empty((E,), dtype=torch.int32, device=dev)
        self.y = torch.empty((T, H), dtype=torch.bfloat16 if out_dtype == B.OUT_BF16 else torch.float32, device=dev)
        # the FFN path and the layout of the packed weights go together
        gemm = path == B.PATH_GEMM or (path == B.PATH_AUTO and T > 4 and H % 128 == 0 and F % 128 == 0)
        self.layout = B.LAYOUT_TILE if gemm else B.LAYOUT_ROWMAJOR
        self.ws_bytes = B.workspace_bytes(T, H, F, E, k)
        self.ws = torch.empty((self.ws_bytes,), dtype=torch.uint8, device=dev)
        # a decode step on resident formats: dymoe_decode_step (two launches) instead of front end + FFN (three)
        self.use_decode_step = True

    # the individual steps; each is one C call
    def route(self, x, wg, bias, st):
        B._check(B.lib.dymoe_route_topk(self.ctx._h, x.data_ptr(), wg.data_ptr(),
                                        bias.data_ptr() if bias is not None else None, self.T, self.H,
                                        self.E, self.k, 1, self.idx.data_ptr(), self.gate.data_ptr(),
                                        self.probs.data_ptr(), st), "dymoe_route_topk")

    def importance(self, x, st, score=None):
        """score: [T] fp32 token scores to rank the heavy hitters by (prefill); None: the row norms of x."""
        if self.phase == B.PHASE_PREFILL and score is None:
            B._check(B.lib.dymoe_token_score_norm(self.ctx._h, x.data_ptr(), self.T, self.H,
                                                  self.score.data_ptr(), st), "dymoe_token_score_norm")
        if score is None:
            score = self.score
        B._check(B.lib.dymoe_expert_importance(self.ctx._h, self.phase, self.idx.data_ptr(),
                                               self.probs.data_ptr(), score.data_ptr(), self.T,
                                               self.E, self.k, self.k_hh, self.imp.data_ptr(),
                                               self.load.data_ptr(), st), "dymoe_expert_importance")

    def assign(self, st):
        B._check(B.lib.dymoe_assign_precision(self.ctx._h, self.phase, self.imp.data_ptr(),
                                              self.load.data_ptr(), self.E, self._nt,
                                              C.cast(self._tc, C.c_void_p), C.cast(self._tb, C.c_void_p),
                                              self.floor_bits, self.bits.data_ptr(),
                                              self.rank.data_ptr(), st), "dymoe_assign_precision")

    def quantize(self, store, st):
        B._check(B.lib.dymoe_quantize_experts(self.ctx._h, store.table.data_ptr(), self.bits.data_ptr(),
                                              self.load.data_ptr(), self.E, self.H, self.F, self.group,
                                              self.layout, st), "dymoe_quantize_experts")

    def ffn(self, x, store, st):
        B._check(B.lib.dymoe_moe_ffn_mixed(self.ctx._h, x.data_ptr(), self.idx.data_ptr(),
                                           self.gate.data_ptr(), self.bits.data_ptr(),
                                           store.table.data_ptr(), self.T, self.H, self.F, self.E,
                                           self.k, self.group, self.out_dtype, self.path,
                                           self.y.data_ptr(), self.ws.data_ptr(), self.ws_bytes, st),
                 "dymoe_moe_ffn_mixed")

    def front(self, x, wg, bias, st):
        """S1 + S2 + S3 of a small decode step in one launch."""
        B._check(B.lib.dymoe_decode_front(self.ctx._h, x.data_ptr(), wg.data_ptr(),
                                          bias.data_ptr() if bias is not None else None, self.T, self.H,
                                          self.E, self.k, 1, self._nt, C.cast(self._tc, C.c_void_p),
                                          C.cast(self._tb, C.c_void_p), self.floor_bits,
                                          self.idx.data_ptr(), self.gate.data_ptr(), self.probs.data_ptr(),
                                          self.imp.data_ptr(), self.load.data_ptr(), self.bits.data_ptr(),
                                          self.rank.data_ptr(), st), "dymoe_decode_front")

    def decode_step(self, x, wg, bias, store, st):
        """S1 + S2 + S3 + S5 of a small decode step on resident formats in two launches; False when the sizes are
        outside what the fused step covers (the caller then makes the separate calls)."""
        rc = B.lib.dymoe_decode_step(self.ctx._h, x.data_ptr(), wg.data_ptr(), bias.data_ptr() if bias is not None else None,
                                     self.T, self.H, self.F, self.E, self.k, 1, self._nt, C.cast(self._tc, C.c_void_p),
                                     C.cast(self._tb, C.c_void_p), self.floor_bits, store.table.data_ptr(), self.group,
                                     self.out_dtype, self.idx.data_ptr(), self.gate.data_ptr(), self.probs.data_ptr(),
                                     self.imp.data_ptr(), self.load.data_ptr(), self.bits.data_ptr(),
                                     self.rank.data_ptr(), self.y.data_ptr(), self.ws.data_ptr(), self.ws_bytes, st)
        if rc == B.ENOTSUP:
            return False
        B._check(rc, "dymoe_decode_step")
        return True

    def step(self, x, wg, bias, store, quantize=True, stream=None, fused_front=True):
        """The whole hot path for one batch.  quantize=False assumes the formats
        the assignment selects are already materialised in `store`.  Small decode
        steps take the single-launch front end unless fused_front is False."""
        st = B._stream(stream)
        if (fused_front and self.use_decode_step and not quantize and self.phase == B.PHASE_DECODE
                and self.path != B.PATH_GEMM and self.layout == B.LAYOUT_ROWMAJOR
                and self.decode_step(x, wg, bias, store, st)):
            return self.y
        if fused_front and self.phase == B.PHASE_DECODE and self.T <= B.FRONT_MAX_TOKENS:
            self.front(x, wg, bias, st)
        else:
            self.route(x, wg, bias, st)
            self.importance(x, st)
            self.assign(st)
        if quantize:
            self.quantize(store, st)
        self.ffn(x, store, st)
        return self.y
