"""A stack of MoE expert layers with the experts resident in pinned HOST memory
(paper Sec. 4.4: dynamic expert orchestration), decoding one token at a time
or prefilling a batch of tokens.

Per layer the compute stream runs the hot path of `layer.py`; the experts it
needs are brought into device slots, on demand or ahead of time: the next
layer's router applied to the current hidden states (Sec. 4.4.1 Eq. 6) names the
experts to prefetch (decode: the token's own predicted experts, Eq. 8; prefill:
the experts most tokens are predicted to ask for, Eq. 7), which are copied on a
side stream (dymoe_prefetch_submit / dymoe_prefetch_wait) while the current
layer computes.  Copies a layer is waiting for and copies made on a prediction
travel on two different streams, so that a miss never queues behind speculation,
and a speculative copy is only issued when it is expected to pay: with p the
measured share of right predictions, a copy of c milliseconds hides at most the
layer's compute time t when it is right and occupies the link for c when it is
wrong, so it is issued when p * min(c, t) >= (1 - p) * c (`lookahead="expected"`;
"always" issues every predicted copy).

Two ways of moving an expert:
  transfer="bf16"      the bf16 weights travel and are quantised on the device
                       to the width the precision assignment asks for;
  transfer="assigned"  the host also holds the quantised formats (made once
                       by the device quantiser) and the format the assignment
                       asks for travels: fewer bytes on the host link, and the
                       mixed-precision cache of Sec. 4.4.2 decides what stays.

Host control flow and bookkeeping only; every arithmetic step runs in
libdymoe.so.
"""
import collections
import ctypes as C

import torch

from . import binding as B
from .cache import FORMATS, ByteBudgetCache, MixedPrecisionCache
from .layer import MoELayer

FMT_BYTES = C.sizeof(B.ExpertFmt)


def quant_layout(H, F, bits, group=64):
    """Byte offsets of a quantised expert stored as one block: for each matrix
    codes | scale | zero.  Returns ([(codes, scale, zero)] * 3, total bytes)."""
    offs, pos = [], 0
    for n, kk in ((F, H), (F, H), (H, F)):
        codes, sz = n * kk * bits // 8, n * (kk // group) * 2
        offs.append((pos, pos + codes, pos + codes + sz))
        pos += codes + 2 * sz
    return offs, pos


class HostExpertPool:
    """Expert weights in pinned host memory.  To bound memory and set-up time,
    `n_pool` distinct experts are drawn and (layer, expert) maps to entry
    (layer * E + expert) mod n_pool.  A bf16 entry is W1 [F,H] | W3 [F,H] |
    W2 [H,F] back to back, so an expert moves with a single copy."""

    def __init__(self, H, F, E, n_pool, matrices):
        # matrices(i) -> [W1, W3, W2] as uint16 numpy arrays (bf16 bits) of pool entry i
        self.H, self.F, self.E, self.n_pool = H, F, E, n_pool
        self.elems = 3 * H * F
        self.nbytes = {16: 2 * self.elems}
        self.layout = B.LAYOUT_ROWMAJOR     # of the quantised formats, once made
        self.buf = {16: torch.empty((n_pool, 2 * self.elems), dtype=torch.uint8, pin_memory=True)}
        view = self.buf[16].numpy().view("int16")
        for i in range(n_pool):
            w1, w3, w2 = matrices(i)
            view[i, :H * F] = w1.reshape(-1).view("int16")
            view[i, H * F:2 * H * F] = w3.reshape(-1).view("int16")
            view[i, 2 * H * F:] = w2.reshape(-1).view("int16")

    def add_quantised(self, ctx, device, formats=(4, 2), layout=B.LAYOUT_ROWMAJOR, factors=None):
        """Quantised copies (by default int4 and int2) of every entry, made by the device quantiser and
        kept in pinned host memory, in the layout the FFN path that will read them expects (row-major for
        the GEMV, tiles for the grouped GEMM).
        factors: None for the plain quantiser, or {H: U_H, F: U_F}, the inverse-Hessian factors
        (dymoe_gptq_factor) of the inputs of W1 / W3 and of W2: the error-compensated quantiser the paper
        prepares its experts with (Sec. 5)."""
        H, F = self.H, self.F
        self.layout = layout
        wdev = torch.empty((self.elems,), dtype=torch.bfloat16, device=device)
        st = torch.cuda.current_stream().cuda_stream
        if factors is not None:
            self._add_compensated(ctx, device, formats, layout, factors, wdev)
            return
        for b in formats:
            offs, total = quant_layout(H, F, b)
            self.nbytes[b] = total
            self.buf[b] = torch.empty((self.n_pool, total), dtype=torch.uint8, pin_memory=True)
            stage = torch.empty((total,), dtype=torch.uint8, device=device)
            fmt = B.ExpertFmt()
            for m in range(3):
                fmt.w[m] = wdev.data_ptr() + m * H * F * 2
            _Slot._point(fmt, b, stage.data_ptr(), offs)
            table = torch.frombuffer(bytearray(bytes(fmt)), dtype=torch.uint8).to(device)
            want = torch.tensor([b], dtype=torch.uint8, device=device)
            for i in range(self.n_pool):
                wdev.view(torch.uint8).copy_(self.buf[16][i], non_blocking=True)
                B._check(B.lib.dymoe_quantize_experts(ctx._h, table.data_ptr(), want.data_ptr(), None, 1, H, F, 64,
                                                      layout, st), "dymoe_quantize_experts")
                self.buf[b][i].copy_(stage, non_blocking=True)
            torch.cuda.synchronize()

    def _add_compensated(self, ctx, device, formats, layout, factors, wdev):
        H, F = self.H, self.F
        shapes = ((F, H), (F, H), (H, F))
        ws = {K: torch.empty((int(B.lib.dymoe_gptq_workspace_bytes(n, K)),), dtype=torch.uint8, device=device)
              for n, K in ((F, H), (H, F))}
        for b in formats:
            offs, total = quant_layout(H, F, b)
            self.nbytes[b] = total
            self.buf[b] = torch.empty((self.n_pool, total), dtype=torch.uint8, pin_memory=True)
            stage = torch.empty((total,), dtype=torch.uint8, device=device)
            for i in range(self.n_pool):
                wdev.view(torch.uint8).copy_(self.buf[16][i], non_blocking=True)
                for m, (n, K) in enumerate(shapes):
                    co, so, zo = offs[m]
                    out = (stage[co:so].view(n, K * b // 8), stage[so:zo].view(torch.float16).view(n, K // 64),
                           stage[zo:zo + n * (K // 64) * 2].view(torch.float16).view(n, K // 64))
                    w = wdev[m * H * F:(m + 1) * H * F].view(n, K)
                    if layout == B.LAYOUT_ROWMAJOR:
                        ctx.gptq_quantize_pack(w, factors[K], b, out=out, workspace=ws[K])
                    else:
                        tiles = ctx.pack_code_tiles(ctx.gptq_quantize_pack(w, factors[K], b, workspace=ws[K]), b)
                        for dst, src in zip(out, tiles):
                            dst.copy_(src)
                self.buf[b][i].copy_(stage, non_blocking=True)
            torch.cuda.synchronize()

    def entry(self, layer, e):
        return (layer * self.E + e) % self.n_pool

    def host_ptr(self, layer, e, fmt=16):
        return self.buf[fmt].data_ptr() + self.entry(layer, e) * self.nbytes[fmt]


class _Slot:
    """Device buffers of one resident expert in one transferred format.  A bf16
    slot also carries a buffer for each of `quant_formats`, which the device
    quantiser writes ("bf16" transfer mode)."""

    def __init__(self, H, F, fmt_bits, device, quant_formats, mem=None):
        """mem: None (the slot allocates its buffers) or a uint8 view of the slot's bytes in an arena."""
        fmt = B.ExpertFmt()
        self.fmt_bits = fmt_bits
        pos = 0

        def take(nbytes):
            nonlocal pos
            if mem is None:
                return torch.empty((nbytes,), dtype=torch.uint8, device=device)
            view = mem[pos:pos + nbytes]
            pos += (nbytes + 255) // 256 * 256
            return view

        if fmt_bits == 16:
            self.buf = take(6 * H * F)
            for i in range(3):
                fmt.w[i] = self.buf.data_ptr() + i * H * F * 2
            self.qbuf = {}
            for b in quant_formats:
                offs, total = quant_layout(H, F, b)
                self.qbuf[b] = take(total)
                self._point(fmt, b, self.qbuf[b].data_ptr(), offs)
        else:
            offs, total = quant_layout(H, F, fmt_bits)
            self.buf = take(total)
            self._point(fmt, fmt_bits, self.buf.data_ptr(), offs)
        self.fmt = torch.frombuffer(bytearray(bytes(fmt)), dtype=torch.uint8).pin_memory()
        self.copy_event = None   # event of a copy not yet waited for on the compute stream
        self.last_use = None     # torch event: the compute stream has finished reading the slot
        self.prefetched = False  # filled ahead of time and not used yet

    @staticmethod
    def nbytes(H, F, fmt_bits, quant_formats):
        """Bytes of a slot of this format inside an arena (pieces aligned to 256 bytes)."""
        r = lambda n: (n + 255) // 256 * 256
        if fmt_bits == 16:
            return r(6 * H * F) + sum(r(quant_layout(H, F, b)[1]) for b in quant_formats)
        return r(quant_layout(H, F, fmt_bits)[1])

    @staticmethod
    def _point(fmt, b, base, offs):
        for i in range(3):
            co, so, zo = offs[i]
            getattr(fmt, "q%d" % b)[i] = base + co
            getattr(fmt, "s%d" % b)[i] = base + so
            getattr(fmt, "z%d" % b)[i] = base + zo


class ExpertStack:
    def __init__(self, ctx, T, phase, H, F, E, k, routers, pool, slots, tier_count, tier_bits, floor_bits=None,
                 prefetch=True, transfer="bf16", alpha=0.125, k_hh=0, predict_t=None, device="cuda:0",
                 budget_bytes=None, lookahead="always", eviction="lru"):
        """T tokens per step; phase "decode" (gate-score importance, Eq. 3; the k experts the next layer is
        predicted to route the token to are fetched ahead, Eq. 8 with t = k) or "prefill" (heavy-hitter
        importance over the k_hh highest-norm tokens, Eq. 2; the predict_t experts of highest predicted
        token frequency are fetched ahead, Eq. 7).
        routers: list over layers of wg [E,H] bf16 device tensors.  slots: number of bf16 slots
        (transfer="bf16") or {16: n, 8: n, 4: n, 2: n} (transfer="assigned"; formats left out get none).
        budget_bytes: instead of `slots`, one byte budget of device memory shared by the formats (the
        library's dymoe_cache_*).
        floor_bits: per-layer floor of the assignment (list) or None.  tier_count: one tuple for every
        layer, or a list of per-layer tuples (e.g. (t_l, E - t_l) from the depth schedule of Sec. 4.3)."""
        if transfer not in ("bf16", "assigned"):
            raise ValueError("transfer must be 'bf16' or 'assigned'")
        if lookahead not in ("always", "expected"):
            raise ValueError("lookahead must be 'always' or 'expected'")
        self.lookahead = lookahead
        if phase not in ("decode", "prefill"):
            raise ValueError("phase must be 'decode' or 'prefill'")
        self.ctx, self.T, self.phase, self.H, self.F, self.E, self.k = ctx, T, phase, H, F, E, k
        self.L = len(routers)
        self.routers, self.pool, self.transfer = routers, pool, transfer
        self.floor = list(floor_bits) if floor_bits is not None else [0] * self.L
        self.prefetch, self.alpha, self.dev = prefetch, alpha, device
        self.predict_t = int(predict_t) if predict_t is not None else k
        # a layer's experts are all resident while it runs, next to the ones fetched ahead
        need = min(E, T * k) + (self.predict_t if prefetch else 0)
        # formats the device quantiser may be asked for when bf16 weights are moved
        made = sorted({int(b) for b in list(tier_bits) + self.floor if int(b) in (8, 4, 2)}) if transfer == "bf16" else []
        self._slot_args = (H, F, device, made)
        if budget_bytes is None:
            counts = {16: int(slots)} if transfer == "bf16" else {b: int(slots.get(b, 0)) for b in FORMATS}
            if any(0 < n < need for n in counts.values()) or not any(counts.values()):
                raise ValueError("every configured pool needs at least %d slots" % need)
            self.cache = MixedPrecisionCache(counts)
            self.arena = None
            self.slots = {(b, i): _Slot(H, F, b, device, made) for b, n in counts.items() for i in range(n)}
        else:
            held = (16,) if transfer == "bf16" else tuple(b for b in FORMATS if b in pool.nbytes)
            sizes = {b: _Slot.nbytes(H, F, b, made) for b in held}
            self.cache = ByteBudgetCache(int(budget_bytes), sizes)
            n_blocks = int(budget_bytes) // self.cache.block_bytes
            if n_blocks * (self.cache.block_bytes // max(sizes.values())) < need:
                raise ValueError("the budget holds fewer than %d experts of the largest format" % need)
            self.arena = torch.empty((n_blocks * self.cache.block_bytes,), dtype=torch.uint8, device=device)
            self._slot_bytes = sizes
            self.slots = {}                         # (format, offset) -> _Slot, made when first handed out
        # eviction order of the expert cache: least recently used (the paper's), or "cyclic": the layers are visited in
        # the same order in every step, so what goes first is the resident whose layer comes up last
        if eviction not in ("lru", "cyclic"):
            raise ValueError("eviction: 'lru' or 'cyclic'")
        self.eviction = eviction
        if eviction == "cyclic":
            self.cache.set_cyclic(self.L)
        per_layer = isinstance(tier_count[0], (tuple, list))
        self.tiers = [tuple(tc) for tc in tier_count] if per_layer else [tuple(tier_count)] * self.L
        if len(self.tiers) != self.L or any(len(tc) != len(tier_bits) for tc in self.tiers):
            raise ValueError("tier_count: one tuple, or one per layer, as long as tier_bits")
        self.tier_arrays = [(C.c_int32 * len(tc))(*[int(v) for v in tc]) for tc in self.tiers]
        path = B.PATH_GEMV if T == 1 else B.PATH_AUTO
        mk = lambda: MoELayer(ctx, T, H, F, E, k, phase, self.tiers[0], tier_bits, k_hh=k_hh, out_dtype=B.OUT_F32,
                              path=path, device=device)
        self.layer, self.ahead = mk(), mk()     # buffers of the current layer, and of the look-ahead prediction
        if transfer == "assigned" and pool.layout != self.layer.layout:
            raise ValueError("the pool's quantised formats are not in the layout the FFN path reads")
        self.tables = torch.zeros((self.L, E, FMT_BYTES), dtype=torch.uint8, device=device)
        self.table_slot = {}                    # (layer, e) -> slot written in the table
        self.h = [torch.empty((T, H), dtype=torch.bfloat16, device=device) for _ in range(2)]
        self.score = torch.empty((T,), dtype=torch.float32, device=device)
        self.side = torch.cuda.Stream(device=device)       # copies a layer is waiting for
        self.spec = torch.cuda.Stream(device=device)       # copies made on a prediction (same priority)
        # what the look-ahead rule goes by: the link's rate (one timed copy), a layer's compute time (timed over the
        # first steps) and the share of right predictions so far (a prior of 3 in 4 until there is evidence)
        self.link_gbps = self._measure_link()
        self.layer_ms = None
        self._layer_events = []
        self._pred_seen, self._pred_right = 4, 3
        self._last_pred = None
        self._idle_lookahead, self._probe_now = False, True
        # What the host reads back per layer sits in one device buffer per runner and travels in one copy:
        # idx [T,k] int32 | load [E] int32 | rank [E] int32 | bits [E] uint8 | mark [E] uint8.  rank and mark are the
        # look-ahead runner's Eq. 7 selection (position of every expert by predicted frequency; 16 for the
        # predict_t most frequent, 0 for the rest), written by dymoe_assign_precision with tiers (t, E - t).
        n_idx, n_load, n_e = T * k * 4, E * 4, (E + 3) // 4 * 4
        self._meta_tail = n_idx                 # T > 1: idx stays on the device

        def views(buf):
            o = n_idx + 2 * n_load
            return (buf[:n_idx].view(torch.int32).view(T, k), buf[n_idx:n_idx + n_load].view(torch.int32),
                    buf[n_idx + n_load:o].view(torch.int32), buf[o:o + E], buf[o + n_e:o + n_e + E])

        def pack(lay):
            lay.meta = torch.zeros((n_idx + 2 * n_load + 2 * n_e,), dtype=torch.uint8, device=device)
            lay.idx, lay.load, lay.sel_rank, lay.bits, lay.sel_mark = views(lay.meta)
            host = torch.zeros(lay.meta.shape, dtype=torch.uint8).pin_memory()
            return (host,) + views(host)

        self.host_meta, self.host_idx, self.host_load, _, self.host_bits, _ = pack(self.layer)
        self.host_pmeta, self.host_pidx, self.host_pload, self.host_prank, self.host_pbits, self.host_pmark = pack(self.ahead)
        t_sel = min(self.predict_t, E)
        self._sel_tc = (C.c_int32 * 2)(t_sel, E - t_sel)
        self._sel_tb = (C.c_uint8 * 2)(16, 0)
        self.stats = collections.Counter()
        self.measure_overlap = False    # set True to time every copy and every wait of the compute stream (overlap_report)
        self._copy_events, self._stall_events = [], []
        self.trace = []     # per step and layer: (experts, assigned bits, bits they were run at)
        self.predictions = []   # per step and layer (but the last): experts fetched ahead for the next layer

    def _measure_link(self):
        """Host link rate in GB/s from one copy out of the pool (64 MiB at most), on the demand stream."""
        fmt = 16 if 16 in self.pool.buf else sorted(self.pool.buf)[-1]
        n = min(self.pool.nbytes[fmt], 64 << 20)
        dst = torch.empty((n,), dtype=torch.uint8, device=self.dev)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        rates = []
        for _ in range(2):                       # the second copy is the one that counts
            e0.record(self.side)
            ev = self.ctx.prefetch_submit(self.pool.buf[fmt].data_ptr(), dst.data_ptr(), n, self.side.cuda_stream)
            e1.record(self.side)
            e1.synchronize()
            self.ctx.prefetch_release(ev)
            rates.append(n / (e0.elapsed_time(e1) * 1e-3) / 1e9)
        return rates[-1]

    def _worth_fetching_ahead(self, nbytes):
        """The expected-value rule of the module's header."""
        if self.lookahead == "always":
            return True
        if self.layer_ms is None:                # no compute time measured yet: wait for it
            return False
        p = self._pred_right / self._pred_seen
        c = nbytes / (self.link_gbps * 1e6)      # ms
        return p * min(c, self.layer_ms) >= (1.0 - p) * c

    def _slot(self, name):
        slot = self.slots.get(name)
        if slot is None:        # byte-budget mode: a view of the arena
            bits, off = name
            H, F, device, made = self._slot_args
            slot = self.slots[name] = _Slot(H, F, bits, device, made, mem=self.arena[off:off + self._slot_bytes[bits]])
        return slot

    def _fill(self, act, key, ahead):
        """Copy the format `act.load_bits` of expert `key` into the slot the cache chose: on the demand stream, or
        (ahead) on the stream of speculative copies."""
        stream = self.spec if ahead else self.side
        slot = self._slot(act.slot)

        def settle(old):
            """Order the new copy behind whatever still touches the memory `old` names."""
            if old.prefetched:
                self.stats["prefetch_wasted"] += 1
                old.prefetched = False
            if old.copy_event is not None:        # an unused earlier copy, possibly on the other stream
                self.ctx.prefetch_wait(old.copy_event, stream.cuda_stream)
                self.ctx.prefetch_release(old.copy_event)
                old.copy_event = None
            if old.last_use is not None:          # the compute stream may still be reading the old content
                stream.wait_event(old.last_use)
                old.last_use = None

        for name in act.freed:                    # slots given up whose memory the new one may overlap
            old = self.slots.get(name)
            if old is not None:
                settle(old)
        settle(slot)
        layer, e = key
        nbytes = self.pool.nbytes[act.load_bits]
        if self.measure_overlap:
            c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            c0.record(stream)
        slot.copy_event = self.ctx.prefetch_submit(self.pool.host_ptr(layer, e, act.load_bits), slot.buf.data_ptr(),
                                                   nbytes, stream.cuda_stream)
        if self.measure_overlap:
            c1.record(stream)
            self._copy_events.append((c0, c1))
        slot.prefetched = ahead
        self.stats["bytes_copied"] += nbytes
        self.stats["copies_%d" % act.load_bits] += 1

    def _front(self, lay, h, wg, st):
        """S1 + S2 + S3 into the buffers of `lay`."""
        if self.phase == "decode" and self.T <= B.FRONT_MAX_TOKENS:
            lay.front(h, wg, None, st)
        else:
            lay.route(h, wg, None, st)
            lay.importance(h, st, score=self.score if self.phase == "prefill" else None)
            lay.assign(st)

    def step(self, h0, token_score=None):
        """One step (T tokens) through all layers.  h0: [T,H] bf16 on the device.  Returns the final hidden states.
        Prefill: token_score [T] fp32 ranks the heavy-hitter tokens in every layer (a token's score is a
        property of the token, Sec. 4.2.1); None takes the row norms of h0 (the layers' own inputs are
        normalised and carry no such signal)."""
        lay, nxt_lay, ctx = self.layer, self.ahead, self.ctx
        cs = torch.cuda.current_stream()
        st = cs.cuda_stream
        h = self.h[0]
        h.copy_(h0)
        if self.phase == "prefill":
            if token_score is not None:
                self.score.copy_(token_score)
            else:
                B._check(B.lib.dymoe_token_score_norm(ctx._h, h.data_ptr(), self.T, self.H, self.score.data_ptr(), st),
                         "dymoe_token_score_norm")
        step_trace, step_pred = [], []
        # when the rule turned every copy of the last step down, the prediction itself (a router launch per layer) is
        # only made every 8th step, to keep the share of right predictions current
        self._probe_now = not self._idle_lookahead or self.stats["steps"] % 8 == 0
        declined0, issued0 = self.stats["prefetch_declined"], self.stats["prefetch_issued"]
        for l in range(self.L):
            lay.floor_bits, lay._tc = self.floor[l], self.tier_arrays[l]
            self._front(lay, h, self.routers[l], st)
            look = self.prefetch and l + 1 < self.L and self._probe_now
            if look:     # Eq. 6: the next layer's router (and precision rule) on the current hidden states
                nxt_lay.floor_bits, nxt_lay._tc = self.floor[l + 1], self.tier_arrays[l + 1]
                self._front(nxt_lay, h, self.routers[l + 1], st)
                if self.T > 1:   # Eq. 7: the predict_t experts of highest predicted frequency, chosen on the device
                    B._check(B.lib.dymoe_assign_precision(ctx._h, B.PHASE_PREFILL, nxt_lay.load.data_ptr(), None, self.E,
                                                          2, C.cast(self._sel_tc, C.c_void_p),
                                                          C.cast(self._sel_tb, C.c_void_p), 0,
                                                          nxt_lay.sel_mark.data_ptr(), nxt_lay.sel_rank.data_ptr(), st),
                             "dymoe_assign_precision")
                a = 0 if self.T == 1 else self._meta_tail
                self.host_pmeta[a:].copy_(nxt_lay.meta[a:], non_blocking=True)
            a = 0 if self.T == 1 else self._meta_tail
            self.host_meta[a:].copy_(lay.meta[a:], non_blocking=True)
            cs.synchronize()
            if self.T == 1:      # in routing order
                active = [int(e) for e in self.host_idx[0].tolist()]
            else:                # every expert some token was routed to
                active = [e for e, c in enumerate(self.host_load.tolist()) if c > 0]
            abits = [int(self.host_bits[e]) for e in active]
            if self._last_pred is not None:       # how the look-ahead of the layer before did
                self._pred_seen += len(self._last_pred)
                self._pred_right += sum(1 for e in self._last_pred if e in active)
                self._last_pred = None
            want = lambda b: 16 if self.transfer == "bf16" else b
            need = [(e, b) for e, b in zip(active, abits) if b != 0]
            # this layer's experts: resident, arriving, or fetched now (what is already resident is
            # protected first, so that fetching one expert cannot evict another one of the layer)
            protect = set()
            for e, b in need:
                if self.cache.covers((l, e), want(b)):
                    protect.add(self.cache.resident((l, e)))
            used_bits = dict(zip(active, abits))
            override = False
            if self.measure_overlap:
                w0 = torch.cuda.Event(enable_timing=True)
                w0.record(cs)
            for e, b in need:
                key = (l, e)
                act = self.cache.request(key, want(b), protect, position=l if self.eviction == "cyclic" else None)
                protect.add(act.slot)
                slot = self._slot(act.slot)
                if act.load_bits:
                    self._fill(act, key, ahead=False)
                    self.stats[act.kind] += 1
                else:
                    self.stats["hit_prefetched" if slot.prefetched else "hit_resident"] += 1
                slot.prefetched = False
                if slot.copy_event is not None:
                    ctx.prefetch_wait(slot.copy_event, st)
                    ctx.prefetch_release(slot.copy_event)
                    slot.copy_event = None
                if self.table_slot.get(key) != act.slot:
                    self.tables[l, e].copy_(slot.fmt, non_blocking=True)
                    self.table_slot[key] = act.slot
                if self.transfer == "assigned" and act.use_bits != b:     # Conservative Reuse: run at the resident precision
                    self.host_bits[e] = act.use_bits
                    used_bits[e] = act.use_bits
                    override = True
                    self.stats["reused_higher"] += 1
            if self.measure_overlap:
                w1 = torch.cuda.Event(enable_timing=True)
                w1.record(cs)
                self._stall_events.append((w0, w1))
            if override:
                lay.bits.copy_(self.host_bits, non_blocking=True)
            step_trace.append((tuple(active), tuple(abits), tuple(used_bits[e] for e in active)))
            # the next layer's predicted experts, copied while this layer computes
            if look:
                if self.T == 1:      # Eq. 8: the token's own predicted experts
                    ahead = [int(v) for v in self.host_pidx[0].tolist()][:self.predict_t]
                else:                # Eq. 7: the experts most tokens are predicted to ask for (nobody's are left out)
                    mark, rank, freq = self.host_pmark.tolist(), self.host_prank.tolist(), self.host_pload.tolist()
                    ahead = sorted((e for e in range(self.E) if mark[e] and freq[e] > 0), key=lambda e: rank[e])
                step_pred.append(tuple(ahead))
                self._last_pred = tuple(ahead)
                for e in ahead:
                    pb = int(self.host_pbits[e])
                    key = (l + 1, e)
                    if pb == 0:
                        continue
                    if self.cache.covers(key, want(pb)):
                        protect.add(self.cache.resident(key))
                        continue
                    if not self._worth_fetching_ahead(self.pool.nbytes[want(pb)]):
                        self.stats["prefetch_declined"] += 1
                        continue
                    act = self.cache.request(key, want(pb), protect, position=l + 1 if self.eviction == "cyclic" else None)
                    protect.add(act.slot)
                    self._fill(act, key, ahead=True)
                    self.stats["prefetch_issued"] += 1
            table = self.tables[l]
            timing = self.layer_ms is None
            if timing:
                t0 = torch.cuda.Event(enable_timing=True)
                t0.record(cs)
            if self.transfer == "bf16":      # S4 on arrival
                B._check(B.lib.dymoe_quantize_experts(ctx._h, table.data_ptr(), lay.bits.data_ptr(),
                                                      lay.load.data_ptr(), self.E, self.H, self.F, 64,
                                                      lay.layout, st), "dymoe_quantize_experts")
            B._check(B.lib.dymoe_moe_ffn_mixed(ctx._h, h.data_ptr(), lay.idx.data_ptr(), lay.gate.data_ptr(),
                                               lay.bits.data_ptr(), table.data_ptr(), self.T, self.H, self.F, self.E,
                                               self.k, 64, B.OUT_F32, lay.path, lay.y.data_ptr(),
                                               lay.ws.data_ptr(), lay.ws_bytes, st), "dymoe_moe_ffn_mixed")
            nxt = self.h[(l + 1) % 2]
            B._check(B.lib.dymoe_residual_rmsnorm(ctx._h, h.data_ptr(), lay.y.data_ptr(), B.OUT_F32,
                                                  float(self.alpha), self.T, self.H, nxt.data_ptr(), st),
                     "dymoe_residual_rmsnorm")
            if timing:
                t1 = torch.cuda.Event(enable_timing=True)
                t1.record(cs)
                self._layer_events.append((t0, t1))
            done = torch.cuda.Event()
            done.record(cs)
            for e, b in need:
                self._slot(self.cache.resident((l, e))).last_use = done
            h = nxt
        self._last_pred = None
        if self._probe_now and self.lookahead == "expected" and self.layer_ms is not None:
            self._idle_lookahead = (self.stats["prefetch_issued"] == issued0 and self.stats["prefetch_declined"] > declined0)
        if self.layer_ms is None and self.stats["steps"] >= 1:      # the second step on: a layer's compute time is known
            cs.synchronize()
            ms = sorted(a.elapsed_time(b) for a, b in self._layer_events[self.L:])
            self.layer_ms, self._layer_events = ms[len(ms) // 2], []
        self.trace.append(step_trace)
        self.predictions.append(step_pred)
        self.stats["steps"] += 1
        return h

    def overlap_report(self):
        """With measure_overlap: time the host link was busy, time the compute stream stood waiting for copies
        (between the first and the last wait of each layer), and the share of the copy time that was hidden
        behind compute.  Clears the recorded events."""
        torch.cuda.synchronize()
        copy_ms = sum(a.elapsed_time(b) for a, b in self._copy_events)
        stall_ms = sum(a.elapsed_time(b) for a, b in self._stall_events)
        self._copy_events, self._stall_events = [], []
        hidden = 1.0 - stall_ms / copy_ms if copy_ms > 0 else None
        return {"copy_ms": copy_ms, "stall_ms": stall_ms, "copy_time_hidden": hidden}

    def close(self):
        torch.cuda.synchronize()
        for slot in self.slots.values():
            if slot.copy_event is not None:
                self.ctx.prefetch_release(slot.copy_event)
                slot.copy_event = None


class DecodeStack(ExpertStack):
    """One token per step (Sec. 4.2.2 importance, Eq. 8 prefetch)."""

    def __init__(self, ctx, H, F, E, k, routers, pool, slots, tier_count, tier_bits, floor_bits=None,
                 prefetch=True, transfer="bf16", alpha=0.125, device="cuda:0", budget_bytes=None, lookahead="always",
                 eviction="lru"):
        super().__init__(ctx, 1, "decode", H, F, E, k, routers, pool, slots, tier_count, tier_bits,
                         floor_bits=floor_bits, prefetch=prefetch, transfer=transfer, alpha=alpha, device=device,
                         budget_bytes=budget_bytes, lookahead=lookahead, eviction=eviction)


class PrefillStack(ExpertStack):
    """T tokens per step (Sec. 4.2.1 importance over the k_hh highest-norm tokens, Eq. 7 prefetch of
    the predict_t most frequently predicted experts)."""

    def __init__(self, ctx, T, H, F, E, k, k_hh, routers, pool, slots, tier_count, tier_bits, floor_bits=None,
                 prefetch=True, predict_t=None, transfer="bf16", alpha=0.125, device="cuda:0", budget_bytes=None,
                 lookahead="always"):
        super().__init__(ctx, T, "prefill", H, F, E, k, routers, pool, slots, tier_count, tier_bits,
                         floor_bits=floor_bits, prefetch=prefetch, transfer=transfer, alpha=alpha, k_hh=k_hh,
                         predict_t=predict_t if predict_t is not None else min(E, max(k, E // 2)), device=device,
                         budget_bytes=budget_bytes, lookahead=lookahead)


class ResidentDecodeStack:
    """One token per step through a stack whose experts are all resident in DEVICE memory, in every format the
    precision assignment may name (a 288 GB device holds a whole model of the paper's size, Sec. 6.1).

    Nothing is copied and nothing is decided on the host: the importance of an expert and its bit width are still
    chosen per token and layer on the device (Sec. 4.2.2, Sec. 4.3), and the FFN reads, through the layer's format
    table, the format the assignment names.  A step is therefore a fixed chain of launches (per layer
    dymoe_decode_step, or dymoe_decode_front and dymoe_moe_ffn_mixed with fused=False, then dymoe_residual_rmsnorm),
    enqueued one by one or (graph=True) replayed as one HIP graph.

    pool: a HostExpertPool holding every format in `tier_bits` and the floors (row-major codes); its entries are
    copied to the device once.  tier_count: one tuple, or one per layer; floor_bits: per layer or None."""

    def __init__(self, ctx, H, F, E, k, routers, pool, tier_count, tier_bits, floor_bits=None, alpha=0.125,
                 device="cuda:0", graph=True, fused=True):
        self.ctx, self.H, self.F, self.E, self.k = ctx, H, F, E, k
        self.fused = bool(fused)
        self.L = L = len(routers)
        self.routers, self.alpha, self.dev = routers, float(alpha), device
        self.floor = [int(b) for b in floor_bits] if floor_bits is not None else [0] * L
        per_layer = isinstance(tier_count[0], (tuple, list))
        tiers = [tuple(tc) for tc in tier_count] if per_layer else [tuple(tier_count)] * L
        if len(tiers) != L or any(len(tc) != len(tier_bits) for tc in tiers):
            raise ValueError("tier_count: one tuple, or one per layer, as long as tier_bits")
        self._tc = [(C.c_int32 * len(tc))(*[int(v) for v in tc]) for tc in tiers]
        self._tb = (C.c_uint8 * len(tier_bits))(*[int(b) for b in tier_bits])
        self._nt = len(tier_bits)
        formats = sorted({int(b) for b in list(tier_bits) + self.floor if int(b) != 0})
        missing = [b for b in formats if b not in pool.buf]
        if missing:
            raise ValueError("the pool holds no %s-bit format" % missing)
        if any(b != 16 for b in formats) and pool.layout != B.LAYOUT_ROWMAJOR:
            raise ValueError("the decode path reads row-major codes")
        self.weights = {b: pool.buf[b].to(device) for b in formats}     # [n_pool, bytes of the format]
        table = bytearray()
        for l in range(L):
            for e in range(E):
                fmt, i = B.ExpertFmt(), pool.entry(l, e)
                for b in formats:
                    base = self.weights[b].data_ptr() + i * pool.nbytes[b]
                    if b == 16:
                        for m in range(3):
                            fmt.w[m] = base + m * H * F * 2
                    else:
                        _Slot._point(fmt, b, base, quant_layout(H, F, b)[0])
                table += bytes(fmt)
        self.tables = torch.frombuffer(table, dtype=torch.uint8).to(device).view(L, E, FMT_BYTES)
        i32 = lambda *s: torch.zeros(s, dtype=torch.int32, device=device)
        f32 = lambda *s: torch.zeros(s, dtype=torch.float32, device=device)
        self.idx, self.gate = i32(L, 1, k), f32(L, 1, k)                 # kept per layer: what `trace` reports
        self.bits = torch.zeros((L, E), dtype=torch.uint8, device=device)
        self.probs, self.imp, self.load, self.rank = f32(1, E), f32(E), i32(E), i32(E)
        self.y = f32(1, H)
        self.ws_bytes = B.workspace_bytes(1, H, F, E, k)
        self.ws = torch.empty((self.ws_bytes,), dtype=torch.uint8, device=device)
        self.h = [torch.zeros((1, H), dtype=torch.bfloat16, device=device) for _ in range(2)]
        self._graph = None if graph else False

    def _enqueue(self, st):
        ctx, H, F, E, k = self.ctx._h, self.H, self.F, self.E, self.k
        for l in range(self.L):
            h, nxt = self.h[l % 2], self.h[(l + 1) % 2]
            idx, gate, bits, table = self.idx[l].data_ptr(), self.gate[l].data_ptr(), self.bits[l].data_ptr(), \
                self.tables[l].data_ptr()
            rc = B.ENOTSUP
            if self.fused:       # front end and FFN in two launches; sizes it does not cover take the separate calls
                rc = B.lib.dymoe_decode_step(ctx, h.data_ptr(), self.routers[l].data_ptr(), None, 1, H, F, E, k, 1,
                                             self._nt, C.cast(self._tc[l], C.c_void_p), C.cast(self._tb, C.c_void_p),
                                             self.floor[l], table, 64, B.OUT_F32, idx, gate, self.probs.data_ptr(),
                                             self.imp.data_ptr(), self.load.data_ptr(), bits, self.rank.data_ptr(),
                                             self.y.data_ptr(), self.ws.data_ptr(), self.ws_bytes, st)
                if rc != B.ENOTSUP:
                    B._check(rc, "dymoe_decode_step")
            if rc == B.ENOTSUP:
                B._check(B.lib.dymoe_decode_front(ctx, h.data_ptr(), self.routers[l].data_ptr(), None, 1, H, E, k, 1,
                                                  self._nt, C.cast(self._tc[l], C.c_void_p), C.cast(self._tb, C.c_void_p),
                                                  self.floor[l], idx, gate, self.probs.data_ptr(), self.imp.data_ptr(),
                                                  self.load.data_ptr(), bits, self.rank.data_ptr(), st),
                         "dymoe_decode_front")
                B._check(B.lib.dymoe_moe_ffn_mixed(ctx, h.data_ptr(), idx, gate, bits, table, 1, H, F, E, k, 64, B.OUT_F32,
                                                   B.PATH_GEMV, self.y.data_ptr(), self.ws.data_ptr(), self.ws_bytes, st),
                         "dymoe_moe_ffn_mixed")
            B._check(B.lib.dymoe_residual_rmsnorm(ctx, h.data_ptr(), self.y.data_ptr(), B.OUT_F32, self.alpha, 1, H,
                                                  nxt.data_ptr(), st), "dymoe_residual_rmsnorm")

    def step(self, h0):
        """h0: [1,H] bf16 on the device.  Returns the final hidden states (a buffer the next step overwrites)."""
        self.h[0].copy_(h0)
        if self._graph is False:
            self._enqueue(torch.cuda.current_stream().cuda_stream)
        else:
            if self._graph is None:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=torch.cuda.Stream(device=self.dev)):
                    self._enqueue(torch.cuda.current_stream().cuda_stream)
                self._graph = g
            self._graph.replay()
        return self.h[self.L % 2]

    def trace(self):
        """Per layer of the last step: (selected experts in routing order, their assigned bit widths).  Synchronises."""
        idx, bits = self.idx.cpu(), self.bits.cpu()
        return [(tuple(int(e) for e in idx[l, 0]), tuple(int(bits[l, e]) for e in idx[l, 0])) for l in range(self.L)]
