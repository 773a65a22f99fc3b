"""A stack of MoE expert layers decoding one token at a time with the experts
resident in pinned HOST memory (paper Sec. 4.4: dynamic expert orchestration).

Per layer the compute stream runs the hot path of `layer.py`; the experts it
needs are brought into a small set of device slots, on demand or ahead of time:
the next layer's router applied to the current hidden state (Sec. 4.4.1 Eq. 6)
names the t experts to prefetch (Eq. 8), and their bf16 weights are copied on a
side stream (dymoe_prefetch_submit / dymoe_prefetch_wait) while the current
layer computes.  Experts arrive as bf16 and are quantised on the device to the
width the precision assignment asks for (S4 on arrival).

Host control flow and bookkeeping only; every arithmetic step runs in
libdymoe.so.  The device slots are a plain LRU cache keyed by (layer, expert);
the paper's mixed-precision cache rules are not modelled here.
"""
import collections
import ctypes as C

import torch

from . import binding as B
from .layer import MoELayer

FMT_BYTES = C.sizeof(B.ExpertFmt)


class HostExpertPool:
    """bf16 expert weights in pinned host memory.  To bound memory and set-up
    time, `n_pool` distinct experts are drawn and (layer, expert) maps to entry
    (layer * E + expert) mod n_pool.  One entry is W1 [F,H] | W3 [F,H] | W2 [H,F]
    back to back, so an expert moves with a single copy."""

    def __init__(self, H, F, E, n_pool, matrices):
        # matrices(i) -> [W1, W3, W2] as uint16 numpy arrays (bf16 bits) of pool entry i
        self.H, self.F, self.E, self.n_pool = H, F, E, n_pool
        self.elems = 3 * H * F
        self.nbytes = 2 * self.elems
        self.buf = torch.empty((n_pool, self.elems), dtype=torch.int16, pin_memory=True)
        view = self.buf.numpy()
        for i in range(n_pool):
            w1, w3, w2 = matrices(i)
            view[i, :H * F] = w1.reshape(-1).view("int16")
            view[i, H * F:2 * H * F] = w3.reshape(-1).view("int16")
            view[i, 2 * H * F:] = w2.reshape(-1).view("int16")

    def entry(self, layer, e):
        return (layer * self.E + e) % self.n_pool

    def host_ptr(self, layer, e):
        return self.buf.data_ptr() + self.entry(layer, e) * self.nbytes


class _Slot:
    """Device buffers of one resident expert."""

    def __init__(self, H, F, device, group=64):
        self.w = torch.empty((3 * H * F,), dtype=torch.bfloat16, device=device)
        self.q = {}
        for b in (4, 2):
            self.q[b] = [(torch.empty((n, kk * b // 8), dtype=torch.uint8, device=device),
                          torch.empty((n, kk // group), dtype=torch.float16, device=device),
                          torch.empty((n, kk // group), dtype=torch.float16, device=device))
                         for n, kk in ((F, H), (F, H), (H, F))]
        fmt = B.ExpertFmt()
        base = self.w.data_ptr()
        for i in range(3):
            fmt.w[i] = base + i * H * F * 2
            for b in (4, 2):
                cd, sc, zr = self.q[b][i]
                getattr(fmt, "q%d" % b)[i] = cd.data_ptr()
                getattr(fmt, "s%d" % b)[i] = sc.data_ptr()
                getattr(fmt, "z%d" % b)[i] = zr.data_ptr()
        self.fmt = torch.frombuffer(bytearray(bytes(fmt)), dtype=torch.uint8).pin_memory()
        self.key = None          # (layer, expert) held
        self.copy_event = None   # event of a copy not yet waited for on the compute stream
        self.last_use = None     # torch event: the compute stream has finished reading the slot
        self.prefetched = False  # filled ahead of time and not used yet


class DecodeStack:
    def __init__(self, ctx, H, F, E, k, routers, pool, n_slots, tier_count, tier_bits,
                 floor_bits=None, prefetch_t=2, prefetch=True, alpha=0.125, device="cuda:0"):
        """routers: list over layers of wg [E,H] bf16 device tensors.  floor_bits: per-layer
        floor of the assignment (list) or None.  prefetch_t: experts fetched ahead per layer (Eq. 8)."""
        if n_slots < k + (prefetch_t if prefetch else 0):
            raise ValueError("need at least k + prefetch_t slots")
        self.ctx, self.H, self.F, self.E, self.k = ctx, H, F, E, k
        self.L = len(routers)
        self.routers, self.pool = routers, pool
        self.floor = list(floor_bits) if floor_bits is not None else [0] * self.L
        self.t, self.prefetch, self.alpha = prefetch_t, prefetch, alpha
        self.dev = device
        self.layer = MoELayer(ctx, 1, H, F, E, k, "decode", tier_count, tier_bits, out_dtype=B.OUT_F32,
                              path=B.PATH_GEMV, device=device)
        self.slots = [_Slot(H, F, device) for _ in range(n_slots)]
        self.lru = collections.OrderedDict((i, None) for i in range(n_slots))   # slot ids, oldest first
        self.where = {}                                                        # (layer, e) -> slot id
        self.tables = torch.zeros((self.L, E, FMT_BYTES), dtype=torch.uint8, device=device)
        self.table_slot = {}                                                   # (layer, e) -> slot id written in the table
        self.pred = torch.empty((1, max(1, prefetch_t)), dtype=torch.int32, device=device)
        self.pred_w = torch.empty((1, max(1, prefetch_t)), dtype=torch.float32, device=device)
        self.h = [torch.empty((1, H), dtype=torch.bfloat16, device=device) for _ in range(2)]
        self.side = torch.cuda.Stream(device=device)
        self.host_idx = torch.empty((1, k), dtype=torch.int32).pin_memory()
        self.host_bits = torch.empty((E,), dtype=torch.uint8).pin_memory()
        self.host_pred = torch.empty((1, max(1, prefetch_t)), dtype=torch.int32).pin_memory()
        self.stats = collections.Counter()
        self.trace = []     # per step and layer: (idx, bits of the active experts)

    # -- residency
    def _touch(self, sid):
        self.lru.move_to_end(sid)

    def _fill(self, key, protect, ahead):
        """Bring expert `key` into a slot (evicting the least recently used one
        outside `protect`), by a copy on the side stream.  Returns the slot id."""
        sid = next(s for s in self.lru if s not in protect)
        slot = self.slots[sid]
        if slot.key is not None:
            self.where.pop(slot.key, None)
            if slot.prefetched:
                self.stats["prefetch_wasted"] += 1
        if slot.copy_event is not None:           # an unused earlier copy: same stream, ordered before this one
            self.ctx.prefetch_release(slot.copy_event)
        if slot.last_use is not None:             # the compute stream may still be reading the old content
            self.side.wait_event(slot.last_use)
        layer, e = key
        slot.copy_event = self.ctx.prefetch_submit(self.pool.host_ptr(layer, e), slot.w.data_ptr(),
                                                   self.pool.nbytes, self.side.cuda_stream)
        slot.key, slot.prefetched = key, ahead
        self.where[key] = sid
        self._touch(sid)
        self.stats["bytes_copied"] += self.pool.nbytes
        return sid

    def step(self, h0):
        """One decode step through all layers.  h0: [1,H] bf16 on the device.  Returns the final hidden state."""
        lay, ctx = self.layer, self.ctx
        cs = torch.cuda.current_stream()
        st = cs.cuda_stream
        h = self.h[0]
        h.copy_(h0)
        step_trace = []
        for l in range(self.L):
            lay.floor_bits = self.floor[l]
            lay.front(h, self.routers[l], None, st)
            look = self.prefetch and l + 1 < self.L
            if look:     # Eq. 6: the next layer's router on the current hidden state; Eq. 8: its top t
                B._check(B.lib.dymoe_route_topk(ctx._h, h.data_ptr(), self.routers[l + 1].data_ptr(), None, 1,
                                                self.H, self.E, self.t, 1, self.pred.data_ptr(),
                                                self.pred_w.data_ptr(), None, st), "dymoe_route_topk")
                self.host_pred.copy_(self.pred, non_blocking=True)
            self.host_idx.copy_(lay.idx, non_blocking=True)
            self.host_bits.copy_(lay.bits, non_blocking=True)
            cs.synchronize()
            active = [int(e) for e in self.host_idx[0].tolist()]
            abits = [int(self.host_bits[e]) for e in active]
            step_trace.append((tuple(active), tuple(abits)))
            need = [e for e, b in zip(active, abits) if b != 0]
            # this layer's experts: resident, arriving, or fetched now (the resident ones are
            # protected first, so that fetching one expert cannot evict another one of the layer)
            used = set(self.where[(l, e)] for e in need if (l, e) in self.where)
            for e in need:
                key = (l, e)
                sid = self.where.get(key)
                if sid is None:
                    sid = self._fill(key, used, ahead=False)
                    self.stats["miss"] += 1
                else:
                    self.stats["hit_prefetched" if self.slots[sid].prefetched else "hit_resident"] += 1
                    self._touch(sid)
                used.add(sid)
                slot = self.slots[sid]
                slot.prefetched = False
                if slot.copy_event is not None:
                    ctx.prefetch_wait(slot.copy_event, st)
                    ctx.prefetch_release(slot.copy_event)
                    slot.copy_event = None
                if self.table_slot.get(key) != sid:
                    self.tables[l, e].copy_(slot.fmt, non_blocking=True)
                    self.table_slot[key] = sid
            # the next layer's predicted experts, copied while this layer computes
            if look:
                protect = set(used)
                for e in [int(v) for v in self.host_pred[0].tolist()]:
                    key = (l + 1, e)
                    sid = self.where.get(key)
                    if sid is None:
                        sid = self._fill(key, protect, ahead=True)
                        self.stats["prefetch_issued"] += 1
                    protect.add(sid)
            table = self.tables[l]
            B._check(B.lib.dymoe_quantize_experts(ctx._h, table.data_ptr(), lay.bits.data_ptr(), lay.load.data_ptr(),
                                                  self.E, self.H, self.F, 64, B.LAYOUT_ROWMAJOR, st),
                     "dymoe_quantize_experts")
            B._check(B.lib.dymoe_moe_ffn_mixed(ctx._h, h.data_ptr(), lay.idx.data_ptr(), lay.gate.data_ptr(),
                                               lay.bits.data_ptr(), table.data_ptr(), 1, self.H, self.F, self.E,
                                               self.k, 64, B.OUT_F32, B.PATH_GEMV, lay.y.data_ptr(),
                                               lay.ws.data_ptr(), lay.ws_bytes, st), "dymoe_moe_ffn_mixed")
            nxt = self.h[(l + 1) % 2]
            B._check(B.lib.dymoe_residual_rmsnorm(ctx._h, h.data_ptr(), lay.y.data_ptr(), B.OUT_F32,
                                                  float(self.alpha), 1, self.H, nxt.data_ptr(), st),
                     "dymoe_residual_rmsnorm")
            done = torch.cuda.Event()
            done.record(cs)
            for sid in used:
                self.slots[sid].last_use = done
            h = nxt
        self.trace.append(step_trace)
        self.stats["steps"] += 1
        return h

    def close(self):
        torch.cuda.synchronize()
        for slot in self.slots:
            if slot.copy_event is not None:
                self.ctx.prefetch_release(slot.copy_event)
                slot.copy_event = None
