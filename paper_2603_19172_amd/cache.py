"""Mixed-precision expert cache (paper Sec. 4.4.2): host-side bookkeeping only.

Two managers with the same interface: `MixedPrecisionCache` below divides the
device memory into a fixed number of slots per format; `ByteBudgetCache` wraps
the library's dymoe_cache_*, which shares one byte budget between the formats.

The device memory set aside for experts is divided into slots of three sizes,
one pool per stored format (16, 8, 4 or 2 bits per weight); each pool is kept in
least-recently-used order.  The three rules of the paper:

  No Duplication        an expert is resident in at most one format;
  Precision Promotion   asked for a higher precision than the resident one:
                        a miss; the higher format is loaded and the lower
                        one dropped;
  Conservative Reuse    asked for a lower precision than the resident one:
                        a hit; the resident (higher) format is used.

`request` returns what the caller has to do (nothing, or copy the expert's
`load_bits` format into slot `slot`) and which precision the layer then runs
the expert at.  No GPU call is made here.
"""
import collections

FORMATS = (16, 8, 4, 2)


class Action:
    __slots__ = ("kind", "slot", "use_bits", "load_bits", "evicted", "dropped", "freed")

    def __init__(self, kind, slot, use_bits, load_bits=0, evicted=None, dropped=None, freed=()):
        self.kind = kind            # "hit", "miss" or "promote"
        self.slot = slot            # (format, index) holding the expert after the request
        self.use_bits = use_bits    # precision the expert is run at
        self.load_bits = load_bits  # format to copy into `slot` (0: nothing to copy)
        self.evicted = evicted      # key that lost `slot`, if any
        self.dropped = dropped      # (format, index) freed by a promotion, if any
        self.freed = tuple(freed)   # slots other than `slot` whose contents were given up and whose memory `slot` may overlap

    def __repr__(self):
        return "Action(%s, slot=%s, use=%d, load=%d, evicted=%s, dropped=%s)" % (
            self.kind, self.slot, self.use_bits, self.load_bits, self.evicted, self.dropped)


class MixedPrecisionCache:
    def __init__(self, slots):
        """slots: {16: n16, 8: n8, 4: n4, 2: n2} slot counts per format (missing: none)."""
        self.capacity = {b: int(slots.get(b, 0)) for b in FORMATS}
        # per format: slot index -> key (None when free), least recently used first
        self.pool = {b: collections.OrderedDict((i, None) for i in range(self.capacity[b])) for b in FORMATS}
        self.where = {}      # key -> (format, index)

    def resident(self, key):
        """(format, index) of the expert, or None."""
        return self.where.get(key)

    def covers(self, key, want_bits):
        """True when a request for `want_bits` would be a hit."""
        loc = self.where.get(key)
        return loc is not None and loc[0] >= want_bits

    def _take(self, fmt, protect):
        """A slot of pool `fmt`: a free one, else the least recently used one not in `protect`."""
        pool = self.pool[fmt]
        for i, k in pool.items():
            if k is None:
                return i, None
        for i, k in pool.items():
            if (fmt, i) not in protect:
                return i, k
        raise RuntimeError("no evictable %d-bit slot" % fmt)

    def request(self, key, want_bits, protect=()):
        if want_bits not in FORMATS:
            raise ValueError("want_bits must be one of %s" % (FORMATS,))
        if self.capacity[want_bits] == 0 and not self.covers(key, want_bits):
            raise ValueError("no %d-bit slots configured" % want_bits)
        loc = self.where.get(key)
        if loc is not None and loc[0] >= want_bits:          # Conservative Reuse (or an exact hit)
            self.pool[loc[0]].move_to_end(loc[1])
            return Action("hit", loc, loc[0])
        dropped = None
        if loc is not None:                                  # Precision Promotion: the lower format goes
            self.pool[loc[0]][loc[1]] = None
            self.pool[loc[0]].move_to_end(loc[1], last=False)
            del self.where[key]
            dropped = loc
        i, old = self._take(want_bits, protect)
        if old is not None:
            del self.where[old]
        self.pool[want_bits][i] = key
        self.pool[want_bits].move_to_end(i)
        self.where[key] = (want_bits, i)
        return Action("promote" if dropped else "miss", (want_bits, i), want_bits, want_bits, old, dropped)


class ByteBudgetCache:
    """The library's byte-budget cache (dymoe_cache_*) behind the interface of MixedPrecisionCache.
    A slot is named (format, byte offset into the caller's arena).  Keys may be any hashable values."""

    def __init__(self, budget_bytes, slot_bytes):
        """slot_bytes: {bits: bytes of one expert in that format}."""
        import ctypes as C
        from . import binding as B
        self._B, self._C = B, C
        self.formats = tuple(sorted(slot_bytes, reverse=True))
        fb = (C.c_int32 * len(self.formats))(*self.formats)
        sb = (C.c_size_t * len(self.formats))(*[int(slot_bytes[b]) for b in self.formats])
        h = C.c_void_p()
        B._check(B.lib.dymoe_cache_create(C.byref(h), int(budget_bytes), len(self.formats), C.cast(fb, C.c_void_p),
                                          C.cast(sb, C.c_void_p)), "dymoe_cache_create")
        self._h = h
        self.block_bytes = int(B.lib.dymoe_cache_block_bytes(h))
        self._id, self._key = {}, {}       # key <-> int64 id
        self.where = {}                    # key -> (format, offset), mirrored for inspection
        self._at = {}                      # slot -> key

    def close(self):
        if self._h is not None and self._B.lib is not None:
            self._B.lib.dymoe_cache_destroy(self._h)
        self._h = None

    __del__ = close

    def _ident(self, key):
        i = self._id.get(key)
        if i is None:
            i = len(self._id)
            self._id[key] = i
            self._key[i] = key
        return i

    def resident(self, key):
        return self.where.get(key)

    def covers(self, key, want_bits):
        loc = self.where.get(key)
        return loc is not None and loc[0] >= want_bits

    def bytes_resident(self):
        return int(self._B.lib.dymoe_cache_bytes_resident(self._h))

    def request(self, key, want_bits, protect=()):
        """protect: slots (format, offset) whose experts must stay."""
        C, B = self._C, self._B
        keep = [self._ident(self._at[s]) for s in protect if s in self._at]
        arr = (C.c_int64 * max(len(keep), 1))(*keep)
        act = B.CacheAction()
        rc = B.lib.dymoe_cache_request(self._h, self._ident(key), int(want_bits), C.cast(arr, C.c_void_p), len(keep),
                                       C.byref(act))
        if rc == B.ENOSPC:
            raise RuntimeError("no evictable room for a %d-bit expert" % want_bits)
        B._check(rc, "dymoe_cache_request")
        evicted = [self._key[act.evicted[i]] for i in range(act.n_evicted)]
        freed = []
        for k in evicted:
            freed.append(self.where.pop(k))
            self._at.pop(freed[-1], None)
        dropped = None
        if act.dropped_offset >= 0:
            dropped = self.where.pop(key)
            self._at.pop(dropped, None)
            freed.append(dropped)
        slot = (act.use_bits, int(act.offset))
        self.where[key] = slot
        self._at[slot] = key
        kind = ("hit", "miss", "promote")[act.kind]
        return Action(kind, slot, act.use_bits, act.load_bits, evicted if evicted else None, dropped,
                      [f for f in freed if f != slot])
