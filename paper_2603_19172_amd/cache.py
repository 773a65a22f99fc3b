"""Mixed-precision expert cache (paper Sec. 4.4.2): thin wrappers of the library's host-side
bookkeeping (dymoe_cache_*; no GPU call is made there or here).

The three rules of the paper:

  No Duplication        an expert is resident in at most one format;
  Precision Promotion   asked for a higher precision than the resident one:
                        a miss; the higher format is loaded and the lower
                        one dropped;
  Conservative Reuse    asked for a lower precision than the resident one:
                        a hit; the resident (higher) format is used.

Two ways of dividing the device memory set aside for experts, one interface:
`MixedPrecisionCache` gives every stored format (16, 8, 4 or 2 bits per weight) a fixed
number of slots (dymoe_cache_create_pools), `ByteBudgetCache` shares one byte budget
between the formats (dymoe_cache_create).  Either keeps least-recently-used order, or, told the length of a cyclic
schedule (`set_cyclic(L)`, requests then carry `position=`), evicts what the schedule comes back to last.

`request` returns what the caller has to do (nothing, or copy the expert's
`load_bits` format into slot `slot`) and which precision the layer then runs
the expert at.  A request that cannot be served raises and leaves the cache as it was.
"""
import ctypes as C

FORMATS = (16, 8, 4, 2)


class Action:
    __slots__ = ("kind", "slot", "use_bits", "load_bits", "evicted", "dropped", "freed")

    def __init__(self, kind, slot, use_bits, load_bits=0, evicted=None, dropped=None, freed=()):
        self.kind = kind            # "hit", "miss" or "promote"
        self.slot = slot            # name of the slot holding the expert after the request
        self.use_bits = use_bits    # precision the expert is run at
        self.load_bits = load_bits  # format to copy into `slot` (0: nothing to copy)
        self.evicted = evicted      # what lost its slot, if anything (one key for fixed pools, a list for a budget)
        self.dropped = dropped      # slot freed by a promotion, if any
        self.freed = tuple(freed)   # slots other than `slot` whose contents were given up and whose memory `slot` may overlap

    def __repr__(self):
        return "Action(%s, slot=%s, use=%d, load=%d, evicted=%s, dropped=%s)" % (
            self.kind, self.slot, self.use_bits, self.load_bits, self.evicted, self.dropped)


class _NativeCache:
    """What the two managers share: keys of any hashable type mapped to the library's int64 ids, the mirror of
    who is where, and the request itself.  Subclasses create the handle and name the slots."""

    def _init(self, handle):
        from . import binding as B
        self._B = B
        self._h = handle
        self._id, self._key = {}, {}       # key <-> int64 id
        self.where = {}                    # key -> slot name, mirrored for inspection
        self._at = {}                      # slot name -> key

    def close(self):
        if getattr(self, "_h", None) is not None and self._B.lib is not None:
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

    def _name(self, bits, offset):
        return (bits, int(offset))

    def resident(self, key):
        """Name of the slot the expert is in, or None."""
        return self.where.get(key)

    def covers(self, key, want_bits):
        """True when a request for `want_bits` would be a hit."""
        loc = self.where.get(key)
        return loc is not None and loc[0] >= want_bits

    def bytes_resident(self):
        return int(self._B.lib.dymoe_cache_bytes_resident(self._h))

    def set_cyclic(self, n_positions):
        """Requests walk a cyclic schedule of n_positions positions (0: back to least-recently-used order)."""
        self._B._check(self._B.lib.dymoe_cache_set_cyclic(self._h, int(n_positions)), "dymoe_cache_set_cyclic")
        self._cyclic = int(n_positions)

    def _request(self, key, want_bits, protect, position=None):
        """protect: slot names whose experts must stay."""
        B = self._B
        keep = [self._ident(self._at[s]) for s in protect if s in self._at]
        arr = (C.c_int64 * max(len(keep), 1))(*keep)
        act = B.CacheAction()
        if position is None:
            rc = B.lib.dymoe_cache_request(self._h, self._ident(key), int(want_bits), C.cast(arr, C.c_void_p), len(keep),
                                           C.byref(act))
        else:
            rc = B.lib.dymoe_cache_request_at(self._h, self._ident(key), int(want_bits), C.cast(arr, C.c_void_p),
                                              len(keep), int(position), C.byref(act))
        if rc == B.ENOSPC:
            raise RuntimeError("no evictable room for a %d-bit expert" % want_bits)
        if rc == B.EINVAL:
            raise ValueError("no %d-bit slots configured, or a position outside the cyclic schedule" % want_bits)
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
        slot = self._name(act.use_bits, act.offset)
        self.where[key] = slot
        self._at[slot] = key
        kind = ("hit", "miss", "promote")[act.kind]
        return kind, slot, act, evicted, dropped, [f for f in freed if f != slot]


class MixedPrecisionCache(_NativeCache):
    """A fixed number of slots per format.  A slot is named (format, index)."""

    def __init__(self, slots):
        """slots: {16: n16, 8: n8, 4: n4, 2: n2} slot counts per format (missing or 0: none)."""
        from . import binding as B
        self.capacity = {b: int(slots.get(b, 0)) for b in FORMATS}
        fmts = [b for b in FORMATS if self.capacity[b] > 0]
        if not fmts:
            raise ValueError("no slots configured")
        # only the order of the slots matters here: the caller owns the memory, one buffer per slot
        self._unit = 256
        fb = (C.c_int32 * len(fmts))(*fmts)
        sb = (C.c_size_t * len(fmts))(*[self._unit] * len(fmts))
        nb = (C.c_int32 * len(fmts))(*[self.capacity[b] for b in fmts])
        h = C.c_void_p()
        B._check(B.lib.dymoe_cache_create_pools(C.byref(h), len(fmts), C.cast(fb, C.c_void_p), C.cast(sb, C.c_void_p),
                                                C.cast(nb, C.c_void_p)), "dymoe_cache_create_pools")
        self._init(h)
        self._base, pos = {}, 0
        for b in fmts:
            self._base[b] = pos
            pos += self.capacity[b] * self._unit

    def _name(self, bits, offset):
        return (bits, (int(offset) - self._base[bits]) // self._unit)

    def held(self, bits):
        """Keys resident in the pool of this format."""
        return [k for k, (b, _) in self.where.items() if b == bits]

    def request(self, key, want_bits, protect=(), position=None):
        if want_bits not in FORMATS:
            raise ValueError("want_bits must be one of %s" % (FORMATS,))
        kind, slot, act, evicted, dropped, freed = self._request(key, want_bits, protect, position)
        return Action(kind, slot, act.use_bits, act.load_bits, evicted[0] if evicted else None, dropped)


class ByteBudgetCache(_NativeCache):
    """One byte budget shared by the formats.  A slot is named (format, byte offset into the caller's arena)."""

    def __init__(self, budget_bytes, slot_bytes):
        """slot_bytes: {bits: bytes of one expert in that format}."""
        from . import binding as B
        self.formats = tuple(sorted(slot_bytes, reverse=True))
        fb = (C.c_int32 * len(self.formats))(*self.formats)
        sb = (C.c_size_t * len(self.formats))(*[int(slot_bytes[b]) for b in self.formats])
        h = C.c_void_p()
        B._check(B.lib.dymoe_cache_create(C.byref(h), int(budget_bytes), len(self.formats), C.cast(fb, C.c_void_p),
                                          C.cast(sb, C.c_void_p)), "dymoe_cache_create")
        self._init(h)
        self.block_bytes = int(B.lib.dymoe_cache_block_bytes(h))

    def request(self, key, want_bits, protect=(), position=None):
        kind, slot, act, evicted, dropped, freed = self._request(key, want_bits, protect, position)
        return Action(kind, slot, act.use_bits, act.load_bits, evicted if evicted else None, dropped, freed)
