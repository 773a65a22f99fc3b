"""Mixed-precision expert cache (paper Sec. 4.4.2): host-side bookkeeping only.

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
    __slots__ = ("kind", "slot", "use_bits", "load_bits", "evicted", "dropped")

    def __init__(self, kind, slot, use_bits, load_bits=0, evicted=None, dropped=None):
        self.kind = kind            # "hit", "miss" or "promote"
        self.slot = slot            # (format, index) holding the expert after the request
        self.use_bits = use_bits    # precision the expert is run at
        self.load_bits = load_bits  # format to copy into `slot` (0: nothing to copy)
        self.evicted = evicted      # key that lost `slot`, if any
        self.dropped = dropped      # (format, index) freed by a promotion, if any

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
