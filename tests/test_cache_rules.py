"""Table-driven CPU tests of the mixed-precision expert cache (paper Sec. 4.4.2):
No Duplication, Precision Promotion, Conservative Reuse, and least-recently-used
eviction, over a fixed partition (dymoe_cache_create_pools) and over one byte budget
(dymoe_cache_create).  Host logic of the library only; no GPU."""
import pytest

from paper_2603_19172_amd.cache import MixedPrecisionCache


def run(cache, script):
    """script: list of (key, want_bits, expected kind, expected use_bits, expected evicted key)."""
    for step, (key, want, kind, use, evicted) in enumerate(script):
        a = cache.request(key, want)
        assert (a.kind, a.use_bits, a.evicted) == (kind, use, evicted), (step, key, want, a)
        assert a.load_bits == (0 if kind == "hit" else want)
        # No Duplication: after any request every expert is resident exactly once
        locs = list(cache.where.values())
        assert len(locs) == len(set(locs))
        if hasattr(cache, "capacity"):        # fixed pools: nobody sits outside its pool
            assert all(0 <= i < cache.capacity[b] for b, i in locs)


def test_exact_hits_and_lru_eviction_within_a_pool():
    c = MixedPrecisionCache({16: 0, 4: 2, 2: 0})
    run(c, [
        ("a", 4, "miss", 4, None),
        ("b", 4, "miss", 4, None),
        ("a", 4, "hit", 4, None),       # a is now the most recently used
        ("c", 4, "miss", 4, "b"),       # so b goes
        ("b", 4, "miss", 4, "a"),
    ])


def test_conservative_reuse_serves_a_lower_request_from_the_higher_format():
    c = MixedPrecisionCache({16: 1, 4: 1, 2: 1})
    run(c, [
        ("a", 16, "miss", 16, None),
        ("a", 4, "hit", 16, None),      # asked for int4, bf16 resident: used as it is, nothing moves
        ("a", 2, "hit", 16, None),
        ("b", 4, "miss", 4, None),
        ("b", 2, "hit", 4, None),
    ])
    assert c.resident("a") == (16, 0) and c.resident("b") == (4, 0)
    assert c.held(2) == []                                  # the int2 pool was never touched


def test_precision_promotion_is_a_miss_that_drops_the_lower_format():
    c = MixedPrecisionCache({16: 1, 4: 2, 2: 2})
    run(c, [
        ("a", 2, "miss", 2, None),
        ("b", 2, "miss", 2, None),
        ("a", 4, "promote", 4, None),   # int2 of a dropped, int4 loaded
        ("c", 2, "miss", 2, None),      # takes the slot a left, nobody is evicted
        ("a", 2, "hit", 4, None),
        ("a", 16, "promote", 16, None),
        ("b", 16, "promote", 16, "a"),  # one bf16 slot only: a leaves the cache altogether
    ])
    assert c.resident("a") is None
    assert c.resident("b") == (16, 0) and c.resident("c") is not None


def test_protected_slots_are_not_evicted():
    c = MixedPrecisionCache({4: 2})
    a = c.request("a", 4)
    b = c.request("b", 4)
    x = c.request("c", 4, protect={a.slot})
    assert x.evicted == "b" and x.slot == b.slot
    with pytest.raises(RuntimeError):
        c.request("d", 4, protect={a.slot, x.slot})
    with pytest.raises(ValueError):
        c.request("e", 16)               # no bf16 slots configured
    with pytest.raises(ValueError):
        c.request("e", 8)


def test_a_promotion_that_finds_no_room_leaves_the_cache_as_it_was():
    """One slot per format; A resident at 2 bits, B protected in the only int4 slot: asking for A at 4 bits cannot be
    served, and A must still be resident at 2 bits afterwards (both managers)."""
    c = MixedPrecisionCache({4: 1, 2: 1})
    c.request("A", 2)
    b = c.request("B", 4)
    with pytest.raises(RuntimeError):
        c.request("A", 4, protect={b.slot})
    assert c.resident("A") == (2, 0) and c.resident("B") == (4, 0) and c.covers("A", 2)
    assert c.request("A", 2).kind == "hit"
    from paper_2603_19172_amd.cache import ByteBudgetCache
    d = ByteBudgetCache(2 * 1024, {4: 1024, 2: 512})        # two blocks of one int4 or two int2 experts
    d.request("A", 2)
    b = d.request("B", 4)
    x = d.request("X", 2)                                   # shares A's block
    with pytest.raises(RuntimeError):
        d.request("A", 4, protect={b.slot, x.slot})         # B's block is protected, A's own block holds X
    assert d.resident("A") == (2, 0) and d.request("A", 2).kind == "hit" and d.resident("X") is not None


def test_covers_predicts_the_outcome_of_a_request():
    c = MixedPrecisionCache({16: 1, 4: 1, 2: 1})
    c.request("a", 4)
    assert c.covers("a", 4) and c.covers("a", 2) and not c.covers("a", 16) and not c.covers("b", 2)


def test_four_formats_form_one_ladder():
    c = MixedPrecisionCache({16: 1, 8: 1, 4: 1, 2: 1})
    run(c, [
        ("a", 4, "miss", 4, None),
        ("a", 8, "promote", 8, None),   # int4 dropped, int8 loaded
        ("a", 4, "hit", 8, None),       # Conservative Reuse from the 8-bit copy
        ("b", 8, "miss", 8, "a"),       # one 8-bit slot: a leaves
        ("a", 2, "miss", 2, None),
        ("a", 16, "promote", 16, None),
        ("a", 8, "hit", 16, None),
    ])
    assert c.resident("b") == (8, 0) and c.resident("a") == (16, 0)


# ------------------------------------------------------------------ one byte budget (dymoe_cache_*)

from paper_2603_19172_amd.cache import ByteBudgetCache

MB = 1 << 20
SIZES = {16: 352 * MB, 4: 99 * MB, 2: 55 * MB}      # a Mixtral expert: 1, 3 and 6 slots per 352 MB block


def _consistent(c):
    """No Duplication, and no two experts in one slot."""
    locs = list(c.where.values())
    assert len(locs) == len(set(locs))
    assert c.bytes_resident() == sum(-(-SIZES[b] // 256) * 256 for b, _ in locs)
    for (b, off) in locs:
        assert off % 256 == 0 and off + SIZES[b] <= c.n_blocks * c.block_bytes


def _cache(n_blocks):
    c = ByteBudgetCache(n_blocks * 352 * MB + 1000, SIZES)
    c.n_blocks = n_blocks
    assert c.block_bytes == 352 * MB
    return c


def test_budget_cache_fills_blocks_format_by_format():
    c = _cache(2)
    a = c.request("a", 16)
    assert (a.kind, a.slot, a.load_bits, a.evicted) == ("miss", (16, 0), 16, None)
    offs = [c.request("q%d" % i, 4).slot[1] for i in range(3)]
    assert offs == [352 * MB + i * 99 * MB for i in range(3)]         # three int4 experts share the second block
    _consistent(c)
    # both blocks are taken: a fourth int4 expert evicts the least recently used int4 one, not the newer bf16 block...
    c.request("a", 16)
    x = c.request("q3", 4)
    assert x.kind == "miss" and x.evicted == ["q0"] and x.slot == (4, 352 * MB)
    # ...and an int2 expert takes over the least recently used block as a whole (here the bf16 one is older)
    c.request("q1", 4); c.request("q2", 4); c.request("q3", 4)
    y = c.request("t0", 2)
    assert y.evicted == ["a"] and y.slot == (2, 0)
    assert [c.request("t%d" % i, 2).slot[1] for i in range(1, 6)] == [i * 55 * MB for i in range(1, 6)]
    _consistent(c)
    # a bf16 expert needs a whole block: the int4 block is the older one now and goes with all three residents
    z = c.request("b", 16)
    assert sorted(z.evicted) == ["q1", "q2", "q3"] and z.slot == (16, 352 * MB)
    _consistent(c)


def test_budget_cache_rules_and_protection():
    c = _cache(2)
    run(c, [
        ("a", 4, "miss", 4, None),
        ("a", 2, "hit", 4, None),          # Conservative Reuse
        ("a", 16, "promote", 16, None),    # Precision Promotion into the free block; the int4 copy is dropped
        ("a", 4, "hit", 16, None),
    ])
    assert c.resident("a") == (16, 352 * MB) and len(c.where) == 1
    r = c.request("b", 2)
    assert r.slot == (2, 0)                # the block the dropped int4 copy left
    # protected experts stay: with both blocks protected nothing can make room for bf16
    with pytest.raises(RuntimeError):
        c.request("c", 16, protect=[c.resident("a"), c.resident("b")])
    assert c.resident("a") == (16, 352 * MB) and c.resident("b") == (2, 0)       # unchanged
    r = c.request("c", 16, protect=[c.resident("a")])
    assert r.evicted == ["b"] and r.slot == (16, 0)
    # promotion when the only room is the block the lower format itself sits in
    d = _cache(1)
    d.request("x", 2)
    p = d.request("x", 16)
    assert (p.kind, p.slot, p.dropped, p.evicted) == ("promote", (16, 0), (2, 0), None)
    _consistent(d)


def test_budget_cache_random_walk_keeps_its_invariants():
    import random
    rnd = random.Random(7)
    c = _cache(3)
    for step in range(3000):
        key = rnd.randrange(40)
        want = rnd.choice((16, 4, 4, 2, 2, 2))
        before = c.resident(key)
        a = c.request(key, want)
        if before is not None and before[0] >= want:
            assert a.kind == "hit" and a.slot == before and a.use_bits == before[0] and a.load_bits == 0
        else:
            assert a.kind == ("promote" if before is not None else "miss")
            assert a.use_bits == want and a.load_bits == want and a.slot[0] == want
            assert (a.dropped == before) if before is not None else a.dropped is None
        assert c.resident(key) == a.slot
        for k in a.evicted or ():
            assert c.resident(k) is None and k != key
        _consistent(c)
    assert c.bytes_resident() <= 3 * 352 * MB


def test_budget_cache_rejects_bad_arguments():
    from paper_2603_19172_amd import binding as B
    import ctypes as C
    h = C.c_void_p()
    fb = (C.c_int32 * 2)(16, 4)
    sb = (C.c_size_t * 2)(1000, 100)
    cr = B.lib.dymoe_cache_create
    assert cr(C.byref(h), 999, 2, C.cast(fb, C.c_void_p), C.cast(sb, C.c_void_p)) == B.ENOSPC
    assert cr(C.byref(h), 10000, 0, C.cast(fb, C.c_void_p), C.cast(sb, C.c_void_p)) == B.EINVAL
    assert cr(C.byref(h), 10000, 2, C.cast((C.c_int32 * 2)(16, 16), C.c_void_p), C.cast(sb, C.c_void_p)) == B.EINVAL
    assert cr(C.byref(h), 10000, 2, C.cast((C.c_int32 * 2)(16, 3), C.c_void_p), C.cast(sb, C.c_void_p)) == B.EINVAL
    assert cr(C.byref(h), 1 << 20, 2, C.cast(fb, C.c_void_p), C.cast((C.c_size_t * 2)(65536, 256), C.c_void_p)) == B.ENOTSUP
    assert cr(C.byref(h), 10000, 2, C.cast(fb, C.c_void_p), C.cast(sb, C.c_void_p)) == B.OK
    act = B.CacheAction()
    assert B.lib.dymoe_cache_request(h, 1, 8, None, 0, C.byref(act)) == B.EINVAL       # not a configured format
    assert B.lib.dymoe_cache_request(h, 1, 4, None, 1, C.byref(act)) == B.EINVAL
    assert B.lib.dymoe_cache_request(h, 1, 4, None, 0, C.byref(act)) == B.OK and act.kind == B.CACHE_MISS
    assert B.lib.dymoe_cache_lookup(h, 1, None, None) == 1 and B.lib.dymoe_cache_lookup(h, 2, None, None) == 0
    B.lib.dymoe_cache_destroy(h)


# ------------------------------------------------------------------ eviction order under a cyclic schedule

def _cycle_misses(cache, n_pos, per_pos, cycles, position_arg):
    """Every position asks for its `per_pos` keys in every cycle; returns the misses of the last cycle."""
    misses = 0
    for c in range(cycles):
        misses = 0
        for pos in range(n_pos):
            for j in range(per_pos):
                a = cache.request((pos, j), 4, position=pos if position_arg else None)
                misses += a.kind != "hit"
    return misses


def test_cyclic_schedule_keeps_what_comes_up_next_where_lru_keeps_nothing():
    """Four positions visited in a circle, one key each, three slots: least-recently-used order evicts every key
    just before its turn (four misses per cycle, for ever); told the schedule, the cache evicts the key whose
    position comes up last and misses once per cycle, which is the least any policy can (Belady)."""
    lru = MixedPrecisionCache({4: 3})
    assert _cycle_misses(lru, 4, 1, 6, position_arg=False) == 4
    cyc = MixedPrecisionCache({4: 3})
    cyc.set_cyclic(4)
    assert _cycle_misses(cyc, 4, 1, 6, position_arg=True) == 1
    # the same under one byte budget
    b = ByteBudgetCache(3 * 1024, {4: 1024})
    b.set_cyclic(4)
    assert _cycle_misses(b, 4, 1, 6, position_arg=True) == 1
    b.set_cyclic(0)                                     # back to least recently used
    assert _cycle_misses(b, 4, 1, 6, position_arg=False) == 4


def test_cyclic_order_step_by_step_and_its_arguments():
    c = MixedPrecisionCache({4: 3})
    c.set_cyclic(4)
    seq = [(("k0", 0), "miss", None), (("k1", 1), "miss", None), (("k2", 2), "miss", None),
           # at position 3 the residents come up in 1 (k0), 2 (k1) and 3 (k2) positions: k2, used last, goes first
           (("k3", 3), "miss", "k2"),
           (("k0", 0), "hit", None), (("k1", 1), "hit", None),
           # at position 2: k3 comes up next, k0 in 2, k1 in 3
           (("k2", 2), "miss", "k1"),
           (("k3", 3), "hit", None), (("k0", 0), "hit", None),
           # a key that is not asked for at its own position is a whole cycle away: at position 1, k0 (position 0) is 3
           # away, k2 1 away, k3 2 away, so k0 goes; a second key at position 1 then finds ... k1 itself protected
           (("k1", 1), "miss", "k0")]
    for (key, pos), kind, evicted in seq:
        a = c.request(key, 4, position=pos)
        assert (a.kind, a.evicted) == (kind, evicted), (key, pos, a)
    a = c.request("other", 4, protect=[c.resident("k1")], position=1)     # k2 comes up next, k3 after it: k3 goes
    assert a.evicted == "k3"
    with pytest.raises(ValueError):
        c.request("k9", 4, position=4)                  # outside the schedule
    with pytest.raises(ValueError):
        c.request("k9", 4, position=-1)
    from paper_2603_19172_amd import binding as B
    assert B.lib.dymoe_cache_set_cyclic(None, 4) == B.EINVAL and B.lib.dymoe_cache_set_cyclic(c._h, -1) == B.EINVAL


def test_cyclic_order_random_walk_keeps_the_rules():
    """The three rules, protection and consistency do not depend on the eviction order."""
    import random
    rnd = random.Random(11)
    c = _cache(3)
    c.set_cyclic(5)
    for step in range(3000):
        pos = step % 5
        key = (pos, rnd.randrange(8))
        want = rnd.choice((16, 4, 4, 2, 2, 2))
        before = c.resident(key)
        a = c.request(key, want, position=pos)
        if before is not None and before[0] >= want:
            assert a.kind == "hit" and a.slot == before and a.load_bits == 0
        else:
            assert a.kind == ("promote" if before is not None else "miss") and a.use_bits == want
        assert c.resident(key) == a.slot
        for k in a.evicted or ():
            assert c.resident(k) is None and k != key
        _consistent(c)
