"""Table-driven CPU tests of the mixed-precision expert cache (paper Sec. 4.4.2):
No Duplication, Precision Promotion, Conservative Reuse, and least-recently-used
eviction inside each format's pool.  Host logic only; no GPU."""
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
        held = [(b, i) for b in cache.pool for i, k in cache.pool[b].items() if k is not None]
        assert sorted(held) == sorted(locs)


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
    assert all(k is None for k in c.pool[2].values())       # the int2 pool was never touched


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
