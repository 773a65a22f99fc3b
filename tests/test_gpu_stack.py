"""GPU tests of the host-resident expert stack: the side-stream copy calls, the
residual + normalisation glue kernel, and a small stack of layers decoded with
and without look-ahead prefetch against the oracle's composition."""
import numpy as np
import pytest
import torch

from oracle import dymoe_oracle as O
from paper_2603_19172_amd import binding as B
from paper_2603_19172_amd import synth
from paper_2603_19172_amd.stack import DecodeStack, HostExpertPool, PrefillStack, ResidentDecodeStack
from gpu_helpers import DEV, bits_of, margin_ok, to_bf16

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = B.Context(0)
    yield c
    c.close()


def test_prefetch_copy_is_ordered_before_the_compute_stream(ctx):
    n = 8 << 20
    g = torch.Generator().manual_seed(11)
    host = torch.randint(0, 256, (n,), dtype=torch.uint8, generator=g).pin_memory()
    dev = torch.zeros((n,), dtype=torch.uint8, device=DEV)
    out = torch.zeros_like(dev)
    side = torch.cuda.Stream()
    cs = torch.cuda.current_stream()
    ev = ctx.prefetch_submit(host.data_ptr(), dev.data_ptr(), n, side.cuda_stream)
    ctx.prefetch_wait(ev, cs.cuda_stream)
    ctx.stream_copy(dev, out)            # on the compute stream: must see the copied bytes
    torch.cuda.synchronize()
    assert ctx.prefetch_done(ev)
    ctx.prefetch_release(ev)
    assert torch.equal(out.cpu(), host)
    # an empty copy still gives an event that completes
    ev = ctx.prefetch_submit(None, None, 0, side.cuda_stream)
    torch.cuda.synchronize()
    assert ctx.prefetch_done(ev)
    ctx.prefetch_release(ev)


@pytest.mark.parametrize("T,H,alpha", [(1, 256, 1.0), (5, 4096, 0.125), (3, 264, 0.5), (2, 250, 0.5), (3, 6152, 0.25)])
def test_residual_rmsnorm_against_the_oracle(ctx, T, H, alpha):
    rng = np.random.default_rng(3)
    h = synth.f32_to_bf16_bits(rng.standard_normal((T, H)).astype(np.float32))
    y = (2.0 * rng.standard_normal((T, H))).astype(np.float32)
    h[T - 1] = 0
    y[T - 1] = 0.0                                   # a zero row stays zero
    ref = O.residual_rmsnorm(h, y.astype(np.float64), alpha)
    for yt in (torch.from_numpy(y).to(DEV), to_bf16(synth.f32_to_bf16_bits(y))):
        yref = ref if yt.dtype == torch.float32 else O.residual_rmsnorm(
            h, synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(y)).astype(np.float64), alpha)
        out = ctx.residual_rmsnorm(to_bf16(h), yt, alpha)
        torch.cuda.synchronize()
        got = bits_of(out).astype(np.int64)
        # fp32 arithmetic on the device, fp64 in the oracle: at most one bf16 step apart
        assert np.abs(got - yref.astype(np.int64)).max() <= 1
        assert (got[T - 1] == 0).all()


TIERS3 = ((1, 3, 4), (16, 4, 2))
TIERS4 = ((1, 2, 2, 3), (16, 8, 4, 2))


def _small_stack(ctx, L, slots, prefetch, seed0, transfer="bf16", pool=None, tiers=TIERS3, budget_bytes=None,
                 eviction="lru"):
    H, F, E, k = 256, 512, 8, 2
    cfgs = [synth.scaled(synth.CONFIGS["tiny"], T=1, phase="decode", config_id=seed0 + l) for l in range(L)]
    routers_np = [synth.router(c)[0] for c in cfgs]
    n_pool = 12
    pool_cfg = synth.scaled(synth.CONFIGS["tiny"], config_id=seed0 + 50)
    mats = {i: synth.expert_weights(pool_cfg, i) for i in range(n_pool)}
    if pool is None:
        pool = HostExpertPool(H, F, E, n_pool, lambda i: mats[i])
        if transfer == "assigned":
            pool.add_quantised(ctx, DEV, formats=[b for b in tiers[1] if b != 16])
    floor = [4] + [0] * (L - 2) + [4]
    stack = DecodeStack(ctx, H, F, E, k, [to_bf16(r) for r in routers_np], pool, slots, tiers[0], tiers[1],
                        floor_bits=floor, prefetch=prefetch, transfer=transfer, alpha=0.25, device=DEV,
                        budget_bytes=budget_bytes, eviction=eviction)
    expert_matrices = lambda l, e: mats[pool.entry(l, e)]
    return stack, routers_np, expert_matrices, floor, cfgs[0]


def _uses(st):
    return st.get("miss", 0) + st.get("promote", 0) + st.get("hit_resident", 0) + st.get("hit_prefetched", 0)


def _check_against_oracle(outs, trace, routers_np, expert_matrices, floor, tiers=TIERS3):
    checked = 0
    for s, (x, h_dev) in enumerate(outs):
        run_bits = [dict(zip(ex, used)) for (ex, _, used) in trace[s]]
        ref_h, log, _ = O.decode_stack(x, routers_np, expert_matrices, 2, tiers[0], tiers[1], floor, 0.25,
                                       run_bits=run_bits)
        # decisions are compared layer by layer up to the first near tie of the oracle's logits (from there on the
        # two sides may legitimately part); the hidden state only when no layer had one
        clear = 0
        for l, (idx, bts, lg, _) in enumerate(log):
            if not margin_ok(lg, 2).all():
                break
            assert trace[s][l][0] == tuple(int(v) for v in idx[0])
            assert trace[s][l][1] == tuple(int(v) for v in bts)            # the assignment itself
            clear += 1
        if clear < len(log):
            continue
        checked += 1
        got = synth.bf16_bits_to_f32(bits_of(h_dev)).astype(np.float64)
        want = synth.bf16_bits_to_f32(ref_h).astype(np.float64)
        # unit-RMS rows; the FFN tolerance (2e-2 of a row's RMS, scaled by alpha) accumulates over the layers
        assert np.abs(got - want).max() <= 2e-2
    # the seeded inputs are fixed: near ties (a gap under 1e-4 somewhere in L layers x top-3 logits) may take out a
    # third of a run's steps at most
    assert checked >= max(1, (2 * len(outs)) // 3), (checked, len(outs))


def test_stack_decode_matches_the_oracle_and_prefetch_changes_nothing(ctx):
    L, steps = 4, 3
    outs, traces, stats = {}, {}, {}
    for prefetch in (False, True):
        stack, routers_np, expert_matrices, floor, cfg0 = _small_stack(ctx, L, 4, prefetch, 300)
        hs = []
        for s in range(steps):
            x, _ = synth.activations(synth.scaled(cfg0, config_id=400 + s))
            hs.append((x, stack.step(to_bf16(x)).clone()))
        stack.close()
        outs[prefetch], traces[prefetch], stats[prefetch] = hs, stack.trace, dict(stack.stats)
    # look-ahead copies change when the weights arrive, never what is computed
    for (x0, a), (x1, b) in zip(outs[False], outs[True]):
        assert torch.equal(a, b)
    assert traces[False] == traces[True]
    for st in stats.values():
        assert _uses(st) == L * 2 * steps
    assert stats[False].get("hit_prefetched", 0) == 0 and stats[False].get("prefetch_issued", 0) == 0
    assert stats[True]["prefetch_issued"] > 0
    assert stats[True]["miss"] <= stats[False]["miss"]
    _check_against_oracle(outs[True], traces[True], routers_np, expert_matrices, floor)


def test_stack_lookahead_by_the_expected_value_rule_changes_nothing_but_the_copies(ctx):
    """lookahead="expected": no speculative copy before a layer's compute time has been measured (two steps), then
    copies whose expected gain covers their expected cost; the hidden states are those of the run without look-ahead."""
    L, steps = 4, 6
    outs, stats = {}, {}
    for mode in ("off", "expected"):
        H, F, E, k = 256, 512, 8, 2
        stack, routers_np, expert_matrices, floor, cfg0 = _small_stack(ctx, L, 6, mode != "off", 2100)
        stack.lookahead = "expected"
        hs = []
        for s in range(steps):
            x, _ = synth.activations(synth.scaled(cfg0, config_id=2200 + s))
            hs.append(stack.step(to_bf16(x)).clone())
        stack.close()
        outs[mode], stats[mode] = hs, dict(stack.stats)
        if mode == "expected":
            assert stack.layer_ms is not None and stack.layer_ms > 0 and stack.link_gbps > 0
            assert 0.0 < stack._pred_right / stack._pred_seen <= 1.0
    for a, b in zip(outs["off"], outs["expected"]):
        assert torch.equal(a, b)
    st = stats["expected"]
    assert st.get("prefetch_declined", 0) > 0                       # the first two steps at least
    assert st.get("prefetch_issued", 0) + st.get("prefetch_declined", 0) > 0
    assert _uses(st) == L * 2 * steps


def test_stack_eviction_by_the_layer_schedule_changes_the_copies_not_the_results(ctx):
    """eviction="cyclic": the cache is told that the layers come round in order and evicts the expert whose layer
    comes up last.  With bf16 travelling, what is run does not depend on what is resident, so every hidden state and
    decision is what the least-recently-used order gives; with fewer slots than a step's experts LRU order never hits,
    the schedule order does."""
    L, steps = 4, 10
    outs, stats, traces = {}, {}, {}
    for ev in ("lru", "cyclic"):
        stack, routers_np, expert_matrices, floor, cfg0 = _small_stack(ctx, L, 5, False, 2600, eviction=ev)
        hs = []
        for s in range(steps):
            x, _ = synth.activations(synth.scaled(cfg0, config_id=2700 + s % 3))     # three tokens in turn: some reuse
            hs.append(stack.step(to_bf16(x)).clone())
        stack.close()
        outs[ev], stats[ev], traces[ev] = hs, dict(stack.stats), list(stack.trace)
    assert traces["lru"] == traces["cyclic"]
    for a, b in zip(outs["lru"], outs["cyclic"]):
        assert torch.equal(a, b)
    assert _uses(stats["lru"]) == _uses(stats["cyclic"]) == L * 2 * steps
    # 5 slots, 8 expert uses per step
    assert stats["lru"].get("hit_resident", 0) == 0 and stats["cyclic"].get("hit_resident", 0) > 0
    assert stats["cyclic"]["bytes_copied"] < stats["lru"]["bytes_copied"]


def test_stack_eviction_by_the_layer_schedule_under_one_budget_keeps_the_cache_rules(ctx):
    """The same order with the assigned formats under one byte budget: what is run may differ from the LRU run (an
    expert found resident at a higher precision is run at it), so the check is the oracle told what was run."""
    L, steps = 4, 6
    budget = 5 * (6 * 256 * 512 + 400 * 1024)           # five blocks of the bf16 size: evictions all the time
    stack, routers_np, expert_matrices, floor, cfg0 = _small_stack(ctx, L, None, False, 2800, transfer="assigned",
                                                                   budget_bytes=budget, eviction="cyclic")
    outs = []
    for s in range(steps):
        x, _ = synth.activations(synth.scaled(cfg0, config_id=2900 + s % 3))
        outs.append((x, stack.step(to_bf16(x)).clone()))
    stack.close()
    assert _uses(stack.stats) == L * 2 * steps
    for step in stack.trace:
        for (ex, assigned, used) in step:
            assert all(u >= a for a, u in zip(assigned, used))      # never below the assigned precision
    _check_against_oracle(outs, stack.trace, routers_np, expert_matrices, floor)


def test_stack_with_room_for_everything_copies_each_expert_once(ctx):
    L, steps = 3, 4
    stack, _, _, _, cfg0 = _small_stack(ctx, L, 3 * 8, True, 500)
    for s in range(steps):
        x, _ = synth.activations(synth.scaled(cfg0, config_id=600 + s))
        stack.step(to_bf16(x))
    stack.close()
    st = stack.stats
    copies = st["bytes_copied"] // stack.pool.nbytes[16]
    assert copies == len(stack.cache.where) <= L * 8          # nothing was ever evicted
    assert st["miss"] + st.get("prefetch_issued", 0) == copies


def test_stack_moving_the_assigned_format_follows_the_cache_rules(ctx):
    """transfer="assigned": the int4 / int2 / bf16 format the assignment asks for travels; an expert
    resident at a higher precision is run at that precision (Conservative Reuse), which the
    oracle is told through run_bits; everything else is the oracle's own chain."""
    L, steps = 4, 6
    slots = {16: 4, 4: 4, 2: 4}
    stack, routers_np, expert_matrices, floor, cfg0 = _small_stack(ctx, L, slots, True, 700, transfer="assigned")
    outs = []
    for s in range(steps):
        x, _ = synth.activations(synth.scaled(cfg0, config_id=800 + (s % 3)))     # tokens come back: reuse happens
        outs.append((x, stack.step(to_bf16(x)).clone()))
    stack.close()
    st = stack.stats
    assert _uses(st) == L * 2 * steps
    # bytes on the link: only the formats asked for, never more than bf16 for everything
    moved = sum(st.get("copies_%d" % b, 0) * stack.pool.nbytes[b] for b in (16, 4, 2))
    assert moved == st["bytes_copied"]
    assert st["copies_4"] + st["copies_2"] > 0
    for step in stack.trace:
        for (ex, assigned, used) in step:
            assert all(u >= a for a, u in zip(assigned, used))       # never run below the assigned precision
    _check_against_oracle(outs, stack.trace, routers_np, expert_matrices, floor)


@pytest.mark.parametrize("transfer", ["bf16", "assigned"])
def test_stack_with_an_8_bit_tier(ctx, transfer):
    """Four tiers (16 / 8 / 4 / 2 bits): the 8-bit format is quantised on the device after a bf16
    transfer, or travels as such and has a pool of its own in the cache."""
    L, steps = 3, 4
    slots = 4 if transfer == "bf16" else {16: 4, 8: 4, 4: 4, 2: 4}
    stack, routers_np, expert_matrices, floor, cfg0 = _small_stack(ctx, L, slots, True, 900, transfer=transfer,
                                                                   tiers=TIERS4)
    outs = []
    for s in range(steps):
        x, _ = synth.activations(synth.scaled(cfg0, config_id=950 + (s % 3)))
        outs.append((x, stack.step(to_bf16(x)).clone()))
    stack.close()
    assert _uses(stack.stats) == L * 2 * steps
    assigned = [a for step in stack.trace for (_, bits, _) in step for a in bits]
    assert 8 in assigned                                   # the tier is exercised
    if transfer == "assigned":
        assert stack.stats["copies_8"] > 0
    _check_against_oracle(outs, stack.trace, routers_np, expert_matrices, floor, tiers=TIERS4)


# ------------------------------------------------------------------ prefill: Eq. 2 importance, Eq. 7 prefetch

def _small_prefill_stack(ctx, T, L, slots, prefetch, seed0, transfer="bf16", predict_t=4, pool=None):
    H, F, E, k, k_hh = 256, 512, 8, 2, 3
    cfgs = [synth.scaled(synth.CONFIGS["tiny"], T=T, config_id=seed0 + l) for l in range(L)]
    routers_np = [synth.router(c)[0] for c in cfgs]
    n_pool = 12
    pool_cfg = synth.scaled(synth.CONFIGS["tiny"], config_id=seed0 + 50)
    mats = {i: synth.expert_weights(pool_cfg, i) for i in range(n_pool)}
    if pool is None:
        pool = HostExpertPool(H, F, E, n_pool, lambda i: mats[i])
        if transfer == "assigned":
            pool.add_quantised(ctx, DEV, layout=B.LAYOUT_TILE)       # T > 4: the grouped GEMM reads tiles
    floor = [4] + [0] * (L - 1)
    stack = PrefillStack(ctx, T, H, F, E, k, k_hh, [to_bf16(r) for r in routers_np], pool, slots, (1, 3, 4),
                         (16, 4, 2), floor_bits=floor, prefetch=prefetch, predict_t=predict_t, transfer=transfer,
                         alpha=0.25, device=DEV)
    return stack, routers_np, (lambda l, e: mats[pool.entry(l, e)]), floor, cfgs[0], k_hh


def _check_prefill_against_oracle(outs, stack, routers_np, expert_matrices, floor, k_hh, predict_t):
    checked = 0
    for s, (x, h_dev) in enumerate(outs):
        run_bits = [dict(zip(ex, used)) for (ex, _, used) in stack.trace[s]]
        ref_h, log, preds = O.prefill_stack(x, routers_np, expert_matrices, 2, k_hh, (1, 3, 4), (16, 4, 2), floor,
                                            0.25, predict_t=predict_t, run_bits=run_bits)
        if not all(margin_ok(lg, 2).all() for (_, _, lg, _, _) in log):
            continue                     # a near tie somewhere in the stack: decisions may legitimately differ
        checked += 1
        for l, (idx, bts, _, imp, load) in enumerate(log):
            active = tuple(int(e) for e in np.nonzero(load)[0])
            assert stack.trace[s][l][0] == active                               # Eq. 7's counts are exact integers
            assert stack.trace[s][l][1] == tuple(int(bts[e]) for e in active)   # Eq. 2 importance -> assignment
        if stack.prefetch:
            # first layer: both sides predict from the same input, so Eq. 7's list is the same, in order
            c, want, plg = preds[0]
            if margin_ok(plg, 2).all():
                assert list(stack.predictions[s][0]) == want
            # deeper layers predict from the GPU's own hidden states (within the FFN tolerance of the
            # oracle's): one token routed differently moves a count by one, so compare the sets where
            # the counts at the cut are further apart than that
            for l, (c, want, _) in enumerate(preds):
                srt = sorted(c.tolist(), reverse=True)
                if len(srt) > predict_t and srt[predict_t - 1] - srt[predict_t] < 2:
                    continue
                assert set(stack.predictions[s][l]) == set(want)
        got = synth.bf16_bits_to_f32(bits_of(h_dev)).astype(np.float64)
        want_h = synth.bf16_bits_to_f32(ref_h).astype(np.float64)
        assert np.abs(got - want_h).max() <= 2e-2
    assert checked >= 1


@pytest.mark.parametrize("T", [24, 150])
def test_prefill_stack_matches_the_oracle_and_prefetch_changes_nothing(ctx, T):
    L, steps, predict_t = 3, 2, 4
    outs, traces = {}, {}
    for prefetch in (False, True):
        stack, routers_np, expert_matrices, floor, cfg0, k_hh = _small_prefill_stack(ctx, T, L, 12, prefetch, 1100,
                                                                                     predict_t=predict_t)
        hs = []
        for s in range(steps):
            x, _ = synth.activations(synth.scaled(cfg0, config_id=1200 + s))
            hs.append((x, stack.step(to_bf16(x)).clone()))
        stack.close()
        outs[prefetch], traces[prefetch] = hs, stack.trace
        if prefetch:
            assert stack.stats["prefetch_issued"] > 0 and stack.stats["hit_prefetched"] > 0
            assert all(len(p) == predict_t for step in stack.predictions for p in step)
            _check_prefill_against_oracle(hs, stack, routers_np, expert_matrices, floor, k_hh, predict_t)
    for (x0, a), (x1, b) in zip(outs[False], outs[True]):
        assert torch.equal(a, b)
    assert traces[False] == traces[True]


def test_prefill_stack_moving_the_assigned_format_in_tile_layout(ctx):
    T, L, steps = 40, 3, 3
    slots = {16: 12, 4: 12, 2: 12}
    stack, routers_np, expert_matrices, floor, cfg0, k_hh = _small_prefill_stack(ctx, T, L, slots, True, 1300,
                                                                                 transfer="assigned", predict_t=4)
    outs = []
    for s in range(steps):
        x, _ = synth.activations(synth.scaled(cfg0, config_id=1400 + (s % 2)))
        outs.append((x, stack.step(to_bf16(x)).clone()))
    stack.close()
    st = stack.stats
    assert st["copies_4"] + st["copies_2"] > 0
    moved = sum(st.get("copies_%d" % b, 0) * stack.pool.nbytes[b] for b in (16, 4, 2))
    assert moved == st["bytes_copied"]
    for step in stack.trace:
        for (ex, assigned, used) in step:
            assert all(u >= a for a, u in zip(assigned, used))
    _check_prefill_against_oracle(outs, stack, routers_np, expert_matrices, floor, k_hh, 4)


@pytest.mark.parametrize("transfer", ["assigned", "bf16"])
def test_stack_with_one_byte_budget_shared_by_the_formats(ctx, transfer):
    """The library's byte-budget cache: blocks of the bf16 size change hands between the formats as the
    demand shifts, slots are views of one arena, and a slot that takes over the memory of evicted experts
    waits for their last use.  Results against the oracle as in the fixed-pool tests."""
    L, steps = 4, 8
    bf16_bytes = 6 * 256 * 512
    budget = (5 if transfer == "assigned" else 6) * (bf16_bytes + 400 * 1024)     # few blocks: evictions all the time
    stack, routers_np, expert_matrices, floor, cfg0 = _small_stack(ctx, L, None, True, 1500, transfer=transfer,
                                                                   budget_bytes=budget)
    outs = []
    for s in range(steps):
        x, _ = synth.activations(synth.scaled(cfg0, config_id=1600 + (s % 4)))
        outs.append((x, stack.step(to_bf16(x)).clone()))
    stack.close()
    st = stack.stats
    assert _uses(st) == L * 2 * steps
    assert stack.cache.bytes_resident() <= stack.arena.numel()
    # every resident expert sits in its own, non-overlapping piece of the arena
    spans = sorted((off, off + stack._slot_bytes[b]) for (b, off) in stack.cache.where.values())
    assert all(a[1] <= b[0] for a, b in zip(spans, spans[1:])) and spans[-1][1] <= stack.arena.numel()
    if transfer == "assigned":
        assert st["copies_4"] + st["copies_2"] > 0
        assert len({b for (b, _) in stack.slots}) >= 2                  # blocks served more than one format
    for step in stack.trace:
        for (ex, assigned, used) in step:
            assert all(u >= a for a, u in zip(assigned, used))
    _check_against_oracle(outs, stack.trace, routers_np, expert_matrices, floor)


def test_stack_overlap_report_accounts_for_copy_and_waiting_time(ctx):
    L, steps = 4, 3
    rep = {}
    for prefetch in (False, True):
        stack, _, _, _, cfg0 = _small_stack(ctx, L, 4, prefetch, 1700)
        stack.measure_overlap = True
        for s in range(steps):
            x, _ = synth.activations(synth.scaled(cfg0, config_id=1800 + s))
            stack.step(to_bf16(x))
        rep[prefetch] = stack.overlap_report()
        stack.close()
        assert rep[prefetch]["copy_ms"] > 0 and rep[prefetch]["stall_ms"] >= 0
        assert rep[prefetch]["copy_time_hidden"] <= 1.0
    # (how much of the copy time the look-ahead hides is a measurement: bench.py reports it per plan)


@pytest.mark.parametrize("layout", [B.LAYOUT_ROWMAJOR, B.LAYOUT_TILE])
def test_pool_prepared_with_the_compensated_quantizer(ctx, layout):
    """The paper prepares its experts off line with GPTQ (Sec. 5): the pool's quantised formats made by
    dymoe_gptq_quantize_pack hold the oracle's compensated codes, in either layout, and a stack runs on them."""
    from paper_2603_19172_amd.stack import quant_layout
    from gpu_helpers import rowmajor_from_tiles
    H, F, E, n_pool = 256, 512, 8, 3
    pool_cfg = synth.scaled(synth.CONFIGS["tiny"], config_id=950)
    mats = {i: synth.expert_weights(pool_cfg, i) for i in range(n_pool)}
    U = {K: O.gptq_factor(O.gptq_hessian(synth.calibration_inputs(950 + K, 1024, K))).astype(np.float32) for K in (H, F)}
    pool = HostExpertPool(H, F, E, n_pool, lambda i: mats[i])
    pool.add_quantised(ctx, DEV, formats=(4, 2), layout=layout, factors={K: torch.from_numpy(U[K]).to(DEV) for K in U})
    for b in (4, 2):
        offs, total = quant_layout(H, F, b)
        assert pool.nbytes[b] == total
        for i in (0, n_pool - 1):
            blob = pool.buf[b][i].numpy()
            for m, (n, K) in enumerate(((F, H), (F, H), (H, F))):
                co, so, zo = offs[m]
                codes = blob[co:so].reshape(n, K * b // 8)
                scale = blob[so:zo].view(np.uint16).reshape(n, K // 64)
                zero = blob[zo:zo + n * (K // 64) * 2].view(np.uint16).reshape(n, K // 64)
                if layout == B.LAYOUT_TILE:
                    codes, scale, zero = rowmajor_from_tiles(codes, scale, zero, b)
                want = O.gptq_quantize_pack(mats[i][m], U[K], b)
                assert np.array_equal(codes, want[0]) and np.array_equal(scale, want[1]) and np.array_equal(zero, want[2])
    if layout == B.LAYOUT_ROWMAJOR:
        L = 3
        cfgs = [synth.scaled(synth.CONFIGS["tiny"], T=1, phase="decode", config_id=960 + l) for l in range(L)]
        routers = [to_bf16(synth.router(c)[0]) for c in cfgs]
        stack = DecodeStack(ctx, H, F, E, 2, routers, pool, {4: 6, 2: 6}, (3, 5), (4, 2), prefetch=True,
                            transfer="assigned", alpha=0.25, device=DEV)
        for s in range(3):
            x, _ = synth.activations(synth.scaled(cfgs[0], config_id=970 + s))
            h = stack.step(to_bf16(x))
            torch.cuda.synchronize()
            assert torch.isfinite(h.float()).all()
        stack.close()
        assert stack.stats["copies_4"] + stack.stats["copies_2"] > 0


@pytest.mark.parametrize("tiers,floor_rule", [(TIERS3, True), (((3, 5), (4, 2)), False), (TIERS4, True)])
def test_resident_stack_replayed_as_a_graph_matches_eager_launches_and_the_oracle(ctx, tiers, floor_rule):
    """Every expert in every format in device memory: no copies, no host decisions, a step is one HIP graph.  The
    graph is replayed several times with other inputs, eager steps and synchronisations in between, and every
    replay must give exactly what eager launches give; the chain itself is the oracle's (assigned precisions)."""
    H, F, E, k, L = 256, 512, 8, 2, 5
    cfgs = [synth.scaled(synth.CONFIGS["tiny"], T=1, phase="decode", config_id=2300 + l) for l in range(L)]
    routers_np = [synth.router(c)[0] for c in cfgs]
    n_pool = 12
    pool_cfg = synth.scaled(synth.CONFIGS["tiny"], config_id=2350)
    mats = {i: synth.expert_weights(pool_cfg, i) for i in range(n_pool)}
    pool = HostExpertPool(H, F, E, n_pool, lambda i: mats[i])
    pool.add_quantised(ctx, DEV, formats=[b for b in tiers[1] if b != 16])
    floor = ([4] + [0] * (L - 2) + [4]) if floor_rule else [0] * L
    routers = [to_bf16(r) for r in routers_np]
    make = lambda graph, fused=True: ResidentDecodeStack(ctx, H, F, E, k, routers, pool, tiers[0], tiers[1],
                                                         floor_bits=floor, alpha=0.25, device=DEV, graph=graph, fused=fused)
    eager, replayed, separate = make(False), make(True), make(False, fused=False)
    outs, traces = [], []
    for s in (0, 1, 2, 1, 0, 3):
        x, _ = synth.activations(synth.scaled(cfgs[0], config_id=2400 + s))
        a = eager.step(to_bf16(x)).clone()
        torch.cuda.synchronize()
        b = replayed.step(to_bf16(x)).clone()
        assert torch.equal(a, b)
        assert eager.trace() == replayed.trace()
        c = separate.step(to_bf16(x)).clone()      # front end and FFN as separate calls: the same bits
        assert torch.equal(a, c) and eager.trace() == separate.trace()
        outs.append((x, b))
        traces.append([(ex, bts, bts) for (ex, bts) in replayed.trace()])
    _check_against_oracle(outs, traces, routers_np, lambda l, e: mats[pool.entry(l, e)], floor, tiers=tiers)


def test_resident_stack_refuses_a_pool_without_the_formats_it_may_need(ctx):
    H, F, E, k = 256, 512, 8, 2
    pool_cfg = synth.scaled(synth.CONFIGS["tiny"], config_id=2350)
    pool = HostExpertPool(H, F, E, 4, lambda i: synth.expert_weights(pool_cfg, i))
    routers = [to_bf16(synth.router(synth.scaled(synth.CONFIGS["tiny"], T=1, phase="decode", config_id=2300))[0])]
    with pytest.raises(ValueError):
        ResidentDecodeStack(ctx, H, F, E, k, routers, pool, (1, 3, 4), (16, 4, 2), device=DEV)
