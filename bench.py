#!/usr/bin/env python3
"""Benchmark of the DyMoE mixed-precision MoE layer on one MI355X.

A step is one pass of the whole hot path over one batch: router gating + top-k
-> expert importance -> bit-width assignment -> quantize-and-pack of the experts
the assignment sends to int4 / int2 -> dequant-fused SwiGLU expert FFN.

Headline (`value`): tokens/s of that full step on the Mixtral-8x7B-shaped decode
layer (batch 1, BASELINE configs[1]).  The same JSON line also carries, each under
its own key: the FFN alone with the selected formats already resident and the two
active experts forced to each pair of formats; the 512-token prefill of the same
layer (configs[2]); the fine-grained 128-expert layer (configs[3]); the 32-layer
decode stack with the experts in pinned host memory, 64 steps (configs[4]); the
roofline of the dominant kernel of the timed step and of the two paths the targets
are stated on (timed with HIP events attached to the dispatches by the library's
per-kernel timers, over the same steps launched eagerly right after the timed
region); the matrix rate and copy rate this machine sustains; and the CPU oracle
timed on this host for the decode step and for a sample of the prefill.

  python bench.py --gpus 1 --steps 200 --warmup 20
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
LAYER_COPIES = 4   # distinct weight copies rotated through, so that no step finds its weights in the 256 MB last-level cache


def bytes_per_weight(bits):
    # packed codes + fp16 scale and zero per group of 64
    return 2.0 if bits == 16 else bits / 8.0 + 4.0 / 64.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--launch", choices=("both", "eager", "hip_graph"), default="both",
                    help="how a step's launches reach the GPU: enqueued one by one (eager) or replayed as a captured HIP "
                         "graph; both (default) times either way and reports the faster one as the step's time")
    ap.add_argument("--no-graph", action="store_true", help="the same as --launch eager")
    ap.add_argument("--skip-prefill", action="store_true")
    ap.add_argument("--stack-steps", type=int, default=64,
                    help="decode steps through the 32-layer stack with the experts in pinned host memory "
                         "(BASELINE configs[4] names 64); 0 skips the stack")
    ap.add_argument("--stack-plans", default="literal,budget,paper",
                    help="which plans of the host-resident stack to run, each with look-ahead off and on: literal (bf16 "
                         "travels and is quantised on arrival, as configs[4] words it), pools (the assigned format "
                         "travels, fixed pools per format), budget (the assigned format, one byte budget), paper "
                         "(4/2 tiers with the cosine depth schedule, one byte budget), paper-pools")
    ap.add_argument("--stack-warmup", type=int, default=1,
                    help="untimed steps of the stack before the timed ones, cycling through the same inputs (as many as "
                         "--stack-steps with a large budget: every expert the timed steps need is then resident)")
    ap.add_argument("--stack-budget-gb", type=float, default=24.0,
                    help="device bytes set aside for expert slots in the stack run")
    ap.add_argument("--skip-cpu", action="store_true")
    ap.add_argument("--no-format-sweep", action="store_true",
                    help="skip the pass that times the decode FFN kernels with the two active experts forced to bf16, "
                         "int8, int4, int4+int2 and int2 (for a profiler run over the default workload: its extra "
                         "launches would blur the per-kernel averages)")
    ap.add_argument("--skip-fine-grained", action="store_true",
                    help="skip the fine-grained layer (BASELINE configs[3]: 2048 tokens, 128 experts, top-8)")
    ap.add_argument("--attention-long", action="store_true",
                    help="also time the attention-derived token score at 2048 and 8192 tokens (32 query / 8 key heads of "
                         "128), causal and not: the sizes its LDS-staged kernels serve")
    ap.add_argument("--gptq", action="store_true",
                    help="also time the error-compensated quantizer (Hessian, inverse factor, column sweep) on the three "
                         "matrices of one Mixtral-shaped expert with 2048 synthetic calibration tokens")
    ap.add_argument("--prefill-steps", type=int, default=20)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run dymoe_pack_tiles on a 1 GiB bf16 matrix: a permuting copy of known traffic "
                         "(1 GiB read in 32-byte pieces, 1 GiB written), a second reference for a profiler's "
                         "byte counters beside the plain stream copy that every run makes")
    args = ap.parse_args()
    if args.no_graph:
        args.launch = "eager"
    args.format_sweep = not args.no_format_sweep
    args.fine_grained = not args.skip_fine_grained
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2603_19172_amd import binding as B
    from paper_2603_19172_amd import synth
    from paper_2603_19172_amd.layer import ExpertStore, MoELayer

    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS["mixtral_decode"]
    H, F, E, k = cfg.H, cfg.F, cfg.E, cfg.k

    def bf16(a):
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(dev).view(torch.bfloat16)

    t_setup = time.perf_counter()
    host_w = synth.expert_weights_many(cfg, range(E), workers=min(16, os.cpu_count() or 8))
    x_np, _ = synth.activations(cfg)
    wg_np, bias_np = synth.router(cfg)
    ctx = B.Context(0)
    stores = [ExpertStore([[bf16(m) for m in host_w[e]] for e in range(E)], H, F, dev, ctx=ctx,
                          formats=(8, 4, 2) if args.format_sweep else (4, 2))]
    for _ in range(LAYER_COPIES - 1):
        stores.append(stores[0].clone())
    x = bf16(x_np)
    wg = bf16(wg_np)
    layer = MoELayer(ctx, cfg.T, H, F, E, k, "decode", cfg.tier_count, cfg.tier_bits,
                     out_dtype=B.OUT_BF16, device=dev)
    torch.cuda.synchronize()
    setup_s = time.perf_counter() - t_setup
    # plain copy of 1 GiB: the copy rate this machine sustains, and a known quantity
    # of traffic for a profiler's byte counters
    src = torch.zeros((1 << 30,), dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    for _ in range(2):
        ctx.stream_copy(src, dst)
    ctx.timing_enable(["stream_copy"])
    for _ in range(10):
        ctx.stream_copy(src, dst)
    ms, n = ctx.timing_read("stream_copy")
    ctx.timing_enable([])
    copy_gbps = 2.0 * src.numel() * n / (ms * 1e-3) / 1e9
    # register-only bf16 MFMA loop: the matrix rate this machine sustains (about 50 ms of it, so that the clock
    # settles where it stays under that load), one and two wavefronts per SIMD
    sink = torch.empty((1 << 18,), dtype=torch.float32, device=dev)
    mfma_rate = {}
    for wps in (1, 2):
        ctx.mfma_peak(2000, wps, sink)
        ctx.timing_enable(["mfma_peak"])
        fl = sum(ctx.mfma_peak(20000, wps, sink) for _ in range(6))
        ms, n = ctx.timing_read("mfma_peak")
        ctx.timing_enable([])
        mfma_rate[wps] = fl / (ms * 1e-3) / 1e12
    mfma_measured = max(mfma_rate.values())
    if args.calibrate_copy:
        src2 = src.view(torch.bfloat16).view(32768, 16384)
        for _ in range(3):
            ctx.pack_tiles(src2)
    torch.cuda.synchronize()
    del src, dst

    def timed_loop(fns, steps, warmup):
        """fns: one callable per weight copy; returns seconds for `steps` calls."""
        for i in range(warmup):
            fns[i % len(fns)]()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            fns[i % len(fns)]()
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    def make_fns(lay, xin, wgt, bias, quantize, mode):
        eager = [(lambda s=s: lay.step(xin, wgt, bias, s, quantize=quantize)) for s in stores]
        if mode == "eager":
            return eager
        graphs = []
        side = torch.cuda.Stream()
        for fn in eager:
            fn()                      # first call outside capture (module load, lazy init)
        torch.cuda.synchronize()
        for fn in eager:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                fn()
            graphs.append(g)
        return [g.replay for g in graphs]

    def time_step(lay, xin, wgt, bias, quantize, steps, warmup):
        """Seconds for `steps` steps in each launch mode asked for; returns (best seconds, its mode, its callables,
        {mode: microseconds per step})."""
        modes = ("eager", "hip_graph") if args.launch == "both" else (args.launch,)
        best, per_mode = None, {}
        for mode in modes:
            fns_ = make_fns(lay, xin, wgt, bias, quantize, mode)
            sec_ = timed_loop(fns_, steps, warmup)
            per_mode[mode] = round(sec_ / steps * 1e6, 2)
            if best is None or sec_ < best[0]:
                best = (sec_, mode, fns_)
        return best[0], best[1], best[2], per_mode

    def time_call(fn, steps, warmup):
        """One callable timed in each launch mode asked for: (best seconds per step, its mode, {mode: us per step})."""
        modes = ("eager", "hip_graph") if args.launch == "both" else (args.launch,)
        best, per_mode = None, {}
        for mode in modes:
            run = fn
            if mode == "hip_graph":
                fn()
                torch.cuda.synchronize()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=torch.cuda.Stream()):
                    fn()
                run = g.replay
            dt = timed_loop([run], steps, warmup) / steps
            per_mode[mode] = round(dt * 1e6, 2)
            if best is None or dt < best[0]:
                best = (dt, mode)
        return best[0], best[1], per_mode

    def step_spread(fns, steps):
        """A second, untimed-for-the-headline pass with an event between the steps: median / min / max of a step."""
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        cur = torch.cuda.current_stream()
        evs[0].record(cur)
        for i in range(steps):
            fns[i % len(fns)]()
            evs[i + 1].record(cur)
        torch.cuda.synchronize()
        us = sorted(evs[i].elapsed_time(evs[i + 1]) * 1e3 for i in range(steps))
        return {"median": round(us[len(us) // 2], 2), "min": round(us[0], 2), "max": round(us[-1], 2),
                "note": "separate pass with an event after every step (the events add about a microsecond each)"}

    # ---------------------------------------------------------------- decode, full hot path
    sec, launch_mode, fns, launch_us = time_step(layer, x, wg, None, True, args.steps, args.warmup)
    ms_per_step = sec / args.steps * 1e3
    value = cfg.T * args.steps / sec
    spread = step_spread(fns, min(args.steps, 200))
    bits_host = layer.bits.cpu().numpy()
    idx_host = layer.idx.cpu().numpy()
    active = [int(e) for e in idx_host[0]]
    active_bits = [int(bits_host[e]) for e in active]
    y_gpu = layer.y.float().cpu().numpy().astype(np.float64)

    # FFN alone, formats resident (what an offline-quantised deployment pays)
    sec_ffn, ffn_mode, _, ffn_launch_us = time_step(layer, x, wg, None, False, args.steps, args.warmup)
    ffn_bytes = sum(3.0 * H * F * bytes_per_weight(b) for b in active_bits)

    # ---------------------------------------------------------------- per-kernel timing (eager, HIP events)
    kernels = ["decode_front", "quantize", "gemv_phase1", "gemv_phase2"]
    ctx.timing_enable(kernels)
    n_timed = min(args.steps, 100)
    for i in range(n_timed):
        layer.step(x, wg, None, stores[i % len(stores)], quantize=True)
    torch.cuda.synchronize()
    kt = {}
    for name in kernels:
        ms, n = ctx.timing_read(name)
        kt[name] = (ms / max(n, 1) * 1e3, n)   # us per launch
    ctx.timing_enable(())
    q_bits = [b for b in active_bits if b in (2, 4)]
    alg_bytes = {
        "quantize": sum(3.0 * H * F * (2.0 + bytes_per_weight(b)) for b in q_bits),
        "gemv_phase1": sum(2.0 * H * F * bytes_per_weight(b) for b in active_bits),
        "gemv_phase2": sum(1.0 * H * F * bytes_per_weight(b) for b in active_bits),
    }
    dominant = max(alg_bytes, key=lambda n: kt[n][0])
    dom_us = kt[dominant][0]
    achieved = alg_bytes[dominant] / (dom_us * 1e-6) / 1e9 if dom_us > 0 else 0.0
    kname = B.lib.dymoe_kernel_name(B.KERNELS.index(dominant)).decode()
    # HBM bytes per launch as counted by rocprofv3 (FETCH_SIZE + WRITE_SIZE, scaled by the
    # same counters' reading for a copy kernel of known size); written down from the
    # profiling runs documented under profiles/, null when no such file is there
    traffic_all = {}
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            traffic_all = json.load(f)
    traffic = traffic_all.get("mixtral_decode", {}).get(kname)
    # the longest kernel of the timed step (the quantiser: it reads bf16 and writes codes, so it says nothing
    # about running on packed weights; that is `roofline_decode_packed` below)
    roofline = {"kernel": kname,
                "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "algorithmic_bytes_per_launch": alg_bytes[dominant], "avg_launch_us": round(dom_us, 2),
                "note": "dominant kernel of the timed step by duration"}
    # decode on packed weights: the two dequant GEMV launches together
    gemv_us = kt["gemv_phase1"][0] + kt["gemv_phase2"][0]
    gemv_bytes = alg_bytes["gemv_phase1"] + alg_bytes["gemv_phase2"]
    gemv_gbs = gemv_bytes / (gemv_us * 1e-6) / 1e9 if gemv_us > 0 else 0.0
    gemv_traffic = [traffic_all.get("mixtral_decode", {}).get(n_) for n_ in ("gemv_phase1_kernel", "gemv_phase2_kernel")]
    roofline_decode = {"kernels": ["gemv_phase1_kernel", "gemv_phase2_kernel"], "bound": "hbm",
                       "achieved": round(gemv_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                       "frac": round(gemv_gbs / HBM_PEAK_GBS, 4),
                       "traffic": sum(gemv_traffic) if all(v is not None for v in gemv_traffic) else None,
                       "algorithmic_bytes_per_step": gemv_bytes, "sum_of_launch_us": round(gemv_us, 2),
                       "note": "S5 on packed weights (bf16 + int4 expert), kernel time only; the step-level figure, "
                               "gaps and front end included, is decode_ffn_only.frac_hbm"}
    kernels_report = {}
    for name in kernels:
        entry = {"avg_us": round(kt[name][0], 2), "launches": kt[name][1]}
        if name in alg_bytes and kt[name][0] > 0:
            gbs = alg_bytes[name] / (kt[name][0] * 1e-6) / 1e9
            entry.update({"algorithmic_bytes": alg_bytes[name], "GBps": round(gbs, 1),
                          "frac_hbm": round(gbs / HBM_PEAK_GBS, 4)})
        kernels_report[name] = entry

    # ---------------------------------------------------------------- S5 alone with the active pair forced to each format
    sweep = {}
    st0 = B._stream(None)
    only_active = torch.zeros((E,), dtype=torch.int32, device=dev)
    only_active[active] = 1
    for ba, bb in (((16, 16), (8, 8), (4, 4), (4, 2), (2, 2)) if args.format_sweep else ()):
        forced = torch.full((E,), 2, dtype=torch.uint8, device=dev)
        forced[active[0]], forced[active[1]] = ba, bb
        for s_ in stores:
            ctx.quantize_experts(s_.table, forced, only_active, E, H, F, layout=layer.layout)
        layer.bits.copy_(forced)
        for i in range(4):
            layer.ffn(x, stores[i % len(stores)], st0)
        torch.cuda.synchronize()
        ctx.timing_enable(["gemv_phase1", "gemv_phase2"])
        n_sw = 40
        for i in range(n_sw):
            layer.ffn(x, stores[i % len(stores)], st0)
        torch.cuda.synchronize()
        us = {n_: ctx.timing_read(n_)[0] / n_sw * 1e3 for n_ in ("gemv_phase1", "gemv_phase2")}
        ctx.timing_enable(())
        nbytes = 3.0 * H * F * (bytes_per_weight(ba) + bytes_per_weight(bb))
        tot = sum(us.values())
        sweep["%d+%d" % (ba, bb)] = {"algorithmic_bytes": nbytes, "kernels_us": {k_: round(v_, 1) for k_, v_ in us.items()},
                                     "GBps": round(nbytes / (tot * 1e-6) / 1e9, 1),
                                     "frac_hbm": round(nbytes / (tot * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)}
    layer.bits.copy_(torch.from_numpy(bits_host).to(dev))

    out = {
        "metric": "MoE-layer tokens/s, decode b=1, full hot path (route, importance, precision, quantize-pack, mixed FFN)",
        "value": round(value, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "step_us": spread, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16 weights/activations, int4+int2 codes, fp32 accumulate",
        "data": "synthetic",
        "config": {"workload": "mixtral_decode (BASELINE configs[1]): H=4096 F=14336 E=8 top-2, 1 token, tiers 1 bf16 / 3 int4 / 4 int2, group 64",
                   "active_experts": active, "active_bits": active_bits, "launch": launch_mode,
                   "us_per_step_by_launch_mode": launch_us,
                   "weight_copies_rotated": LAYER_COPIES, "setup_s": round(setup_s, 1)},
        "roofline": roofline,
        "roofline_decode_packed": roofline_decode,
        "machine": {"stream_copy_GBps": round(copy_gbps, 1),
                    "mfma_bf16_TFLOPs_register_loop": {"one_wave_per_simd": round(mfma_rate[1], 1),
                                                       "two_waves_per_simd": round(mfma_rate[2], 1)},
                    "note": "what this GPU sustains on the library's two measurement aids (dymoe_stream_copy: 1 GiB read + "
                            "1 GiB written; dymoe_mfma_peak: v_mfma_f32_32x32x16_bf16 on registers only): the practical "
                            "ceilings beside the data sheet's 8 TB/s and 2.5 PFLOP/s that every fraction here is priced against"},
        "hot_path_hbm": {"algorithmic_bytes_per_step": sum(alg_bytes.values()),
                         "GBps": round(sum(alg_bytes.values()) / (ms_per_step * 1e-3) / 1e9, 1),
                         "frac_hbm": round(sum(alg_bytes.values()) / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                         "stream_copy_GBps": round(copy_gbps, 1),
                         "note": "all kernels of a step and the gaps between them over the step's algorithmic "
                                 "bytes; stream_copy_GBps is a plain 1 GiB copy (read + write bytes) on this GPU"},
        "kernels": kernels_report,
        "decode_ffn_format_sweep": {"note": "S5 kernels alone (sum of their execution times, eager launches, 4 rotating weight "
                                            "copies), the two active experts forced to the named bit-widths",
                                    "pairs": sweep} if args.format_sweep else None,
        "decode_ffn_only": {"tokens_per_s": round(cfg.T * args.steps / sec_ffn, 1),
                            "us_per_step": round(sec_ffn / args.steps * 1e6, 2),
                            "algorithmic_bytes": ffn_bytes,
                            "GBps": round(ffn_bytes / (sec_ffn / args.steps) / 1e9, 1),
                            "frac_hbm": round(ffn_bytes / (sec_ffn / args.steps) / 1e9 / HBM_PEAK_GBS, 4),
                            "launch": ffn_mode, "us_per_step_by_launch_mode": ffn_launch_us,
                            "note": "S1+S2+S3+S5 with the selected formats already materialised (dymoe_decode_step: two launches)"},
    }

    # ---------------------------------------------------------------- prefill 512 on the same layer
    if not args.skip_prefill:
        pcfg = synth.CONFIGS["mixtral_prefill"]
        px_np, _ = synth.activations(pcfg)
        pwg_np, _ = synth.router(pcfg)
        px, pwg = bf16(px_np), bf16(pwg_np)
        play = MoELayer(ctx, pcfg.T, H, F, E, k, "prefill", pcfg.tier_count, pcfg.tier_bits,
                        k_hh=pcfg.k_hh, out_dtype=B.OUT_BF16, device=dev)
        psec, pmode, _, p_launch_us = time_step(play, px, pwg, None, True, args.prefill_steps, 3)
        psec2, pmode2, _, p_launch_us2 = time_step(play, px, pwg, None, False, args.prefill_steps, 3)
        pbits = play.bits.cpu().numpy()
        pload = play.load.cpu().numpy()
        flops = float(pload.sum()) * 6.0 * H * F
        wbytes = sum(3.0 * H * F * bytes_per_weight(int(b)) for b, l in zip(pbits, pload) if l > 0)
        ctx.timing_enable(["gemm1", "gemm2", "quantize", "plan", "gemm_combine"])
        for i in range(5):
            play.step(px, pwg, None, stores[i % len(stores)], quantize=True)
        torch.cuda.synchronize()
        pk = {n: ctx.timing_read(n) for n in ("gemm1", "gemm2", "quantize", "plan", "gemm_combine")}
        ctx.timing_enable(())
        g_us = (pk["gemm1"][0] / max(pk["gemm1"][1], 1) + pk["gemm2"][0] / max(pk["gemm2"][1], 1)) * 1e3
        out["prefill_512"] = {
            "workload": "mixtral_prefill (BASELINE configs[2]): 512 tokens, 26 heavy hitters x8, precision assigned at run time; expert weights shared with the decode workload",
            "tokens_per_s_full_path": round(pcfg.T * args.prefill_steps / psec, 1),
            "us_per_step_full_path": round(psec / args.prefill_steps * 1e6, 1),
            "tokens_per_s_formats_resident": round(pcfg.T * args.prefill_steps / psec2, 1),
            "us_per_step_formats_resident": round(psec2 / args.prefill_steps * 1e6, 1),
            "launch": {"full_path": pmode, "formats_resident": pmode2},
            "us_per_step_by_launch_mode": {"full_path": p_launch_us, "formats_resident": p_launch_us2},
            "bits": [int(b) for b in pbits], "load": [int(l) for l in pload],
            "gemm_flops": flops, "weight_bytes": wbytes,
            "grouped_gemm_us": round(g_us, 1),
            "grouped_gemm_TFLOPs": round(flops / (g_us * 1e-6) / 1e12, 1) if g_us > 0 else None,
            "grouped_gemm_frac_mfma_bf16_peak": round(flops / (g_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4) if g_us > 0 else None,
            "grouped_gemm_frac_of_measured_mfma_rate": round(flops / (g_us * 1e-6) / 1e12 / mfma_measured, 4) if g_us > 0 else None,
            "kernels_us": {n: round(v[0] / max(v[1], 1) * 1e3, 1) for n, v in pk.items()},
        }
        gt = traffic_all.get("mixtral_prefill", {})
        out["roofline_prefill_gemm"] = {
            "kernels": ["gemm_kernel<1>", "gemm_kernel<2>"], "bound": "mfma",
            "achieved": round(flops / (g_us * 1e-6) / 1e12, 1) if g_us > 0 else None, "peak": MFMA_BF16_PEAK_TFLOPS,
            "unit": "TFLOP/s", "frac": round(flops / (g_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4) if g_us > 0 else None,
            "traffic": (gt.get("gemm_kernel<1>", 0) + gt.get("gemm_kernel<2>", 0)) or None,
            "algorithmic_flops_per_step": flops, "algorithmic_weight_bytes_per_step": wbytes,
            "sum_of_launch_us": round(g_us, 1),
            "note": "2*3*H*F flops per (token, expert) pair over the two GEMM launches of one 512-token step"}
        # the oracle on a seeded sample of the same step: routing, importance and assignment in full, the FFN on
        # a few token rows; its time per (token, expert) pair extrapolated to the 1024 pairs of the step
        if not args.skip_cpu:
            from oracle import dymoe_oracle as O
            t0 = time.perf_counter()
            ridx, rw, rp, _ = O.route_topk(px_np, pwg_np, None, k)
            rimp, rload, _ = O.expert_importance_prefill(ridx, O.token_score_norm(px_np), E, pcfg.k_hh)
            rbits, _ = O.assign_precision(rimp, rload, pcfg.tier_count, pcfg.tier_bits)
            t_front = time.perf_counter() - t0
            rows = np.random.default_rng(5).choice(pcfg.T, 4, replace=False)
            need = sorted(set(int(e) for e in ridx[rows].ravel()))
            t0 = time.perf_counter()
            ex = [({"w": host_w[e]} if rbits[e] == 16 else {"q": [O.quantize_pack(m, int(rbits[e])) for m in host_w[e]]})
                  if e in need else {} for e in range(E)]
            t_quant = time.perf_counter() - t0
            mb = np.array([rbits[e] if e in need else 0 for e in range(E)], np.uint8)
            t0 = time.perf_counter()
            pref = O.moe_ffn_mixed(px_np[rows], ridx[rows], rw[rows], mb, ex)
            t_ffn = time.perf_counter() - t0
            n_q = sum(1 for e in need if rbits[e] != 16)
            n_q_all = int(sum(1 for e in range(E) if rload[e] > 0 and rbits[e] != 16))
            est = t_front + t_quant / max(n_q, 1) * n_q_all + t_ffn / (len(rows) * k) * (pcfg.T * k)
            got = play.y.float().cpu().numpy().astype(np.float64)[rows]
            prms = np.sqrt((pref ** 2).mean(axis=1, keepdims=True))
            out["prefill_512"]["cpu_baseline"] = {
                "value": round(pcfg.T / est, 4), "unit": "tokens/s", "cores": 1, "kind": "oracle", "extrapolated": True,
                "sample": "route + importance + assignment of all 512 tokens (%.2f s), quantize-pack of %d of the %d "
                          "quantised experts (%.1f s), FFN of %d token rows = %d (token, expert) pairs (%.1f s); the step's "
                          "time is extrapolated from these: quantize-pack per expert x %d, FFN per pair x %d"
                          % (t_front, n_q, n_q_all, t_quant, len(rows), len(rows) * k, t_ffn, n_q_all, pcfg.T * k),
                "seconds_per_step_extrapolated": round(est, 1),
                "ffn_max_err_over_rms_on_the_sample_bf16_out": round(float((np.abs(got - pref) / prms).max()), 5)}
        # the attention-derived token score of the same 512 tokens (32 query heads, 8 key heads of 128)
        a_heads, a_kv, a_d = 32, 8, 128
        aq_np, ak_np, _ = synth.attention_inputs(pcfg, a_heads, a_kv, a_d)
        aq = torch.from_numpy(aq_np.view(np.int16)).to(dev).view(torch.bfloat16)
        ak = torch.from_numpy(ak_np.view(np.int16)).to(dev).view(torch.bfloat16)
        a_ws = torch.empty((int(B.lib.dymoe_attention_workspace_bytes(pcfg.T, a_heads)),), dtype=torch.uint8, device=dev)
        a_out = torch.empty((pcfg.T,), dtype=torch.float32, device=dev)
        for _ in range(3):
            ctx.token_score_attention(aq, ak, causal=True, out=a_out, workspace=a_ws)
        torch.cuda.synchronize()
        ctx.timing_enable(["attn_stats", "attn_colsum"])
        for _ in range(args.prefill_steps):
            ctx.token_score_attention(aq, ak, causal=True, out=a_out, workspace=a_ws)
        torch.cuda.synchronize()
        ak_us = {n: ctx.timing_read(n) for n in ("attn_stats", "attn_colsum")}
        ctx.timing_enable(())
        a_us = sum(v[0] / max(v[1], 1) for v in ak_us.values()) * 1e3
        a_flops = 2 * 2.0 * pcfg.T * (pcfg.T + 32) / 2 * a_d * a_heads     # two passes over the causal half (32-token tiles)
        out["prefill_512"]["attention_token_score"] = {
            "workload": "512 tokens, 32 query / 8 key heads of 128, causal",
            "kernels_us": {n: round(v[0] / max(v[1], 1) * 1e3, 1) for n, v in ak_us.items()},
            "TFLOPs": round(a_flops / (a_us * 1e-6) / 1e12, 1) if a_us > 0 else None}

    # ---------------------------------------------------------------- attention score, long sequences (opt-in)
    if args.attention_long:
        a_heads, a_kv, a_d = 32, 8, 128
        rows = []
        for aT in (2048, 8192):
            acfg = synth.scaled(synth.CONFIGS["mixtral_prefill"], T=aT, k_hh=max(1, aT // 20), config_id=70)
            aq_np, ak_np, _ = synth.attention_inputs(acfg, a_heads, a_kv, a_d)
            aq = torch.from_numpy(aq_np.view(np.int16)).to(dev).view(torch.bfloat16)
            ak = torch.from_numpy(ak_np.view(np.int16)).to(dev).view(torch.bfloat16)
            a_ws = torch.empty((int(B.lib.dymoe_attention_workspace_bytes(aT, a_heads)),), dtype=torch.uint8, device=dev)
            a_out = torch.empty((aT,), dtype=torch.float32, device=dev)
            for causal in (True, False):
                for _ in range(3):
                    ctx.token_score_attention(aq, ak, causal=causal, out=a_out, workspace=a_ws)
                torch.cuda.synchronize()
                ctx.timing_enable(["attn_stats", "attn_colsum"])
                for _ in range(args.prefill_steps):
                    ctx.token_score_attention(aq, ak, causal=causal, out=a_out, workspace=a_ws)
                torch.cuda.synchronize()
                ak_us = {n: ctx.timing_read(n) for n in ("attn_stats", "attn_colsum")}
                ctx.timing_enable(())
                a_us = sum(v[0] / max(v[1], 1) for v in ak_us.values()) * 1e3
                # two passes of T x T x d products per head; the causal mask leaves the 32-token tiles on or below the diagonal
                a_flops = 2 * 2.0 * a_d * a_heads * (aT * (aT + 32) / 2 if causal else float(aT) * aT)
                rows.append({"tokens": aT, "causal": causal,
                             "kernels_us": {n: round(v[0] / max(v[1], 1) * 1e3, 1) for n, v in ak_us.items()},
                             "TFLOPs": round(a_flops / (a_us * 1e-6) / 1e12, 1),
                             "frac_mfma_bf16_peak": round(a_flops / (a_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)})
            del aq, ak, a_ws
        out["attention_token_score_long"] = {"workload": "32 query / 8 key heads of 128", "runs": rows}

    # ---------------------------------------------------------------- fine-grained layer (opt-in)
    if args.fine_grained:
        fcfg = synth.CONFIGS["fine_grained"]
        fhw = synth.expert_weights_many(fcfg, range(fcfg.E), workers=16)
        fstore = ExpertStore([[bf16(m) for m in fhw[e]] for e in range(fcfg.E)], fcfg.H, fcfg.F, dev, ctx=ctx)
        fx_np, _ = synth.activations(fcfg)
        fwg_np, fbias_np = synth.router(fcfg)
        fx, fwg, fbias = bf16(fx_np), bf16(fwg_np), torch.from_numpy(fbias_np).to(dev)
        flay = MoELayer(ctx, fcfg.T, fcfg.H, fcfg.F, fcfg.E, fcfg.k, "prefill", fcfg.tier_count, fcfg.tier_bits,
                        k_hh=fcfg.k_hh, out_dtype=B.OUT_BF16, device=dev)
        for _ in range(3):
            flay.step(fx, fwg, fbias, fstore)
        torch.cuda.synchronize()
        # throughput: the step in either launch mode, the faster one reported, as for the other workloads
        fdt, fmode, f_launch_us = time_call(lambda: flay.step(fx, fwg, fbias, fstore), args.prefill_steps, 3)
        # per-kernel times: eager launches with events on the dispatches
        fnames = ["route", "route_select", "token_norm", "importance", "assign", "quantize", "plan", "gemm1", "gemm2", "gemm_combine"]
        ctx.timing_enable(fnames)
        for _ in range(args.prefill_steps):
            flay.step(fx, fwg, fbias, fstore)
        torch.cuda.synchronize()
        fk = {n: ctx.timing_read(n) for n in fnames}
        ctx.timing_enable(())
        fg_us = (fk["gemm1"][0] / max(fk["gemm1"][1], 1) + fk["gemm2"][0] / max(fk["gemm2"][1], 1)) * 1e3
        fflops = 2.0 * 3 * fcfg.H * fcfg.F * fcfg.T * fcfg.k
        out["fine_grained_2048"] = {
            "workload": "fine_grained (BASELINE configs[3]): 2048 tokens, 128 experts of 768, top-8, Zipf router bias, tiers 13/39/76",
            "tokens_per_s_full_path": round(fcfg.T / fdt, 1), "us_per_step_full_path": round(fdt * 1e6, 1),
            "launch": fmode, "us_per_step_by_launch_mode": f_launch_us,
            "experts_with_load": int((flay.load > 0).sum()), "max_load": int(flay.load.max()),
            "grouped_gemm_us": round(fg_us, 1),
            "grouped_gemm_frac_mfma_bf16_peak": round(fflops / (fg_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
            "kernels_us": {n: round(v[0] / max(v[1], 1) * 1e3, 1) for n, v in fk.items()}}
        # one decode token on the same layer (the selected experts rank first, so all eight run in bf16):
        # 75 MB of weights, a step made of launch latencies rather than bandwidth
        dcfg = synth.scaled(fcfg, T=1, phase="decode", k_hh=0, config_id=45)
        dx = bf16(synth.activations(dcfg)[0])
        dlay = MoELayer(ctx, 1, fcfg.H, fcfg.F, fcfg.E, fcfg.k, "decode", fcfg.tier_count, fcfg.tier_bits,
                        out_dtype=B.OUT_BF16, device=dev)
        ddt, dmode, d_launch_us = time_call(lambda: dlay.step(dx, fwg, fbias, fstore), 200, 5)
        dsel = dlay.idx.cpu().numpy().ravel()
        dbits = dlay.bits.cpu().numpy()
        dbytes = sum({16: 2.0, 8: 1.0625, 4: 0.5625, 2: 0.3125}[int(dbits[e])] * 3 * fcfg.H * fcfg.F for e in dsel)
        out["fine_grained_2048"]["decode_1_token"] = {
            "us_per_step_full_path": round(ddt * 1e6, 1), "tokens_per_s": round(1.0 / ddt, 1),
            "selected_bits": [int(dbits[e]) for e in dsel], "weight_bytes": dbytes,
            "GBps": round(dbytes / ddt / 1e9, 1), "launch": dmode, "us_per_step_by_launch_mode": d_launch_us,
            "note": "same weights hot in the caches from step to step: a latency figure, not a bandwidth one"}
        del fstore, flay, dlay
        torch.cuda.empty_cache()

    # ---------------------------------------------------------------- error-compensated quantizer (opt-in)
    if args.gptq:
        gnames = ["gptq_hessian", "gptq_factor", "gptq_group", "gptq_trail"]
        n_cal = 2048
        res = {}
        for label, (gN, gK) in (("W1/W3 [F,H]", (F, H)), ("W2 [H,F]", (H, F))):
            gw = bf16(host_w[0][0 if gK == H else 2])
            gx = bf16(synth.calibration_inputs(31, n_cal, gK))
            hess = torch.empty((gK, gK), dtype=torch.float32, device=dev)
            gu = torch.empty_like(hess)
            fws = torch.empty((int(B.lib.dymoe_gptq_factor_workspace_bytes(gK)),), dtype=torch.uint8, device=dev)
            sws = torch.empty((int(B.lib.dymoe_gptq_workspace_bytes(gN, gK)),), dtype=torch.uint8, device=dev)
            gout = None
            for rep in range(2):                        # the second pass is the one reported
                ctx.timing_enable(gnames)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                ctx.gptq_hessian(gx, out=hess)
                ctx.gptq_factor(hess, out=gu, workspace=fws)
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                fac = {n_: ctx.timing_read(n_) for n_ in gnames}
                gout = ctx.gptq_quantize_pack(gw, gu, 4, workspace=sws, out=gout)
                torch.cuda.synchronize()
                t2 = time.perf_counter()
                swp = {n_: ctx.timing_read(n_) for n_ in gnames}
                ctx.timing_enable(())
            trail_flops = 2.0 * gN * gK * (gK - 64) / 2.0       # one FMA per (row, column pair c < j across groups)
            res[label] = {
                "N": gN, "K": gK, "calibration_tokens": n_cal,
                "hessian_ms": round(fac["gptq_hessian"][0], 3),
                "hessian_TFLOPs_bf16": round(2.0 * n_cal * gK * gK / 2 / (fac["gptq_hessian"][0] * 1e-3) / 1e12, 1),
                "factor_ms_wall": round((t1 - t0) * 1e3 - fac["gptq_hessian"][0], 2),
                "factor_kernels_ms": {"chol_diag": round(fac["gptq_factor"][0], 2), "group": round(fac["gptq_group"][0], 2),
                                      "trail": round(fac["gptq_trail"][0], 2)},
                "sweep_ms_wall": round((t2 - t1) * 1e3, 2),
                "sweep_kernels_ms": {"group": round(swp["gptq_group"][0], 2), "trail": round(swp["gptq_trail"][0], 2)},
                "sweep_trail_TFLOPs_fp32": round(trail_flops / (swp["gptq_trail"][0] * 1e-3) / 1e12, 1),
                # 157.3 TFLOP/s is the packed-fp32 figure; one v_fma_f32 per lane (this build emits no packed fp32) peaks at half
                "sweep_trail_frac_fp32_fma_peak_78p6": round(trail_flops / (swp["gptq_trail"][0] * 1e-3) / 1e12 / 78.65, 3),
                "finite": bool(torch.isfinite(gu).all())}
            del hess, gu, fws, sws, gx, gw, gout
            torch.cuda.empty_cache()
        out["gptq_one_expert"] = {
            "note": "int4, group 64; the factor of [F,H] serves W1 and W3; wall times include the launch gaps of the "
                    "per-group launches (timed launches carry events, untimed runs are a little faster)",
            "matrices": res,
            "expert_total_ms": round(res["W1/W3 [F,H]"]["hessian_ms"] + res["W1/W3 [F,H]"]["factor_ms_wall"]
                                     + 2 * res["W1/W3 [F,H]"]["sweep_ms_wall"] + res["W2 [H,F]"]["hessian_ms"]
                                     + res["W2 [H,F]"]["factor_ms_wall"] + res["W2 [H,F]"]["sweep_ms_wall"], 1)}

    # ---------------------------------------------------------------- CPU oracle on this host
    if not args.skip_cpu:
        from oracle import dymoe_oracle as O
        def oracle_step():
            ridx, rw, rp, rl = O.route_topk(x_np, wg_np, bias_np, k)
            rimp = O.expert_importance_decode(rp)
            rload = np.bincount(ridx.ravel(), minlength=E).astype(np.int32)
            rbits, _ = O.assign_precision(rimp, rload, cfg.tier_count, cfg.tier_bits)
            experts = []
            for e in range(E):
                b = int(rbits[e])
                if e not in ridx[0]:
                    experts.append({})
                elif b == 16:
                    experts.append({"w": host_w[e]})
                else:
                    experts.append({"q": [O.quantize_pack(m, b) for m in host_w[e]]})
            ob = rbits.copy()
            for e in range(E):
                if e not in ridx[0]:
                    ob[e] = 0
            return ridx, rbits, O.moe_ffn_mixed(x_np, ridx, rw, ob, experts)

        # whole steps, repeated until about 10 s of oracle work have been timed
        t0 = time.perf_counter()
        cpu_steps = 0
        while cpu_steps < 64 and (cpu_steps == 0 or time.perf_counter() - t0 < 10.0):
            ridx, rbits, ref = oracle_step()
            cpu_steps += 1
        cpu_s = time.perf_counter() - t0
        rms = np.sqrt((ref ** 2).mean(axis=1, keepdims=True))
        err = float((np.abs(y_gpu - ref) / rms).max())
        out["cpu_baseline"] = {"value": round(cfg.T * cpu_steps / cpu_s, 4), "unit": "tokens/s", "cores": 1,
                               "kind": "oracle",
                               "sample": "%d full steps of 1 token each (route, importance, assignment, quantize-pack of the active "
                                         "int4 expert, FFN over the 2 active experts), %.1f s in all" % (cpu_steps, cpu_s),
                               "host_cpus": os.cpu_count()}
        out["parity_vs_oracle"] = {"topk_equal": bool(np.array_equal(idx_host, ridx)),
                                   "bits_equal": bool(np.array_equal(bits_host, rbits)),
                                   "ffn_max_err_over_rms_bf16_out": round(err, 5)}
    # ---------------------------------------------------------------- 32-layer stack, experts in host memory
    if args.stack_steps > 0:
        t_stack = time.perf_counter()
        from paper_2603_19172_amd.stack import DecodeStack, HostExpertPool
        L, n_pool = 32, 16
        del stores[1:]
        torch.cuda.empty_cache()
        pool = HostExpertPool(H, F, E, n_pool, lambda i: host_w[i % E] if i < E else
                              synth.expert_weights(synth.scaled(cfg, config_id=50), i % E))
        pool.add_quantised(ctx, dev)
        routers = [bf16(synth.router(synth.scaled(cfg, config_id=100 + l))[0]) for l in range(L)]
        floor = [4 if (l < 4 or l >= L - 4) else 2 for l in range(L)]
        xs = [bf16(synth.activations(synth.scaled(cfg, config_id=200 + s))[0]) for s in range(args.stack_steps)]
        gb = {b: pool.nbytes[b] / 1e9 for b in (16, 4, 2)}
        budget = float(args.stack_budget_gb)
        # one byte budget, spent three ways: bf16 slots that also hold what the device quantiser writes;
        # fixed pools of the three formats (a quarter / half / quarter of the bytes); the library's
        # byte-budget cache, whose blocks change hands between the formats as the demand shifts
        # the paper's "4/2" mode: t_l Critical experts in 4 bits (cosine depth schedule, lambda = 0.5), the rest in 2
        paper_tiers = [(B.depth_schedule(l, L, 0.5, E), E - B.depth_schedule(l, L, 0.5, E)) for l in range(L)]
        all_plans = {
            "literal": ("bf16", int(budget / (gb[16] + gb[4] + gb[2])), "1/3/4 bf16/int4/int2", cfg.tier_count, cfg.tier_bits, floor),
            "pools": ("assigned", {16: int(0.25 * budget / gb[16]), 4: int(0.5 * budget / gb[4]),
                                   2: int(0.25 * budget / gb[2])}, "1/3/4 bf16/int4/int2", cfg.tier_count, cfg.tier_bits, floor),
            "budget": ("assigned", "budget", "1/3/4 bf16/int4/int2", cfg.tier_count, cfg.tier_bits, floor),
            "paper-pools": ("assigned", {4: int(0.75 * budget / gb[4]), 2: int(0.25 * budget / gb[2])},
                            "4/2 with the cosine depth schedule", paper_tiers, (4, 2), None),
            "paper": ("assigned", "budget", "4/2 with the cosine depth schedule", paper_tiers, (4, 2), None)}
        plans = [all_plans[n_.strip()] for n_ in args.stack_plans.split(",") if n_.strip()]
        results = []
        for transfer, slots, tier_name, tcount, tbits, flr in plans:
            # look-ahead off and on under the paper's least-recently-used eviction, then eviction by the layer schedule
            for prefetch, eviction in ((False, "lru"), (True, "lru"), (False, "cyclic")):
                by_budget = slots == "budget"
                stack = DecodeStack(ctx, H, F, E, k, routers, pool, None if by_budget else slots, tcount, tbits,
                                    floor_bits=flr, prefetch=prefetch, transfer=transfer, alpha=0.125, device=dev,
                                    budget_bytes=int(budget * 1e9) if by_budget else None, lookahead="expected",
                                    eviction=eviction)
                for s in range(max(1, args.stack_warmup)):      # warm-up (fills the slots it can)
                    stack.step(xs[s % len(xs)])
                torch.cuda.synchronize()
                stack.stats.clear()
                stack.measure_overlap = True
                t0 = time.perf_counter()
                for s in range(args.stack_steps):
                    stack.step(xs[s])
                torch.cuda.synchronize()
                dt = time.perf_counter() - t0
                ovl = stack.overlap_report()
                stack.close()
                stt = stack.stats
                results.append({"transfer": transfer, "tiers": tier_name, "slots": slots, "prefetch": prefetch,
                                "eviction": eviction,
                                "steps_per_s": round(args.stack_steps / dt, 3),
                                "ms_per_layer": round(dt / args.stack_steps / L * 1e3, 3),
                                "expert_uses": stt["miss"] + stt["promote"] + stt["hit_resident"] + stt["hit_prefetched"],
                                "miss": stt["miss"], "promote": stt["promote"], "hit_resident": stt["hit_resident"],
                                "hit_prefetched": stt["hit_prefetched"], "reused_higher": stt["reused_higher"],
                                "prefetch_issued": stt["prefetch_issued"], "prefetch_wasted": stt["prefetch_wasted"],
                                "prefetch_declined": stt["prefetch_declined"],
                                "predictions_right": round(stack._pred_right / stack._pred_seen, 3) if prefetch else None,
                                "layer_compute_ms": None if stack.layer_ms is None else round(stack.layer_ms, 3),
                                "link_GBps_one_copy": round(stack.link_gbps, 1),
                                "GB_moved_per_step": round(stt["bytes_copied"] / args.stack_steps / 1e9, 2),
                                "host_link_GBps": round(stt["bytes_copied"] / dt / 1e9, 1),
                                "copy_ms_per_step": round(ovl["copy_ms"] / args.stack_steps, 2),
                                "compute_stream_waiting_ms_per_step": round(ovl["stall_ms"] / args.stack_steps, 2),
                                "copy_time_hidden": None if ovl["copy_time_hidden"] is None else round(ovl["copy_time_hidden"], 3)})
                del stack
                torch.cuda.empty_cache()
        # the same stack with every format of every expert resident on the device: one HIP graph per step
        from paper_2603_19172_amd.stack import ResidentDecodeStack
        resident = []
        for tier_name, tcount, tbits, flr in (("1/3/4 bf16/int4/int2", cfg.tier_count, cfg.tier_bits, floor),
                                              ("4/2 with the cosine depth schedule", paper_tiers, (4, 2), None)):
            for graph in (False, True):
                rs = ResidentDecodeStack(ctx, H, F, E, k, routers, pool, tcount, tbits, floor_bits=flr, alpha=0.125,
                                         device=dev, graph=graph)
                for s in range(2):
                    rs.step(xs[s % len(xs)])
                torch.cuda.synchronize()
                n_rs = max(args.stack_steps, 32)
                t0 = time.perf_counter()
                for s in range(n_rs):
                    rs.step(xs[s % len(xs)])
                torch.cuda.synchronize()
                dt = time.perf_counter() - t0
                tr = rs.trace()
                nbytes = sum(pool.nbytes[b] for (_, bts) in tr for b in bts)
                resident.append({"tiers": tier_name, "launch": "hip_graph" if graph else "eager", "steps": n_rs,
                                 "steps_per_s": round(n_rs / dt, 1), "us_per_layer": round(dt / n_rs / L * 1e6, 1),
                                 "weight_GB_read_in_the_last_step": round(nbytes / 1e9, 3),
                                 "GBps_last_step_bytes_at_mean_rate": round(nbytes / (dt / n_rs) / 1e9, 1)})
                del rs
                torch.cuda.empty_cache()
        out["stack_decode_resident"] = {"workload": "the same 32 layers with every expert resident in device memory in every "
                                                    "format its tiers may name: no copies, no host decisions, a step is "
                                                    "128 launches replayed as one HIP graph", "runs": resident}
        out["stack_decode"] = {"workload": "32 Mixtral-shaped layers, 1 token per step, experts in pinned host memory "
                                           "(16 distinct experts shared by the 256 layer-experts), every step a different token; eviction 'lru' is the "
                                           "paper's least-recently-used order, 'cyclic' evicts the expert whose layer comes up last; look-ahead of the next layer's 2 "
                                           "experts on a copy stream of its own, issued when p * min(c, t) >= (1 - p) * c (p share of "
                                           "right predictions, c the copy's time, t a layer's compute time); the 1/3/4 tiers carry "
                                           "an int4 floor in the first and last 4 layers",
                               "device_budget_GB": budget, "steps": args.stack_steps, "warmup_steps": max(1, args.stack_warmup),
                               "host_pool_GB": round(sum(pool.buf[b].numel() for b in pool.buf) / 1e9, 2),
                               "section_wall_s": round(time.perf_counter() - t_stack, 1),
                               "runs": results}
    # the two acceptance figures of the benchmark spec, side by side with what was measured in this run
    pg = out.get("prefill_512", {}).get("grouped_gemm_frac_mfma_bf16_peak")
    out["targets"] = {
        "decode_frac_hbm_on_packed_weights": {"target": 0.70, "kernels_only": roofline_decode["frac"],
                                              "step_level_formats_resident": out["decode_ffn_only"]["frac_hbm"],
                                              "step_level_full_hot_path": out["hot_path_hbm"]["frac_hbm"],
                                              "met": bool(out["decode_ffn_only"]["frac_hbm"] >= 0.70)},
        "prefill_grouped_gemm_frac_mfma_bf16_peak": {"target": 0.50, "measured": pg,
                                                     "met": bool(pg is not None and pg >= 0.50)}}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
