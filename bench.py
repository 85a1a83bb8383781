#!/usr/bin/env python3
"""Benchmark of the POP pruned-FFN hot path on one MI355X.

Workload (the Llama-2-7B-shaped configuration the metric is quoted on): bf16 SwiGLU FFN layers with
d = 4096, m = 11008, synthetic N(0, 0.02^2) weights, Gaussian activations with 0.1 % heavy-tailed outlier
channels; prompt of 512 tokens, then 128 decode steps at batch 1; channel sparsity r = 0.35 with a
candidate band of 0.1 (regions 0.60 / 0.10 / 0.30), plus r = 0.20 and 0.50 as extra lines.

A "step" is one request: prefill partition of the prompt (importance reduction + three-region partition)
on each of `--layers` independent layers, then 128 decode tokens, each running decode-mask + pruned-FFN
on every layer in turn.  Rotating over several independent layers (default 8, 1.5 GB of active weights
per token) keeps the weights out of the 256 MB last-level cache between tokens, as in a real decoder
where one layer's weights are touched once per token; `--layers 1` gives the cache-warm single-layer
number, which is also reported as `warm_us_per_token`.

The reported value is decode microseconds per token per layer, measured with events on the stream the
kernels run on, inside the timed region; all inputs are resident in HBM before timing starts.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402
import torch  # noqa: E402

HBM_PEAK_GBS = 8000.0
PROMPT, DECODE_STEPS = 512, 128
F_CAND = 0.10


def region_fractions(r: float):
    """(f_ret, f_cand) for channel sparsity r with candidate band F_CAND centred on the pruning threshold."""
    return 1.0 - r - F_CAND / 2, F_CAND


def byte_model(d, n_ret, n_cand, k, esize=2):
    """Algorithmic HBM bytes of one decode token on one layer (weights only dominate; vectors included)."""
    n_rc, a = n_ret + n_cand, n_ret + k
    gateup = 2 * n_rc * d * esize + d * esize + 4 * n_rc * 2 + 4 * n_rc
    down = a * d * esize + 4 * a * 2 + 4 * d
    active = 3 * a * d * esize
    return dict(gateup=gateup, down=down, algorithmic=gateup + down, active=active)


class BenchLayer:
    def __init__(self, pop, synth, cfg, layer_id, r_list):
        L = synth.make_layer(cfg, layer_id)
        to_dev = lambda a: torch.from_numpy(a.view(np.int16)).cuda()  # noqa: E731
        self.pop = pop
        self.d, self.m = cfg.d, cfg.m
        wg, wu, wd = to_dev(L.w_gate), to_dev(L.w_up), to_dev(L.w_down)
        self.handle = pop.pop_layer_create(cfg.d, cfg.m, pop.POP_BF16, wg, wu, wd, PROMPT, 1)
        del wg, wu, wd
        self.x_prompt = to_dev(synth.make_activations(L, PROMPT, "prompt", layer_id))
        self.x_decode = to_dev(synth.make_activations(L, DECODE_STEPS, "decode", layer_id))
        self.y = torch.empty(cfg.d, dtype=torch.int16, device="cuda")
        self.host_layer = L

    def close(self):
        self.pop.pop_layer_destroy(self.handle)


def run(args):
    from paper_2602_06822_amd import binding as pop
    from paper_2602_06822_amd import synth

    torch.cuda.set_device(0)
    cfg = synth.CFG2
    lib = pop.raw()
    stream = torch.cuda.current_stream()
    sp = C.c_void_p(stream.cuda_stream)
    if args.other_shapes_only:
        # only the timings of the other workload shapes (for kernel traces of the batched decode kernels)
        print(json.dumps({"other_shapes": time_other_shapes(pop, synth, lib, stream)}))
        return
    layers = [BenchLayer(pop, synth, cfg, i, None) for i in range(args.layers)]
    d, m = cfg.d, cfg.m
    torch.cuda.synchronize()

    def counts(r):
        f_ret, f_cand = region_fractions(r)
        n_ret, n_cand, _ = pop.pop_region_counts(m, f_ret, f_cand)
        return n_ret, n_cand, pop.pop_k_for_ratio(m, r, n_ret, n_cand)

    if args.stack_only:
        # only the 32-layer stack (for a kernel trace of the eager call sequences against the captured graph)
        print(json.dumps({"stack_of_32_layers": time_layer_stack(pop, synth, lib, layers, counts(0.35), 32)}))
        for L in layers:
            L.close()
        return

    def make_calls(r):
        n_ret, n_cand, k = r if isinstance(r, tuple) else counts(r)  # explicit region sizes, or a sparsity
        karr = (C.c_int * 1)(k)
        prefill, decode = [], []
        for L in layers:
            prefill.append((L.handle, C.c_void_p(L.x_prompt.data_ptr()), PROMPT, n_ret, n_cand, None, None, None,
                            None, sp))
            per_tok = []
            for t in range(DECODE_STEPS):
                xt = C.c_void_p(L.x_decode.data_ptr() + t * d * 2)
                yp = C.c_void_p(L.y.data_ptr())
                per_tok.append(((L.handle, xt, 1, karr, None, None, None, None, sp),
                                (L.handle, None, 1, None, 0, yp, pop.POP_BF16, sp),
                                (L.handle, xt, 1, karr, yp, pop.POP_BF16, None, None, None, None, sp)))
            decode.append(per_tok)
        return prefill, decode

    def check(rc):
        if rc != 0:
            raise pop.PopError(rc, "bench")

    def one_request(calls, ev=None, probe=None, single=False):
        prefill, decode = calls
        if ev:
            ev[0].record(stream)
        for a in prefill:
            check(lib.pop_prefill_partition(*a))
        if ev:
            ev[1].record(stream)
        for t in range(DECODE_STEPS):
            for li in range(len(layers)):
                a_mask, a_ffn, a_step = decode[li][t]
                if single:
                    # the whole step in one call (pop_decode_step: the same launches as the two calls)
                    check(lib.pop_decode_step(*a_step))
                elif probe is not None and (t * len(layers) + li) % probe["every"] == 0:
                    e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
                    e0.record(stream)
                    check(lib.pop_decode_mask(*a_mask))
                    e1.record(stream)
                    check(lib.pop_pruned_ffn(*a_ffn))
                    e2.record(stream)
                    probe["events"].append((e0, e1, e2))
                else:
                    check(lib.pop_decode_mask(*a_mask))
                    check(lib.pop_pruned_ffn(*a_ffn))
        if ev:
            ev[2].record(stream)

    def timed(r, steps, warmup, probe_every=None, single=False):
        calls = make_calls(r)
        for _ in range(warmup):
            one_request(calls, single=single)
        torch.cuda.synchronize()
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
        probe = dict(every=probe_every, events=[]) if probe_every else None
        t0 = time.perf_counter()
        for s in range(steps):
            one_request(calls, evs[s], probe, single)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        for L in layers:  # raises if a bounded in-kernel wait expired during the last request
            pop.pop_layer_sync_status(L.handle)
        prefill_ms = sum(e[0].elapsed_time(e[1]) for e in evs)
        decode_ms = sum(e[1].elapsed_time(e[2]) for e in evs)
        n_tok_layers = steps * DECODE_STEPS * len(layers)
        out = dict(wall_s=wall, ms_per_step=1e3 * wall / steps,
                   decode_us_per_token=1e3 * decode_ms / n_tok_layers,
                   prefill_us_per_layer=1e3 * prefill_ms / (steps * len(layers)))
        if probe:
            mk = [a.elapsed_time(b) * 1e3 for a, b, _ in probe["events"]]
            dn = [b.elapsed_time(c) * 1e3 for _, b, c in probe["events"]]
            out["probe_mask_us"] = float(np.mean(mk))
            out["probe_ffn_us"] = float(np.mean(dn))
            out["probe_n"] = len(mk)
            tot = np.asarray(mk) + np.asarray(dn)
            out["probe_token_us_p10_p50_p90"] = [round(float(np.percentile(tot, q)), 3) for q in (10, 50, 90)]
        return out

    r_main = 0.35
    # the timed region proper: every step through the one-call entry point (pop_decode_step: the fused kernel and the
    # small kernel that sums its partial outputs), nothing between the calls.  A separate, shorter pass brackets every
    # n-th step's two calls with events (which costs that step its overlap with the next launch) for the percentiles.
    if args.variant2_only:
        # only the step that re-scores every channel (Variant 2: top-k over all m keys; batch-general kernels), for a
        # kernel trace of its launches
        cnt = pop.pop_strategy_counts(pop.POP_STRATEGY_RESCORE_ALL, m, r_main, 0.0)
        t = timed(cnt, max(1, args.steps // 4), 1)["decode_us_per_token"]
        print(json.dumps({"variant2_rescore_all": dict(n_ret=cnt[0], n_cand=cnt[1], k=cnt[2], us_per_token=round(t, 3))}))
        for L in layers:
            L.close()
        return
    main = timed(r_main, args.steps, args.warmup, single=True)
    probed = timed(r_main, max(1, args.steps // 4), 1, probe_every=args.probe_every)
    for key in ("probe_mask_us", "probe_ffn_us", "probe_token_us_p10_p50_p90"):
        main[key] = probed.get(key)
    main["two_calls_us_per_token"] = probed["decode_us_per_token"]
    n_ret, n_cand, k = counts(r_main)
    bm = byte_model(d, n_ret, n_cand, k)
    us = main["decode_us_per_token"]

    extra = {}
    if not args.quick:
        for r in (0.20, 0.50):
            t = timed(r, max(1, args.steps // 2), 1)
            nr, nc, kk = counts(r)
            b = byte_model(d, nr, nc, kk)
            extra[f"r={r:.2f}"] = dict(us_per_token=round(t["decode_us_per_token"], 3),
                                       active_GBps=round(b["active"] / t["decode_us_per_token"] / 1e3, 1),
                                       frac_of_peak_active=round(b["active"] / t["decode_us_per_token"] / 1e3 / HBM_PEAK_GBS, 4))
    # The paper's ablation of the decode strategy (Sec. 5, trade-off table), in time and bytes on this shape: a
    # static prefill mask (Variant 1: no candidates), POP with candidate bands of 5 / 10 / 20 % of the channels,
    # and re-scoring every channel at each step (Variant 2: every channel a candidate); all at r = 0.35.
    ablation = None
    if not args.quick:
        rows = [("dense", (m, 0, 0)),
                ("variant1_static_mask", pop.pop_strategy_counts(pop.POP_STRATEGY_STATIC_MASK, m, r_main, 0.0))]
        for g in (0.05, 0.10, 0.20):
            rows.append((f"pop_gamma_{g:.2f}", pop.pop_strategy_counts(pop.POP_STRATEGY_POP, m, r_main, g)))
        rows.append(("variant2_rescore_all", pop.pop_strategy_counts(pop.POP_STRATEGY_RESCORE_ALL, m, r_main, 0.0)))
        ablation = {}
        for name, cnt in rows:
            t = timed(cnt, 1, 1)["decode_us_per_token"]
            ablation[name] = dict(n_ret=cnt[0], n_cand=cnt[1], k=cnt[2], us_per_token=round(t, 3),
                                  MB_per_token=round(byte_model(d, *cnt)["algorithmic"] / 1e6, 2))
        base_t = ablation["variant1_static_mask"]["us_per_token"]
        base_b = ablation["variant1_static_mask"]["MB_per_token"]
        for name, row in ablation.items():
            row["overhead_vs_static_mask_pct"] = dict(time=round(100 * (row["us_per_token"] / base_t - 1), 2),
                                                      bytes=round(100 * (row["MB_per_token"] / base_b - 1), 2))
    # cache-warm single-layer figure (same layer every token)
    warm = None
    if not args.quick and len(layers) > 1:
        keep = layers
        layers = layers[:1]
        warm = timed(r_main, max(1, args.steps // 2), 1)["decode_us_per_token"]
        layers = keep
    # the same step as its two calls (pop_decode_mask, pop_pruned_ffn), without probes, for comparison
    single = None
    if not args.quick:
        single = timed(r_main, max(1, args.steps // 2), 1)["decode_us_per_token"]

    # the prefilling stage with its output (pop_prefill_forward: contraction that keeps H, partition, prefill mask,
    # gathered columns, down-projection GEMM over the active channels), rotated over the layers
    forward = None
    if not args.quick or args.forward:
        yp = torch.empty((PROMPT, d), dtype=torch.int16, device="cuda")
        fcalls = [(L.handle, C.c_void_p(L.x_prompt.data_ptr()), PROMPT, n_ret, n_cand, k, C.c_void_p(yp.data_ptr()),
                   pop.POP_BF16, None, None, None, None, None, sp) for L in layers]
        for a in fcalls:
            check(lib.pop_prefill_forward(*a))
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 4
        e0.record(stream)
        for _ in range(reps):
            for a in fcalls:
                check(lib.pop_prefill_forward(*a))
        e1.record(stream)
        torch.cuda.synchronize()
        f_us = 1e3 * e0.elapsed_time(e1) / (reps * len(layers))
        f_flop = 4.0 * PROMPT * m * d + 2.0 * PROMPT * (n_ret + k) * d
        forward = dict(us_per_layer=round(f_us, 2), flop=f_flop, TFLOPs=round(f_flop / f_us / 1e6, 1),
                       frac_of_bf16_mfma_peak=round(f_flop / f_us / 1e6 / 2500.0, 4),
                       note="whole call: both GEMMs, partition, mask, gather and the small kernels between them")
        del yp

    # configs[2]: a 32-layer stack of this layer shape, one token through all layers (each layer its own weights,
    # partition and input), as eager calls and as one captured HIP graph of the 32 steps
    stack = None
    if not args.quick:
        stack = time_layer_stack(pop, synth, lib, layers, counts(r_main), 32)

    # duration of the dominant kernel: the same launches as in the timed region (every token of every layer, layers
    # rotated), issued back to back without the tail kernel between them, bracketed by two events on the launch
    # stream; consecutive launches abut, as in the dispatch records of a kernel trace
    def kernel_only(which):
        pre, calls = make_calls(r_main)
        for a in pre:
            check(lib.pop_prefill_partition(*a))
        def sweep():
            for t in range(DECODE_STEPS):
                for li in range(len(layers)):
                    a_mask, a_ffn, _ = calls[li][t]
                    check(lib.pop_decode_mask(*a_mask) if which == "mask" else lib.pop_pruned_ffn(*a_ffn))
        if which == "ffn":  # the tail needs a step to finish: one per layer, then the tail alone repeatedly
            for li in range(len(layers)):
                check(lib.pop_decode_mask(*calls[li][0][0]))
        sweep()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        sweep()
        e1.record(stream)
        torch.cuda.synchronize()
        return 1e3 * e0.elapsed_time(e1) / (DECODE_STEPS * len(layers))

    # The box's own read ceiling for these bytes: bare read kernels (no arithmetic) launched exactly like the fused
    # kernel above, back to back over the rotated layers: a contiguous read of the step's algorithmic byte count, and
    # a gathered read of exactly the step's rows out of each layer's channel-major weights.
    def read_legs():
        sink = torch.zeros(1, dtype=torch.int32, device="cuda")
        nbytes = bm["algorithmic"] // 16 * 16
        bufs = [torch.ones(nbytes, dtype=torch.uint8, device="cuda") for _ in layers]
        n_wg = torch.cuda.get_device_properties(0).multi_processor_count
        out = {}
        for name in ("bare_read_us", "gathered_read_us"):
            def sweep():
                for t in range(DECODE_STEPS):
                    for li, L in enumerate(layers):
                        if name == "bare_read_us":
                            check(lib.pop_probe_read(C.c_void_p(bufs[li].data_ptr()), C.c_size_t(nbytes), n_wg,
                                                     C.c_void_p(sink.data_ptr()), sp))
                        else:
                            check(lib.pop_probe_step_read(L.handle, k, n_wg, C.c_void_p(sink.data_ptr()), sp))
            sweep()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            sweep()
            e1.record(stream)
            torch.cuda.synchronize()
            out[name] = 1e3 * e0.elapsed_time(e1) / (DECODE_STEPS * len(layers))
        del bufs
        return out

    fused_us = kernel_only("mask")
    tail_us = kernel_only("ffn")
    reads = read_legs()
    for L in layers:  # no in-kernel bounded wait may have expired anywhere above
        pop.pop_layer_sync_status(L.handle)
    roofline = None
    if fused_us:
        # dominant kernel: the fused decode kernel behind pop_decode_mask (B = 1).  It streams every weight byte of
        # the step (gate+up rows of retained and candidate channels, down columns of retained and selected ones);
        # pop_pruned_ffn only reduces the per-workgroup partial sums.
        ach = bm["algorithmic"] / fused_us / 1e3  # GB/s
        roofline = dict(bound="hbm", kernel="decode_fused_kernel (pop_decode_mask, B=1)",
                        achieved=round(ach, 1), peak=HBM_PEAK_GBS, unit="GB/s", frac=round(ach / HBM_PEAK_GBS, 4),
                        traffic=measured_traffic(), algorithmic_bytes_per_launch=bm["algorithmic"],
                        avg_launch_us=round(fused_us, 3), tail_kernel_us=round(tail_us, 3),
                        in_sequence_probe_us=[round(main.get("probe_mask_us") or 0.0, 3),
                                              round(main.get("probe_ffn_us") or 0.0, 3)],
                        bare_read_us=round(reads["bare_read_us"], 3),
                        gathered_read_us=round(reads["gathered_read_us"], 3),
                        token_us_over_gathered_read=round(us / reads["gathered_read_us"], 4),
                        traffic_source="profiles/decode_fused_cfg2_r35_hbm_traffic.txt (committed rocprofv3 "
                                       "FETCH_SIZE/WRITE_SIZE summary of this command; not read live in this run)",
                        note="avg_launch_us: back-to-back launches of the kernel between two events; "
                             "in_sequence_probe_us: fused and tail launch bracketed one by one inside the timed "
                             "region (adds the event and launch gaps); bare_read_us / gathered_read_us: read-only "
                             "kernels (pop_probe_read: the algorithmic byte count, contiguous; pop_probe_step_read: "
                             "exactly the step's weight rows) launched the same way over the same rotated layers")

    # the same workload under the input-side reading of the importance (selection first, then the forward pass over
    # retained + selected channels; separate launches, no fused kernel); last use of these layers
    input_side = None
    if not args.quick:
        for L in layers:
            pop.pop_layer_set_importance(L.handle, pop.POP_IMPORTANCE_INPUT_SIDE)
        t = timed(r_main, 1, 1, single=True)
        input_side = dict(decode_us_per_token=round(t["decode_us_per_token"], 3),
                          prefill_us_per_layer=round(t["prefill_us_per_layer"], 2),
                          MB_per_token=round((3 * (n_ret + k) + 2 * (n_cand - k)) * d * 2 / 1e6, 2))

    other_configs = None
    host_layer0 = layers[0].host_layer
    if not args.quick:
        for L in layers:
            L.close()
        layers = []
        torch.cuda.empty_cache()
        other_configs = time_other_shapes(pop, synth, lib, stream)

    cpu = None if args.no_cpu_baseline else cpu_baseline(synth, host_layer0, n_ret, n_cand, k, args.cpu_tokens)

    # the box's own copy bandwidth (plain device-to-device copy of 1 GiB, bytes read + written per second), as a
    # second yardstick next to the published peak
    copy_gbps = None
    if not args.quick:
        ca = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        cb = torch.empty_like(ca)
        for _ in range(2):
            cb.copy_(ca)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(5):
            cb.copy_(ca)
        e1.record(stream)
        torch.cuda.synchronize()
        copy_gbps = 5 * 2.0 * (1 << 30) / (e0.elapsed_time(e1) * 1e-3) / 1e9
        del ca, cb
        if roofline:
            roofline["measured_copy_GBps"] = round(copy_gbps, 1)
            roofline["frac_of_measured_copy"] = round(roofline["achieved"] / copy_gbps, 4)

    if args.pmc_calibration:
        # a plain device-to-device copy of known size, for scaling the rocprofv3 FETCH_SIZE / WRITE_SIZE counters
        a = torch.zeros(256 << 20, dtype=torch.uint8, device="cuda")
        bb = torch.empty_like(a)
        for _ in range(3):
            bb.copy_(a)
        torch.cuda.synchronize()

    for L in layers:
        L.close()

    result = {
        "metric": "pruned-FFN decode us/token (per layer, Llama-2-7B shape, 1 GPU)",
        "value": round(us, 3),
        "unit": "us/token",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(main["ms_per_step"], 3),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"configs[1]: Llama-2-7B-shaped FFN layer, bf16, d=4096 m=11008, prompt {PROMPT} + 128 "
                               "decode steps at batch 1, channel sparsity 0.35 (regions .60/.10/.30, k=550)",
                   "layers_rotated": args.layers,
                   "step": "prefill partition + 128 decode tokens (pop_decode_step) on every layer",
                   "n_ret": n_ret, "n_cand": n_cand, "k": k},
        "tokens_per_s_per_layer": round(1e6 / us, 1),
        "prefill_us_per_layer": round(main["prefill_us_per_layer"], 2),
        "prefill_TFLOPs_whole_call": round(4.0 * PROMPT * m * d / main["prefill_us_per_layer"] / 1e6, 1),
        "probed_token_us_p10_p50_p90": main.get("probe_token_us_p10_p50_p90"),
        "two_calls_with_probes_us_per_token": round(main["two_calls_us_per_token"], 3),
        "prefill_forward": forward,
        "stack_of_32_layers": stack,
        "input_side_importance_reading": input_side,
        "active_GBps": round(bm["active"] / us / 1e3, 1),
        "algorithmic_GBps": round(bm["algorithmic"] / us / 1e3, 1),
        "frac_of_peak_active_bytes": round(bm["active"] / us / 1e3 / HBM_PEAK_GBS, 4),
        "warm_us_per_token": None if warm is None else round(warm, 3),
        "other_sparsities": extra,
        "two_calls_us_per_token": None if single is None else round(single, 3),
        "ablation_r0.35": ablation,
        "other_shapes": other_configs,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(result))


def time_layer_stack(pop, synth, lib, bench_layers, cnt, n_layers):
    """One decode token through n_layers independent layers of the benchmark shape (device copies of the bench
    layers' weights, each with its own partition and its own inputs): per-token time of the eager call sequence
    (two calls per layer), of the one-call steps, and of one captured graph of the one-call steps."""
    n_ret, n_cand, k = cnt
    cfg = bench_layers[0].host_layer.cfg
    d = cfg.d
    to_dev = lambda a: torch.from_numpy(a.view(np.int16)).cuda()  # noqa: E731
    hs, xs = [], []
    t_stack = 2048  # configs[2]'s prompt length (it shapes the partitions; the decode steps do not depend on it)
    prompts = [to_dev(synth.make_activations(src.host_layer, t_stack, "prompt_stack", i))
               for i, src in enumerate(bench_layers)]
    for i in range(n_layers):
        src = bench_layers[i % len(bench_layers)]
        L = src.host_layer
        h = pop.pop_layer_create(cfg.d, cfg.m, pop.POP_BF16, to_dev(L.w_gate), to_dev(L.w_up), to_dev(L.w_down),
                                 t_stack, 1)
        pop.pop_prefill_partition(h, prompts[i % len(bench_layers)], t_stack, n_ret, n_cand)
        hs.append(h)
        xs.append(src.x_decode[i // len(bench_layers)].clone())
    y = torch.empty(d, dtype=torch.int16, device="cuda")
    karr = (C.c_int * 1)(k)
    side = torch.cuda.Stream()
    out = {"layers": n_layers, "prompt_tokens": t_stack}
    torch.cuda.synchronize()

    def token(sp, single):
        for h, x in zip(hs, xs):
            if single:
                rc = lib.pop_decode_step(h, C.c_void_p(x.data_ptr()), 1, karr, C.c_void_p(y.data_ptr()), pop.POP_BF16,
                                         None, None, None, None, sp)
            else:
                rc = lib.pop_decode_mask(h, C.c_void_p(x.data_ptr()), 1, karr, None, None, None, None, sp)
                rc = rc or lib.pop_pruned_ffn(h, None, 1, None, 0, C.c_void_p(y.data_ptr()), pop.POP_BF16, sp)
            if rc:
                raise pop.PopError(rc, "bench stack")

    def timeit(fn, reps=8):
        fn()
        side.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(side)
        for _ in range(reps):
            fn()
        e1.record(side)
        side.synchronize()
        return 1e3 * e0.elapsed_time(e1) / reps

    with torch.cuda.stream(side):
        sp = C.c_void_p(side.cuda_stream)
        out["eager_two_calls_us_per_token"] = round(timeit(lambda: token(sp, False)), 1)
        out["eager_one_call_us_per_token"] = round(timeit(lambda: token(sp, True)), 1)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            token(C.c_void_p(torch.cuda.current_stream().cuda_stream), True)
        out["graph_us_per_token"] = round(timeit(g.replay), 1)
        for h in hs:
            if pop.raw().pop_layer_sync_status(h, sp) != 0:
                raise RuntimeError("a bounded wait expired during the stack benchmark")
    del g
    for h in hs:
        pop.pop_layer_destroy(h)
    torch.cuda.empty_cache()
    return out


def time_other_shapes(pop, synth, lib, stream):
    """Decode step time of the other workload shapes (the parity tests cover them; these are the timings):
    Llama-2-13B-shaped layer at batch 1, 4 and 8 (sparsity .50) and one Mixtral-shaped expert at batch 1 (.35).
    Four independent layers rotated per step (cache-cold weights), short prompt for the partition."""
    sp = C.c_void_p(stream.cuda_stream)
    out = {}
    for name, cfg, r, batches in (("llama2_13b_layer_r0.50", synth.CFG4, 0.50, (1, 4, 8)),
                                  ("mixtral_expert_r0.35", synth.CFG5, 0.35, (1,))):
        n_layers, T = 4, 128
        to_dev = lambda a: torch.from_numpy(a.view(np.int16)).cuda()  # noqa: E731
        n_ret, n_cand, _ = pop.pop_region_counts(cfg.m, *region_fractions(r))
        k = pop.pop_k_for_ratio(cfg.m, r, n_ret, n_cand)
        hs, xds, host_layers = [], [], []
        for i in range(n_layers):
            L = synth.make_layer(cfg, i)
            h = pop.pop_layer_create(cfg.d, cfg.m, pop.POP_BF16, to_dev(L.w_gate), to_dev(L.w_up), to_dev(L.w_down),
                                     T, max(batches))
            pop.pop_prefill_partition(h, to_dev(synth.make_activations(L, T, "prompt", i)), T, n_ret, n_cand)
            hs.append(h)
            xds.append(to_dev(synth.make_activations(L, 64, "decode", i)))
            host_layers.append(L)
        bm = byte_model(cfg.d, n_ret, n_cand, k)
        res = {}
        for B in batches:
            y = torch.empty(B * cfg.d, dtype=torch.int16, device="cuda")
            karr = (C.c_int * B)(*([k] * B))
            steps = 64 // B

            def loop():
                for t in range(steps):
                    for h, xd in zip(hs, xds):
                        xt = C.c_void_p(xd.data_ptr() + t * B * cfg.d * 2)
                        rc = lib.pop_decode_mask(h, xt, B, karr, None, None, None, None, sp)
                        rc = rc or lib.pop_pruned_ffn(h, None, B, None, 0, C.c_void_p(y.data_ptr()), pop.POP_BF16, sp)
                        if rc:
                            raise pop.PopError(rc, "bench")
            loop()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            loop()
            loop()
            e1.record(stream)
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / (2 * steps * n_layers)
            # bytes the step really streams: gate+up rows of retained and candidate channels, down rows of the
            # retained channels and of the union of the B selections (data-dependent; taken from one step's masks)
            mk = torch.empty((B, cfg.m), dtype=torch.uint8, device="cuda")
            rc = lib.pop_decode_mask(hs[0], C.c_void_p(xds[0].data_ptr()), B, karr, None, C.c_void_p(mk.data_ptr()),
                                     None, None, sp)
            if rc:
                raise pop.PopError(rc, "bench")
            torch.cuda.synchronize()
            union = int(mk.any(dim=0).sum().item())
            streamed = (2 * (n_ret + n_cand) + union) * cfg.d * 2
            res[f"B={B}"] = dict(us_per_step=round(us, 2), us_per_token=round(us / B, 2),
                                 tokens_per_s=round(1e6 * B / us, 1),
                                 active_GBps_one_sequence=round(bm["active"] / us / 1e3, 1),
                                 union_channels=union, MB_streamed=round(streamed / 1e6, 2),
                                 streamed_GBps=round(streamed / us / 1e3, 1))
        # The whole workload the shape stands for, per token: configs[3] is a stack of 40 such layers (each with its
        # own weights - device copies of the four above -, partition and input), configs[4] a layer of 8 experts of
        # which every token runs 2 (the router is harness-side; here a seeded draw).
        n_units = 40 if cfg is synth.CFG4 else 8
        units = list(hs)
        for i in range(n_layers, n_units):
            L = host_layers[i % n_layers]
            h = pop.pop_layer_create(cfg.d, cfg.m, pop.POP_BF16, to_dev(L.w_gate), to_dev(L.w_up), to_dev(L.w_down),
                                     T, max(batches))
            pop.pop_prefill_partition(h, to_dev(synth.make_activations(L, T, "prompt", i)), T, n_ret, n_cand)
            units.append(h)
        del host_layers

        def time_tokens(token, reps):
            token(0)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for t in range(reps):
                token(t + 1)
            e1.record(stream)
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e3 / reps

        def one_step(h, xd, t, B, karr, y):
            xt = C.c_void_p(xd.data_ptr() + (t % (64 // B)) * B * cfg.d * 2)
            rc = lib.pop_decode_step(h, xt, B, karr, C.c_void_p(y.data_ptr()), pop.POP_BF16, None, None, None, None, sp)
            if rc:
                raise pop.PopError(rc, "bench")

        if cfg is synth.CFG4:
            stack = {"layers": n_units}
            for B in batches:
                y = torch.empty(B * cfg.d, dtype=torch.int16, device="cuda")
                karr = (C.c_int * B)(*([k] * B))
                us = time_tokens(lambda t: [one_step(h, xds[i % n_layers], t, B, karr, y) for i, h in enumerate(units)], 6)
                stack[f"B={B}"] = dict(us_per_step=round(us, 1), us_per_token=round(us / B, 1))
            res["stack_of_40_layers"] = stack
        else:
            y = torch.empty(cfg.d, dtype=torch.int16, device="cuda")
            karr = (C.c_int * 1)(k)
            draw = np.random.default_rng(20260206)
            routes = [draw.choice(n_units, size=2, replace=False) for _ in range(65)]
            us = time_tokens(lambda t: [one_step(units[e], xds[e % n_layers], t, 1, karr, y) for e in routes[t]], 64)
            res["moe_layer_8_experts_top2"] = dict(us_per_token=round(us, 2), experts_per_token=2,
                                                   note="two expert steps per token; router harness-side, not timed")
        for h in units:
            pop.pop_layer_destroy(h)
        torch.cuda.empty_cache()
        out[name] = dict(d=cfg.d, m=cfg.m, n_ret=n_ret, n_cand=n_cand, k=k, layers_rotated=n_layers, **res)
    return out


def measured_traffic():
    """HBM bytes per launch of the fused kernel from the committed rocprofv3 counter summary, if present."""
    path = os.path.join(ROOT, "profiles", "decode_fused_cfg2_r35_hbm_traffic.txt")
    try:
        for ln in open(path):
            if ln.startswith("traffic_bytes_per_launch:"):
                return int(float(ln.split(":", 1)[1]))
    except OSError:
        pass
    return None


def cpu_baseline(synth, L, n_ret, n_cand, k, n_tokens, n_prompt=64):
    """The oracle (double precision, as it stands) timed on the host cores: decode steps of one layer for n_tokens
    tokens, and the prefilling stage (hidden activations of all channels, importance, partition) for the first
    n_prompt prompt tokens."""
    from oracle import pop_oracle as oracle
    flags = oracle.use_timed_build()  # the same source, compiled -O3 -march=native for the timed leg
    region, ret, cand = oracle.partition(synth.make_scores(L.cfg.m, "cpu_baseline_scores", "none"), n_ret, n_cand)
    xt = synth.make_activations(L, n_tokens, "decode")
    oracle.decode(xt[0], L.w_gate, L.w_up, L.w_down, L.cfg.dtype, region, cand, k)  # warm the pages
    t0 = time.perf_counter()
    for t in range(n_tokens):
        oracle.decode(xt[t], L.w_gate, L.w_up, L.w_down, L.cfg.dtype, region, cand, k)
    dt = time.perf_counter() - t0
    xp = synth.make_activations(L, n_prompt, "prompt")
    t0 = time.perf_counter()
    oracle.prefill(xp, L.w_gate, L.w_up, L.w_down, L.cfg.dtype, n_ret, n_cand)
    dp = time.perf_counter() - t0
    return {"value": round(1e6 * dt / n_tokens, 1), "unit": "us/token", "cores": oracle.num_threads(), "kind": "oracle",
            "compiler_flags": " ".join(flags),
            "sample": f"{n_tokens} decode tokens of one layer (pass 1 over retained+candidate channels, re-score, "
                      f"top-k, down projection), same shape and sparsity; prefill timed apart",
            "prefill_us_per_prompt_token": round(1e6 * dp / n_prompt, 1),
            "prefill_sample": f"prefilling stage of one layer on the first {n_prompt} of the {PROMPT} prompt tokens"}


def main():
    global PROMPT
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=8)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--layers", type=int, default=8, help="independent layers rotated per token (cache-cold weights)")
    ap.add_argument("--probe-every", type=int, default=8, help="bracket every n-th decode call pair with events")
    ap.add_argument("--cpu-tokens", type=int, default=2048)
    ap.add_argument("--prompt", type=int, default=PROMPT,
                    help="prompt length of the prefill legs (512 = the workload; 2048 = the 32-layer configuration's)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pmc-calibration", action="store_true", help="also run three 256 MiB device copies")
    ap.add_argument("--other-shapes-only", action="store_true",
                    help="run only the 13B-shaped (B = 1, 4, 8) and Mixtral-expert timings")
    ap.add_argument("--variant2-only", action="store_true",
                    help="run only the decode step that re-scores all channels (ablation Variant 2)")
    ap.add_argument("--stack-only", action="store_true",
                    help="run only the 32-layer stack: eager two-call steps, eager one-call steps, captured graph")
    ap.add_argument("--forward", action="store_true", help="with --quick: keep the prefill-forward section")
    ap.add_argument("--quick", action="store_true", help="main line only: skip other sparsities and the warm figure")
    args = ap.parse_args()
    PROMPT = args.prompt
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only; --gpus must be 1 (nothing here shards across GPUs)")
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    run(args)


if __name__ == "__main__":
    main()
