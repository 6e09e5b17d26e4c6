#!/usr/bin/env python3
"""Benchmark of the quantized LoRA linear layer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

A step is one forward plus one backward of the whole hot path (all kernels the C ABI launches) on the
LLaMA-7B q_proj workload: K = N = 4096, M = 2048 tokens, INT4 codes, group size 128, LoRA r = 8, fp16.
Inputs are synthetic, seeded, and resident in HBM before the timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_F16_TFLOPS = 2516.6   # 256 CU x 4096 flop/clk/CU x 2.4 GHz, dense fp16/bf16
PEAK_HBM_GBPS = 8000.0
# HBM bytes per launch of the two GEMM kernels on the headline workload, from rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE runs of this script, scaled by a 1 GiB copy in the same runs (profiles/qgemm_c2_hbm_traffic.md).
EVENT_EVERY = 5
GEMM_TRAFFIC_BYTES = {"fwd": 86.5e6, "bwd": 88.6e6}


def _mean(v):
    return sum(v) / len(v)


def run_headline(inp, steps: int, warmup: int):
    import torch
    from paper_2306_08162_amd import binding as ql
    from paper_2306_08162_amd.device import DeviceLayer
    from paper_2306_08162_amd.hiprt import Event

    cfg = inp.cfg
    layer = DeviceLayer(inp, "cuda:0")
    stream = torch.cuda.current_stream().cuda_stream or None

    for _ in range(warmup):
        layer.forward()
        layer.backward()
    torch.cuda.synchronize()

    # The GEMM kernels are timed with HIP events inside the timed region, on every EVENT_EVERY-th step only: an event
    # record costs a few microseconds of GPU time, which would otherwise weigh on every step of the measured loop.
    # A pair of events around one kernel also measures the latency of dispatching that kernel behind an event (3-5 us
    # here), which an untimed pass does not pay: there the GEMM follows the adapter kernel t = x A^T (u = dY B).  So the
    # sampled steps take turns with three spans: the GEMM alone -- an upper bound of the kernel's duration, the figure
    # the roofline is priced with --, adapter kernel + GEMM, and adapter kernel alone; the difference of the last two
    # (a lower bound: the event behind the lone adapter kernel waits for that kernel's end-of-kernel write-back, which
    # the GEMM's start overlaps) is reported beside it.  The profiler's kernel durations lie between the two.
    sampled = [i for i in range(steps) if i % EVENT_EVERY == 0]
    ev = {i: [Event() for _ in range(4)] for i in sampled}
    span_of = {i: n % 3 for n, i in enumerate(sampled)}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        if i in ev:
            ql.qlora_profile_gemm_span(span_of[i])
            ql.qlora_profile_gemm(ev[i][0].handle, ev[i][1].handle)
            layer.forward(stream=stream or 0)
            ql.qlora_profile_gemm(ev[i][2].handle, ev[i][3].handle)
            layer.backward(stream=stream or 0)
            ql.qlora_profile_gemm(None, None)
            ql.qlora_profile_gemm_span(0)
        else:
            layer.forward(stream=stream or 0)
            layer.backward(stream=stream or 0)
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    ms_per_step = (t1 - t0) * 1e3 / steps
    by_span = {sp: [e for i, e in ev.items() if span_of[i] == sp] for sp in range(3)}
    fwd = {sp: _mean([e[0].elapsed_ms(e[1]) for e in es]) if es else None for sp, es in by_span.items()}
    bwd = {sp: _mean([e[2].elapsed_ms(e[3]) for e in es]) if es else None for sp, es in by_span.items()}
    fwd_ms, bwd_ms = fwd[0], bwd[0]
    diff_ms = None
    if fwd[1] is not None and fwd[2] is not None:
        diff_ms = {"fwd": fwd[1] - fwd[2], "bwd": bwd[1] - bwd[2]}
    return cfg, layer, ms_per_step, fwd_ms, bwd_ms, diff_ms


def _graph_time(launch_all, iters: int):
    """Capture `launch_all` (a burst of library calls) into a HIP graph and time its replays with HIP events.

    The passes are only a few microseconds long, so issuing them from Python one by one would measure the
    interpreter; a captured graph replays them back to back.  The library records no memsets, so the replays are safe.
    """
    import torch
    from paper_2306_08162_amd.hiprt import Event

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        launch_all()                      # warm-up outside capture (first touch of every buffer)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        launch_all()
    graph.replay()
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream().cuda_stream or None
    e0, e1 = Event(), Event()
    e0.record(stream)
    for _ in range(iters):
        graph.replay()
    e1.record(stream)
    e1.synchronize()
    return e0.elapsed_ms(e1) * 1e3 / iters       # microseconds per replay


def run_small_m(M: int = 16, iters: int = 5, headline_layer: bool = True, bit_widths=(2, 8), sibling_calls: bool = True):
    """Packed-weight GB/s at M tokens.

    Every measured burst walks a pool of distinct weight sets larger than 1 GB (the last-level cache is 256 MB),
    forward over the whole pool and backward over the whole pool, so each pass streams its weights from HBM.
    Reported: the headline layer's weights (INT4 q_proj) and one LLaMA-7B decoder block (seven projections) at
    INT2 and INT8.  GB/s counts weight-side bytes only (packed codes + scales + zero-points).
    """
    import torch
    from paper_2306_08162_amd import binding as ql
    from paper_2306_08162_amd import workloads as wl
    from paper_2306_08162_amd.device import DeviceLayer, DeviceSiblings

    def pool_of(layers, target_bytes):
        """Clones of the layers' weight buffers (distinct addresses) until the pool exceeds target_bytes."""
        per_set = sum(l.cfg.weight_side_bytes for l in layers)
        n_sets = 1 + target_bytes // per_set
        sets = []
        for i in range(n_sets):
            sets.append([(l, l.packed if i == 0 else l.packed.clone(), l.scales if i == 0 else l.scales.clone(),
                          l.zeros if i == 0 else l.zeros.clone()) for l in layers])
        return sets, per_set

    def measure(layers, label, groups=None):
        """groups: lists of indices into `layers` that are called together through the sibling entry points
        (projections reading the same x); None: one call per layer."""
        sets, per_set = pool_of(layers, 1 << 30)
        out = {"weight_side_bytes_per_set": per_set, "pool_sets": len(sets)}
        calls = layers if groups is None else [layers[g[0]] if len(g) == 1 else DeviceSiblings([layers[i] for i in g])
                                               for g in groups]

        def sweep(which):
            for st in sets:
                for l, pk, sc, zr in st:
                    l.packed, l.scales, l.zeros = pk, sc, zr
                for c in calls:
                    (c.forward if which == "fwd" else c.backward)()

        total = 0.0
        for which in ("fwd", "bwd"):
            us = _graph_time(lambda: sweep(which), iters) / len(sets)
            total += us
            out[which] = {"us_per_set": round(us, 2), "packed_weight_GBps": round(per_set / us * 1e-3, 1)}
        out["fwd_bwd_packed_weight_GBps"] = round(2 * per_set / total * 1e-3, 1)
        out["frac_of_hbm_peak"] = round(out["fwd_bwd_packed_weight_GBps"] / PEAK_HBM_GBPS, 4)
        if groups is None:
            # The floor of this regime: one launch per projection of a kernel that only reads the projection's packed
            # words (16-byte loads over the whole chip, an exclusive-or, nothing else), over the same pool.
            words = torch.empty(ql.STREAM_PROBE_WORDS, dtype=torch.int32, device="cuda:0")

            def probe():
                for st in sets:
                    for l, pk, sc, zr in st:
                        ql.qlora_stream_probe(pk, pk.numel() * pk.element_size(), words, check=False)

            packed_bytes = sum(pk.numel() * pk.element_size() for _, pk, _, _ in sets[0])
            us = _graph_time(probe, iters) / len(sets)
            out["stream_only_floor"] = {"us_per_set": round(us, 2), "packed_GBps": round(packed_bytes / us * 1e-3, 1),
                                        "what": "one read-only launch per projection over its packed words"}
        return label, out

    results = {}
    if headline_layer:
        q4 = DeviceLayer(wl.make_inputs(wl.config2().with_tokens(M)), "cuda:0")
        k, v = measure([q4], "q_proj_int4")
        results[k] = v
        del q4
    for bits in bit_widths:
        cfgs = wl.config5(bits, M)
        by_shape = {}
        layers = []
        for c in cfgs:
            key = (c.K, c.N)
            if key not in by_shape:
                by_shape[key] = wl.make_inputs(c)
            inp = by_shape[key]
            layers.append(DeviceLayer(wl.LayerInputs(c, inp.codes, inp.scales, inp.zeros, inp.A, inp.B, inp.x, inp.dy),
                                      "cuda:0"))
        k, v = measure(layers, f"decoder_block_int{bits}")
        results[k] = v
        if sibling_calls:
            # the same block with q/k/v and gate/up handed over together (they read the same activations)
            names = [c.name.split("_")[1] for c in cfgs]
            groups = [[names.index(n) for n in g] for g in (("q", "k", "v"), ("o",), ("gate", "up"), ("down",))]
            k, v = measure(layers, f"decoder_block_int{bits}_sibling_calls", groups)
            results[k] = v
        del layers, by_shape
        torch.cuda.empty_cache()
    def overall(keys):
        tot_b = sum(2 * results[k]["weight_side_bytes_per_set"] for k in keys)
        tot_us = sum(results[k]["fwd"]["us_per_set"] + results[k]["bwd"]["us_per_set"] for k in keys)
        return round(tot_b / tot_us * 1e-3, 1)

    first = ["q_proj_int4"] if headline_layer else []
    per_layer = overall(first + [f"decoder_block_int{b}" for b in bit_widths])
    results["all_fwd_bwd_packed_weight_GBps"] = per_layer                       # one call per projection
    results["all_frac_of_hbm_peak"] = round(per_layer / PEAK_HBM_GBPS, 4)
    if sibling_calls:
        siblings = overall(first + [f"decoder_block_int{b}_sibling_calls" for b in bit_widths])
        results["all_sibling_calls_fwd_bwd_packed_weight_GBps"] = siblings       # q/k/v and gate/up together
        results["all_sibling_calls_frac_of_hbm_peak"] = round(siblings / PEAK_HBM_GBPS, 4)
    return results


def _event_time(call, warm: int, iters: int) -> float:
    """Microseconds per call of `call`, HIP events on the stream the library launches on around `iters` back-to-back
    calls (for passes long enough that issuing them from Python does not starve the GPU)."""
    import torch
    from paper_2306_08162_amd.hiprt import Event
    for _ in range(warm):
        call()
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream().cuda_stream or None
    e0, e1 = Event(), Event()
    e0.record(stream)
    for _ in range(iters):
        call()
    e1.record(stream)
    e1.synchronize()
    return e0.elapsed_ms(e1) * 1e3 / iters


def _layer_times(cfg, graph: bool):
    """Forward and backward microseconds of one layer drawn on the device.  graph: replay a captured burst that
    rotates weight copies beyond the last-level cache (passes of tens of microseconds); else plain event timing."""
    import torch
    from paper_2306_08162_amd.device import DeviceLayer
    layer = DeviceLayer.drawn_on_device(cfg)
    if not graph:
        us = {"fwd": _event_time(layer.forward, 5, 20), "bwd": _event_time(layer.backward, 5, 20)}
    else:
        wbytes = cfg.weight_side_bytes
        copies = max(2, min(32, 1 + (300 << 20) // wbytes))
        pool = [(layer.packed, layer.scales, layer.zeros)] + [
            (layer.packed.clone(), layer.scales.clone(), layer.zeros.clone()) for _ in range(copies - 1)]

        def sweep(which):
            for pk, sc, zr in pool:
                layer.packed, layer.scales, layer.zeros = pk, sc, zr
                (layer.forward if which == "fwd" else layer.backward)()

        us = {w: _graph_time(lambda w=w: sweep(w), 5) / copies for w in ("fwd", "bwd")}
    del layer
    torch.cuda.empty_cache()
    return us


def run_configs():
    """The other named workloads, timed in the library's own launch configuration: config 3 (gate/up, INT2, bf16,
    rank 16), config 4 (down, INT3 stream, M = 4096) and the decoder block of config 5 at INT2 and INT8 for M = 256
    and M = 4096 (its M = 1 and M = 16 passes are priced in GB/s under "small_m").  TFLOP/s counts 4MNK + 6Mr(K+N)
    per forward + backward; the fraction is of the fp16 / bf16 MFMA peak."""
    from paper_2306_08162_amd import workloads as wl
    out = {}

    def entry(cfgs_with_mult, graph):
        f_us = b_us = 0.0
        flops = 0
        shapes = {}
        for cfg, mult in cfgs_with_mult:
            us = _layer_times(cfg, graph)
            f_us += mult * us["fwd"]
            b_us += mult * us["bwd"]
            flops += mult * cfg.flops_fwd_bwd
            shapes[f"{cfg.K}x{cfg.N}"] = {"fwd_us": round(us["fwd"], 1), "bwd_us": round(us["bwd"], 1),
                                          "TFLOPs": round(cfg.flops_fwd_bwd / (us["fwd"] + us["bwd"]) * 1e-6, 1)}
        tf = flops / (f_us + b_us) * 1e-6
        return {"fwd_us": round(f_us, 1), "bwd_us": round(b_us, 1), "TFLOPs": round(tf, 1),
                "frac_of_mfma_peak": round(tf / PEAK_MFMA_F16_TFLOPS, 4), "per_shape_KxN": shapes}

    for cfg in (wl.config3(), wl.config4()):
        e = entry([(cfg, 1)], graph=False)
        e.pop("per_shape_KxN")
        e["workload"] = f"M={cfg.M} K={cfg.K} N={cfg.N} INT{cfg.bits} G={cfg.group_size} r={cfg.rank} {cfg.dtype}"
        out[cfg.name] = e
    for bits in (2, 8):
        for M in (256, 4096):
            block = {c.name.split("_")[1]: c for c in wl.config5(bits, M)}
            out[f"c5_decoder_block_int{bits}_M{M}"] = entry([(block["q"], 4), (block["gate"], 2), (block["down"], 1)],
                                                            graph=M <= 512)
    return out


def run_lrec_loss(M: int = 2048, V: int = 32000, iters: int = 20):
    """The LREC objective + gradient over M token rows of a LLaMA vocabulary (widened row of the scope table).

    HBM-bound: both logit rows are read once and the gradient written once, 6 bytes per logit.  Four input sets are
    rotated so that no launch finds its rows in the 256 MB last-level cache (a set is 262 MB).
    """
    import numpy as np
    import torch
    from paper_2306_08162_amd import binding as ql
    from paper_2306_08162_amd import workloads as wl
    from paper_2306_08162_amd.hiprt import Event
    dev = torch.device("cuda:0")
    rows = 64                                   # seeded rows generated on the host, tiled over the M tokens
    zt = wl.normal(0x10551, rows * V).reshape(rows, V) * 4.0
    zs = 0.7 * zt + wl.normal(0x10552, rows * V).reshape(rows, V) * 1.2
    up = lambda a: torch.from_numpy(wl.to_bits(a.ravel(), "f16").view(np.int16).reshape(rows, V)).to(dev)
    sets = []
    for i in range(4):
        sets.append((up(zs).roll(i, 0).repeat(M // rows, 1).contiguous(), up(zt).roll(i, 0).repeat(M // rows, 1).contiguous()))
    labels = torch.from_numpy((wl.splitmix64(0x10553, 0, M) % np.uint64(V)).astype(np.int32)).to(dev)
    kl = torch.empty(M, dtype=torch.float32, device=dev)
    ce = torch.empty_like(kl)
    mean = torch.empty(1, dtype=torch.float32, device=dev)
    grad = torch.empty((M, V), dtype=torch.int16, device=dev)
    ws = torch.empty(ql.qlora_lrec_workspace_bytes(M), dtype=torch.uint8, device=dev)
    call = lambda i: ql.qlora_lrec_loss(sets[i % 4][0], sets[i % 4][1], labels, 1.0, 120.0, kl, ce, mean, grad, M, V,
                                        ql.QLORA_F16, ws)
    for i in range(4):
        call(i)
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream().cuda_stream or None
    e0, e1 = Event(), Event()
    e0.record(stream)
    for i in range(iters):
        call(i)
    e1.record(stream)
    e1.synchronize()
    us = e0.elapsed_ms(e1) * 1e3 / iters
    nbytes = 6 * M * V
    # for scale: what a plain device-to-device copy of the same volume reaches on this machine (reads + writes counted)
    src = grad.view(-1)
    dst = torch.empty_like(src)
    for _ in range(2):
        dst.copy_(src)
    e0.record(stream)
    for _ in range(10):
        dst.copy_(src)
    e1.record(stream)
    e1.synchronize()
    copy_gbps = 2 * src.numel() * 2 / (e0.elapsed_ms(e1) * 1e-3 / 10) * 1e-9
    return {"workload": f"M={M} tokens x V={V} logits, fp16, lambda_kl=1 lambda_ce=120", "us_per_call": round(us, 2),
            "algorithmic_bytes": nbytes, "GBps": round(nbytes / us * 1e-3, 1),
            "frac_of_hbm_peak": round(nbytes / us * 1e-3 / PEAK_HBM_GBPS, 4),
            "plain_copy_GBps_same_box": round(copy_gbps, 1), "loss_mean": float(mean.cpu()[0])}


def run_actorder_gather(M: int = 2048, K: int = 4096, G: int = 128, iters: int = 20):
    """The run-time cost of an activation-order checkpoint: one column gather of x before the forward call and one
    of dX after the backward call (4 bytes per element each: read once, written once).  Eight buffers are rotated."""
    import numpy as np
    import torch
    from paper_2306_08162_amd import binding as ql
    from paper_2306_08162_amd import workloads as wl
    dev = torch.device("cuda:0")
    perm = np.empty(K, dtype=np.int32)
    ql.qlora_actorder_perm(wl.actorder_g_idx(0xAC7, K, G), perm, None, K, G)
    idx = torch.from_numpy(perm).to(dev)
    src = [torch.zeros((M, K), dtype=torch.int16, device=dev) for _ in range(8)]
    dst = [torch.empty((M, K), dtype=torch.int16, device=dev) for _ in range(8)]
    def burst():
        for i in range(8):
            ql.qlora_gather_columns(src[i], idx, dst[i], M, K)
    us = _graph_time(burst, iters) / 8
    def copies():
        for i in range(8):
            dst[i].copy_(src[i])
    copy_us = _graph_time(copies, iters) / 8
    nbytes = 4 * M * K
    return {"workload": f"gather of {M} x {K} 16-bit columns by a seeded activation order (G={G})",
            "us_per_call": round(us, 2), "algorithmic_bytes": nbytes, "GBps": round(nbytes / us * 1e-3, 1),
            "frac_of_hbm_peak": round(nbytes / us * 1e-3 / PEAK_HBM_GBPS, 4),
            "plain_copy_us_same_box": round(copy_us, 2), "calls_per_fwd_bwd": 2}


def run_stacked(iters: int = 20):
    """Variants of the headline layer that training runs of the paper use.  Stacked adapters on the headline projection (App. D: a frozen rank-32 recovery pair plus a trainable rank-8
    pair): the backward pass with gradients for all 40 adapter columns against the one that forms them for the
    trainable 8 only.  HIP events around `iters` back-to-back calls."""
    import dataclasses
    import torch
    from paper_2306_08162_amd import workloads as wl
    from paper_2306_08162_amd.device import DeviceLayer
    from paper_2306_08162_amd.hiprt import Event
    cfg = dataclasses.replace(wl.config2(), rank=40, alpha=80.0, name="c2_qproj_int4_rank32+8")
    layer = DeviceLayer(wl.make_inputs(cfg))
    layer.forward()
    stream = torch.cuda.current_stream().cuda_stream or None
    out = {}
    for label, call in (("all_40_columns", lambda: layer.backward()), ("trainable_8_only", lambda: layer.backward_stacked(32))):
        for _ in range(5):
            call()
        torch.cuda.synchronize()
        e0, e1 = Event(), Event()
        e0.record(stream)
        for _ in range(iters):
            call()
        e1.record(stream)
        e1.synchronize()
        out[label + "_bwd_us"] = round(e0.elapsed_ms(e1) * 1e3 / iters, 2)
    out["workload"] = f"{cfg.name}: M={cfg.M} K={cfg.K} N={cfg.N} INT{cfg.bits} fp16, backward pass"
    # the rank LREC trains at (App. C: r = 32 on every layer), whole step
    cfg32 = dataclasses.replace(wl.config2(), rank=32, alpha=64.0, name="c2_qproj_int4_rank32")
    del layer
    layer = DeviceLayer(wl.make_inputs(cfg32))
    def step():
        layer.forward()
        layer.backward()
    for _ in range(100):                 # as for the headline: the clocks settle over the first ~20 ms
        step()
    torch.cuda.synchronize()
    e0, e1 = Event(), Event()
    e0.record(stream)
    for _ in range(200):
        step()
    e1.record(stream)
    e1.synchronize()
    us = e0.elapsed_ms(e1) * 1e3 / 200
    out["rank32_fwd_bwd_us"] = round(us, 2)
    out["rank32_fwd_bwd_TFLOPs"] = round(cfg32.flops_fwd_bwd / us * 1e-6, 1)
    # the headline layer with LoRA dropout (App. B: rate 0.05), mask drawn by a seeded generator on the host
    import numpy as np
    del layer
    cfg = wl.config2()
    layer = DeviceLayer(wl.make_inputs(cfg))
    u01 = wl.splitmix64(0xD809, 0, cfg.M * cfg.K).astype(np.float64) / 2.0 ** 64
    bits = (u01 >= 0.05).astype(np.uint64).reshape(cfg.M, cfg.K // 32, 32)
    words = (bits << np.arange(32, dtype=np.uint64)).sum(axis=2).astype(np.uint32)
    km = torch.from_numpy(words.view(np.int32)).to(layer.device)
    def dstep():
        layer.forward_dropout(km, 1.0 / 0.95)
        layer.backward_dropout(km, 1.0 / 0.95)
    for _ in range(100):
        dstep()
    torch.cuda.synchronize()
    e0, e1 = Event(), Event()
    e0.record(stream)
    for _ in range(200):
        dstep()
    e1.record(stream)
    e1.synchronize()
    out["dropout_0.05_fwd_bwd_us"] = round(e0.elapsed_ms(e1) * 1e3 / 200, 2)
    return out


def run_mfma_probe(iters: int = 40000, reps: int = 4):
    """What the matrix cores of this machine sustain: register-resident MFMAs and nothing else (no memory, no LDS, no
    other arithmetic), two waves per SIMD, about 10 ms per launch, the last of `reps` launches reported.  With constant
    operands the published peak is reached; with random operands that change from MFMA to MFMA the chip's power
    management lowers the clock.  Context for the roofline fraction, which is priced at the published peak."""
    import torch
    from paper_2306_08162_amd import binding as ql
    from paper_2306_08162_amd.hiprt import Event

    out = torch.empty(ql.MFMA_PROBE_FLOATS, dtype=torch.float32, device="cuda:0")
    stream = torch.cuda.current_stream().cuda_stream or None
    res = {}
    for name, rnd in (("constant_operands", False), ("random_operands", True)):
        tf = 0.0
        for _ in range(reps):
            e0, e1 = Event(), Event()
            e0.record(stream)
            ql.qlora_mfma_probe(out, iters, rnd, stream=stream)
            e1.record(stream)
            e1.synchronize()
            tf = iters * ql.MFMA_PROBE_FLOP_PER_ITER / (e0.elapsed_ms(e1) * 1e-3) / 1e12
        res[name + "_TFLOPs"] = round(tf, 1)
    res["what"] = "register-resident v_mfma_f32_32x32x16_f16 only, 2 waves per SIMD, ~10 ms launches"
    return res


def run_dense_library_context(M: int, K: int, N: int, iters: int = 200):
    """CONTEXT ONLY, never part of `value`: the vendor library's dense fp16 GEMM (torch.matmul) on already
    dequantised weights of the headline shape, in the two operand orders of the layer's passes.  It reads four
    times the weight bytes, has no LoRA term, and shares nothing with this library's kernels."""
    import torch
    x = torch.randn(M, K, device="cuda:0", dtype=torch.float16)
    dy = torch.randn(M, N, device="cuda:0", dtype=torch.float16)
    w = torch.randn(N, K, device="cuda:0", dtype=torch.float16)
    out = {}
    for name, fn in (("fwd_x_wT_us", lambda: x @ w.t()), ("bwd_dy_w_us", lambda: dy @ w)):
        for _ in range(50):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        out[name] = round(e0.elapsed_time(e1) / iters * 1e3, 2)
    out["note"] = "vendor dense fp16 GEMM of the same shape on fp16 weights: context, not this library"
    return out


def run_cpu_baseline(inp, max_rows: int):
    """The fp64 oracle as it stands, on the host cores: forward + backward on the first `max_rows` token rows."""
    import oracle
    c = inp.cfg
    rows = min(c.M, max_rows)
    t0 = time.perf_counter()
    lo = oracle.LayerOracle(inp.codes, inp.scales, inp.zeros, inp.A, inp.B, bits=c.bits, group_size=c.group_size,
                            alpha=c.alpha, dtype=c.dtype)
    lo.forward(inp.x[:rows])
    lo.backward_dx(inp.dy[:rows])
    lo.backward_adapters(inp.dy[:rows], inp.x[:rows])
    dt = time.perf_counter() - t0
    flops = 4 * rows * c.N * c.K + 6 * rows * c.rank * (c.K + c.N)
    return {"value": round(flops / dt / 1e12, 5), "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"fp64 C/OpenMP oracle, unpack+dequant+fwd+bwd on the first {rows} of {c.M} token rows of the "
                      f"same workload, {dt:.1f} s"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)   # 35 ms of timed work: the clocks settle over the first ~20 ms
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--cpu-rows", type=int, default=2048, help="token rows the CPU oracle baseline is timed on")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-small-m", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy, so a rocprofv3 --pmc run of this command holds a kernel of "
                         "known HBM traffic to scale FETCH_SIZE / WRITE_SIZE by")
    ap.add_argument("--library-context", action="store_true",
                    help="also time the vendor library's dense fp16 GEMM of the headline shape (context only)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the layer has no multi-GPU path); use --gpus 1",
              file=sys.stderr)
        return 2

    if args.calibrate_copy:
        import torch
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)              # reads 1 GiB, writes 1 GiB: far larger than every cache
        torch.cuda.synchronize()
        del src, dst
    from paper_2306_08162_amd import workloads as wl
    inp = wl.make_inputs(wl.config2())      # drawn on the host first, so that nothing but the upload separates the
                                            # sections below from the headline's warm-up steps
    # The sections that widen the headline run first: the headline's W warm-up steps and K timed steps then start on a
    # GPU that has been working for seconds, as a layer inside a training job does (with W = 5 and K = 20 after an idle
    # stretch the whole measurement would sit inside the few milliseconds the clocks take to come up).
    extras = {}
    if not args.no_small_m:
        extras["configs"] = run_configs()
        extras["small_m"] = {"M": 16, "timing": "HIP-graph replays over a >1 GB pool of distinct weight sets",
                             **run_small_m(16)}
        extras["small_m_M1"] = {"M": 1, "timing": "as small_m", **run_small_m(1, headline_layer=False)}
        extras["small_m_M32"] = {"M": 32, "timing": "as small_m; two 16-row token blocks per weight fragment",
                                 **run_small_m(32, bit_widths=(2,), sibling_calls=False)}
        extras["lrec_loss"] = run_lrec_loss()
        extras["actorder_gather"] = run_actorder_gather()
        extras["stacked_adapters"] = run_stacked()
    cfg, layer, ms_per_step, fwd_ms, bwd_ms, diff_ms = run_headline(inp, args.steps, args.warmup)
    del layer
    flops = cfg.flops_fwd_bwd
    value = flops / (ms_per_step * 1e-3) / 1e12

    # dominant kernel: the fused dequantise + MFMA GEMM (one launch per pass); take the slower of the two
    gemm_flops = {"fwd": 2 * cfg.M * cfg.N * cfg.K + 2 * cfg.M * cfg.rank * cfg.N,
                  "bwd": 2 * cfg.M * cfg.N * cfg.K + 2 * cfg.M * cfg.rank * cfg.K}
    gemm_ms = {"fwd": fwd_ms, "bwd": bwd_ms}
    dom = "bwd" if bwd_ms >= fwd_ms else "fwd"
    achieved = gemm_flops[dom] / (gemm_ms[dom] * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": f"qgemm_kernel ({dom} GEMM, INT4 fp16)", "achieved": round(achieved, 2),
                "peak": PEAK_MFMA_F16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_MFMA_F16_TFLOPS, 4),
                "traffic": GEMM_TRAFFIC_BYTES[dom],
                "traffic_unit": "bytes per launch, not measured in this run: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE "
                                "runs of this command, see profiles/qgemm_c2_hbm_traffic.md",
                "kernel_us": {k: round(v * 1e3, 2) for k, v in gemm_ms.items()},
                "kernel_us_lower_bound": {k: round(v * 1e3, 2) for k, v in diff_ms.items()} if diff_ms else None,
                "kernel_tflops": {k: round(gemm_flops[k] / (gemm_ms[k] * 1e-3) / 1e12, 2) for k in gemm_ms}}

    result = {
        "metric": "quant-LoRA linear fwd+bwd TFLOP/s (4096^2, M=2048) + packed-weight GB/s @ M=16",
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": cfg.name, "M": cfg.M, "K": cfg.K, "N": cfg.N, "bits": cfg.bits,
                   "group_size": cfg.group_size, "rank": cfg.rank, "alpha": cfg.alpha,
                   "flops_per_step": flops},
        "frac_of_mfma_peak": round(value / PEAK_MFMA_F16_TFLOPS, 4),
        "roofline": roofline,
    }
    result.update(extras)
    if not args.no_small_m:
        result["mfma_probe"] = run_mfma_probe()
        result["frac_of_sustained_mfma_rate"] = round(value / result["mfma_probe"]["random_operands_TFLOPs"], 4)
    if args.library_context:
        result["dense_library_context"] = run_dense_library_context(cfg.M, cfg.K, cfg.N)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = run_cpu_baseline(inp, args.cpu_rows)
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
