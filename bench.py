#!/usr/bin/env python3
"""Benchmark of the MX hot path on one MI355X.

Headline: Slice-and-Scale MXFP8 (E4M3) -> MXFP4 (E2M1) over a
Llama-8B-shaped decoder checkpoint (224 linear weights, 6 979 321 856 elements, block 32), as
GB/s of algorithmic traffic (anchor codes + anchor scales read, target codes + target scales
written) and as a fraction of the 8 TB/s HBM peak.  One step = one such pass over the whole
checkpoint in one batched launch, the anchor already resident in HBM.  The other rows of the
hot path (quantize, dequantize, fake-quant, the other conversions, the column-axis kernels, the
fused consumer GEMM) are timed in the same run and reported under "rows", in groups that --only
selects.  The CPU oracle is timed beside the headline on a bounded sample.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--layers L] [--no-rows] [--no-cpu] [--only GROUPS]
"""
import argparse
import hashlib
import json
import os
import statistics
import sys
import time

HBM_PEAK_GBS = 8000.0
FP8_MFMA_PEAK = 5.0e15
ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

GROUPS = ("ss", "dense", "fq", "cols", "blocks", "gemm")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


WARM_MS = 30.0   # secondary rows: untimed calls for at least this long first (the GPU takes ~10 ms of sustained
                 # work to reach its steady state: clocks, page tables; measured 72-80 % -> 82-83 % on one kernel)


def time_region(torch, fn, steps, warmup, warm_ms=0.0):
    """Milliseconds per call from HIP events on the current stream (the stream the library launches on), bracketed
    by synchronize: (mean over the whole timed region, median of the calls, fastest call, wall-clock mean)."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    if warm_ms > 0.0:
        t0 = time.perf_counter()
        while (time.perf_counter() - t0) * 1e3 < warm_ms:
            for _ in range(4):
                fn()
            torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    ev[0].record()
    for i in range(steps):
        fn()
        ev[i + 1].record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    per = [ev[i].elapsed_time(ev[i + 1]) for i in range(steps)]
    return ev[0].elapsed_time(ev[steps]) / steps, statistics.median(per), min(per), wall_ms / steps


def time_graph(torch, fn, calls, steps=20, warmup=4):
    """Milliseconds per call of fn when `calls` of them are replayed as one captured HIP graph (the kernels without the
    host between the launches): time_region's tuple, divided by `calls`."""
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for _ in range(calls):
            fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        for _ in range(calls):
            fn()
    t = time_region(torch, graph.replay, steps, warmup, WARM_MS)
    del graph
    return tuple(x / calls for x in t)


def build_checkpoint(torch, mx, synth, layers, anchor_elem):
    """Quantize the synthetic decoder weights to one packed anchor arena; returns per-tensor views."""
    tensors = synth.llama8b_tensor_list(layers)
    total_blocks = sum(r * c // 32 for _, r, c in tensors)
    codes = torch.empty((total_blocks, 32), dtype=torch.uint8, device="cuda")
    scales = torch.empty((total_blocks,), dtype=torch.uint8, device="cuda")
    fmt = mx.make_format(anchor_elem)
    views, b0 = [], 0
    for i, (_, r, c) in enumerate(tensors):
        w = synth.torch_config3_weight(i, r, c)
        nb = r * c // 32
        cv = codes[b0:b0 + nb].view(r, c // 32, 32)
        sv = scales[b0:b0 + nb].view(r, c // 32)
        mx.mx_quantize(w, fmt, cv, sv)
        views.append((cv, sv))
        b0 += nb
        del w
    torch.cuda.synchronize()
    return tensors, codes, scales, views


def alloc_targets(torch, mx, views, target_elem):
    bb = 32 * mx.mx_elem_bits(target_elem) // 8
    total = sum(s.numel() for _, s in views)
    codes = torch.empty((total, bb), dtype=torch.uint8, device="cuda")
    scales = torch.empty((total,), dtype=torch.uint8, device="cuda")
    out, b0 = [], 0
    for _, s in views:
        nb = s.numel()
        out.append((codes[b0:b0 + nb].view(tuple(s.shape) + (bb,)), scales[b0:b0 + nb].view(s.shape)))
        b0 += nb
    return codes, scales, out


def ss_bytes(nblocks, anchor_bits, target_bits):
    return nblocks * (4 * anchor_bits + 4 * target_bits + 2)


def row(nbytes, timing, **extra):
    """A bandwidth row: GB/s and the fraction of HBM peak from the median call, the fastest call beside it."""
    _, med, fastest, _ = timing
    gbs = nbytes / (med * 1e-3) / 1e9
    out = {"ms": round(med, 4), "ms_min": round(fastest, 4), "GB/s": round(gbs, 1), "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)}
    out.update(extra)
    return out


# HBM bytes per launch of the headline kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs, scaled by the same
# counters on a plain copy of known size (profiles/ss_batched_e4m3_e2m1_llama8b_checkpoint.md: 7204.4 MB fetched + 3707.8 MB written).  The figure belongs to the
# kernel sources it was measured with: when they have changed since, the field is null, not a stale number.
MEASURED_TRAFFIC = {"bytes": 10912200000, "bytes_per_step": 10905190400,
                    "sources_sha256": "20e66e4729090a90"}   # first 16 hex digits over mx_ss.hip + mx_device.h
TRAFFIC_SOURCES = ("paper_2604_00529_amd/csrc/mx_ss.hip", "paper_2604_00529_amd/csrc/mx_device.h")


def kernel_sources_hash():
    h = hashlib.sha256()
    for rel in TRAFFIC_SOURCES:
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(bytes_per_step):
    if MEASURED_TRAFFIC["bytes_per_step"] != bytes_per_step or MEASURED_TRAFFIC["sources_sha256"] != kernel_sources_hash():
        return None
    return MEASURED_TRAFFIC["bytes"]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--layers", type=int, default=32, help="decoder layers of the synthetic checkpoint (32 = the 8B shape)")
    ap.add_argument("--no-rows", action="store_true", help="skip the secondary rows")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline")
    ap.add_argument("--warm-ms", type=float, default=None,
                    help="untimed warm-up time per secondary row in ms (default 30; 0 keeps counter profiles small)")
    ap.add_argument("--only", default=None,
                    help="profiling aid: run only these groups of secondary rows (comma list of %s; no headline, no CPU baseline)"
                         % ", ".join(GROUPS))
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (for scaling the profiler's FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no collectives exist in this path); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2604_00529_amd as mx
    from paper_2604_00529_amd import synth
    mx.binding.lib()
    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)

    global WARM_MS
    if args.warm_ms is not None:
        WARM_MS = args.warm_ms
    if args.calibrate_copy:
        calibrate_copy(torch)
    if args.only is not None:
        groups = [g for g in args.only.split(",") if g]
        assert all(g in GROUPS for g in groups), "--only takes a comma list of %s" % ", ".join(GROUPS)
        rows = {}
        run_groups(torch, mx, synth, rows, groups, args, None)
        print(json.dumps({"rows": rows}), flush=True)
        return

    # ---------------------------------------------------------------- headline: SS E4M3 -> E2M1, whole checkpoint
    log("[bench] building the MXFP8 anchor checkpoint (%d layers)" % args.layers)
    ckpt = build_checkpoint(torch, mx, synth, args.layers, "e4m3")
    tensors, a_codes, a_scales, a_views = ckpt
    nblocks = a_scales.numel()
    n_elem = nblocks * 32
    fa, ft = mx.make_format("e4m3"), mx.make_format("e2m1")
    t_codes, t_scales, t_views = alloc_targets(torch, mx, a_views, "e2m1")
    ws = torch.empty(mx.binding.lib().mx_slice_and_scale_batched_workspace(len(a_views), nblocks), dtype=torch.uint8,
                     device="cuda")
    batch = mx.SsBatch(a_views, fa, ft, t_views, ws)      # descriptors marshalled once; run() is one C call

    log("[bench] timing Slice-and-Scale E4M3 -> E2M1: %d tensors, %d elements" % (len(a_views), n_elem))
    ms, ms_med, ms_min, wall_ms = time_region(torch, batch.run, args.steps, args.warmup)
    nbytes = ss_bytes(nblocks, 8, 4)
    # one clock for the whole line: HIP events around the K steps (on the stream the kernels run on), inside the
    # synchronize bracket; the wall-clock figure of the same region is given beside it
    value = nbytes / (ms * 1e-3) / 1e9
    log("[bench] %.4f ms/step by events (median %.4f, min %.4f; wall clock %.4f): %.1f GB/s, %.1f %% of HBM peak"
        % (ms, ms_med, ms_min, wall_ms, value, 100 * value / HBM_PEAK_GBS))

    result = {
        "metric": "Slice-and-Scale GB/s and % of HBM peak, 8B-shaped checkpoint MXFP8->MXFP4",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 4), "ms_per_step_median": round(ms_med, 4), "ms_per_step_min": round(ms_min, 4),
        "ms_per_step_wall_clock": round(wall_ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {"workload": "configs[2]: Llama-8B-shaped decoder checkpoint, %d layers, %d linear weights, "
                               "%d elements, MXFP8 E4M3 anchor -> MXFP4 E2M1, block 32, one batched launch"
                               % (args.layers, len(a_views), n_elem),
                   "bytes_per_step": nbytes, "pct_hbm_peak": round(100 * value / HBM_PEAK_GBS, 2)},
        "roofline": {"bound": "hbm", "kernel": "ss_batched_kernel<E4M3,E2M1>", "achieved": round(value, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(value / HBM_PEAK_GBS, 4),
                     "traffic": measured_traffic(nbytes)},
    }
    del batch, t_codes, t_scales, t_views

    # ---------------------------------------------------------------- the measured ceiling of a plain copy beside it
    # a device-to-device copy of the anchor's codes by the runtime's own copy (read = write: a mix with more writes than
    # the conversion's 2 : 1), same clock
    dst = torch.empty_like(a_codes)
    c_ms, c_med, _, _ = time_region(torch, lambda: dst.copy_(a_codes), 10, 3)
    copy_gbs = 2 * a_codes.numel() / (c_med * 1e-3) / 1e9
    del dst
    torch.cuda.empty_cache()
    result["config"]["copy_ceiling"] = {"GB/s": round(copy_gbs, 1), "kind": "torch device-to-device copy of the anchor codes (%d B read + written)" % a_codes.numel()}
    result["config"]["pct_of_copy_ceiling"] = round(100 * value / copy_gbs, 1)

    # ---------------------------------------------------------------- CPU oracle beside it (bounded sample)
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(torch, a_views, tensors)

    # ---------------------------------------------------------------- the other rows of the hot path
    if not args.no_rows:
        rows = {}
        run_groups(torch, mx, synth, rows, GROUPS, args, ckpt)
        result["rows"] = rows

    print(json.dumps(result), flush=True)


def calibrate_copy(torch):
    src = torch.full((1 << 30,), 7, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst


def run_groups(torch, mx, synth, rows, groups, args, ckpt):
    if "ss" in groups:
        ss_rows(torch, mx, synth, rows, args, ckpt)
    del ckpt
    torch.cuda.empty_cache()
    if "dense" in groups:
        dense_rows(torch, mx, synth, rows)
    if "fq" in groups:
        fake_quant_rows(torch, mx, synth, rows)
    if "cols" in groups:
        column_rows(torch, mx, synth, rows)
    if "blocks" in groups:
        block_size_rows(torch, mx, synth, rows)
    if "gemm" in groups:
        gemm_rows(torch, mx, synth, rows)


def ss_rows(torch, mx, synth, rows, args, ckpt):
    """The other Slice-and-Scale conversions of configs[2] on the whole checkpoint (HBM), then configs[0] and [1]
    (single small tensors that stay in the 256 MB last-level cache: flagged, not roofline rows)."""
    steps2 = max(3, min(args.steps, 20))
    if ckpt is None:
        ckpt = build_checkpoint(torch, mx, synth, args.layers, "e4m3")
    tensors, a_codes, a_scales, a_views = ckpt
    del ckpt
    nblocks = a_scales.numel()
    fa = mx.make_format("e4m3")
    ws = torch.empty(mx.binding.lib().mx_slice_and_scale_batched_workspace(len(a_views), nblocks), dtype=torch.uint8,
                     device="cuda")
    for tgt in ("e3m2", "e2m3"):
        c2, s2, v2 = alloc_targets(torch, mx, a_views, tgt)
        t = time_region(torch, mx.SsBatch(a_views, fa, mx.make_format(tgt), v2, ws).run, steps2, 2, WARM_MS)
        rows["ss_e4m3_%s" % tgt] = row(ss_bytes(nblocks, 8, 6), t)
        del c2, s2, v2
    # every lower MXFP format from ONE pass over the anchor (read once, three targets written)
    trip = [alloc_targets(torch, mx, a_views, t) for t in ("e3m2", "e2m3", "e2m1")]
    tv = [[trip[q][2][i] for q in range(3)] for i in range(len(a_views))]
    b3 = mx.SsBatch(a_views, fa, [mx.make_format(t) for t in ("e3m2", "e2m3", "e2m1")], tv, ws)
    rows["ss_e4m3_to_e3m2_e2m3_e2m1_one_pass"] = row(nblocks * (32 + 1 + 24 + 24 + 16 + 3), time_region(torch, b3.run, steps2, 2, WARM_MS))
    del trip, tv, b3
    # MXINT8 anchor -> MXINT6 / MXINT4: the anchor arena is re-quantized in place of the FP8 one
    del a_codes, a_scales, a_views
    torch.cuda.empty_cache()
    tensors, a_codes, a_scales, a_views = build_checkpoint(torch, mx, synth, args.layers, "int8")
    fi = mx.make_format("int8")
    for tgt, bits in (("int4", 4), ("int6", 6)):
        c2, s2, v2 = alloc_targets(torch, mx, a_views, tgt)
        t = time_region(torch, mx.SsBatch(a_views, fi, mx.make_format(tgt), v2, ws).run, steps2, 2, WARM_MS)
        rows["ss_int8_%s" % tgt] = row(ss_bytes(nblocks, 8, bits), t)
        del c2, s2, v2
    del a_codes, a_scales, a_views, ws
    torch.cuda.empty_cache()
    # configs[0]: fp32 1024 x 1024 -> MXINT8 -> MXINT6 / MXINT4; configs[1]: bf16 4096 x 4096 -> E4M3 -> E3M2 / E2M3 / E2M1,
    # blocks along rows.  5 MiB and 48 MiB of traffic: last-level-cache resident, launch-latency sized
    import numpy as np
    for name, w, anchor, targets in (("config1_1024x1024", torch.from_numpy(synth.config1_weight()).cuda(), "int8", ("int6", "int4")),
                                     ("config2_4096x4096", torch.from_numpy(synth.config2_weight().view(np.int16)).view(torch.bfloat16).cuda(), "e4m3", ("e3m2", "e2m3", "e2m1"))):
        f = mx.make_format(anchor)
        pc, ps = mx.mx_quantize(w, f)
        nb = ps.numel()
        t = time_region(torch, lambda: mx.mx_quantize(w, f, pc, ps), 20, 5, WARM_MS)
        rows["quantize_%s_%s" % (name, anchor)] = row(w.numel() * w.element_size() + nb * 33, t, cache_resident=True)
        # launches this short are timed by the host's pace; 16 of them replayed as one graph give the kernel's own time
        t = time_graph(torch, lambda: mx.mx_quantize(w, f, pc, ps), 16)
        rows["quantize_%s_%s_graph" % (name, anchor)] = row(w.numel() * w.element_size() + nb * 33, t, cache_resident=True, calls_per_replay=16)
        for tg in targets:
            ftg = mx.make_format(tg)
            oc, os_ = mx.mx_slice_and_scale(pc, ps, f, ftg)
            t = time_region(torch, lambda: mx.mx_slice_and_scale(pc, ps, f, ftg, oc, os_), 20, 5, WARM_MS)
            rows["ss_%s_%s_%s" % (name, anchor, tg)] = row(ss_bytes(nb, 8, mx.mx_elem_bits(tg)), t, cache_resident=True)
            t = time_graph(torch, lambda: mx.mx_slice_and_scale(pc, ps, f, ftg, oc, os_), 16)
            rows["ss_%s_%s_%s_graph" % (name, anchor, tg)] = row(ss_bytes(nb, 8, mx.mx_elem_bits(tg)), t, cache_resident=True, calls_per_replay=16)
        del pc, ps, w


def dense_rows(torch, mx, synth, rows):
    """Quantize / dequantize along rows on eight stacked copies of the largest decoder weight (gate_proj 14336 x 4096;
    114688 x 4096 = 469.8 M elements: 940 MB as bf16, 1.88 GB as fp32 -- several times the 256 MB last-level cache, so
    every pass streams HBM)."""
    r, c = 8 * 14336, 4096
    wbig = torch.cat([synth.torch_config3_weight(1000 + i, 14336, c) for i in range(8)], dim=0)
    for dt_name, esz in (("bf16", 2), ("f32", 4)):
        src = wbig if dt_name == "bf16" else wbig.float()
        formats = (("e4m3", 8), ("int8", 8), ("e2m1", 4), ("int4", 4), ("e3m2", 6)) if dt_name == "bf16" else (("e4m3", 8), ("int8", 8), ("e2m1", 4))
        for elem, bits in formats:
            f = mx.make_format(elem)
            pc, ps = mx.mx_quantize(src, f)
            nbytes = r * c * esz + r * c // 32 * (4 * bits + 1)
            rows["quantize_%s_%s" % (dt_name, elem)] = row(nbytes, time_region(torch, lambda: mx.mx_quantize(src, f, pc, ps), 20, 3, WARM_MS))
            deq = torch.empty((r, c), dtype=src.dtype, device="cuda")
            rows["dequant_%s_%s" % (elem, dt_name)] = row(nbytes, time_region(torch, lambda: mx.mx_dequant(pc, ps, f, r, c, out=deq), 20, 3, WARM_MS))
            del pc, ps, deq
        del src
    del wbig
    torch.cuda.empty_cache()


def fake_quant_rows(torch, mx, synth, rows):
    """Fake-quant step of multi-format QAT (configs[3]): activations 32768 x 4096 (256 MiB as bf16, 512 MiB as fp32),
    blocks along the reduction axis, one sampled format per step, direct and through the 8-bit anchor (Eq. (7))."""
    act16 = synth.torch_config4_activations()
    sched = synth.config4_format_schedule(steps=64)
    for dt_name, act in (("bf16", act16), ("f32", None)):
        if act is None:
            act = act16.float()
        out = torch.empty_like(act)
        nby = act.numel() * act.element_size() * 2
        for via in (False, True):
            st = {"k": 0}

            def fq():
                elem = sched[st["k"] % len(sched)]
                st["k"] += 1
                anchor = None
                if via and elem not in ("int8", "e4m3"):
                    anchor = mx.make_format("int8" if elem.startswith("int") else "e4m3")
                mx.mx_fake_quant(act, mx.make_format(elem), anchor, out)
            rows["fake_quant_%s_mixed_formats" % dt_name + ("_via_anchor" if via else "")] = row(nby, time_region(torch, fq, 64, 6, WARM_MS))
        for elem in ("int8", "int4", "e4m3", "e3m2", "e2m1"):
            f = mx.make_format(elem)
            rows["fake_quant_%s_%s" % (dt_name, elem)] = row(nby, time_region(torch, lambda: mx.mx_fake_quant(act, f, None, out), 20, 3, WARM_MS))
        # for scale: the framework's own device-to-device copy of the same tensor (same bytes read and written per
        # element as fake-quant; not a kernel of this library)
        rows["reference_torch_copy_%s" % dt_name] = row(nby, time_region(torch, lambda: out.copy_(act), 20, 3, WARM_MS))
        del out, act
    del act16
    torch.cuda.empty_cache()


def column_rows(torch, mx, synth, rows):
    """Blocks down the columns (axis 0): the 256 MiB activation tensor of configs[3], the weight leg of configs[3] --
    bf16 4096 x 14336, blocks along K, 112 MiB dense -- and configs[1]'s column-axis quantization (32 MiB, cache
    resident, flagged).  Every call of a row works on the next of several buffer sets (4 for the activations, 6 for the
    weight), so that neither the dense nor the packed side of a call is still in the 256 MB last-level cache from the
    call before: with one set the packed tensor (67-134 MB) stays there and quantize / dequantize read 7 / 25-35 points
    better than they stream from HBM."""
    import numpy as np
    NA, NW = 4, 6
    act0 = synth.torch_config4_activations()
    acts = [act0] + [act0.clone() for _ in range(NA - 1)]
    outs = [torch.empty_like(act0) for _ in range(NA)]
    nby = act0.numel() * 4
    st = {"k": 0}

    def nxt(n):
        st["k"] = (st["k"] + 1) % n
        return st["k"]
    for elem, bits in (("e2m1", 4), ("int4", 4), ("e4m3", 8)):
        f0 = mx.make_format(elem, axis=0)

        def fq():
            i = nxt(NA)
            mx.mx_fake_quant(acts[i], f0, None, outs[i])
        rows["fake_quant_bf16_%s_axis0" % elem] = row(nby, time_region(torch, fq, 20, 4, WARM_MS))
        packs = [mx.mx_quantize(a, f0) for a in acts]
        nbytes = act0.numel() * 2 + act0.numel() // 32 * (4 * bits + 1)

        def qz():
            i = nxt(NA)
            mx.mx_quantize(acts[i], f0, packs[i][0], packs[i][1])

        def dq():
            i = nxt(NA)
            mx.mx_dequant(packs[i][0], packs[i][1], f0, act0.shape[0], act0.shape[1], out=outs[i])
        rows["quantize_bf16_%s_axis0" % elem] = row(nbytes, time_region(torch, qz, 20, 4, WARM_MS))
        rows["dequant_%s_bf16_axis0" % elem] = row(nbytes, time_region(torch, dq, 20, 4, WARM_MS))
        del packs
    del act0, acts, outs
    torch.cuda.empty_cache()
    w0 = synth.torch_config3_weight(2000, 4096, 14336)               # [K, N]: the weight of x @ W, blocks down its columns
    ws = [w0] + [w0.clone() for _ in range(NW - 1)]
    wos = [torch.empty_like(w0) for _ in range(NW)]
    sched = synth.config4_format_schedule(steps=64)
    sk = {"k": 0}

    def fqw():
        elem = sched[sk["k"] % len(sched)]
        sk["k"] += 1
        i = nxt(NW)
        mx.mx_fake_quant(ws[i], mx.make_format(elem, axis=0), None, wos[i])
    rows["fake_quant_bf16_config4_weight_4096x14336_axis0_mixed_formats"] = row(w0.numel() * 4, time_region(torch, fqw, 64, 6, WARM_MS))
    f8 = mx.make_format("e4m3", axis=0)
    wpacks = [mx.mx_quantize(w, f8) for w in ws]

    def qw():
        i = nxt(NW)
        mx.mx_quantize(ws[i], f8, wpacks[i][0], wpacks[i][1])
    rows["quantize_bf16_config4_weight_4096x14336_e4m3_axis0"] = row(w0.numel() * 2 + w0.numel() // 32 * 33, time_region(torch, qw, 24, 6, WARM_MS))
    del w0, ws, wos, wpacks
    w2 = torch.from_numpy(synth.config2_weight().view(np.int16)).view(torch.bfloat16).cuda()
    pc, ps = mx.mx_quantize(w2, f8)
    rows["quantize_config2_4096x4096_e4m3_axis0"] = row(w2.numel() * 2 + w2.numel() // 32 * 33, time_region(torch, lambda: mx.mx_quantize(w2, f8, pc, ps), 20, 5, WARM_MS), cache_resident=True)
    del w2, pc, ps
    torch.cuda.empty_cache()


def block_size_rows(torch, mx, synth, rows):
    """Block sizes other than the benchmark's 32 (the paper evaluates 64 and sweeps 16 .. 128, Sec. 4.3): quantize,
    Slice-and-Scale and fake-quant with blocks along rows on four stacked copies of the largest decoder weight (470 MB as
    bf16), and quantize / fake-quant with blocks of 64 rows down the columns of configs[3]'s activations."""
    r, c = 4 * 14336, 4096
    w = torch.cat([synth.torch_config3_weight(1000 + i, 14336, c) for i in range(4)], dim=0)
    out = torch.empty_like(w)
    for k in (64, 16, 128):
        f8, f4 = mx.make_format("e4m3", block=k), mx.make_format("e2m1", block=k)
        pc, ps = mx.mx_quantize(w, f8)
        nb = r * c // k
        rows["quantize_bf16_e4m3_block%d" % k] = row(r * c * 2 + r * c + nb, time_region(torch, lambda: mx.mx_quantize(w, f8, pc, ps), 20, 3, WARM_MS))
        tc, ts = mx.mx_slice_and_scale(pc, ps, f8, f4)
        rows["ss_e4m3_e2m1_block%d" % k] = row(r * c + r * c // 2 + 2 * nb, time_region(torch, lambda: mx.mx_slice_and_scale(pc, ps, f8, f4, tc, ts), 20, 3, WARM_MS))
        rows["fake_quant_bf16_e2m1_via_e4m3_block%d" % k] = row(r * c * 4, time_region(torch, lambda: mx.mx_fake_quant(w, f4, f8, out), 20, 3, WARM_MS))
        del pc, ps, tc, ts
    del w, out
    torch.cuda.empty_cache()
    # down the columns of config 4's activations, four buffer sets in turn (see column_rows)
    act0 = synth.torch_config4_activations()
    acts = [act0] + [act0.clone() for _ in range(3)]
    outs = [torch.empty_like(act0) for _ in range(4)]
    f8c, f4c = mx.make_format("e4m3", axis=0, block=64), mx.make_format("e2m1", axis=0, block=64)
    packs = [mx.mx_quantize(a, f8c) for a in acts]
    st = {"k": 0}

    def qz():
        i = st["k"] = (st["k"] + 1) % 4
        mx.mx_quantize(acts[i], f8c, packs[i][0], packs[i][1])

    def fq():
        i = st["k"] = (st["k"] + 1) % 4
        mx.mx_fake_quant(acts[i], f4c, None, outs[i])
    rows["quantize_bf16_e4m3_axis0_block64"] = row(act0.numel() * 3 + act0.numel() // 64, time_region(torch, qz, 20, 4, WARM_MS))
    rows["fake_quant_bf16_e2m1_axis0_block64"] = row(act0.numel() * 4, time_region(torch, fq, 20, 4, WARM_MS))
    del act0, acts, outs, packs
    torch.cuda.empty_cache()


def gemm_rows(torch, mx, synth, rows):
    """Fused consumer GEMM (configs[4]): bf16 activations -> MXFP8 (not timed), weight anchor E4M3 [N, K/32, 32],
    Slice-and-Scale to E2M1 and the scaled MX MFMA.  8 different anchors are rotated (484 MB) so that W streams from
    HBM.  Decode (M = 16) is bound by reading the anchor; prefill (M = 2048) by the matrix cores (operand A is FP8, so
    the FP8 dense peak applies).  The prefill shape is timed on both of its paths, by name: `_fused` slices the anchor
    in registers inside the product kernel (W_t never exists in memory); `_hoisted` writes W_t into a workspace with the
    Slice-and-Scale kernel and multiplies it with a second kernel (its bytes count the workspace's write and re-read).
    `_kept_w_t` rows multiply by a W_t converted beforehand (mx_gemm_fp8_fp4; the conversion is not timed).
    `_with_activation_quantize_graph` rows time the whole consumer call as a model makes it: mx_quantize of the bf16
    activations to MXFP8 along K, then the anchor-fed product on its default path.
    Rows time the Python call (events per call); `_graph` rows replay a captured HIP graph of 8 calls, which takes the
    host's call overhead (3-5 us, a fifth of the decode kernel's time) out of the figure."""
    f8 = mx.make_format("e4m3")
    L = mx.binding.lib()
    wlist = []
    for i in range(8):
        w = synth.torch_config3_weight(3000 + i, 14336, 4096)
        wlist.append(mx.mx_quantize(w, f8))
        del w
    # last shape: a down_proj with few rows (M = 64, N = 4096, K = 14336; the same anchors' bytes read as [4096, 14336]):
    # few tiles and a long K, which the library splits over several workgroups per tile when it is lent a workspace
    for Mg, Ng, Kg, name in ((16, 14336, 4096, "gemm_ss_fp4_M16"), (2048, 14336, 4096, "gemm_ss_fp4_M2048"),
                             (64, 4096, 14336, "gemm_ss_fp4_M64_N4096_K14336")):
        a = torch.randn((Mg, Kg), device="cuda", dtype=torch.float32, generator=torch.Generator(device="cuda").manual_seed(1005)).to(torch.bfloat16)
        ac, asc = mx.mx_quantize(a, f8)
        cbuf = torch.empty((Mg, Ng), dtype=torch.float32, device="cuda")
        wv = [(c.view(Ng, Kg // 32, 32), sc.view(Ng, Kg // 32)) for c, sc in wlist]
        need = L.mx_gemm_ss_fp4_workspace(Ng, Kg)
        wsp = torch.empty(max(16, need), dtype=torch.uint8, device="cuda")      # allocated once, outside every timed call
        flops = 2.0 * Mg * Ng * Kg
        base_bytes = Ng * Kg + Ng * Kg // 32 + Mg * Kg + Mg * Kg // 32 + Mg * Ng * 4
        # `_kept_w_t`: the anchors converted to MXFP4 beforehand (one Slice-and-Scale per precision switch, not timed) and
        # multiplied by mx_gemm_fp8_fp4, which then streams half the bytes
        f4 = mx.make_format("e2m1")
        w4 = [mx.mx_slice_and_scale(c, sc, f8, f4) for c, sc in wv + wv]   # 16 buffers (500 MB): beyond the 256 MB cache, like the anchors
        kept_bytes = Ng * Kg // 2 + Ng * Kg // 32 + Mg * Kg + Mg * Kg // 32 + Mg * Ng * 4
        kept_need = L.mx_gemm_fp8_fp4_workspace(Mg, Ng, Kg)                      # > 0: the library splits K for this shape
        kept_ws = torch.empty(kept_need, dtype=torch.uint8, device="cuda") if kept_need else False
        paths = [("", False, base_bytes)] if Mg < mx.GEMM_WORKSPACE_MIN_ROWS else \
                [("_fused", False, base_bytes), ("_hoisted" if Mg >= mx.GEMM_HOIST_MIN_ROWS else "_k_slices", wsp,
                  base_bytes + (2 * need if Mg >= mx.GEMM_HOIST_MIN_ROWS else 0))]
        paths.append(("_kept_w_t", "kept", kept_bytes))
        for suffix, workspace, nbytes_g in paths:
            st = {"i": 0}

            def gemm():
                i = st["i"] = (st["i"] + 1) % 16
                if workspace == "kept":
                    mx.mx_gemm_fp8_fp4(ac, asc, w4[i][0], w4[i][1], cbuf, workspace=kept_ws)
                else:
                    mx.mx_gemm_ss_fp4(ac, asc, wv[i % 8][0], wv[i % 8][1], cbuf, workspace=workspace)

            def gemm_row(timing, **extra):
                _, med, fastest, _ = timing
                out = {"ms": round(med, 4), "ms_min": round(fastest, 4), "TFLOP/s": round(flops / (med * 1e-3) / 1e12, 1),
                       "frac_fp8_mfma_peak": round(flops / (med * 1e-3) / FP8_MFMA_PEAK, 4),
                       "GB/s": round(nbytes_g / (med * 1e-3) / 1e9, 1),
                       "frac_hbm_peak": round(nbytes_g / (med * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
                out.update(extra)
                return out
            rows[name + suffix] = gemm_row(time_region(torch, gemm, 24, 8, WARM_MS))
            # the same 8 calls as one captured graph: per-call time without the host between the launches
            rows[name + suffix + "_graph"] = gemm_row(time_graph(torch, gemm, 8), calls_per_replay=8)
        # the whole consumer call as a model makes it: bf16 activations quantized to MXFP8 along K (mx_quantize) and the
        # product, anchor-fed by the default path; 8 such pairs per graph replay
        st2 = {"i": 0}
        ws_default = wsp if Mg >= mx.GEMM_WORKSPACE_MIN_ROWS else False

        def quant_gemm():
            i = st2["i"] = (st2["i"] + 1) % 8
            mx.mx_quantize(a, f8, ac, asc)
            mx.mx_gemm_ss_fp4(ac, asc, wv[i][0], wv[i][1], cbuf, workspace=ws_default)
        t = time_graph(torch, quant_gemm, 8)
        nbytes_g = base_bytes + Mg * Kg * 2 + (2 * need if Mg >= mx.GEMM_HOIST_MIN_ROWS else 0)   # (read by gemm_row) + the bf16 activations
        rows[name + "_with_activation_quantize_graph"] = gemm_row(t, calls_per_replay=8)
        del a, ac, asc, cbuf, wv, wsp, w4, kept_ws
    del wlist
    torch.cuda.empty_cache()


def cpu_baseline(torch, a_views, tensors):
    """The CPU oracle, as it stands, on a bounded sample of the same anchor (whole tensors from layer 0 on): with one
    OpenMP thread per host core that this process may use, and with a single thread beside it."""
    import oracle
    oracle.build()
    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    threads = max(1, min(cores, int(os.environ.get("OMP_NUM_THREADS", cores))))

    def leg(nthreads, seconds):
        oracle.set_threads(nthreads)
        # calibrate on the smallest tensor (k_proj), then take whole tensors worth roughly `seconds`
        c0 = a_views[1][0].cpu().numpy()
        s0 = a_views[1][1].cpu().numpy()
        t0 = time.perf_counter()
        oracle.slice_and_scale(c0, s0, "e4m3", "e2m1")
        rate = s0.size / (time.perf_counter() - t0)           # blocks per second
        budget_blocks = rate * seconds
        sample, used = [], 0
        for (cv, sv), (name, r, c) in zip(a_views, tensors):
            if used and used + sv.numel() > budget_blocks:
                break
            sample.append((cv.cpu().numpy(), sv.cpu().numpy(), name))
            used += sv.numel()
        log("[bench] CPU oracle on %d tensors (%d elements), %d thread(s)" % (len(sample), used * 32, nthreads))
        t0 = time.perf_counter()
        for cv, sv, _ in sample:
            oracle.slice_and_scale(cv, sv, "e4m3", "e2m1")
        dt = time.perf_counter() - t0
        gbs = ss_bytes(used, 8, 4) / dt / 1e9
        return round(gbs, 4), ("Slice-and-Scale E4M3->E2M1 of the first %d tensors of the same anchor (%s..%s), %d elements, %.1f s"
                               % (len(sample), sample[0][2], sample[-1][2], used * 32, dt))

    v_all, s_all = leg(threads, 12.0)
    v_one, s_one = leg(1, 6.0)
    return {"value": v_all, "unit": "GB/s", "cores": threads, "kind": "oracle", "sample": s_all,
            "host_cores_available": cores,
            "one_thread": {"value": v_one, "unit": "GB/s", "cores": 1, "sample": s_one}}


if __name__ == "__main__":
    main()
