#!/usr/bin/env python3
"""Benchmark of the MX hot path on one MI355X.

Headline: Slice-and-Scale MXFP8 (E4M3) -> MXFP4 (E2M1) over a
Llama-8B-shaped decoder checkpoint (224 linear weights, 6 979 321 856 elements, block 32), as
GB/s of algorithmic traffic (anchor codes + anchor scales read, target codes + target scales
written) and as a fraction of the 8 TB/s HBM peak.  One step = one such pass over the whole
checkpoint in one batched launch, the anchor already resident in HBM.  The other rows of the
hot path (quantize, dequantize, fake-quant, the other conversions) are timed in the same run
and reported under "rows".  The CPU oracle is timed beside it on a bounded sample.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--layers L] [--no-rows] [--no-cpu]
"""
import argparse
import json
import os
import sys
import time

HBM_PEAK_GBS = 8000.0
ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


WARM_MS = 30.0   # secondary rows: untimed calls for at least this long first (the GPU takes ~10 ms of sustained
                 # work to reach its steady state: clocks, page tables; measured 72-80 % -> 82-83 % on one kernel)


def time_region(torch, fn, steps, warmup, warm_ms=0.0):
    """Average milliseconds per call: events on the current stream, bracketed by synchronize."""
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
    return sum(per) / steps, min(per), wall_ms / steps


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
    ap.add_argument("--only", default=None, choices=["gemm"],
                    help="profiling aid: run only this group of secondary rows (no headline, no CPU baseline)")
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
    if args.only == "gemm":
        rows = {}
        gemm_rows(torch, mx, synth, rows)
        print(json.dumps({"rows": rows}), flush=True)
        return

    # ---------------------------------------------------------------- headline: SS E4M3 -> E2M1, whole checkpoint
    log("[bench] building the MXFP8 anchor checkpoint (%d layers)" % args.layers)
    tensors, a_codes, a_scales, a_views = build_checkpoint(torch, mx, synth, args.layers, "e4m3")
    nblocks = a_scales.numel()
    n_elem = nblocks * 32
    fa, ft = mx.make_format("e4m3"), mx.make_format("e2m1")
    t_codes, t_scales, t_views = alloc_targets(torch, mx, a_views, "e2m1")
    ws = torch.empty(mx.binding.lib().mx_slice_and_scale_batched_workspace(len(a_views), nblocks), dtype=torch.uint8,
                     device="cuda")

    batch = mx.SsBatch(a_views, fa, ft, t_views, ws)      # descriptors marshalled once; run() is one C call

    def step():
        batch.run()

    log("[bench] timing Slice-and-Scale E4M3 -> E2M1: %d tensors, %d elements" % (len(a_views), n_elem))
    ms, ms_min, wall_ms = time_region(torch, step, args.steps, args.warmup)
    nbytes = ss_bytes(nblocks, 8, 4)
    value = nbytes / (wall_ms * 1e-3) / 1e9
    achieved = nbytes / (ms * 1e-3) / 1e9
    log("[bench] %.3f ms/step (events avg %.3f, min %.3f): %.1f GB/s, %.1f %% of HBM peak"
        % (wall_ms, ms, ms_min, value, 100 * achieved / HBM_PEAK_GBS))

    result = {
        "metric": "Slice-and-Scale GB/s and % of HBM peak, 8B-shaped checkpoint MXFP8->MXFP4",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall_ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {"workload": "configs[2]: Llama-8B-shaped decoder checkpoint, %d layers, %d linear weights, "
                               "%d elements, MXFP8 E4M3 anchor -> MXFP4 E2M1, block 32, one batched launch"
                               % (args.layers, len(a_views), n_elem),
                   "bytes_per_step": nbytes, "pct_hbm_peak": round(100 * value / HBM_PEAK_GBS, 2)},
        "roofline": {"bound": "hbm", "kernel": "ss_batched_kernel<E4M3,E2M1>", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": MEASURED_TRAFFIC.get("ss_e4m3_e2m1")},
    }

    if args.calibrate_copy:
        src = torch.full((1 << 30,), 7, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---------------------------------------------------------------- CPU oracle beside it (bounded sample)
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(torch, a_views, tensors)

    # ---------------------------------------------------------------- the other rows of the hot path
    if not args.no_rows:
        rows = {}
        steps2 = max(3, min(args.steps, 10))
        for tgt in ("e3m2", "e2m3"):
            c2, s2, v2 = alloc_targets(torch, mx, a_views, tgt)
            f2 = mx.make_format(tgt)
            m, _, _ = time_region(torch, mx.SsBatch(a_views, fa, f2, v2, ws).run, steps2, 2, WARM_MS)
            rows["ss_e4m3_%s" % tgt] = row(ss_bytes(nblocks, 8, 6), m)
            del c2, s2, v2
        # every lower MXFP format from ONE pass over the anchor (read once, three targets written)
        trip = [alloc_targets(torch, mx, a_views, t) for t in ("e3m2", "e2m3", "e2m1")]
        tv = [[trip[q][2][i] for q in range(3)] for i in range(len(a_views))]
        b3 = mx.SsBatch(a_views, fa, [mx.make_format(t) for t in ("e3m2", "e2m3", "e2m1")], tv, ws)
        m, _, _ = time_region(torch, b3.run, steps2, 2, WARM_MS)
        rows["ss_e4m3_to_e3m2_e2m3_e2m1_one_pass"] = row(nblocks * (32 + 1 + 24 + 24 + 16 + 3), m)
        del trip, tv, b3
        del t_codes, t_scales, t_views, batch
        torch.cuda.empty_cache()
        # MXINT8 anchor -> MXINT6 / MXINT4: the anchor arena is re-quantized in place of the FP8 one
        del a_codes, a_scales, a_views
        torch.cuda.empty_cache()
        tensors, a_codes, a_scales, a_views = build_checkpoint(torch, mx, synth, args.layers, "int8")
        fi = mx.make_format("int8")
        for tgt, bits in (("int4", 4), ("int6", 6)):
            c2, s2, v2 = alloc_targets(torch, mx, a_views, tgt)
            f2 = mx.make_format(tgt)
            m, _, _ = time_region(torch, mx.SsBatch(a_views, fi, f2, v2, ws).run, steps2, 2, WARM_MS)
            rows["ss_int8_%s" % tgt] = row(ss_bytes(nblocks, 8, bits), m)
            del c2, s2, v2
        del a_codes, a_scales, a_views
        torch.cuda.empty_cache()
        # quantize / dequantize on eight stacked copies of the largest decoder weight (gate_proj 14336 x 4096 bf16;
        # 114688 x 4096 = 469.8 M elements, 940 MB dense): several times the 256 MB last-level cache, so every pass
        # streams HBM
        r, c = 8 * 14336, 4096
        wbig = torch.cat([synth.torch_config3_weight(1000 + i, 14336, c) for i in range(8)], dim=0)
        for elem, bits in (("e4m3", 8), ("int8", 8), ("e2m1", 4), ("int4", 4), ("e3m2", 6)):
            f = mx.make_format(elem)
            pc, ps = mx.mx_quantize(wbig, f)
            m, _, _ = time_region(torch, lambda: mx.mx_quantize(wbig, f, pc, ps), 10, 3, WARM_MS)
            rows["quantize_bf16_%s" % elem] = row(r * c * 2 + r * c // 32 * (4 * bits + 1), m)
            deq = torch.empty((r, c), dtype=torch.bfloat16, device="cuda")
            m, _, _ = time_region(torch, lambda: mx.mx_dequant(pc, ps, f, r, c, out=deq), 10, 3, WARM_MS)
            rows["dequant_%s_bf16" % elem] = row(r * c * 2 + r * c // 32 * (4 * bits + 1), m)
            del pc, ps, deq
        del wbig
        torch.cuda.empty_cache()
        # fake-quant step of multi-format QAT (configs[3]): bf16 activations 32768 x 4096, blocks along the
        # reduction axis, one sampled format per step, direct and through the 8-bit anchor
        act = synth.torch_config4_activations()
        out = torch.empty_like(act)
        sched = synth.config4_format_schedule(steps=64)
        nby = act.numel() * 4
        for via in (False, True):
            st = {"k": 0}

            def fq():
                elem = sched[st["k"] % len(sched)]
                st["k"] += 1
                anchor = None
                if via and elem not in ("int8", "e4m3"):
                    anchor = mx.make_format("int8" if elem.startswith("int") else "e4m3")
                mx.mx_fake_quant(act, mx.make_format(elem), anchor, out)
            m, _, _ = time_region(torch, fq, 64, 6, WARM_MS)
            rows["fake_quant_bf16_mixed_formats" + ("_via_anchor" if via else "")] = row(nby, m)
        for elem in ("int8", "int4", "e4m3", "e3m2", "e2m1"):
            f = mx.make_format(elem)
            m, _, _ = time_region(torch, lambda: mx.mx_fake_quant(act, f, None, out), 10, 3, WARM_MS)
            rows["fake_quant_bf16_%s" % elem] = row(nby, m)
        # for scale: the framework's own device-to-device copy of the same tensor (same 2 B read + 2 B written per
        # element as fake-quant; not a kernel of this library)
        m, _, _ = time_region(torch, lambda: out.copy_(act), 10, 3, WARM_MS)
        rows["reference_torch_copy_bf16"] = row(nby, m)
        # blocks down the columns (axis 0) on the same 256 MiB activation tensor: fake-quant, quantize, dequantize
        for elem, bits in (("e2m1", 4), ("int4", 4), ("e4m3", 8)):
            f0 = mx.make_format(elem, axis=0)
            m, _, _ = time_region(torch, lambda: mx.mx_fake_quant(act, f0, None, out), 10, 3, WARM_MS)
            rows["fake_quant_bf16_%s_axis0" % elem] = row(nby, m)
            pc, ps = mx.mx_quantize(act, f0)
            m, _, _ = time_region(torch, lambda: mx.mx_quantize(act, f0, pc, ps), 10, 3, WARM_MS)
            rows["quantize_bf16_%s_axis0" % elem] = row(act.numel() * 2 + act.numel() // 32 * (4 * bits + 1), m)
            m, _, _ = time_region(torch, lambda: mx.mx_dequant(pc, ps, f0, act.shape[0], act.shape[1], out=out), 10, 3, WARM_MS)
            rows["dequant_%s_bf16_axis0" % elem] = row(act.numel() * 2 + act.numel() // 32 * (4 * bits + 1), m)
            del pc, ps
        gemm_rows(torch, mx, synth, rows)
        result["rows"] = rows

    print(json.dumps(result), flush=True)


def gemm_rows(torch, mx, synth, rows):
    # fused consumer GEMM (configs[4]): bf16 activations -> MXFP8 (not timed), weight anchor E4M3 [N, K/32, 32]
    # sliced to E2M1 in registers, scaled MX MFMA.  Decode (M = 16) is bound by reading the anchor: 8 weights are
    # rotated (484 MB) so that they stream from HBM; prefill (M = 2048) is bound by the matrix cores (operand A is
    # FP8, so the FP8 dense peak applies).
    f8 = mx.make_format("e4m3")
    wlist = []
    for i in range(8):
        w = synth.torch_config3_weight(3000 + i, 14336, 4096)
        wlist.append(mx.mx_quantize(w, f8))
        del w
    # third row: a down_proj shape with few rows (M = 64, N = 4096, K = 14336; the same anchors' bytes read as
    # [4096, 14336]): few tiles and a long K, which the library splits over several workgroups per tile
    for Mg, Ng, Kg, name in ((16, 14336, 4096, "gemm_ss_fp4_M16"), (2048, 14336, 4096, "gemm_ss_fp4_M2048"),
                             (64, 4096, 14336, "gemm_ss_fp4_M64_N4096_K14336")):
        a = torch.randn((Mg, Kg), device="cuda", dtype=torch.float32, generator=torch.Generator(device="cuda").manual_seed(1005)).to(torch.bfloat16)
        ac, asc = mx.mx_quantize(a, f8)
        cbuf = torch.empty((Mg, Ng), dtype=torch.float32, device="cuda")
        ws = [(c.view(Ng, Kg // 32, 32), sc.view(Ng, Kg // 32)) for c, sc in wlist]
        st = {"i": 0}

        def gemm():
            i = st["i"] = (st["i"] + 1) % 8
            mx.mx_gemm_ss_fp4(ac, asc, ws[i][0], ws[i][1], cbuf)
        m, _, _ = time_region(torch, gemm, 24, 8, WARM_MS)
        flops = 2.0 * Mg * Ng * Kg
        nbytes_g = Ng * Kg + Ng * Kg // 32 + Mg * Kg + Mg * Kg // 32 + Mg * Ng * 4
        rows[name] = {"ms": round(m, 4), "TFLOP/s": round(flops / (m * 1e-3) / 1e12, 1),
                      "frac_fp8_mfma_peak": round(flops / (m * 1e-3) / 5.0e15, 4),
                      "GB/s": round(nbytes_g / (m * 1e-3) / 1e9, 1),
                      "frac_hbm_peak": round(nbytes_g / (m * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        del a, ac, asc, cbuf, ws
    del wlist


def row(nbytes, ms):
    gbs = nbytes / (ms * 1e-3) / 1e9
    return {"ms": round(ms, 4), "GB/s": round(gbs, 1), "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)}


# HBM bytes per launch of the headline kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs,
# scaled by the same counters on a plain copy of known size (see profiles/); None until measured.
MEASURED_TRAFFIC = {"ss_e4m3_e2m1": 10912164270}   # profiles/ss_e4m3_e2m1_llama8b_checkpoint.md


def cpu_baseline(torch, a_views, tensors):
    """The CPU oracle on a bounded sample of the same anchor: whole tensors from layer 0 on."""
    import numpy as np
    import oracle
    oracle.build()
    threads = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "16")), 16)
    oracle.set_threads(threads)
    # calibrate on the smallest tensor (k_proj), then take whole tensors worth roughly 15 s
    c0 = a_views[1][0].cpu().numpy()
    s0 = a_views[1][1].cpu().numpy()
    t0 = time.perf_counter()
    oracle.slice_and_scale(c0, s0, "e4m3", "e2m1")
    rate = s0.size / (time.perf_counter() - t0)           # blocks per second
    budget_blocks = rate * 15.0
    sample, used = [], 0
    for (cv, sv), (name, r, c) in zip(a_views, tensors):
        if used and used + sv.numel() > budget_blocks:
            break
        sample.append((cv.cpu().numpy(), sv.cpu().numpy(), name))
        used += sv.numel()
    log("[bench] CPU oracle on %d tensors (%d elements), %d threads" % (len(sample), used * 32, threads))
    t0 = time.perf_counter()
    for cv, sv, _ in sample:
        oracle.slice_and_scale(cv, sv, "e4m3", "e2m1")
    dt = time.perf_counter() - t0
    gbs = ss_bytes(used, 8, 4) / dt / 1e9
    return {"value": round(gbs, 4), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": "Slice-and-Scale E4M3->E2M1 of the first %d tensors of the same anchor (%s..%s), %d elements, %.1f s"
                      % (len(sample), sample[0][2], sample[-1][2], used * 32, dt)}


if __name__ == "__main__":
    main()
