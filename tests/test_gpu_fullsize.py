"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

Config 3 (Llama-8B-shaped checkpoint, 224 tensors, one batched launch): every output byte of every
conversion (4-bit and 6-bit targets) is checked against tables that the oracle computes -- the element map of
Eq. (4) / Eq. (6) is a pure function of one anchor byte (256 calls of the oracle's slice_code), the place of every
code bit inside a packed block is read off the oracle's pack_block on one-bit patterns, and torch on the GPU only
gathers through those tables -- every scale byte against the oracle's scale step, and windows of the 6-bit
conversions and of the anchor quantization against the oracle proper as well.  Config 4 (fake-quant of 32768 x 4096 activations and of a
4096 x 14336 weight down its columns): sampled rows / columns against the oracle.
"""
import os
import sys

import numpy as np
import pytest

from paper_2604_00529_amd import synth

pytestmark = pytest.mark.gpu
sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available()
    import paper_2604_00529_amd as mx
    mx.binding.lib()
    import bench
    return torch, mx, bench


def _bf16_to_host(t):
    import torch
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def _packing_runs(oracle, bits):
    """Where the oracle puts every code bit of a block of 32: for each output byte, the runs (element, first code bit,
    first byte bit, length) that make it up, found from pack_block on patterns with a single bit set."""
    nbytes = 32 * bits // 8
    src = {}                                                  # output bit position -> (element, code bit)
    for e in range(32):
        for b in range(bits):
            codes = np.zeros(32, dtype=np.uint8)
            codes[e] = 1 << b
            packed = oracle.pack_block(codes, bits)
            assert packed.size == nbytes
            pos = [8 * j + t for j in range(nbytes) for t in range(8) if (packed[j] >> t) & 1]
            assert len(pos) == 1
            src[pos[0]] = (e, b)
    assert len(src) == 32 * bits                              # a bijection: nothing overlaps, nothing is dropped
    runs = []
    for j in range(nbytes):
        byte_runs, t = [], 0
        while t < 8:
            e, b = src[8 * j + t]
            n = 1
            while t + n < 8 and src[8 * j + t + n] == (e, b + n):
                n += 1
            byte_runs.append((e, b, t, n))
            t += n
        runs.append(byte_runs)
    return runs


def _expected_packed(m, runs):
    """m: [n, 32] element codes (one per byte, on the GPU) -> the packed blocks [n, bytes] by the oracle's bit layout."""
    import torch
    out = torch.zeros((m.shape[0], len(runs)), dtype=torch.uint8, device=m.device)
    for j, byte_runs in enumerate(runs):
        for e, b, t, n in byte_runs:
            out[:, j] |= ((m[:, e] >> b) & ((1 << n) - 1)) << t
    return out


def _windows(rng, nblocks, width, count):
    out = [(0, min(width, nblocks)), (max(0, nblocks - width), nblocks)]
    for _ in range(count):
        s = int(rng.integers(0, max(1, nblocks - width)))
        out.append((s, min(nblocks, s + width)))
    return out


@pytest.mark.parametrize("anchor,target4,targets6", [("e4m3", "e2m1", ("e3m2", "e2m3")), ("int8", "int4", ("int6",))])
def test_config3_checkpoint(env, oracle, anchor, target4, targets6):
    torch, mx, bench = env
    rng = np.random.default_rng(33)
    tensors, a_codes, a_scales, a_views = bench.build_checkpoint(torch, mx, synth, 32, anchor)
    assert len(a_views) == 224 and a_scales.numel() == 218103808
    fa = mx.make_format(anchor)

    # --- anchor quantization itself: windows of rows of a few tensors, regenerated from their seeds
    for ti in (0, 1, 4, 6, 223):
        _, r, c = tensors[ti]
        w = synth.torch_config3_weight(ti, r, c)
        for r0 in (0, r - 8, int(rng.integers(0, r - 8))):
            rows = _bf16_to_host(w[r0:r0 + 8].contiguous())
            wc, ws = oracle.quantize(rows, anchor)
            assert np.array_equal(a_views[ti][1][r0:r0 + 8].cpu().numpy(), ws), (ti, r0)
            assert np.array_equal(a_views[ti][0][r0:r0 + 8].cpu().numpy(), wc), (ti, r0)
        del w

    # --- 4-bit target: the whole checkpoint, every byte
    ft = mx.make_format(target4)
    t_codes, t_scales, t_views = bench.alloc_targets(torch, mx, a_views, target4)
    ws_bytes = mx.binding.lib().mx_slice_and_scale_batched_workspace(len(a_views), a_scales.numel())
    wsp = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    t_codes.fill_(0xA5)
    t_scales.fill_(0xA5)
    mx.SsBatch(a_views, fa, ft, t_views, wsp).run()
    torch.cuda.synchronize()
    lut = torch.tensor([oracle.slice_code(anchor, target4, c) for c in range(256)], dtype=torch.uint8, device="cuda")
    slut = torch.tensor([oracle.slice_byte(anchor, target4, b) for b in range(256)], dtype=torch.uint8, device="cuda")
    assert torch.equal(slut[a_scales.long()], t_scales), "scale bytes"
    runs4 = _packing_runs(oracle, 4)
    step = 1 << 21                                   # blocks per comparison slab (64 Mi codes)
    for b0 in range(0, a_scales.numel(), step):
        a = a_codes[b0:b0 + step]                    # [n, 32] anchor codes
        m = lut[a.long()]                            # expected 4-bit codes, one per byte
        assert torch.equal(_expected_packed(m, runs4), t_codes[b0:b0 + step]), "codes in blocks %d.." % b0
        del a, m
    del t_codes, t_scales, t_views

    # --- 6-bit targets: every byte of the whole checkpoint through the oracle's tables, then windows against the oracle
    # proper (first / last blocks of tensors, random interior)
    runs6 = _packing_runs(oracle, 6)
    for tgt in targets6:
        c6, s6, v6 = bench.alloc_targets(torch, mx, a_views, tgt)
        c6.fill_(0xA5)
        s6.fill_(0xA5)
        mx.SsBatch(a_views, fa, mx.make_format(tgt), v6, wsp).run()
        torch.cuda.synchronize()
        lut6 = torch.tensor([oracle.slice_code(anchor, tgt, c) for c in range(256)], dtype=torch.uint8, device="cuda")
        slut6 = torch.tensor([oracle.slice_byte(anchor, tgt, b) for b in range(256)], dtype=torch.uint8, device="cuda")
        assert torch.equal(slut6[a_scales.long()], s6), "scale bytes (%s)" % tgt
        for b0 in range(0, a_scales.numel(), step):
            m = lut6[a_codes[b0:b0 + step].long()]
            assert torch.equal(_expected_packed(m, runs6), c6[b0:b0 + step]), "%s codes in blocks %d.." % (tgt, b0)
            del m
        for ti in (0, 1, 2, 5, 100, 222, 223):
            nb = a_views[ti][1].numel()
            ac = a_views[ti][0].reshape(nb, 32)
            asc = a_views[ti][1].reshape(nb)
            gc = v6[ti][0].reshape(nb, 24)
            gs = v6[ti][1].reshape(nb)
            for s, e in _windows(rng, nb, 4096, 3):
                wc, wsc = oracle.slice_and_scale(ac[s:e].cpu().numpy(), asc[s:e].cpu().numpy(), anchor, tgt)
                assert np.array_equal(gs[s:e].cpu().numpy(), wsc), (tgt, ti, s)
                assert np.array_equal(gc[s:e].cpu().numpy(), wc), (tgt, ti, s)
        del c6, s6, v6
    del a_codes, a_scales, a_views
    torch.cuda.empty_cache()


def test_config3_random_byte_anchor_full_size(env, oracle):
    # adversarial pass at checkpoint scale: uniformly random code and scale bytes (every NaN code, -128, 0 / 254 / 255
    # scales), one flat tensor of 2^27 blocks, all five benchmark conversions checked through the oracle's tables
    torch, mx, _ = env
    nb = 1 << 27
    g = torch.Generator(device="cuda")
    g.manual_seed(5)
    codes = torch.randint(0, 256, (nb, 32), dtype=torch.uint8, device="cuda", generator=g)
    scales = torch.randint(0, 256, (nb,), dtype=torch.uint8, device="cuda", generator=g)
    for anchor, target in (("e4m3", "e2m1"), ("int8", "int4")):
        oc, os_ = mx.mx_slice_and_scale(codes, scales, mx.make_format(anchor), mx.make_format(target))
        lut = torch.tensor([oracle.slice_code(anchor, target, c) for c in range(256)], dtype=torch.uint8, device="cuda")
        slut = torch.tensor([oracle.slice_byte(anchor, target, b) for b in range(256)], dtype=torch.uint8, device="cuda")
        assert torch.equal(slut[scales.long()], os_)
        step = 1 << 21
        runs4 = _packing_runs(oracle, 4)
        for b0 in range(0, nb, step):
            m = lut[codes[b0:b0 + step].long()]
            assert torch.equal(_expected_packed(m, runs4), oc[b0:b0 + step])
        del oc, os_
    runs6 = _packing_runs(oracle, 6)
    for anchor, target in (("e4m3", "e3m2"), ("e4m3", "e2m3"), ("int8", "int6")):
        oc, os_ = mx.mx_slice_and_scale(codes, scales, mx.make_format(anchor), mx.make_format(target))
        lut = torch.tensor([oracle.slice_code(anchor, target, c) for c in range(256)], dtype=torch.uint8, device="cuda")
        slut = torch.tensor([oracle.slice_byte(anchor, target, b) for b in range(256)], dtype=torch.uint8, device="cuda")
        assert torch.equal(slut[scales.long()], os_)
        for b0 in range(0, nb, 1 << 21):
            m = lut[codes[b0:b0 + (1 << 21)].long()]
            assert torch.equal(_expected_packed(m, runs6), oc[b0:b0 + (1 << 21)])
        for s in (0, nb - 2048, 12345678, 99999999):
            wc, wsc = oracle.slice_and_scale(codes[s:s + 2048].cpu().numpy(), scales[s:s + 2048].cpu().numpy(), anchor, target)
            assert np.array_equal(os_[s:s + 2048].cpu().numpy(), wsc) and np.array_equal(oc[s:s + 2048].cpu().numpy(), wc)
        del oc, os_


def test_config4_fake_quant_full_size(env, oracle):
    torch, mx, _ = env
    rng = np.random.default_rng(44)
    act = synth.torch_config4_activations()                          # 32768 x 4096 bf16
    out = torch.empty_like(act)
    rows = np.sort(rng.choice(act.shape[0], size=24, replace=False))
    rows[0], rows[-1] = 0, act.shape[0] - 1
    host = _bf16_to_host(act[torch.as_tensor(rows, device="cuda")].contiguous())
    for elem in synth.QAT_FORMATS:
        for anchor in (None, "int8" if elem.startswith("int") else "e4m3"):
            if anchor == elem:
                continue
            mx.mx_fake_quant(act, mx.make_format(elem), None if anchor is None else mx.make_format(anchor), out)
            got = _bf16_to_host(out[torch.as_tensor(rows, device="cuda")].contiguous())
            want = oracle.fake_quant(host, elem, anchor=anchor)
            assert np.array_equal(got, want), (elem, anchor)
    del act, out
    # weights [K = 4096, N = 14336], blocks down the columns (the reduction axis of x @ W)
    w = synth.torch_config3_weight(2000, 4096, 14336)
    wo = torch.empty_like(w)
    cols = np.sort(rng.choice(14336, size=32, replace=False))
    cols[0], cols[-1] = 0, 14335
    hostw = _bf16_to_host(w[:, torch.as_tensor(cols, device="cuda")].contiguous())
    for elem in ("int4", "e2m1", "e3m2", "int8"):
        mx.mx_fake_quant(w, mx.make_format(elem, axis=0), None, wo)
        got = _bf16_to_host(wo[:, torch.as_tensor(cols, device="cuda")].contiguous())
        want = oracle.fake_quant(hostw, elem, axis=0)
        assert np.array_equal(got, want), elem


def test_offsets_beyond_4_gib(env, oracle):
    """One tensor of 4.3 G elements: element and byte offsets pass 2^31 and 2^32 inside a single call of every entry point
    (row 2^18 starts at byte 2^31 of the bf16 matrix, row 2^19 at byte 2^32 = element 2^31, row 2^20 at element 2^32 = byte
    2^32 of the 8-bit codes = byte 2^31 of the 4-bit codes).  Rows on both sides of each boundary, the first and the last
    row are compared with the oracle."""
    torch, mx, _ = env
    rows, cols = (1 << 20) + 96, 4096
    x = torch.empty((rows, cols), dtype=torch.bfloat16, device="cuda")
    g = torch.Generator(device="cuda").manual_seed(4096)
    for r0 in range(0, rows, 1 << 16):
        r1 = min(rows, r0 + (1 << 16))
        x[r0:r1] = torch.randn((r1 - r0, cols), device="cuda", generator=g, dtype=torch.float32).mul_(0.02).to(torch.bfloat16)
    probe = sorted({0, rows - 1, 699050, 699051} | {b + d for b in (1 << 18, 1 << 19, 3 << 18, 1 << 20) for d in (-1, 0)})
    idx = torch.as_tensor(probe, device="cuda")
    host = _bf16_to_host(x[idx].contiguous())
    f8, f4, f6 = mx.make_format("e4m3"), mx.make_format("e2m1"), mx.make_format("e3m2")

    ac, asc = mx.mx_quantize(x, f8)                                   # 4.3 GB of codes
    oc, osc = oracle.quantize(host, "e4m3")
    assert np.array_equal(ac[idx].cpu().numpy(), oc) and np.array_equal(asc[idx].cpu().numpy(), osc)
    for ft, name in ((f4, "e2m1"), (f6, "e3m2")):                     # 6-bit codes: byte 2^31 falls in row 699050
        tc, ts = mx.mx_slice_and_scale(ac, asc, f8, ft)
        wc, ws = oracle.slice_and_scale(oc, osc, "e4m3", name)
        assert np.array_equal(tc[idx].cpu().numpy(), wc) and np.array_equal(ts[idx].cpu().numpy(), ws), name
        if name == "e2m1":
            y = mx.mx_dequant(tc, ts, ft, rows, cols, dtype=torch.bfloat16)
            want = oracle.dequant(wc, ws, "e2m1", len(probe), cols, out="bf16")
            assert np.array_equal(_bf16_to_host(y[idx].contiguous()), want)
            del y
        del tc, ts
    del ac, asc
    torch.cuda.empty_cache()

    y = torch.empty_like(x)
    mx.mx_fake_quant(x, mx.make_format("int4"), mx.make_format("int8"), y)
    assert np.array_equal(_bf16_to_host(y[idx].contiguous()), oracle.fake_quant(host, "int4", anchor="int8"))
    # blocks down the columns: the row blocks on both sides of each boundary, all columns
    mx.mx_fake_quant(x, mx.make_format("e2m1", axis=0), None, y)
    for b in (1 << 18, 1 << 19, 1 << 20):
        slab = _bf16_to_host(x[b - 32:b + 32].contiguous())
        assert np.array_equal(_bf16_to_host(y[b - 32:b + 32].contiguous()), oracle.fake_quant(slab, "e2m1", axis=0)), b
    del y
    # transposed packed tensor of the column-axis quantizer: whole columns, the last one ends past byte 2^31
    f4c = mx.make_format("e2m1", axis=0)
    cc, cs = mx.mx_quantize(x, f4c)
    pick = [0, 1, 2047, 2048, 4094, 4095]
    hostc = _bf16_to_host(x[:, torch.as_tensor(pick, device="cuda")].contiguous())
    wc, ws = oracle.quantize(hostc, "e2m1", axis=0)
    pidx = torch.as_tensor(pick, device="cuda")
    assert np.array_equal(cc[pidx].cpu().numpy(), wc) and np.array_equal(cs[pidx].cpu().numpy(), ws)
    z = mx.mx_dequant(cc, cs, f4c, rows, cols, dtype=torch.bfloat16)
    want = oracle.dequant(wc, ws, "e2m1", rows, len(pick), axis=0, out="bf16")
    assert np.array_equal(_bf16_to_host(z[:, pidx].contiguous()), want)
