"""GPU parity: every C-ABI entry point against the CPU oracle, element by element, on the same
seeded inputs.  Bar: bit-exact codes, scale bytes and fp32 / bf16 values (NaN compared as NaN)."""
import numpy as np
import pytest

from paper_2604_00529_amd import synth

pytestmark = pytest.mark.gpu

CORE = ["int8", "int6", "int4", "e4m3", "e3m2", "e2m3", "e2m1"]
EXTRA = ["int7", "int5", "int3", "int2", "e3m3", "e2m2"]
SS_PAIRS = [("int8", "int6"), ("int8", "int4"), ("e4m3", "e3m2"), ("e4m3", "e2m3"), ("e4m3", "e2m1"),
            ("int8", "int7"), ("int8", "int5"), ("int8", "int3"), ("int8", "int2"), ("e4m3", "e3m3"), ("e4m3", "e2m2")]
TIES = {"default": 0, "away": 1, "even": 2}


@pytest.fixture(scope="module")
def mx():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2604_00529_amd as mx
    mx.binding.lib()          # fails loudly if libmx.so has not been built
    return mx


def to_gpu(a):
    import torch
    if a.dtype == np.uint16:      # bfloat16 bit patterns
        return torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16).cuda()
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def to_host(t):
    import torch
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def assert_same_values(got, want):
    """fp32 arrays or bf16 bit arrays: identical bits, NaN matching NaN."""
    if want.dtype == np.uint16:
        g_nan = (got & 0x7FFF) > 0x7F80
        w_nan = (want & 0x7FFF) > 0x7F80
    else:
        g_nan, w_nan = np.isnan(got), np.isnan(want)
        got, want = got.view(np.uint32), want.view(np.uint32)
    assert np.array_equal(g_nan, w_nan)
    bad = (got != want) & ~w_nan
    assert not bad.any(), "first mismatch at %s" % (np.argwhere(bad)[:4].tolist(),)


# ------------------------------------------------------------------------------------ Slice-and-Scale
@pytest.mark.parametrize("anchor,target", SS_PAIRS)
@pytest.mark.parametrize("tie", ["default", "away", "even"])
def test_slice_and_scale_random_bytes(mx, oracle, anchor, target, tie):
    # uniformly random code bytes and scale bytes: every anchor code (NaN codes, -128 included) and every
    # scale byte (0, 254, 255 included); sizes span several workgroup tiles and ragged tails
    fa, ft = mx.make_format(anchor, round=tie), mx.make_format(target, round=tie)
    for nblocks, seed in ((1, 1), (15, 2), (17, 3), (1024, 4), (4096 + 5, 5), (3 * 1024 + 77, 6), (20000, 7)):
        codes = synth.random_bytes(seed, nblocks * 32).reshape(nblocks, 32)
        scales = synth.random_bytes(seed + 100, nblocks)
        scales[: min(nblocks, 6)] = np.array([0, 1, 253, 254, 255, 250], dtype=np.uint8)[: min(nblocks, 6)]
        want_c, want_s = oracle.slice_and_scale(codes, scales, anchor, target, tie=TIES[tie])
        got_c, got_s = mx.mx_slice_and_scale(to_gpu(codes), to_gpu(scales), fa, ft)
        assert np.array_equal(to_host(got_s), want_s), (nblocks,)
        assert np.array_equal(to_host(got_c), want_c), (nblocks,)


def test_slice_and_scale_all_codes_in_every_position(mx, oracle):
    # code c at element position i of a block, for all 256 x 32 combinations (catches lane / packing slips)
    blocks = np.zeros((256 * 32, 32), dtype=np.uint8)
    for c in range(256):
        for i in range(32):
            blocks[c * 32 + i, :] = (c * 7 + 13) & 0xFF
            blocks[c * 32 + i, i] = c
    scales = np.full(blocks.shape[0], 120, dtype=np.uint8)
    for anchor, target in SS_PAIRS:
        want_c, want_s = oracle.slice_and_scale(blocks, scales, anchor, target)
        got_c, got_s = mx.mx_slice_and_scale(to_gpu(blocks), to_gpu(scales), mx.make_format(anchor), mx.make_format(target))
        assert np.array_equal(to_host(got_c), want_c), (anchor, target)
        assert np.array_equal(to_host(got_s), want_s)


def test_slice_and_scale_empty(mx):
    import torch
    c = torch.empty((0, 32), dtype=torch.uint8, device="cuda")
    s = torch.empty((0,), dtype=torch.uint8, device="cuda")
    oc, os_ = mx.mx_slice_and_scale(c, s, mx.make_format("e4m3"), mx.make_format("e2m1"))
    assert oc.shape == (0, 16) and os_.shape == (0,)


@pytest.mark.parametrize("anchor,target", SS_PAIRS[:5])
def test_slice_and_scale_batched(mx, oracle, anchor, target):
    # many tensors of unequal size in one launch, against per-tensor oracle results
    import torch
    sizes = [1, 33, 1024, 7, 4096, 5000, 2, 1025, 64, 300] * 8     # 80 tensors: more than one table chunk
    anchors, want = [], []
    for i, nb in enumerate(sizes):
        codes = synth.random_bytes(900 + i, nb * 32).reshape(nb, 32)
        scales = synth.random_bytes(1900 + i, nb)
        anchors.append((to_gpu(codes), to_gpu(scales)))
        want.append(oracle.slice_and_scale(codes, scales, anchor, target))
    got = mx.mx_slice_and_scale_batched(anchors, mx.make_format(anchor), mx.make_format(target))
    torch.cuda.synchronize()
    for i, ((gc, gs), (wc, ws)) in enumerate(zip(got, want)):
        assert np.array_equal(to_host(gs), ws), i
        assert np.array_equal(to_host(gc), wc), i


@pytest.mark.parametrize("anchor,target", [("e4m3", "e2m1"), ("int8", "int6"), ("int8", "int5")])
def test_slice_and_scale_batched_large_segments(mx, oracle, anchor, target):
    # tensors big enough that the launch cuts them into its large segments (1024 workgroups), with ragged ends:
    # a last code segment that is nearly empty, one that is nearly full, and a scale segment of a few bytes
    import torch
    sizes = [(1 << 20) + 37, (1 << 21) - 5, 1 << 20]
    anchors, want = [], []
    for i, nb in enumerate(sizes):
        codes = synth.random_bytes(4100 + i, nb * 32).reshape(nb, 32)
        scales = synth.random_bytes(5100 + i, nb)
        anchors.append((to_gpu(codes), to_gpu(scales)))
        want.append(oracle.slice_and_scale(codes, scales, anchor, target))
    got = mx.mx_slice_and_scale_batched(anchors, mx.make_format(anchor), mx.make_format(target))
    torch.cuda.synchronize()
    for i, ((gc, gs), (wc, ws)) in enumerate(zip(got, want)):
        assert np.array_equal(to_host(gs), ws), i
        assert np.array_equal(to_host(gc), wc), i


MULTI_SETS = [("int8", ["int6", "int4"]), ("e4m3", ["e3m2", "e2m3", "e2m1"]), ("e4m3", ["e3m2", "e2m1"]),
              ("e4m3", ["e2m3", "e2m1"]), ("e4m3", ["e3m2", "e2m3"])]


@pytest.mark.parametrize("anchor,targets", MULTI_SETS)
def test_slice_and_scale_multi_target(mx, oracle, anchor, targets):
    # several targets from one pass over the anchor: each output is what the single conversion gives
    fa = mx.make_format(anchor)
    for nblocks, seed in ((1, 11), (33, 12), (8192 + 17, 13)):
        codes = synth.random_bytes(seed, nblocks * 32).reshape(nblocks, 32)
        scales = synth.random_bytes(seed + 100, nblocks)
        outs = mx.mx_slice_and_scale_multi(to_gpu(codes), to_gpu(scales), fa, [mx.make_format(t) for t in targets])
        for t, (gc, gs) in zip(targets, outs):
            wc, ws = oracle.slice_and_scale(codes, scales, anchor, t)
            assert np.array_equal(to_host(gs), ws), (t, nblocks)
            assert np.array_equal(to_host(gc), wc), (t, nblocks)


def test_slice_and_scale_multi_target_batched(mx, oracle):
    import torch
    sizes = [1, 33, 9000, 7, 4096, 300] * 9            # 54 tensors: more than one table chunk
    anchors, host = [], []
    for i, nb in enumerate(sizes):
        codes = synth.random_bytes(700 + i, nb * 32).reshape(nb, 32)
        scales = synth.random_bytes(1700 + i, nb)
        anchors.append((to_gpu(codes), to_gpu(scales)))
        host.append((codes, scales))
    targets = ["e3m2", "e2m3", "e2m1"]
    got = mx.SsBatch(anchors, mx.make_format("e4m3"), [mx.make_format(t) for t in targets]).run()
    torch.cuda.synchronize()
    for i, row in enumerate(got):
        for t, (gc, gs) in zip(targets, row):
            wc, ws = oracle.slice_and_scale(host[i][0], host[i][1], "e4m3", t)
            assert np.array_equal(to_host(gs), ws), (i, t)
            assert np.array_equal(to_host(gc), wc), (i, t)


def test_slice_and_scale_multi_target_rejections(mx):
    import torch
    c = torch.zeros((4, 32), dtype=torch.uint8, device="cuda")
    s = torch.zeros((4,), dtype=torch.uint8, device="cuda")
    for anchor, targets in (("e4m3", ["e2m1", "e3m2"]),          # not in increasing element order
                            ("int8", ["int6", "int5", "int4"]),  # a set without a kernel
                            ("e4m3", ["e3m2", "int4"])):         # mixed families
        with pytest.raises(mx.MxError):
            mx.mx_slice_and_scale_multi(c, s, mx.make_format(anchor), [mx.make_format(t) for t in targets])


# ------------------------------------------------------------------------------------ quantize
def _quant_inputs(dtype):
    w1 = synth.config1_weight(seed=1001, rows=96, cols=1024 + 96)          # several tiles + ragged tail
    w2 = synth.bf16_bits_to_f32(synth.config2_weight(seed=1002, rows=64, cols=512))
    w3 = synth.edge_case_matrix(seed=21, rows=40, cols=256)
    w4 = synth.special_matrix(cols=128)
    w4 = np.concatenate([w4] * 8, axis=0)                                  # 32 rows so that axis 0 works too
    mats = [w1, w2, w3, w4]
    if dtype == "bf16":
        mats = [synth.f32_to_bf16_bits(m) for m in mats]
    return mats


@pytest.mark.parametrize("fmt", CORE + EXTRA)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("axis", [1, 0])
def test_quantize(mx, oracle, fmt, dtype, axis):
    for tie in (("default",) if fmt in EXTRA else ("default", "away", "even")):
        f = mx.make_format(fmt, axis=axis, round=tie)
        for m in _quant_inputs(dtype):
            if axis == 0:
                m = np.ascontiguousarray(m[: m.shape[0] // 32 * 32])
            want_c, want_s = oracle.quantize(m, fmt, axis=axis, tie=TIES[tie])
            got_c, got_s = mx.mx_quantize(to_gpu(m), f)
            assert np.array_equal(to_host(got_s), want_s), (tie, m.shape)
            assert np.array_equal(to_host(got_c), want_c), (tie, m.shape)


@pytest.mark.parametrize("fmt", ["int8", "e4m3", "e2m1", "e3m2", "int4", "int6"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("axis", [1, 0])
def test_quantize_strided_source(mx, oracle, fmt, dtype, axis):
    # leading dimension larger than the row length (a column slice of a wider matrix)
    m = synth.config1_weight(seed=31, rows=64, cols=640)
    if dtype == "bf16":
        m = synth.f32_to_bf16_bits(m)
    g = to_gpu(m)[:, 64:64 + 512]
    sub = np.ascontiguousarray(m[:, 64:64 + 512])
    f = mx.make_format(fmt, axis=axis)
    want_c, want_s = oracle.quantize(sub, fmt, axis=axis)
    got_c, got_s = mx.mx_quantize(g, f)
    assert np.array_equal(to_host(got_s), want_s)
    assert np.array_equal(to_host(got_c), want_c)


# ------------------------------------------------------------------------------------ dequant
@pytest.mark.parametrize("fmt", CORE + EXTRA)
@pytest.mark.parametrize("out", ["f32", "bf16"])
@pytest.mark.parametrize("axis", [1, 0])
def test_dequant_random_bytes(mx, oracle, fmt, out, axis):
    import torch
    rows, cols = 96, 1024 + 96
    f = mx.make_format(fmt, axis=axis)
    outer, nblocks, bb = mx.packed_shape(f, rows, cols)
    codes = synth.random_bytes(5, outer * nblocks * bb).reshape(outer, nblocks, bb)
    scales = synth.random_bytes(6, outer * nblocks).reshape(outer, nblocks)
    scales.reshape(-1)[:8] = np.array([0, 1, 2, 127, 250, 253, 254, 255], dtype=np.uint8)
    want = oracle.dequant(codes, scales, fmt, rows, cols, axis=axis, out=out)
    got = mx.mx_dequant(to_gpu(codes), to_gpu(scales), f, rows, cols,
                        dtype=torch.float32 if out == "f32" else torch.bfloat16)
    assert_same_values(to_host(got), want)


# ------------------------------------------------------------------------------------ fake-quant
@pytest.mark.parametrize("fmt", CORE + EXTRA)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("axis", [1, 0])
def test_fake_quant_direct(mx, oracle, fmt, dtype, axis):
    for tie in (("default",) if fmt in EXTRA else ("default", "away", "even")):
        f = mx.make_format(fmt, axis=axis, round=tie)
        for m in _quant_inputs(dtype):
            if axis == 0:
                m = np.ascontiguousarray(m[: m.shape[0] // 32 * 32])
            want = oracle.fake_quant(m, fmt, axis=axis, tie=TIES[tie])
            got = mx.mx_fake_quant(to_gpu(m), f)
            assert_same_values(to_host(got), want)


@pytest.mark.parametrize("anchor,target", SS_PAIRS)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("axis", [1, 0])
def test_fake_quant_via_anchor(mx, oracle, anchor, target, dtype, axis):
    for tie in ("default", "away"):
        fa, ft = mx.make_format(anchor, axis=axis, round=tie), mx.make_format(target, axis=axis, round=tie)
        for m in _quant_inputs(dtype):
            if axis == 0:
                m = np.ascontiguousarray(m[: m.shape[0] // 32 * 32])
            want = oracle.fake_quant(m, target, anchor=anchor, axis=axis, tie=TIES[tie])
            got = mx.mx_fake_quant(to_gpu(m), ft, anchor=fa)
            assert_same_values(to_host(got), want)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("k", [32, 16, 64, 128])
def test_fake_quant_down_columns_column_counts_of_4_mod_8(mx, oracle, dtype, k):
    """Down the columns the fake-quant kernel takes 16-byte chunks of a row (8 bf16 / 4 fp32 columns) when the column
    count allows it; bf16 tensors whose column count is 4 mod 8 take the kernels with 4 columns per lane.  Both kinds
    on neighbouring column counts, for every block size, with a padded leading dimension whose padding must stay
    untouched."""
    import torch
    rng = np.random.default_rng(77 + k)
    for cols in (4, 12, 100, 104, 516, 520):
        rows = 256
        ld = (cols + 7) // 8 * 8 + 8
        m = (rng.standard_normal((rows, cols)) * np.exp(rng.uniform(-3, 3, size=(rows, cols)))).astype(np.float32)
        host = synth.f32_to_bf16_bits(m) if dtype == "bf16" else m
        wide = np.zeros((rows, ld), dtype=host.dtype)
        wide[:, :cols] = host
        src = to_gpu(wide)[:, :cols]
        for fmt, anchor in (("e2m1", None), ("e2m1", "e4m3"), ("int4", "int8"), ("e3m2", None), ("int7", None)):
            f = mx.make_format(fmt, axis=0, block=k)
            fa = mx.make_format(anchor, axis=0, block=k) if anchor else None
            out_wide = torch.zeros((rows, ld), dtype=src.dtype, device="cuda")
            mx.mx_fake_quant(src, f, fa, out_wide[:, :cols])
            want = oracle.fake_quant(host, fmt, anchor=anchor, axis=0, k=k)
            assert_same_values(to_host(out_wide[:, :cols].contiguous()), want)
            assert not bool(out_wide[:, cols:].any()), (cols, fmt, anchor)


def test_fake_quant_in_place_and_ste(mx, oracle):
    import torch
    m = synth.config1_weight(seed=8, rows=64, cols=256)
    f = mx.make_format("e2m1")
    want = oracle.fake_quant(m, "e2m1", anchor="e4m3")
    g = to_gpu(m)
    mx.mx_fake_quant(g, f, anchor=mx.make_format("e4m3"), out=g)
    assert_same_values(to_host(g), want)
    # straight-through estimator: the gradient passes unchanged
    w = to_gpu(m).requires_grad_(True)
    y = mx.MxFakeQuantSTE.apply(w, f, mx.make_format("e4m3"))
    grad = torch.randn_like(y)
    y.backward(grad)
    assert torch.equal(w.grad, grad)
    assert_same_values(to_host(y.detach()), want)


# ------------------------------------------------------------------------------------ end to end, configs 1 and 2
def test_config1_end_to_end(mx, oracle):
    w = synth.config1_weight()
    f8 = mx.make_format("int8")
    c8, s8 = mx.mx_quantize(to_gpu(w), f8)
    wc8, ws8 = oracle.quantize(w, "int8")
    assert np.array_equal(to_host(c8), wc8) and np.array_equal(to_host(s8), ws8)
    for t in ("int6", "int4"):
        gc, gs = mx.mx_slice_and_scale(c8, s8, f8, mx.make_format(t))
        wc, ws = oracle.slice_and_scale(wc8, ws8, "int8", t)
        assert np.array_equal(to_host(gc), wc) and np.array_equal(to_host(gs), ws)
        deq = mx.mx_dequant(gc, gs, mx.make_format(t), 1024, 1024)
        assert_same_values(to_host(deq), oracle.dequant(wc, ws, t, 1024, 1024))


@pytest.mark.parametrize("axis", [1, 0])
def test_config2_end_to_end(mx, oracle, axis):
    w = synth.config2_weight()                          # the whole of config 2: 4096 x 4096, every byte compared
    f8 = mx.make_format("e4m3", axis=axis)
    c8, s8 = mx.mx_quantize(to_gpu(w), f8)
    wc8, ws8 = oracle.quantize(w, "e4m3", axis=axis)
    assert np.array_equal(to_host(s8), ws8) and np.array_equal(to_host(c8), wc8)
    for t in ("e3m2", "e2m3", "e2m1"):
        gc, gs = mx.mx_slice_and_scale(c8, s8, f8, mx.make_format(t, axis=axis))
        wc, ws = oracle.slice_and_scale(wc8, ws8, "e4m3", t)
        assert np.array_equal(to_host(gc), wc) and np.array_equal(to_host(gs), ws)
        deq = mx.mx_dequant(gc, gs, mx.make_format(t, axis=axis), 4096, 4096)
        assert_same_values(to_host(deq), oracle.dequant(wc, ws, t, 4096, 4096, axis=axis))


# ------------------------------------------------------------------------------------ every bf16 value
def _all_bf16_blocks():
    """Every one of the 65536 bf16 bit patterns (NaN / Inf included), 31 to a block, behind a leading element that
    sets the block's scale from far below to far above the values' own magnitudes."""
    vals = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    pad = (-len(vals)) % 31
    vals = np.concatenate([vals, np.zeros(pad, dtype=np.uint16)]).reshape(-1, 31)
    rows = []
    for leader in (0x0000, 0x0080, 0x2000, 0x3800, 0x3F80, 0x4300, 0x5000, 0x7F00, 0xBF80):   # 0, 2^-126, ..., 1, 128, ..., -1
        lead = np.full((vals.shape[0], 1), leader, dtype=np.uint16)
        rows.append(np.concatenate([lead, vals], axis=1).reshape(-1))
    flat = np.concatenate(rows)
    cols = 1024
    n = len(flat) // cols * cols
    return flat[:n].reshape(-1, cols)


@pytest.mark.parametrize("fmt", CORE + EXTRA)
def test_every_bf16_value(mx, oracle, fmt):
    m = _all_bf16_blocks()
    g = to_gpu(m)
    anchor = None if fmt in ("int8", "e4m3") else ("int8" if fmt.startswith("int") else "e4m3")
    for tie in ("default", "away", "even"):
        f = mx.make_format(fmt, round=tie)
        want_c, want_s = oracle.quantize(m, fmt, tie=TIES[tie])
        got_c, got_s = mx.mx_quantize(g, f)
        assert np.array_equal(to_host(got_s), want_s), tie
        assert np.array_equal(to_host(got_c), want_c), tie
        assert_same_values(to_host(mx.mx_fake_quant(g, f)), oracle.fake_quant(m, fmt, tie=TIES[tie]))
        if anchor is not None:
            fa = mx.make_format(anchor, round=tie)
            assert_same_values(to_host(mx.mx_fake_quant(g, f, anchor=fa)), oracle.fake_quant(m, fmt, anchor=anchor, tie=TIES[tie]))
