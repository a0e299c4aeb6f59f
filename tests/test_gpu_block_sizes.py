"""Block sizes other than 32 on the GPU (blocks along a row, and down a column): 16, 64 and 128 -- the sizes of the paper's
block-size sweep (Sec. 4.3, App. C; its bit sweep uses 64).  Every entry point against the oracle, bit for bit,
and the paper's own study shape: 100 random (1, 1024) tensors, quantized directly and through Slice-and-Scale."""
import numpy as np
import pytest

from paper_2604_00529_amd import synth
from test_gpu_parity import TIES, assert_same_values, mx, to_gpu, to_host  # noqa: F401  (mx is the module fixture)

pytestmark = pytest.mark.gpu

BLOCKS = [16, 64, 128]
FORMATS = ["int8", "int6", "int5", "int4", "int2", "e4m3", "e3m2", "e2m3", "e2m2", "e2m1"]
SS_PAIRS = [("int8", "int6"), ("int8", "int4"), ("int8", "int3"), ("e4m3", "e3m2"), ("e4m3", "e2m3"), ("e4m3", "e2m1")]


def _inputs(dtype):
    w1 = synth.config1_weight(seed=1101, rows=48, cols=1024 + 384)        # 1408 = 11 * 128: several tiles + a tail
    w3 = synth.edge_case_matrix(seed=23, rows=40, cols=256)
    w4 = synth.special_matrix(cols=128)
    mats = [w1, w3, w4]
    if dtype == "bf16":
        mats = [synth.f32_to_bf16_bits(m) for m in mats]
    return mats


@pytest.mark.parametrize("k", BLOCKS)
@pytest.mark.parametrize("fmt", FORMATS)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_quantize_dequant_fake_quant(mx, oracle, k, fmt, dtype):
    import torch
    for tie in ("default", "away"):
        f = mx.make_format(fmt, block=k, round=tie)
        for m in _inputs(dtype):
            want_c, want_s = oracle.quantize(m, fmt, k=k, tie=TIES[tie])
            got_c, got_s = mx.mx_quantize(to_gpu(m), f)
            assert np.array_equal(to_host(got_s), want_s), (tie, m.shape)
            assert np.array_equal(to_host(got_c), want_c), (tie, m.shape)
            want_f = oracle.fake_quant(m, fmt, k=k, tie=TIES[tie])
            assert_same_values(to_host(mx.mx_fake_quant(to_gpu(m), f)), want_f)
            out = "f32" if dtype == "f32" else "bf16"
            want_d = oracle.dequant(want_c, want_s, fmt, m.shape[0], m.shape[1], k=k, out=out)
            got_d = mx.mx_dequant(got_c, got_s, f, m.shape[0], m.shape[1],
                                  dtype=torch.float32 if out == "f32" else torch.bfloat16)
            assert_same_values(to_host(got_d), want_d)


@pytest.mark.parametrize("k", BLOCKS)
@pytest.mark.parametrize("anchor,target", SS_PAIRS)
def test_slice_and_scale_and_fake_quant_via_anchor(mx, oracle, k, anchor, target):
    fa, ft = mx.make_format(anchor, block=k), mx.make_format(target, block=k)
    bb = k * oracle.elem_bits(anchor) // 8
    for nblocks, seed in ((2, 1), (34, 2), (4096 + 6, 3)):
        codes = synth.random_bytes(seed, nblocks * bb).reshape(nblocks, bb)
        scales = synth.random_bytes(seed + 50, nblocks)
        scales[:2] = np.array([254, 255], dtype=np.uint8)
        want_c, want_s = oracle.slice_and_scale(codes, scales, anchor, target, k=k)
        got_c, got_s = mx.mx_slice_and_scale(to_gpu(codes), to_gpu(scales), fa, ft)
        assert np.array_equal(to_host(got_s), want_s), nblocks
        assert np.array_equal(to_host(got_c), want_c), nblocks
    # several tensors in one launch
    sizes = [2, 66, 1024, 8, 4098]
    anchors, want = [], []
    for i, nb in enumerate(sizes):
        c = synth.random_bytes(300 + i, nb * bb).reshape(nb, bb)
        s = synth.random_bytes(400 + i, nb)
        anchors.append((to_gpu(c), to_gpu(s)))
        want.append(oracle.slice_and_scale(c, s, anchor, target, k=k))
    got = mx.mx_slice_and_scale_batched(anchors, fa, ft)
    for (gc, gs), (wc, ws) in zip(got, want):
        assert np.array_equal(to_host(gs), ws) and np.array_equal(to_host(gc), wc)
    for dtype in ("f32", "bf16"):
        for m in _inputs(dtype):
            want_f = oracle.fake_quant(m, target, anchor=anchor, k=k)
            assert_same_values(to_host(mx.mx_fake_quant(to_gpu(m), ft, anchor=fa)), want_f)


def test_odd_width_needs_whole_runs_of_32_codes(mx):
    import torch
    c = torch.zeros((3, 16), dtype=torch.uint8, device="cuda")      # 3 blocks of 16 codes: 48 codes
    s = torch.zeros((3,), dtype=torch.uint8, device="cuda")
    with pytest.raises(mx.MxError) as e:
        mx.mx_slice_and_scale(c, s, mx.make_format("int8", block=16), mx.make_format("int5", block=16))
    assert e.value.status == 5


@pytest.mark.parametrize("rows,cols", [(1, 16), (3, 48), (5, 80)])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_blocks_of_16_ending_in_half_a_run_of_32_codes(mx, oracle, rows, cols, dtype):
    # an odd number of blocks of 16: the last run of 32 codes is half empty.  8- and 4-bit elements are converted (and
    # nothing is written past the end of the codes: guard bytes behind them stay untouched), the other widths refused
    import torch
    rng = np.random.default_rng(rows * 100 + cols)
    m = (rng.standard_normal((rows, cols)) * 3).astype(np.float32)
    if dtype == "bf16":
        m = synth.f32_to_bf16_bits(m)
    g = to_gpu(m)
    nb = rows * cols // 16
    for fmt in ("int8", "e4m3", "int4", "e2m1"):
        f = mx.make_format(fmt, block=16)
        bb = 16 * oracle.elem_bits(fmt) // 8
        codes = torch.full((nb * bb + 64,), 0xA5, dtype=torch.uint8, device="cuda")
        scales = torch.full((nb + 64,), 0xA5, dtype=torch.uint8, device="cuda")
        mx.mx_quantize(g, f, codes[:nb * bb].view(rows, cols // 16, bb), scales[:nb].view(rows, cols // 16))
        torch.cuda.synchronize()
        want_c, want_s = oracle.quantize(m, fmt, k=16)
        assert np.array_equal(to_host(codes[:nb * bb]).reshape(want_c.shape), want_c), fmt
        assert np.array_equal(to_host(scales[:nb]).reshape(want_s.shape), want_s), fmt
        assert bool((codes[nb * bb:] == 0xA5).all()) and bool((scales[nb:] == 0xA5).all()), fmt
        out = "f32" if dtype == "f32" else "bf16"
        got_d = mx.mx_dequant(codes[:nb * bb].view(rows, cols // 16, bb), scales[:nb].view(rows, cols // 16), f, rows, cols,
                              dtype=torch.float32 if out == "f32" else torch.bfloat16)
        assert_same_values(to_host(got_d), oracle.dequant(want_c, want_s, fmt, rows, cols, k=16, out=out))
        assert_same_values(to_host(mx.mx_fake_quant(g, f)), oracle.fake_quant(m, fmt, k=16))
    for fmt in ("int7", "int6", "int5", "int3", "int2", "e3m3", "e3m2", "e2m3", "e2m2"):
        f = mx.make_format(fmt, block=16)
        with pytest.raises(mx.MxError) as e:
            mx.mx_quantize(g, f)
        assert e.value.status == 5, fmt
        # fake-quant touches no codes and takes every width
        assert_same_values(to_host(mx.mx_fake_quant(g, f)), oracle.fake_quant(m, fmt, k=16))


def _column_inputs(dtype):
    # rows a multiple of 128 (every block size divides them): 1, 3 and 5 tiles of 4 windows, the last one ragged
    # (12 and 20 windows); more than 256 columns and a ragged column tile
    w1 = synth.config1_weight(seed=1201, rows=128, cols=520)
    w2 = synth.config1_weight(seed=1202, rows=384, cols=72)
    w3 = np.ascontiguousarray(np.concatenate([synth.edge_case_matrix(seed=29, rows=40, cols=256)] * 16, axis=0)[:640])
    w4 = np.concatenate([synth.special_matrix(cols=128)] * 32, axis=0)[:128]
    mats = [w1, w2, w3, w4]
    if dtype == "bf16":
        mats = [synth.f32_to_bf16_bits(m) for m in mats]
    return mats


@pytest.mark.parametrize("k", BLOCKS)
@pytest.mark.parametrize("fmt", FORMATS)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_column_blocks_quantize_dequant_fake_quant(mx, oracle, k, fmt, dtype):
    # blocks of 16, 64 and 128 rows down the columns (axis 0): every entry point against the oracle, bit for bit
    import torch
    for tie in ("default", "away"):
        f = mx.make_format(fmt, axis=0, block=k, round=tie)
        for m in _column_inputs(dtype):
            want_c, want_s = oracle.quantize(m, fmt, axis=0, k=k, tie=TIES[tie])
            got_c, got_s = mx.mx_quantize(to_gpu(m), f)
            assert np.array_equal(to_host(got_s), want_s), (tie, m.shape)
            assert np.array_equal(to_host(got_c), want_c), (tie, m.shape)
            want_f = oracle.fake_quant(m, fmt, axis=0, k=k, tie=TIES[tie])
            assert_same_values(to_host(mx.mx_fake_quant(to_gpu(m), f)), want_f)
            out = "f32" if dtype == "f32" else "bf16"
            want_d = oracle.dequant(want_c, want_s, fmt, m.shape[0], m.shape[1], axis=0, k=k, out=out)
            got_d = mx.mx_dequant(got_c, got_s, f, m.shape[0], m.shape[1],
                                  dtype=torch.float32 if out == "f32" else torch.bfloat16)
            assert_same_values(to_host(got_d), want_d)


@pytest.mark.parametrize("k", BLOCKS)
@pytest.mark.parametrize("anchor,target", [("int8", "int4"), ("e4m3", "e2m1"), ("e4m3", "e3m2")])
def test_column_blocks_via_anchor(mx, oracle, k, anchor, target):
    # Eq. (7) with column blocks of every size, and the stored-anchor route (quantize, Slice-and-Scale, dequantize)
    # that it must equal
    import torch
    fa, ft = mx.make_format(anchor, axis=0, block=k), mx.make_format(target, axis=0, block=k)
    for m in _column_inputs("bf16")[:2]:
        want = oracle.fake_quant(m, target, anchor=anchor, axis=0, k=k)
        assert_same_values(to_host(mx.mx_fake_quant(to_gpu(m), ft, anchor=fa)), want)
        c8, s8 = mx.mx_quantize(to_gpu(m), fa)
        ct, st = mx.mx_slice_and_scale(c8, s8, fa, ft)
        got = mx.mx_dequant(ct, st, ft, m.shape[0], m.shape[1], dtype=torch.bfloat16)
        assert_same_values(to_host(got), want)


def test_column_blocks_of_16_need_whole_windows_of_32_rows(mx):
    import torch
    w = torch.zeros((48, 64), dtype=torch.float32, device="cuda")       # 3 blocks of 16 rows: half a window is left over
    with pytest.raises(mx.MxError) as e:
        mx.mx_fake_quant(w, mx.make_format("int4", axis=0, block=16))
    assert e.value.status == 5


@pytest.mark.parametrize("k", [16, 32, 64, 128])
def test_tensor_level_study_shape(mx, oracle, k):
    # Sec. 4.3 / App. C: 100 random (1, 1024) tensors; direct quantization to every lower format and Slice-and-Scale
    # from the 8-bit anchor, both paths bit for bit against the oracle, and on the GPU results the error ratio that the
    # double rounding implies: MSE(sliced) / MSE(direct) = 1 + 3 * 4^-d for d dropped bits of precision (MXINT8 -> 6:
    # d = 2, 1.19; E4M3 -> E3M2: d = 1, 1.75), i.e. Slice-and-Scale stays close to direct quantization
    tensors = synth.random_tensors_1x1024()
    x = np.concatenate(tensors, axis=0)                                  # [100, 1024]
    g = to_gpu(x)
    for anchor, targets in (("int8", ("int6", "int4", "int2")), ("e4m3", ("e3m2", "e2m1"))):
        fa = mx.make_format(anchor, block=k)
        a_c, a_s = mx.mx_quantize(g, fa)
        wa_c, wa_s = oracle.quantize(x, anchor, k=k)
        assert np.array_equal(to_host(a_c), wa_c) and np.array_equal(to_host(a_s), wa_s)
        for t in targets:
            ft = mx.make_format(t, block=k)
            direct = to_host(mx.mx_fake_quant(g, ft))
            sliced = to_host(mx.mx_fake_quant(g, ft, anchor=fa))
            assert_same_values(direct, oracle.fake_quant(x, t, k=k))
            assert_same_values(sliced, oracle.fake_quant(x, t, anchor=anchor, k=k))
            s_c, s_s = mx.mx_slice_and_scale(a_c, a_s, fa, ft)
            w_c, w_s = oracle.slice_and_scale(wa_c, wa_s, anchor, t, k=k)
            assert np.array_equal(to_host(s_c), w_c) and np.array_equal(to_host(s_s), w_s)
            mse_d = float(np.mean((direct.astype(np.float64) - x) ** 2))
            mse_s = float(np.mean((sliced.astype(np.float64) - x) ** 2))
            ratio = mse_s / mse_d
            if t == "int6":
                assert 1.15 < ratio < 1.23, (t, ratio)
            elif t == "e3m2":
                assert 1.5 < ratio < 1.9, (t, ratio)
            elif t == "e2m1":                       # d = 2, less where E2M1 saturates
                assert 1.05 < ratio < 1.25, (t, ratio)
            else:                                   # int4: d = 4, int2: d = 6
                assert 0.999 < ratio < 1.03, (t, ratio)
