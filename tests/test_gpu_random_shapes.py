"""Seeded sweep over random shapes, formats, block sizes, axes, leading dimensions and value mixes: every dense entry
point and Slice-and-Scale against the oracle, bit for bit.  The fixed-shape parity tests pick their sizes by hand; this
one draws them, so that shapes nobody thought of (one row, one block per row, a block count that leaves half a wave,
padded rows) get exercised too.  Every case is small; the whole module is a few seconds on the GPU."""
import numpy as np
import pytest

from paper_2604_00529_amd import synth
from test_gpu_parity import CORE, EXTRA, SS_PAIRS, assert_same_values, to_gpu, to_host, mx  # noqa: F401  (mx: fixture)

pytestmark = pytest.mark.gpu


def _values(rng, rows, cols):
    """A matrix mixing ordinary weights with the degenerate cases, block by block."""
    kind = rng.integers(0, 5)
    if kind == 0:
        m = rng.standard_normal((rows, cols)) * 0.02
    elif kind == 1:
        m = rng.standard_t(3, size=(rows, cols)) * np.exp(rng.uniform(-30, 30))
    elif kind == 2:
        m = rng.integers(-512, 513, size=(rows, cols)) / 32.0                # many exact ties
    elif kind == 3:
        m = rng.standard_normal((rows, cols)) * np.exp(rng.uniform(-60, 60, size=(rows, cols)))
    else:
        m = rng.standard_normal((rows, cols)) * 1e-40                        # fp32 subnormals
    m = m.astype(np.float32)
    for _ in range(int(rng.integers(0, 4))):                                 # a few special entries
        r, c = int(rng.integers(rows)), int(rng.integers(cols))
        m[r, c] = [np.nan, np.inf, -np.inf, 0.0, -0.0, 3.0e38][int(rng.integers(6))]
    if rng.integers(3) == 0:
        m[int(rng.integers(rows))] = 0.0                                     # all-zero blocks
    return m


def _shape(rng, axis, k):
    if axis == 1:
        rows = int(rng.choice([1, 2, 3, 5, 17, 33, 64, 100]))
        cols = k * int(rng.choice([1, 2, 3, 5, 8, 13, 24, 40]))
        cols = (cols + 7) // 8 * 8 if k < 8 else cols
    else:
        rows = max(k, 32) * int(rng.choice([1, 2, 3, 5, 9]))                 # whole blocks, and whole windows of 32 rows
        cols = 8 * int(rng.choice([1, 2, 3, 7, 16, 33, 65, 130]))
    return rows, cols


@pytest.mark.parametrize("seed", range(160))
def test_dense_entry_points_random_case(mx, oracle, seed):
    import torch
    rng = np.random.default_rng(7000 + seed)
    axis = int(rng.integers(0, 2))
    k = int(rng.choice([32, 32, 16, 64, 128])) if axis == 0 else int(rng.choice([16, 32, 64, 128]))
    fmt = str(rng.choice(CORE + EXTRA))
    dtype = str(rng.choice(["f32", "bf16"]))
    tie = str(rng.choice(["default", "away", "even"]))
    tie_id = {"default": 0, "away": 1, "even": 2}[tie]
    rows, cols = _shape(rng, axis, k)
    pad = 8 * int(rng.integers(0, 3))                                        # leading dimension = cols + pad
    m = _values(rng, rows, cols)
    host = synth.f32_to_bf16_bits(m) if dtype == "bf16" else m
    wide = np.zeros((rows, cols + pad), dtype=host.dtype)
    wide[:, :cols] = host
    src = to_gpu(wide)[:, :cols]
    f = mx.make_format(fmt, axis=axis, block=k, round=tie)
    case = (seed, fmt, dtype, axis, k, tie, rows, cols, pad)

    want_c, want_s = oracle.quantize(host, fmt, axis=axis, k=k, tie=tie_id)
    # blocks of 16 ending in half a run of 32 codes: only 8- and 4-bit elements have a packed form on the GPU
    packed_ok = not (k == 16 and (rows * cols) % 32 != 0 and oracle.elem_bits(fmt) not in (8, 4))
    if packed_ok:
        got_c, got_s = mx.mx_quantize(src, f)
        assert np.array_equal(to_host(got_s), want_s), case
        assert np.array_equal(to_host(got_c), want_c), case
    else:
        with pytest.raises(mx.MxError) as e:
            mx.mx_quantize(src, f)
        assert e.value.status == 5, case

    out_wide = torch.zeros((rows, cols + pad), dtype=src.dtype, device="cuda")
    mx.mx_fake_quant(src, f, None, out_wide[:, :cols])
    assert_same_values(to_host(out_wide[:, :cols].contiguous()), oracle.fake_quant(host, fmt, axis=axis, k=k, tie=tie_id))
    assert not bool(out_wide[:, cols:].any()), case                          # the padding is not written

    anchor = "int8" if fmt.startswith("int") else "e4m3"
    if fmt != anchor:
        got = mx.mx_fake_quant(src, f, mx.make_format(anchor, axis=axis, block=k, round=tie))
        assert_same_values(to_host(got), oracle.fake_quant(host, fmt, anchor=anchor, axis=axis, k=k, tie=tie_id))

    # dequantize random bytes (every code, every scale byte) of the same shape
    codes = synth.random_bytes(seed, want_c.size).reshape(want_c.shape)
    scales = synth.random_bytes(seed + 1, want_s.size).reshape(want_s.shape)
    for out in ("f32", "bf16"):
        want = oracle.dequant(codes, scales, fmt, rows, cols, axis=axis, k=k, out=out)
        if not packed_ok:
            with pytest.raises(mx.MxError) as e:
                mx.mx_dequant(to_gpu(codes), to_gpu(scales), f, rows, cols, dtype=torch.float32 if out == "f32" else torch.bfloat16)
            assert e.value.status == 5, case
            continue
        got = mx.mx_dequant(to_gpu(codes), to_gpu(scales), f, rows, cols,
                            dtype=torch.float32 if out == "f32" else torch.bfloat16)
        assert_same_values(to_host(got), want)


@pytest.mark.parametrize("seed", range(96))
def test_slice_and_scale_random_case(mx, oracle, seed):
    rng = np.random.default_rng(9000 + seed)
    anchor, target = SS_PAIRS[int(rng.integers(len(SS_PAIRS)))]
    k = int(rng.choice([16, 32, 32, 64, 128]))
    tie = str(rng.choice(["default", "away", "even"]))
    bits = oracle.elem_bits(target)
    # odd widths are converted in runs of 32 codes: with block 16 the block count must be even
    nblocks = int(rng.choice([1, 2, 3, 31, 63, 64, 65, 127, 1000, 4097, 70001]))
    if bits % 2 and k == 16:
        nblocks += nblocks % 2
    codes = synth.random_bytes(seed, nblocks * k).reshape(nblocks, k)
    scales = synth.random_bytes(seed + 100, nblocks)
    scales[: min(8, nblocks)] = np.array([0, 1, 2, 127, 250, 253, 254, 255], dtype=np.uint8)[: min(8, nblocks)]
    want_c, want_s = oracle.slice_and_scale(codes, scales, anchor, target, k=k, tie={"default": 0, "away": 1, "even": 2}[tie])
    got_c, got_s = mx.mx_slice_and_scale(to_gpu(codes), to_gpu(scales), mx.make_format(anchor, block=k, round=tie),
                                         mx.make_format(target, block=k, round=tie))
    case = (seed, anchor, target, k, tie, nblocks)
    assert np.array_equal(to_host(got_s), want_s), case
    assert np.array_equal(to_host(got_c), want_c), case
