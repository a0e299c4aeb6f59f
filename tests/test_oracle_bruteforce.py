"""Pins of the oracle's arithmetic by exhaustive nearest-value search (definition of
"round to nearest, clamp") and by the hand-computed worked examples."""
import os
from fractions import Fraction

import numpy as np
import pytest

import defs
from paper_2604_00529_amd import synth

TIES = {"default": 0, "away": 1, "even": 2}
SS_PAIRS = [("int8", "int6"), ("int8", "int4"), ("e4m3", "e3m2"), ("e4m3", "e2m3"), ("e4m3", "e2m1"),
            ("int8", "int7"), ("int8", "int5"), ("int8", "int3"), ("int8", "int2"),
            ("e4m3", "e3m3"), ("e4m3", "e2m2")]


@pytest.mark.parametrize("fmt", defs.ALL_FORMATS)
@pytest.mark.parametrize("tie", ["default", "away", "even"])
def test_encode_dense_sweep_is_nearest(oracle, fmt, tie):
    # every multiple of 1/16 up to beyond saturation, both signs: includes all ties of every format here
    top = max(v for _, v in defs.value_table(fmt))
    n = int(min(top * 16 + 40, 600 * 16))
    for i in list(range(0, n + 1)) + ([int(top * 16) + j for j in range(-20, 300, 7)] if n < top * 16 else []):
        for sgn in (1, -1):
            r = Fraction(sgn * i, 16)
            want = defs.nearest_code(fmt, r, tie, negative_zero=(sgn < 0 and i == 0))
            got = oracle.encode(fmt, float(r) if i else (0.0 if sgn > 0 else -0.0), TIES[tie])
            assert got == want, (fmt, tie, r)


@pytest.mark.parametrize("fmt", [f for f in defs.ALL_FORMATS if not defs.is_int(f)])
def test_encode_fine_sweep_near_zero(oracle, fmt):
    # subnormal range and ties below the smallest normal, on a 2^-12 grid
    for i in range(0, 4096 * 2 + 1):
        r = Fraction(i, 4096)
        assert oracle.encode(fmt, float(r), 0) == defs.nearest_code(fmt, r)
        assert oracle.encode(fmt, -float(r), 2) == defs.nearest_code(fmt, -r, "even", negative_zero=(i == 0))


@pytest.mark.parametrize("anchor,target", SS_PAIRS)
@pytest.mark.parametrize("tie", ["default", "away", "even"])
def test_slice_map_all_256_codes(oracle, anchor, target, tie):
    # Eq. (4) / Eq. (6) element step for every anchor code, by exhaustive nearest search on P_h / 2^De
    de = defs.emax(anchor) - defs.emax(target)
    assert de == oracle.delta_e(anchor, target)
    tab = dict(defs.value_table(anchor))
    for code in range(256):
        if code not in tab:                      # E4M3 NaN: +-max normal when the target has no NaN
            val = Fraction(448) * (-1 if code & 0x80 else 1)
        else:
            val = tab[code]
        want = defs.nearest_code(target, val / 2 ** de, tie, negative_zero=(val == 0 and code & 0x80 != 0))
        assert oracle.slice_code(anchor, target, code, TIES[tie]) == want, (hex(code),)


def test_slice_int_equals_shift_and_round_on_dropped_bit(oracle):
    # Sec. 3.3: "right shift by De, drop the De LSBs, round using the most significant dropped bit"
    # (applied to the magnitude), then clip.  A second, integer-only formulation.
    for bl in range(2, 8):
        de = 8 - bl
        lim = 2 ** (bl - 1) - 1
        for code in range(256):
            p = code if code < 128 else code - 256
            mag = abs(p)
            q = (mag >> de) + ((mag >> (de - 1)) & 1)
            q = min(q, lim)
            want = (q if p >= 0 else -q) & (2 ** bl - 1)
            assert oracle.slice_code("int8", f"int{bl}", code) == want


@pytest.mark.parametrize("fmt", defs.ALL_FORMATS)
def test_scale_byte_floor_log2(oracle, fmt):
    em = defs.emax(fmt)
    vals = [2.0 ** e for e in range(-149, 128)] + [1.99, 3.0e38, 1.4e-45, 0.3, 5e-39, 1.1754942e-38]
    for v in vals:
        v = float(np.float32(v))
        for w in (v, np.nextafter(np.float32(v), np.float32(0)), np.nextafter(np.float32(v), np.float32(np.inf))):
            w = float(w)
            if w == 0 or np.isinf(w):
                continue
            want = max(-127, min(127, defs.floor_log2(Fraction(w)) - em)) + 127
            assert oracle.scale_byte(w, fmt) == want
    assert oracle.scale_byte(0.0, fmt) == 0
    assert oracle.scale_byte(float("inf"), fmt) == 255
    assert oracle.scale_byte(float("nan"), fmt) == 255


@pytest.mark.parametrize("fmt", ["int8", "int6", "int4", "e4m3", "e3m2", "e2m3", "e2m1", "int2", "e3m3", "e2m2"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_quantize_small_tensors_bruteforce(oracle, fmt, dtype):
    k = 32
    mats = [synth.edge_case_matrix(seed=11, rows=10, cols=64, dtype=dtype)]
    w = synth.config1_weight(seed=5, rows=4, cols=128)
    mats.append(w if dtype == "f32" else synth.f32_to_bf16_bits(w))
    for m in mats:
        vals = m if dtype == "f32" else synth.bf16_bits_to_f32(m)
        for tie in ("default", "even" if defs.is_int(fmt) else "away"):
            codes, scales = oracle.quantize(m, fmt, axis=1, k=k, tie=TIES[tie])
            un = oracle.unpack(codes, fmt, k)
            for r in range(m.shape[0]):
                for j in range(m.shape[1] // k):
                    byte, want = defs.quantize_block(fmt, [float(v) for v in vals[r, j * k:(j + 1) * k]], tie)
                    assert scales[r, j] == byte, (r, j)
                    assert list(un[r, j]) == want, (r, j)


@pytest.mark.parametrize("k", [16, 64, 128])
@pytest.mark.parametrize("fmt", ["int8", "int4", "e4m3", "e2m1"])
def test_quantize_other_block_sizes_bruteforce(oracle, fmt, k):
    # Eq. (1) / (2) block by block for the block sizes of the paper's sweep (Sec. 4.3): the scale byte comes from the
    # maximum over exactly k consecutive elements and element j of block b sits at position j of that block's codes
    w = synth.config1_weight(seed=6, rows=3, cols=256)
    w[1, 70] = 37.5                                   # an outlier that must move one block's scale only
    codes, scales = oracle.quantize(w, fmt, axis=1, k=k)
    un = oracle.unpack(codes, fmt, k)
    assert scales.shape == (3, 256 // k)
    for r in range(3):
        for j in range(256 // k):
            byte, want = defs.quantize_block(fmt, [float(v) for v in w[r, j * k:(j + 1) * k]], "default")
            assert scales[r, j] == byte, (r, j)
            assert list(un[r, j]) == want, (r, j)


def test_quantize_axis0_is_transpose_of_axis1(oracle):
    # blocks along axis 0 of M are blocks along axis 1 of M^T, packed with outer = cols
    # (for every block size; the block-by-block brute force pins axis 1 for blocks of 32 above and of 16 / 64 / 128 below)
    m = synth.config1_weight(seed=9, rows=128, cols=48)
    for k in (32, 16, 64, 128):
        for fmt in ("int8", "e4m3", "e2m1", "e3m2"):
            c0, s0 = oracle.quantize(m, fmt, axis=0, k=k)
            c1, s1 = oracle.quantize(np.ascontiguousarray(m.T), fmt, axis=1, k=k)
            assert np.array_equal(c0, c1) and np.array_equal(s0, s1)
            assert s0.shape == (48, 128 // k)
            d0 = oracle.dequant(c0, s0, fmt, 128, 48, axis=0, k=k)
            d1 = oracle.dequant(c1, s1, fmt, 48, 128, axis=1, k=k)
            assert np.array_equal(d0, d1.T)
            f0 = oracle.fake_quant(m, fmt, axis=0, k=k)
            assert np.array_equal(f0, d0)


def _read_examples():
    path = os.path.join(defs.GOLDEN, "worked_examples.txt")
    rows = []
    with open(path) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


def test_worked_examples(oracle):
    rows = _read_examples()
    v = None
    anchors = {}
    n_checked = 0
    for row in rows:
        if row[0] == "input":
            v = np.array([[float(t) for t in row[1:]]], dtype=np.float32)
        elif row[0] == "quantize":
            fmt, byte, codes = row[1], int(row[2]), [int(t, 16) for t in row[3:]]
            c, s = oracle.quantize(v, fmt, axis=1, k=v.shape[1])
            assert s[0, 0] == byte
            assert list(oracle.unpack(c, fmt, v.shape[1])[0, 0]) == codes
            anchors[fmt] = (c, s)
            n_checked += 1
        elif row[0] == "slice":
            fa, ft, byte, codes = row[1], row[2], int(row[3]), [int(t, 16) for t in row[4:]]
            c, s = oracle.slice_and_scale(*anchors[fa], fa, ft, k=v.shape[1])
            assert s[0, 0] == byte
            assert list(oracle.unpack(c, ft, v.shape[1])[0, 0]) == codes
            n_checked += 1
        elif row[0] == "tie":
            p, away, even = int(row[1]), int(row[2]), int(row[3])
            assert oracle.slice_code("int8", "int4", p & 0xFF, 0) == away & 0xF
            assert oracle.slice_code("int8", "int4", p & 0xFF, 1) == away & 0xF
            assert oracle.slice_code("int8", "int4", p & 0xFF, 2) == even & 0xF
            n_checked += 1
    assert n_checked >= 14


def test_double_rounding_example(oracle):
    # V/X_h = 7.6 -> P_h = 8 -> slice gives 1; direct MXINT4 of the same block gives 0 for that element.
    # Block max 127/64 keeps floor(log2) = 0 so X_h = 2^-6 and X_l = 2^-2.
    v = np.zeros((1, 32), dtype=np.float32)
    v[0, 0] = 127.0 / 64.0
    v[0, 1] = 7.6 / 64.0
    ca, sa = oracle.quantize(v, "int8")
    assert oracle.unpack(ca, "int8")[0, 0, 1] == 8
    cs, ss = oracle.slice_and_scale(ca, sa, "int8", "int4")
    cd, sd = oracle.quantize(v, "int4")
    assert ss[0, 0] == sd[0, 0] == 125
    assert oracle.unpack(cs, "int4")[0, 0, 1] == 1
    assert oracle.unpack(cd, "int4")[0, 0, 1] == 0
