"""Pins of the oracle by what the paper and the mathematics fix: identity, the paper's scale
equivalence and residual-error statements (Sec. 3.3), the exact reduction of Slice-and-Scale
to direct quantization of the dequantized anchor, idempotence, symmetry, monotonicity and the
closed-form MSE ratio of the tensor-level study (Sec. 4.3 / App. C)."""
import math

import numpy as np
import pytest

from paper_2604_00529_amd import synth

SS_PAIRS = [("int8", "int6"), ("int8", "int4"), ("e4m3", "e3m2"), ("e4m3", "e2m3"), ("e4m3", "e2m1"),
            ("int8", "int7"), ("int8", "int5"), ("int8", "int3"), ("int8", "int2"),
            ("e4m3", "e3m3"), ("e4m3", "e2m2")]
CORE = ["int8", "int6", "int4", "e4m3", "e3m2", "e2m3", "e2m1"]


def _inputs():
    w1 = synth.config1_weight(seed=1001, rows=64, cols=256)
    w2 = synth.bf16_bits_to_f32(synth.config2_weight(seed=1002, rows=64, cols=256))
    w3 = synth.edge_case_matrix(seed=3, rows=12, cols=256)
    return [w1, w2, w3]


def test_identity_slice(oracle):
    # De = 0: same-format Slice-and-Scale returns the anchor unchanged (every byte but INT8 -128,
    # which the symmetric clip maps to -127)
    for fmt in ("int8", "e4m3"):
        for code in range(256):
            want = code
            if fmt == "int8" and code == 0x80:
                want = 0x81
            assert oracle.slice_code(fmt, fmt, code) == want
        for byte in range(256):
            assert oracle.slice_byte(fmt, fmt, byte) == byte


@pytest.mark.parametrize("anchor,target", SS_PAIRS)
def test_scale_equivalence(oracle, anchor, target):
    # Sec. 3.3: the low-precision scale obtained from the anchor's scale equals the one obtained
    # from the full-precision tensor (whenever the anchor's shared exponent was not clamped).
    for w in _inputs():
        ca, sa = oracle.quantize(w, anchor)
        _, ss = oracle.slice_and_scale(ca, sa, anchor, target)
        _, sd = oracle.quantize(w, target)
        ok = sa > 0
        assert ok.any()
        assert np.array_equal(ss[ok], sd[ok])


def _spacing(oracle, fmt, value):
    """Spacing of the element grid of `fmt` at |value| (in element units)."""
    kind, a, b = oracle.FORMATS[fmt]
    if kind == 0:
        return 1.0
    bias = 2 ** (a - 1) - 1
    mag = abs(value)
    e = 1 - bias if mag < 2.0 ** (1 - bias) else math.floor(math.log2(mag))
    e = min(e, oracle.emax(fmt))
    return 2.0 ** (e - b)


@pytest.mark.parametrize("anchor,target", SS_PAIRS)
def test_residual_error_bound_all_codes(oracle, anchor, target):
    # Sec. 3.3 below Eq. (4): X_l P_l ~ X_h P_h, residual only from the low-precision rounding:
    # |P_l - P_h / 2^De| <= half the target spacing there, and below one spacing when clamped.
    de = oracle.delta_e(anchor, target)
    top = oracle.max_normal(target)
    for code in range(256):
        p = oracle.decode(anchor, code)
        if math.isnan(p):
            continue
        r = p / 2.0 ** de
        q = oracle.decode(target, oracle.slice_code(anchor, target, code))
        if abs(r) <= top:
            assert abs(q - r) <= 0.5 * _spacing(oracle, target, r) + 1e-300
        else:
            assert abs(q) == top and abs(r) - top <= _spacing(oracle, target, top)   # equality only for the external INT8 code -128
        assert (q == 0) or (math.copysign(1, q) == math.copysign(1, r))


@pytest.mark.parametrize("anchor,target", SS_PAIRS)
def test_slice_vs_direct_within_one_step(oracle, anchor, target):
    # double rounding: slice and direct codes differ by at most one target step, never more
    for w in _inputs()[:2]:
        ca, sa = oracle.quantize(w, anchor)
        cs, ss = oracle.slice_and_scale(ca, sa, anchor, target)
        cd, sd = oracle.quantize(w, target)
        assert np.array_equal(ss, sd)
        us, ud = oracle.unpack(cs, target).astype(np.int64), oracle.unpack(cd, target).astype(np.int64)
        kind, a, b = oracle.FORMATS[target]
        bits = oracle.elem_bits(target)
        if kind == 0:      # two's complement -> signed value
            vs = np.where(us >= 2 ** (bits - 1), us - 2 ** bits, us)
            vd = np.where(ud >= 2 ** (bits - 1), ud - 2 ** bits, ud)
        else:              # sign-magnitude codes are monotone in the magnitude index
            sign = 2 ** (bits - 1)
            vs = np.where(us & sign, -(us & (sign - 1)), us & (sign - 1))
            vd = np.where(ud & sign, -(ud & (sign - 1)), ud & (sign - 1))
        assert np.abs(vs - vd).max() <= 1
        assert (vs != vd).mean() < 0.6


@pytest.mark.parametrize("anchor,target", SS_PAIRS)
def test_slice_equals_direct_quantization_of_dequantized_anchor(oracle, anchor, target):
    # SS(anchor) == Q_t(DQ(anchor)) exactly for anchors made by Q_A: max|P_h| lies in the top binade,
    # so floor(log2 max|X_h P_h|) = floor(log2 max|V|).  Two different code paths of the oracle
    # (code-to-code slice vs float quantizer) must agree bit for bit.
    for w in _inputs():
        rows, cols = w.shape
        ca, sa = oracle.quantize(w, anchor)
        deq = oracle.dequant(ca, sa, anchor, rows, cols)
        finite = np.isfinite(deq).reshape(rows, cols // 32, 32).all(axis=2) & (sa > 0)
        cs, ss = oracle.slice_and_scale(ca, sa, anchor, target)
        cd, sd = oracle.quantize(deq, target)
        nz = np.abs(deq).reshape(rows, cols // 32, 32).max(axis=2) > 0
        m = finite & nz
        assert m.sum() >= 64
        assert np.array_equal(ss[m], sd[m])
        assert np.array_equal(cs[m], cd[m])


@pytest.mark.parametrize("fmt", CORE + ["int2", "e3m3", "e2m2"])
def test_idempotence(oracle, fmt):
    # Q_f(DQ(Q_f(V))) == Q_f(V)
    for w in _inputs():
        rows, cols = w.shape
        c, s = oracle.quantize(w, fmt)
        d = oracle.dequant(c, s, fmt, rows, cols)
        c2, s2 = oracle.quantize(d, fmt)
        nz = (np.abs(d).reshape(rows, cols // 32, 32).max(axis=2) > 0) & (s > 0)
        assert np.array_equal(s[nz], s2[nz]) and np.array_equal(c[nz], c2[nz])
        # fake-quant is DQ o Q
        assert np.array_equal(oracle.fake_quant(w, fmt), d)


@pytest.mark.parametrize("fmt", CORE)
def test_negation_symmetry(oracle, fmt):
    for w in _inputs():
        rows, cols = w.shape
        c, s = oracle.quantize(w, fmt)
        cn, sn = oracle.quantize(-w, fmt)
        assert np.array_equal(s, sn)
        a = oracle.dequant(c, s, fmt, rows, cols)
        b = oracle.dequant(cn, sn, fmt, rows, cols)
        assert np.array_equal(a, -b)


@pytest.mark.parametrize("anchor,target", SS_PAIRS)
def test_slice_map_symmetric_and_monotone(oracle, anchor, target):
    vals = []
    for code in range(256):
        p = oracle.decode(anchor, code)
        if math.isnan(p) or (anchor == "int8" and code == 0x80):
            continue
        q = oracle.decode(target, oracle.slice_code(anchor, target, code))
        vals.append((p, q))
        # SS(-A) = -SS(A)
        neg = (256 - code) & 0xFF if anchor == "int8" else code ^ 0x80
        qn = oracle.decode(target, oracle.slice_code(anchor, target, neg))
        assert qn == -q
    vals.sort()
    assert all(vals[i][1] <= vals[i + 1][1] for i in range(len(vals) - 1))


def test_fake_quant_via_anchor_composition(oracle):
    # Eq. (7): W_t = Q_{A->t}(Q_A(W)); fake-quant via the anchor is DQ of exactly that
    for w in _inputs():
        rows, cols = w.shape
        for anchor, target in SS_PAIRS[:5]:
            ca, sa = oracle.quantize(w, anchor)
            ct, st = oracle.slice_and_scale(ca, sa, anchor, target)
            want = oracle.dequant(ct, st, target, rows, cols)
            got = oracle.fake_quant(w, target, anchor=anchor)
            assert np.array_equal(got, want, equal_nan=True)
        wb = synth.f32_to_bf16_bits(w)
        got = oracle.fake_quant(wb, "e2m1", anchor="e4m3")
        ca, sa = oracle.quantize(wb, "e4m3")
        ct, st = oracle.slice_and_scale(ca, sa, "e4m3", "e2m1")
        assert np.array_equal(got, oracle.dequant(ct, st, "e2m1", rows, cols, out="bf16"))


def test_nan_inf_and_zero_blocks(oracle):
    m = synth.special_matrix(cols=128)
    for fmt in CORE:
        c, s = oracle.quantize(m, fmt)
        bad = np.zeros((4, 4), dtype=bool)
        bad[0, 0] = bad[1, 1] = bad[2, 2] = bad[3, 0] = bad[3, 3] = True
        assert np.array_equal(s == 255, bad)
        assert (c[bad] == 0).all()
        d = oracle.dequant(c, s, fmt, 4, 128)
        assert np.isnan(d.reshape(4, 4, 32)[bad]).all()
        assert np.isfinite(d.reshape(4, 4, 32)[~bad]).all()
        fq = oracle.fake_quant(m, fmt)
        assert np.array_equal(fq, d, equal_nan=True)
    z = np.zeros((1, 64), dtype=np.float32)
    z[0, 32:] = -0.0
    for fmt in CORE:
        c, s = oracle.quantize(z, fmt)
        assert (s == 0).all()
        assert (oracle.dequant(c, s, fmt, 1, 64) == 0).all()
    # scale byte saturation in Slice-and-Scale, NaN byte stays
    assert oracle.slice_byte("e4m3", "e2m1", 250) == 254
    assert oracle.slice_byte("e4m3", "e2m1", 254) == 254
    assert oracle.slice_byte("e4m3", "e2m1", 255) == 255
    assert oracle.slice_byte("int8", "int4", 0) == 4


def test_mse_ratio_closed_form(oracle):
    # Tensor-level study (Sec. 4.3, App. C): 100 random (1,1024) tensors, block 64.  For MXINT the
    # slice error is the direct error plus the anchor's (uniform, X_h^2/12) plus a deterministic
    # half-step term, giving MSE(SS)/MSE(direct) ~= 1 + 3 * 4^-De.  Statistical check, +-3 %.
    tensors = synth.random_tensors_1x1024(seed=4300, count=100)
    for target, de in (("int7", 1), ("int6", 2), ("int5", 3), ("int4", 4)):
        num = den = 0.0
        for t in tensors:
            ca, sa = oracle.quantize(t, "int8", k=64)
            cs, ss = oracle.slice_and_scale(ca, sa, "int8", target, k=64)
            a = oracle.dequant(cs, ss, target, 1, 1024, k=64).astype(np.float64)
            b = oracle.fake_quant(t, target, k=64).astype(np.float64)
            num += ((a - t) ** 2).mean()
            den += ((b - t) ** 2).mean()
        ratio = num / den
        assert abs(ratio / (1 + 3 * 4.0 ** -de) - 1) < 0.03, (target, ratio)
    # MXFP: the same argument on the mantissa: dropping d = mu_h - mu_l mantissa bits of a normal number
    # gives ~ 1 + 3 * 4^-d (d = 0: only the subnormal range of the target loses bits).  This is the
    # "modestly larger relative gap at intermediate bit-widths" of App. C.  Loose statistical band.
    for target, d in (("e3m3", 0), ("e3m2", 1), ("e2m3", 0), ("e2m2", 1), ("e2m1", 2)):
        num = den = 0.0
        for t in tensors:
            a = oracle.fake_quant(t, target, anchor="e4m3", k=64).astype(np.float64)
            b = oracle.fake_quant(t, target, k=64).astype(np.float64)
            num += ((a - t) ** 2).mean()
            den += ((b - t) ** 2).mean()
        model = 1 + 3 * 4.0 ** -d if d else 1.0
        assert max(1.0, 0.9 * model) <= num / den <= model + 0.15, (target, num / den)
