"""Pins of the oracle's format layer against the public format definitions (value tables),
independent of the oracle's own arithmetic: literal tables, exact rationals, spot values."""
import math
from fractions import Fraction

import numpy as np
import pytest

import defs


def test_literal_tables_are_self_consistent():
    # the typed tables must agree with the sign|exponent|mantissa definition (catches typos in the file)
    g = defs.read_golden_values()
    for fmt in ("e2m1", "e2m3", "e3m2", "e4m3"):
        eta, mu = defs.FP_SHAPES[fmt]
        for code, val in g[fmt].items():
            assert defs.fp_value(eta, mu, code) == val, (fmt, hex(code))
    assert len(g["e2m1"]) == 8 and len(g["e2m3"]) == 32 and len(g["e3m2"]) == 32


@pytest.mark.parametrize("fmt", defs.ALL_FORMATS)
def test_decode_every_code_matches_table(oracle, fmt):
    tab = dict(defs.value_table(fmt))
    n = 2 ** defs.bits_of(fmt)
    for code in range(n):
        got = oracle.decode(fmt, code)
        if code not in tab:
            assert fmt == "e4m3" and code in (0x7F, 0xFF) and math.isnan(got)
            continue
        assert Fraction(got) == tab[code], (fmt, hex(code))
        if tab[code] == 0 and code != 0:          # negative zero keeps its sign
            assert math.copysign(1.0, got) < 0


def test_spot_values(oracle):
    g = defs.read_golden_values()
    for fmt in ("e4m3", "int8"):
        for code, val in g[fmt].items():
            got = oracle.decode(fmt, code)
            if val is None:
                assert math.isnan(got)
            else:
                assert Fraction(got) == val
    for byte, val in g["e8m0"].items():
        got = oracle.scale_value(byte)
        if val is None:
            assert math.isnan(got)
        else:
            assert got == float(val) and Fraction(got) == Fraction(2) ** (byte - 127)


def test_format_constants(oracle):
    # largest normal, e_max (Sec. 3.3 notation) and the De the paper states
    expect = {"e4m3": (448, 8), "e3m2": (28, 4), "e2m3": (7.5, 2), "e2m1": (6, 2),
              "int8": (127, 6), "int6": (31, 4), "int4": (7, 2), "int2": (1, 0)}
    for fmt, (mx, em) in expect.items():
        assert oracle.max_normal(fmt) == mx
        assert oracle.emax(fmt) == em == defs.emax(fmt)
    # "for signed MXINT this is equivalent to De = b_h - b_l" (below Eq. (3))
    for bh in range(2, 9):
        for bl in range(2, bh + 1):
            assert oracle.delta_e(f"int{bh}", f"int{bl}") == bh - bl
    assert oracle.delta_e("e4m3", "e3m2") == 4
    assert oracle.delta_e("e4m3", "e2m3") == 6
    assert oracle.delta_e("e4m3", "e2m1") == 6


@pytest.mark.parametrize("fmt", defs.ALL_FORMATS)
def test_dequant_all_codes_all_scales_exact(oracle, fmt):
    # V^ = X * P for every code and every E8M0 byte, in exact rationals
    tab = dict(defs.value_table(fmt))
    for byte in range(0, 255):
        x = Fraction(2) ** (byte - 127)
        for code, val in tab.items():
            got = oracle.dequant_value(fmt, code, byte)
            assert Fraction(got) == val * x
    for code in tab:
        assert math.isnan(oracle.dequant_value(fmt, code, 255))


def test_int8_matches_ocp_fixed_point_view(oracle):
    # OCP MXINT8 elements are code/64 with X = 2^floor(log2 amax); the integer view stores byte - 6.
    for code in range(256):
        v = code if code < 128 else code - 256
        for byte in (6, 50, 127, 200, 254):
            assert Fraction(oracle.dequant_value("int8", code, byte - 6)) == \
                Fraction(v, 64) * Fraction(2) ** (byte - 127)


@pytest.mark.parametrize("bits", [2, 3, 4, 5, 6, 7, 8])
def test_pack_roundtrip_and_bit_positions(oracle, bits):
    rng = np.random.default_rng(bits)
    for k in (8, 32, 64):
        codes = rng.integers(0, 2 ** bits, size=k, dtype=np.uint8)
        packed = oracle.pack_block(codes, bits)
        assert packed.size == (k * bits + 7) // 8
        # element i occupies bits [i*bits, (i+1)*bits) of the little-endian bit string
        as_int = int.from_bytes(packed.tobytes(), "little")
        for i in range(k):
            assert (as_int >> (i * bits)) & (2 ** bits - 1) == codes[i]
        assert np.array_equal(oracle.unpack_block(packed, k, bits), codes)


def test_bf16_conversion(oracle):
    from paper_2604_00529_amd import synth
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.standard_normal(2000).astype(np.float32) * np.float32(10.0) ** rng.integers(-40, 38, 2000),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-45, 9.2e-41],
                                 dtype=np.float32)]).astype(np.float32)
    a = oracle.bf16_bits(x)
    b = synth.f32_to_bf16_bits(x)        # bit-trick implementation, independent of the oracle's arithmetic one
    assert np.array_equal(a, b)
    assert np.array_equal(oracle.bf16_to_f32(a), synth.bf16_bits_to_f32(b))
