"""Pins of the oracle's reference for the fused consumer GEMM (Sec. 3.5: the model runs with W_t = Q_{A->t}(W_A);
Eq. (6) for the conversion, Sec. 3.3 for the reconstruction V^ = X * P): exact rational arithmetic written out here
from the value tables, and cases with a closed form.  A transposed operand, a scale taken from the wrong block, a
forgotten or doubled 2^De, or the anchor multiplied instead of its slice each fail at least one of them."""
from fractions import Fraction

import numpy as np

import defs

DE = 6   # e_max(E4M3) - e_max(E2M1) = 8 - 2 (Sec. 3.3, Eq. (6))


def _tables():
    e4m3 = dict(defs.value_table("e4m3"))
    e2m1 = dict(defs.value_table("e2m1"))
    return e4m3, e2m1


def _exact_product(a_codes, a_scales, w_codes, w_scales):
    """C[m][n] as Fractions, every step spelled out: activation value = 2^(byte - 127) * value(code); weight code
    sliced with the exhaustive nearest-value search on value / 2^De, its scale byte raised by De."""
    e4m3, e2m1 = _tables()
    M, KB, k = a_codes.shape
    N = w_codes.shape[0]
    out = [[Fraction(0) for _ in range(N)] for _ in range(M)]
    for m in range(M):
        for n in range(N):
            acc = Fraction(0)
            for b in range(KB):
                xa = Fraction(2) ** (int(a_scales[m, b]) - 127)
                xw = Fraction(2) ** (int(w_scales[n, b]) + DE - 127)
                for j in range(k):
                    av = e4m3[int(a_codes[m, b, j])]
                    wv = e4m3[int(w_codes[n, b, j])]
                    wt = e2m1[defs.nearest_code("e2m1", wv / 2 ** DE, negative_zero=bool(w_codes[n, b, j] & 0x80))]
                    acc += (xa * av) * (xw * wt)
            out[m][n] = acc
    return out


def _random_operands(rng, M, N, KB):
    a_codes = rng.integers(0, 256, size=(M, KB, 32), dtype=np.uint8)
    w_codes = rng.integers(0, 256, size=(N, KB, 32), dtype=np.uint8)
    a_codes[(a_codes & 0x7F) == 0x7F] = 0x3A      # no NaN codes: their reading has a pin of its own
    w_codes[(w_codes & 0x7F) == 0x7F] = 0x6B
    a_scales = rng.integers(120, 134, size=(M, KB), dtype=np.uint8)
    w_scales = rng.integers(115, 128, size=(N, KB), dtype=np.uint8)
    return a_codes, a_scales, w_codes, w_scales


def test_gemm_reference_against_exact_rationals(oracle):
    rng = np.random.default_rng(20260401)
    for M, N, KB in [(3, 4, 2), (1, 5, 1), (4, 2, 3)]:
        a_codes, a_scales, w_codes, w_scales = _random_operands(rng, M, N, KB)
        # large anchor codes in some columns, so that the slice is not zero almost everywhere
        w_codes[:, :, ::3] |= 0x60
        w_codes[(w_codes & 0x7F) == 0x7F] = 0x7E
        got, got_abs = oracle.gemm_ss_reference(a_codes, a_scales, w_codes, w_scales, with_abs=True)
        want = _exact_product(a_codes, a_scales, w_codes, w_scales)
        assert got.shape == (M, N)
        for m in range(M):
            for n in range(N):
                w = float(want[m][n])
                assert abs(got[m, n] - w) <= 1e-12 * max(abs(w), float(got_abs[m, n])), (M, N, KB, m, n)
        assert (got_abs >= np.abs(got) * (1 - 1e-12)).all()


def test_gemm_reference_one_hot_activations_read_the_sliced_weight(oracle):
    # A[m] = 1.0 at position p(m) only (code 0x38, scale byte 127): C[m][n] is the dequantized SLICED weight at
    # [n][p(m)] -- not the anchor's value, and not the weight of another row, block or position
    e4m3, e2m1 = _tables()
    rng = np.random.default_rng(7)
    M, N, KB = 5, 6, 2
    _, _, w_codes, w_scales = _random_operands(rng, M, N, KB)
    w_codes |= 0x50                                # magnitudes of 2^3 and more: most slices are non-zero
    w_codes[(w_codes & 0x7F) == 0x7F] = 0x7E
    a_codes = np.zeros((M, KB, 32), dtype=np.uint8)
    a_scales = np.full((M, KB), 127, dtype=np.uint8)
    pos = [(0, 0), (0, 31), (1, 0), (1, 17), (0, 5)]
    for m, (b, j) in enumerate(pos):
        a_codes[m, b, j] = 0x38
    got = oracle.gemm_ss_reference(a_codes, a_scales, w_codes, w_scales)
    differs_from_anchor = 0
    for m, (b, j) in enumerate(pos):
        for n in range(N):
            wv = e4m3[int(w_codes[n, b, j])]
            wt = e2m1[defs.nearest_code("e2m1", wv / 2 ** DE, negative_zero=bool(w_codes[n, b, j] & 0x80))]
            want = Fraction(2) ** (int(w_scales[n, b]) + DE - 127) * wt
            assert got[m, n] == float(want), (m, n)
            differs_from_anchor += want != Fraction(2) ** (int(w_scales[n, b]) - 127) * wv
    assert differs_from_anchor > 0                 # the case can tell the slice from the anchor


def test_gemm_reference_closed_forms(oracle):
    # constant operands: every activation 1.5 * 2^2, every weight anchor 384 * 2^-3 (code 0x7C; 384 / 64 = 6 is E2M1's
    # largest value, kept exactly): C = K * 6 * 48 for every output
    M, N, KB = 2, 3, 4
    a_codes = np.full((M, KB, 32), 0x3C, dtype=np.uint8)
    a_scales = np.full((M, KB), 129, dtype=np.uint8)
    w_codes = np.full((N, KB, 32), 0x7C, dtype=np.uint8)
    w_scales = np.full((N, KB), 124, dtype=np.uint8)
    got = oracle.gemm_ss_reference(a_codes, a_scales, w_codes, w_scales)
    assert (got == KB * 32 * 6.0 * 48.0).all()
    # anchor values below half of E2M1's smallest magnitude times 2^De (0.25 * 64 = 16) slice to zero: C = 0;
    # exactly 16 is a tie between 0 and 0.5 and goes to the even code, 0
    w_codes[:] = 0x58                              # 16
    assert (oracle.gemm_ss_reference(a_codes, a_scales, w_codes, w_scales) == 0).all()
    w_codes[:] = 0x59                              # 18 -> 0.5 * 64 = 32
    assert (oracle.gemm_ss_reference(a_codes, a_scales, w_codes, w_scales) == KB * 32 * 6.0 * 4.0).all()
    # the sign of the weight carries through the slice; a row of activations with alternating signs cancels
    a_codes[:, :, 1::2] ^= 0x80
    assert (oracle.gemm_ss_reference(a_codes, a_scales, w_codes, w_scales) == 0).all()
    # scaling one block's activation scale byte by +1 adds that block's share once more
    a_codes[:, :, 1::2] ^= 0x80
    a_scales[:, 2] += 1
    assert (oracle.gemm_ss_reference(a_codes, a_scales, w_codes, w_scales) == (KB + 1) * 32 * 6.0 * 4.0).all()


def test_wide_reconstruction_against_exact_rationals_at_extreme_scale_bytes(oracle):
    """dequant_f64 / gemm_ss_reference(wide=True): scale bytes 0..5 and 248..254 keep their exact values (where the
    float32 dequantizer underflows or overflows), the sliced byte saturates at 254 (Eq. (6) scale step inside the E8M0
    range), and byte 255 makes the block -- and with it every output that touches it -- NaN."""
    e4m3, e2m1 = _tables()
    rng = np.random.default_rng(20260405)
    # element by element against the tables, every code x the extreme bytes
    codes = np.arange(256, dtype=np.uint8).reshape(8, 1, 32)
    for byte in (0, 1, 5, 126, 127, 250, 254):
        scales = np.full((8, 1), byte, dtype=np.uint8)
        got = oracle.dequant_f64(codes, scales, "e4m3")
        for c in range(256):
            want = e4m3.get(c)
            if want is None:                                  # the two NaN codes (not in the table of finite values)
                assert np.isnan(got[c // 32, c % 32])
            else:
                assert Fraction(float(got[c // 32, c % 32])) == Fraction(2) ** (byte - 127) * want, (byte, c)
    assert np.isnan(oracle.dequant_f64(codes, np.full((8, 1), 255, dtype=np.uint8), "e4m3")).all()
    # wherever the float32 dequantizer is exact (moderate bytes), the two reconstructions agree
    sc = rng.integers(100, 150, size=(8, 1), dtype=np.uint8)
    f32 = oracle.dequant(codes, sc, "e4m3", 8, 32).astype(np.float64)
    f64 = oracle.dequant_f64(codes, sc, "e4m3")
    assert np.array_equal(np.isnan(f32), np.isnan(f64)) and np.array_equal(np.nan_to_num(f32), np.nan_to_num(f64))
    # the product: low bytes on W against ordinary A, high bytes on W against small A, exact rationals
    for w_lo, w_hi, a_lo, a_hi in ((0, 6, 120, 134), (248, 255, 90, 101)):
        a_codes, _, w_codes, _ = _random_operands(rng, 3, 4, 2)
        w_codes[:, :, ::2] |= 0x60
        w_codes[(w_codes & 0x7F) == 0x7F] = 0x7E
        a_scales = rng.integers(a_lo, a_hi, size=(3, 2), dtype=np.uint8)
        w_scales = rng.integers(w_lo, w_hi, size=(4, 2), dtype=np.uint8)
        if w_hi == 255:
            w_scales[0, 0] = 254                              # saturating: 254 + De stays 254
            w_scales[1, 1] = 250                              # 250 + 6 = 256 -> 254
        got, got_abs = oracle.gemm_ss_reference(a_codes, a_scales, w_codes, w_scales, with_abs=True, wide=True)
        for m in range(3):
            for n in range(4):
                acc = Fraction(0)
                for b in range(2):
                    xa = Fraction(2) ** (int(a_scales[m, b]) - 127)
                    xw = Fraction(2) ** (min(int(w_scales[n, b]) + DE, 254) - 127)
                    for j in range(32):
                        wv = e4m3[int(w_codes[n, b, j])]
                        wt = e2m1[defs.nearest_code("e2m1", wv / 2 ** DE, negative_zero=bool(w_codes[n, b, j] & 0x80))]
                        acc += (xa * e4m3[int(a_codes[m, b, j])]) * (xw * wt)
                assert abs(Fraction(float(got[m, n])) - acc) <= Fraction(float(got_abs[m, n])) * Fraction(1, 2 ** 45), (m, n)
    # byte 255 on one block of W / of A: NaN in exactly that column / row
    a_codes, a_scales, w_codes, w_scales = _random_operands(rng, 3, 4, 2)
    w_scales[2, 1] = 255
    a_scales[1, 0] = 255
    got = oracle.gemm_ss_reference(a_codes, a_scales, w_codes, w_scales, wide=True)
    want_nan = np.zeros((3, 4), dtype=bool)
    want_nan[:, 2] = True
    want_nan[1, :] = True
    assert np.array_equal(np.isnan(got), want_nan)


def test_gemm_reference_of_a_kept_fp4_weight_against_exact_rationals(oracle):
    # The product with a W_t that was converted before (Sec. 3.5 "Inference"): the weight's nibbles are read here by hand
    # (code j of a block = bits 4 j .. 4 j + 3 of its 16 bytes, little endian) and multiplied in exact rationals.  A
    # swapped nibble order, a scale from the wrong block or a transposed operand fails.
    e4m3, e2m1 = _tables()
    rng = np.random.default_rng(20260402)
    for M, N, KB in [(2, 3, 2), (3, 1, 1)]:
        a_codes, a_scales, _, _ = _random_operands(rng, M, N, KB)
        w4 = rng.integers(0, 256, size=(N, KB, 16), dtype=np.uint8)
        w4_scales = rng.integers(118, 133, size=(N, KB), dtype=np.uint8)
        got, got_abs = oracle.gemm_reference(a_codes, a_scales, w4, w4_scales, w_fmt="e2m1", with_abs=True)
        wide = oracle.gemm_reference(a_codes, a_scales, w4, w4_scales, w_fmt="e2m1", wide=True)
        for m in range(M):
            for n in range(N):
                acc = Fraction(0)
                for b in range(KB):
                    xa = Fraction(2) ** (int(a_scales[m, b]) - 127)
                    xw = Fraction(2) ** (int(w4_scales[n, b]) - 127)
                    for j in range(32):
                        nib = (int(w4[n, b, j // 2]) >> (4 * (j % 2))) & 0xF
                        acc += (xa * e4m3[int(a_codes[m, b, j])]) * (xw * e2m1[nib])
                w = float(acc)
                assert abs(got[m, n] - w) <= 1e-12 * max(abs(w), float(got_abs[m, n])), (M, N, KB, m, n)
                assert abs(wide[m, n] - w) <= 1e-12 * max(abs(w), float(got_abs[m, n])), (M, N, KB, m, n)
    # and the reference of the fused product is this one applied to the converted anchor
    a_codes, a_scales, w_codes, w_scales = _random_operands(rng, 3, 4, 2)
    tc, ts = oracle.slice_and_scale(w_codes, w_scales, "e4m3", "e2m1")
    assert np.array_equal(oracle.gemm_ss_reference(a_codes, a_scales, w_codes, w_scales),
                          oracle.gemm_reference(a_codes, a_scales, tc, ts, w_fmt="e2m1"))
