"""CPU oracle for the MX quantization / Slice-and-Scale hot path (numpy front end).

TEST INFRASTRUCTURE ONLY.  This package wraps ``mx_oracle.c`` (plain scalar C,
double precision, written from the paper's Sec. 3.3-3.5 and Eq. (1)-(7)) with
ctypes.  It shares nothing with the HIP library and must never be imported by
the product package; only tests, the smoke check and the benchmark's CPU
baseline call it.

Dense tensors are numpy arrays: ``float32`` for fp32, ``uint16`` for bfloat16
bit patterns.  Packed tensors are ``uint8`` arrays ``codes[outer, nblocks,
bytes_per_block]`` and ``scales[outer, nblocks]`` (block axis innermost; for
axis 0 the packed tensor is laid out transposed, ``outer = cols``).

parity unpinned: tie rule, symmetric integer clip, all-zero block, sign of
zero and NaN/Inf conventions (no value in the paper to check against).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mx_oracle.c")
_SO = os.path.join(_HERE, "libmx_oracle.so")

# name -> (kind, a, b): kind 0 = MXINT(a bits), kind 1 = MXFP(eta = a, mu = b)
FORMATS = {
    "int8": (0, 8, 0), "int7": (0, 7, 0), "int6": (0, 6, 0), "int5": (0, 5, 0),
    "int4": (0, 4, 0), "int3": (0, 3, 0), "int2": (0, 2, 0),
    "e4m3": (1, 4, 3), "e3m3": (1, 3, 3), "e3m2": (1, 3, 2), "e2m3": (1, 2, 3),
    "e2m2": (1, 2, 2), "e2m1": (1, 2, 1),
}

TIE_DEFAULT, TIE_HALF_AWAY, TIE_HALF_EVEN = 0, 1, 2


def build(force=False):
    """Compile mx_oracle.c with gcc into libmx_oracle.so (next to the source)."""
    if not force and os.path.exists(_SO) and os.path.getmtime(_SO) >= os.path.getmtime(_SRC):
        return _SO
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
           "-Wall", "-Wextra", "-o", _SO, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _SO


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_SO)
        i, l, d, p = ctypes.c_int, ctypes.c_long, ctypes.c_double, ctypes.c_void_p
        L.mxo_set_threads.argtypes = [i]
        L.mxo_get_threads.restype = i
        L.mxo_elem_bits.argtypes = [i, i, i]
        L.mxo_emax.argtypes = [i, i, i]
        L.mxo_max_normal.argtypes = [i, i, i]
        L.mxo_max_normal.restype = d
        L.mxo_decode.argtypes = [i, i, i, ctypes.c_uint]
        L.mxo_decode.restype = d
        L.mxo_encode.argtypes = [i, i, i, d, i]
        L.mxo_encode.restype = ctypes.c_uint
        L.mxo_scale_byte.argtypes = [d, i, i, i]
        L.mxo_scale_value.argtypes = [i]
        L.mxo_scale_value.restype = d
        L.mxo_delta_e.argtypes = [i, i, i, i, i]
        L.mxo_block_bytes.argtypes = [i, i]
        L.mxo_block_bytes.restype = l
        L.mxo_slice_code.argtypes = [i, i, i, i, i, i, ctypes.c_uint]
        L.mxo_slice_code.restype = ctypes.c_uint
        L.mxo_slice_byte.argtypes = [i, i, i, i, i, i]
        L.mxo_dequant_value.argtypes = [i, i, i, ctypes.c_uint, i]
        L.mxo_dequant_value.restype = d
        L.mxo_pack_block.argtypes = [p, i, i, p]
        L.mxo_unpack_block.argtypes = [p, i, i, p]
        L.mxo_double_to_bf16.argtypes = [d]
        L.mxo_double_to_bf16.restype = ctypes.c_uint16
        L.mxo_bf16_to_double.argtypes = [ctypes.c_uint16]
        L.mxo_bf16_to_double.restype = d
        L.mxo_quantize.argtypes = [p, i, l, l, l, i, i, i, i, i, i, p, p]
        L.mxo_slice_and_scale.argtypes = [i, i, i, i, i, i, i, l, p, p, p, p]
        L.mxo_dequant.argtypes = [i, i, i, i, p, p, l, l, l, i, i, p]
        L.mxo_fake_quant.argtypes = [i, i, i, i, i, i, i, i, p, i, l, l, l, i, i, p, l]
        _lib = L
    return _lib


def set_threads(n):
    lib().mxo_set_threads(int(n))


def get_threads():
    return lib().mxo_get_threads()


def _fmt(name):
    return FORMATS[name]


def elem_bits(fmt):
    return lib().mxo_elem_bits(*_fmt(fmt))


def emax(fmt):
    return lib().mxo_emax(*_fmt(fmt))


def max_normal(fmt):
    return lib().mxo_max_normal(*_fmt(fmt))


def decode(fmt, code):
    return lib().mxo_decode(*_fmt(fmt), int(code))


def encode(fmt, r, tie=TIE_DEFAULT):
    return lib().mxo_encode(*_fmt(fmt), float(r), tie)


def scale_byte(amax, fmt):
    return lib().mxo_scale_byte(float(amax), *_fmt(fmt))


def scale_value(byte):
    return lib().mxo_scale_value(int(byte))


def delta_e(anchor, target):
    ka, ah, bh = _fmt(anchor)
    kt, al, bl = _fmt(target)
    assert ka == kt, "anchor and target must both be MXINT or both MXFP"
    return lib().mxo_delta_e(ka, ah, bh, al, bl)


def slice_code(anchor, target, code, tie=TIE_DEFAULT):
    ka, ah, bh = _fmt(anchor)
    kt, al, bl = _fmt(target)
    assert ka == kt
    return lib().mxo_slice_code(ka, ah, bh, al, bl, tie, int(code))


def slice_byte(anchor, target, byte):
    ka, ah, bh = _fmt(anchor)
    kt, al, bl = _fmt(target)
    assert ka == kt
    return lib().mxo_slice_byte(ka, ah, bh, al, bl, int(byte))


def dequant_value(fmt, code, byte):
    return lib().mxo_dequant_value(*_fmt(fmt), int(code), int(byte))


def block_bytes(fmt, k=32):
    return lib().mxo_block_bytes(k, elem_bits(fmt))


def pack_block(codes, bits):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    k = codes.size
    out = np.zeros(lib().mxo_block_bytes(k, bits), dtype=np.uint8)
    lib().mxo_pack_block(codes.ctypes.data, k, bits, out.ctypes.data)
    return out


def unpack_block(packed, k, bits):
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    out = np.zeros(k, dtype=np.uint8)
    lib().mxo_unpack_block(packed.ctypes.data, k, bits, out.ctypes.data)
    return out


def unpack(codes, fmt, k=32):
    """codes[..., bytes_per_block] -> element codes [..., k] (one per byte)."""
    bits = elem_bits(fmt)
    flat = np.ascontiguousarray(codes, dtype=np.uint8).reshape(-1, codes.shape[-1])
    out = np.zeros((flat.shape[0], k), dtype=np.uint8)
    L, bb = lib(), flat.shape[1]
    src, dst = flat.ctypes.data, out.ctypes.data
    for t in range(flat.shape[0]):
        L.mxo_unpack_block(src + t * bb, k, bits, dst + t * k)
    return out.reshape(codes.shape[:-1] + (k,))


def _dense_dtype(x):
    if x.dtype == np.float32:
        return 0
    if x.dtype == np.uint16:
        return 1
    raise TypeError("dense tensors are float32 or uint16 (bfloat16 bit patterns)")


def _outer_nblk(rows, cols, axis, k):
    if axis == 1:
        assert cols % k == 0
        return rows, cols // k
    assert axis == 0 and rows % k == 0
    return cols, rows // k


def quantize(x, fmt, axis=1, k=32, tie=TIE_DEFAULT):
    """Q_f of Eq. (1)-(2): dense [rows, cols] -> (codes, scales)."""
    x = np.ascontiguousarray(x)
    rows, cols = x.shape
    outer, nblk = _outer_nblk(rows, cols, axis, k)
    bb = block_bytes(fmt, k)
    codes = np.zeros((outer, nblk, bb), dtype=np.uint8)
    scales = np.zeros((outer, nblk), dtype=np.uint8)
    rc = lib().mxo_quantize(x.ctypes.data, _dense_dtype(x), rows, cols, cols, axis, k, *_fmt(fmt), tie,
                            codes.ctypes.data, scales.ctypes.data)
    assert rc == 0
    return codes, scales


def slice_and_scale(codes, scales, anchor, target, k=32, tie=TIE_DEFAULT):
    """Q_{A->t} of Eq. (4) / Eq. (6) on packed blocks (any leading shape)."""
    ka, ah, bh = _fmt(anchor)
    kt, al, bl = _fmt(target)
    assert ka == kt
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.uint8)
    nblocks = scales.size
    assert codes.size == nblocks * block_bytes(anchor, k)
    out_codes = np.zeros(scales.shape + (block_bytes(target, k),), dtype=np.uint8)
    out_scales = np.zeros(scales.shape, dtype=np.uint8)
    rc = lib().mxo_slice_and_scale(ka, ah, bh, al, bl, tie, k, nblocks, codes.ctypes.data, scales.ctypes.data,
                                   out_codes.ctypes.data, out_scales.ctypes.data)
    assert rc == 0
    return out_codes, out_scales


def dequant(codes, scales, fmt, rows, cols, axis=1, k=32, out="f32"):
    """V^ = X * P into a dense [rows, cols] array (float32, or uint16 bf16 bits)."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.uint8)
    outer, nblk = _outer_nblk(rows, cols, axis, k)
    assert scales.size == outer * nblk and codes.size == outer * nblk * block_bytes(fmt, k)
    dst = np.zeros((rows, cols), dtype=np.float32 if out == "f32" else np.uint16)
    rc = lib().mxo_dequant(*_fmt(fmt), k, codes.ctypes.data, scales.ctypes.data, rows, cols, cols, axis,
                           0 if out == "f32" else 1, dst.ctypes.data)
    assert rc == 0
    return dst


def fake_quant(x, target, anchor=None, axis=1, k=32, tie=TIE_DEFAULT, out=None):
    """DQ(Q_t(x)) or, with an anchor, DQ(Q_{A->t}(Q_A(x))) of Eq. (7)."""
    x = np.ascontiguousarray(x)
    rows, cols = x.shape
    kt, al, bl = _fmt(target)
    if anchor is None:
        has, ah, bh = 0, 0, 0
    else:
        ka, ah, bh = _fmt(anchor)
        assert ka == kt
        has = 1
    if out is None:
        out_dtype = x.dtype
    else:
        out_dtype = np.float32 if out == "f32" else np.uint16
    dst = np.zeros((rows, cols), dtype=out_dtype)
    rc = lib().mxo_fake_quant(kt, al, bl, has, ah, bh, tie, k, x.ctypes.data, _dense_dtype(x), rows, cols, cols,
                              axis, 0 if out_dtype == np.float32 else 1, dst.ctypes.data, cols)
    assert rc == 0
    return dst


def dequant_f64(codes, scales, fmt, k=32):
    """V^ = X * P (Sec. 3.3 notation) as float64, element by element from the two scalar definitions
    mxo_decode(code) and mxo_scale_value(byte): no float32 in between, so every scale byte 0..254 keeps its exact
    value (2^-127 .. 2^127 times a minifloat is exact in float64) and byte 255 gives NaN.  codes[..., nblocks,
    bytes_per_block], scales[..., nblocks] -> [..., nblocks * k]."""
    L = lib()
    vals = np.array([L.mxo_decode(*_fmt(fmt), c) for c in range(1 << elem_bits(fmt))], dtype=np.float64)
    xs = np.array([L.mxo_scale_value(b) for b in range(256)], dtype=np.float64)
    el = unpack(codes, fmt, k)                                    # [..., nblocks, k] element codes
    with np.errstate(invalid="ignore"):
        out = vals[el] * xs[np.asarray(scales, dtype=np.uint8)][..., None]
    return out.reshape(el.shape[:-2] + (el.shape[-2] * k,))


def gemm_reference(a_codes, a_scales, w_codes, w_scales, w_fmt="e2m1", k=32, with_abs=False, wide=False):
    """fp64 product of two dequantized MX operands: C = DQ(A) @ DQ(W).T with A in MXFP8 E4M3 [M, K/k blocks] and W
    packed in `w_fmt` [N, K/k blocks] (Sec. 3.3 notation for the reconstruction V^ = X * P; Sec. 3.5 "Inference": the
    model runs with a W_t that was converted before; numpy's matmul is the library step).
    with_abs also returns sum_k |a||w|, the scale of the rounding error of any finite-precision accumulation.
    wide: reconstruct the operands straight in float64 (dequant_f64) instead of through the float32 dequantizer, so
    that scale bytes near 0 and 254 keep their exact values and byte 255 propagates as NaN."""
    M, KB = a_scales.shape
    N = w_scales.shape[0]
    K = KB * k
    if wide:
        a = dequant_f64(a_codes, a_scales, "e4m3", k=k)
        w = dequant_f64(w_codes, w_scales, w_fmt, k=k)
    else:
        a = dequant(a_codes, a_scales, "e4m3", M, K, axis=1, k=k).astype(np.float64)
        w = dequant(w_codes, w_scales, w_fmt, N, K, axis=1, k=k).astype(np.float64)
    if with_abs:
        return a @ w.T, np.abs(a) @ np.abs(w).T
    return a @ w.T


def gemm_ss_reference(a_codes, a_scales, w_codes, w_scales, target="e2m1", k=32, with_abs=False, wide=False):
    """Reference of the fused consumer GEMM: C = DQ(A) @ DQ(Q_{A->t}(W_A)).T with W_A the E4M3 anchor
    [N, K/k blocks]: the anchor converted by Eq. (6) (slice_and_scale), then gemm_reference."""
    tc, ts = slice_and_scale(w_codes, w_scales, "e4m3", target, k=k)
    return gemm_reference(a_codes, a_scales, tc, ts, w_fmt=target, k=k, with_abs=with_abs, wide=wide)


def bf16_bits(x):
    """float32 array -> nearest bfloat16 bit patterns (uint16), ties to even."""
    x = np.asarray(x, dtype=np.float32)
    out = np.zeros(x.shape, dtype=np.uint16)
    flat, oflat = x.reshape(-1), out.reshape(-1)
    for n in range(flat.size):
        oflat[n] = lib().mxo_double_to_bf16(float(flat[n]))
    return out


def bf16_to_f32(h):
    """uint16 bfloat16 bit patterns -> float32 (exact)."""
    h = np.asarray(h, dtype=np.uint16)
    return (h.astype(np.uint32) << 16).view(np.float32)
