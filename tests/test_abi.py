"""The C-ABI library without a GPU: it loads, exports every symbol include/mx.h declares, and its
host-side validation turns bad arguments into status codes before anything could be launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def mx():
    from paper_2604_00529_amd import build
    build.build(verbose=False)               # compiles only if the library is missing or stale
    import paper_2604_00529_amd as mx
    mx.binding.lib()
    return mx


def declared_functions():
    text = open(os.path.join(ROOT, "include", "mx.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mx_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(mx):
    names = declared_functions()
    assert {"mx_quantize", "mx_slice_and_scale", "mx_slice_and_scale_batched", "mx_fake_quant", "mx_dequant",
            "mx_packed_bytes", "mx_status_str"} <= set(names)
    L = mx.binding.lib()
    for n in names:
        assert hasattr(L, n), n


def test_header_is_plain_c(tmp_path):
    # the boundary is a C ABI: the header compiles as strict C99, with no C++ or HIP types in any signature
    import os
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = tmp_path / "use_mx.c"
    src.write_text('#include "mx.h"\n'
                   'int main(void) {\n'
                   '  mx_format_t f = {MX_FP4_E2M1, MX_SCALE_E8M0, 32, 1, MX_ROUND_DEFAULT};\n'
                   '  mx_status_t (*q)(const mx_format_t*, const mx_dense_t*, const mx_packed_t*, void*) = mx_quantize;\n'
                   '  (void)q; return mx_elem_bits(f.elem) == 4 ? 0 : 1;\n'
                   '}\n')
    r = subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.join(root, "include"),
                        "-fsyntax-only", str(src)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


def test_element_table(mx):
    bits = {"int8": 8, "int7": 7, "int6": 6, "int5": 5, "int4": 4, "int3": 3, "int2": 2,
            "e4m3": 8, "e3m3": 7, "e3m2": 6, "e2m3": 6, "e2m2": 5, "e2m1": 4}
    emax = {"int8": 6, "int6": 4, "int4": 2, "int2": 0, "e4m3": 8, "e3m3": 4, "e3m2": 4, "e2m3": 2, "e2m2": 2, "e2m1": 2}
    for k, v in bits.items():
        assert mx.mx_elem_bits(k) == v
    for k, v in emax.items():
        assert mx.mx_elem_emax(k) == v
    assert mx.binding.lib().mx_elem_bits(99) == -1


def test_packed_bytes(mx):
    assert mx.mx_packed_bytes(mx.make_format("e2m1"), 1024, 1024) == (1024 * 1024 // 2, 1024 * 32)
    assert mx.mx_packed_bytes(mx.make_format("e3m2", axis=0), 64, 48) == (48 * 2 * 24, 96)
    assert mx.mx_packed_bytes(mx.make_format("int8"), 0, 64) == (0, 0)
    with pytest.raises(mx.MxError) as e:
        mx.mx_packed_bytes(mx.make_format("int8"), 10, 33)            # 33 is not a multiple of the block
    assert e.value.status == 3
    with pytest.raises(mx.MxError) as e:
        mx.mx_packed_bytes(mx.make_format("int8", block=48), 10, 96)  # k = 16, 32, 64, 128 have kernels
    assert e.value.status == 5
    assert mx.mx_packed_bytes(mx.make_format("int6", block=64), 10, 128) == (10 * 2 * 48, 20)
    assert mx.mx_packed_bytes(mx.make_format("e2m1", block=16), 4, 64) == (4 * 4 * 8, 16)


def _dense(ptr, dtype, rows, cols, ld=None):
    return mx_binding().MxDense(ptr, dtype, rows, cols, cols if ld is None else ld)


def mx_binding():
    from paper_2604_00529_amd import binding
    return binding


def test_validation_returns_codes_without_launching(mx):
    B = mx.binding
    L = B.lib()
    P = 0x10000  # a made-up, aligned device address: never dereferenced because validation fails first
    f = mx.make_format("e4m3")
    ref = ctypes.byref
    # quantize
    d = B.MxDense(P, B.MX_BF16, 64, 128, 128)
    p = B.MxPacked(P, P, 64, 4)
    assert L.mx_quantize(None, ref(d), ref(p), None) == 1
    assert L.mx_quantize(ref(f), None, ref(p), None) == 1
    assert L.mx_quantize(ref(mx.make_format(77)), ref(d), ref(p), None) == 2
    assert L.mx_quantize(ref(f), ref(B.MxDense(P, 5, 64, 128, 128)), ref(p), None) == 2
    assert L.mx_quantize(ref(f), ref(B.MxDense(P, B.MX_BF16, 64, 100, 104)), ref(p), None) == 3      # 100 % 32
    assert L.mx_quantize(ref(f), ref(B.MxDense(P, B.MX_BF16, 64, 128, 64)), ref(p), None) == 3       # ld < cols
    assert L.mx_quantize(ref(f), ref(d), ref(B.MxPacked(P, P, 64, 5)), None) == 3                     # wrong nblocks
    assert L.mx_quantize(ref(f), ref(B.MxDense(P + 4, B.MX_BF16, 64, 128, 128)), ref(p), None) == 4
    assert L.mx_quantize(ref(f), ref(B.MxDense(P, B.MX_BF16, 64, 128, 132)), ref(p), None) == 4      # ld % 8
    assert L.mx_quantize(ref(f), ref(B.MxDense(None, B.MX_BF16, 64, 128, 128)), ref(p), None) == 1
    assert L.mx_quantize(ref(mx.make_format("e4m3", axis=2)), ref(d), ref(p), None) == 3
    f_bad_round = mx.make_format("e4m3")
    f_bad_round.round = 9
    assert L.mx_quantize(ref(f_bad_round), ref(d), ref(p), None) == 2
    # empty tensors are fine and launch nothing
    assert L.mx_quantize(ref(f), ref(B.MxDense(None, B.MX_BF16, 0, 128, 128)), ref(B.MxPacked(None, None, 0, 4)), None) == 0
    # slice-and-scale: must be a down-conversion inside one family from an 8-bit anchor
    a, t = B.MxPacked(P, P, 1, 100), B.MxPacked(P, P, 1, 100)
    assert L.mx_slice_and_scale(ref(mx.make_format("e4m3")), ref(a), ref(mx.make_format("int4")), ref(t), None) == 2
    assert L.mx_slice_and_scale(ref(mx.make_format("e2m1")), ref(a), ref(mx.make_format("e4m3")), ref(t), None) == 2
    assert L.mx_slice_and_scale(ref(mx.make_format("e4m3")), ref(a), ref(mx.make_format("e4m3")), ref(t), None) == 2
    assert L.mx_slice_and_scale(ref(mx.make_format("int6")), ref(a), ref(mx.make_format("int4")), ref(t), None) == 5
    assert L.mx_slice_and_scale(ref(mx.make_format("int8")), ref(a), ref(mx.make_format("int4")),
                                ref(B.MxPacked(P, P, 1, 99)), None) == 3
    assert L.mx_slice_and_scale(ref(mx.make_format("int8")), ref(a), ref(mx.make_format("int4", round="even")),
                                ref(t), None) == 2                                                     # tie rules differ
    assert L.mx_slice_and_scale(ref(mx.make_format("int8")), ref(B.MxPacked(P + 8, P, 1, 100)),
                                ref(mx.make_format("int4")), ref(t), None) == 4
    assert L.mx_slice_and_scale(ref(mx.make_format("int8")), ref(B.MxPacked(None, None, 0, 0)),
                                ref(mx.make_format("int4")), ref(B.MxPacked(None, None, 0, 0)), None) == 0
    # batched: workspace checks
    A = (B.MxPacked * 2)(a, a)
    T = (B.MxPacked * 2)(t, t)
    fa, ft = mx.make_format("e4m3"), mx.make_format("e2m1")
    need = L.mx_slice_and_scale_batched_workspace(2, 200)
    assert need > 0
    assert L.mx_slice_and_scale_batched(ref(fa), ref(ft), 2, A, T, None, need, None) == 1
    assert L.mx_slice_and_scale_batched(ref(fa), ref(ft), 2, A, T, P, 8, None) == 7
    assert L.mx_slice_and_scale_batched(ref(fa), ref(ft), 2, A, T, P + 1, need, None) == 4
    assert L.mx_slice_and_scale_batched(ref(fa), ref(ft), -1, A, T, P, need, None) == 3
    assert L.mx_slice_and_scale_batched(ref(fa), ref(ft), 0, None, None, None, 0, None) == 0
    # fake-quant
    s2 = B.MxDense(P, B.MX_F32, 32, 64, 64)
    d2 = B.MxDense(P + 0x10000, B.MX_F32, 32, 64, 64)
    assert L.mx_fake_quant(ref(mx.make_format("int4")), ref(mx.make_format("e4m3")), ref(s2), ref(d2), None) == 2
    assert L.mx_fake_quant(ref(mx.make_format("int4")), ref(mx.make_format("int6")), ref(s2), ref(d2), None) == 5
    assert L.mx_fake_quant(ref(mx.make_format("int4")), None, ref(s2), ref(B.MxDense(P, B.MX_F32, 32, 32, 32)), None) == 3
    assert L.mx_fake_quant(ref(mx.make_format("int4")), None, ref(s2), ref(B.MxDense(P, B.MX_BF16, 32, 64, 64)), None) == 5
    assert L.mx_fake_quant(ref(mx.make_format("int4", axis=0)), ref(mx.make_format("int8", axis=1)), ref(s2), ref(d2), None) == 2
    # blocks of 16 with an odd number of blocks: codes are packed in runs of 32, so widths that share dwords across
    # lanes are refused (quantize and dequant alike); 8- and 4-bit elements pass validation (0 rows here: no launch)
    for elem, want in (("int7", 5), ("int6", 5), ("int5", 5), ("int3", 5), ("int2", 5), ("e3m3", 5), ("e3m2", 5), ("e2m2", 5)):
        fk = mx.make_format(elem, block=16)
        for dt in (B.MX_F32, B.MX_BF16):
            assert L.mx_quantize(ref(fk), ref(B.MxDense(P, dt, 3, 48, 48)), ref(B.MxPacked(P, P, 3, 3)), None) == want, elem
            assert L.mx_dequant(ref(fk), ref(B.MxPacked(P, P, 1, 1)), ref(B.MxDense(P, dt, 1, 16, 16)), None) == want, elem
    # dequant
    assert L.mx_dequant(ref(f), ref(B.MxPacked(P, P, 32, 3)), ref(s2), None) == 3
    assert L.mx_dequant(ref(f), None, ref(s2), None) == 1
    # fused GEMM: A [M, K / 32 blocks], W anchor [N, K / 32 blocks], C fp32 [M, N]
    ga, gw = B.MxPacked(P, P, 16, 8), B.MxPacked(P, P, 64, 8)
    gc = B.MxDense(P, B.MX_F32, 16, 64, 64)
    assert L.mx_gemm_ss_fp4(None, ref(gw), ref(gc), None) == 1
    assert L.mx_gemm_ss_fp4(ref(ga), ref(gw), None, None) == 1
    assert L.mx_gemm_ss_fp4(ref(ga), ref(B.MxPacked(P, None, 64, 8)), ref(gc), None) == 1
    assert L.mx_gemm_ss_fp4(ref(ga), ref(gw), ref(B.MxDense(P, B.MX_BF16, 16, 64, 64)), None) == 5   # C is fp32 only
    assert L.mx_gemm_ss_fp4(ref(ga), ref(B.MxPacked(P, P, 64, 12)), ref(gc), None) == 3              # K differs
    assert L.mx_gemm_ss_fp4(ref(ga), ref(gw), ref(B.MxDense(P, B.MX_F32, 16, 32, 32)), None) == 3    # N differs
    assert L.mx_gemm_ss_fp4(ref(ga), ref(gw), ref(B.MxDense(P, B.MX_F32, 8, 64, 64)), None) == 3     # M differs
    assert L.mx_gemm_ss_fp4(ref(ga), ref(gw), ref(B.MxDense(P + 4, B.MX_F32, 16, 64, 64)), None) == 4
    assert L.mx_gemm_ss_fp4(ref(B.MxPacked(P, P, 16, 6)), ref(B.MxPacked(P, P, 64, 6)), ref(gc), None) == 5   # K = 192
    assert L.mx_gemm_ss_fp4(ref(B.MxPacked(None, None, 0, 8)), ref(gw), ref(B.MxDense(None, B.MX_F32, 0, 64, 64)), None) == 0
    # the workspace entry point: the same checks in front of any use of the workspace, then the workspace's own
    big = 1 << 20
    assert L.mx_gemm_ss_fp4_ws(None, ref(gw), ref(gc), ctypes.c_void_p(P), big, None) == 1
    assert L.mx_gemm_ss_fp4_ws(ref(ga), ref(B.MxPacked(P, P, 64, 12)), ref(gc), ctypes.c_void_p(P), big, None) == 3
    assert L.mx_gemm_ss_fp4_ws(ref(ga), ref(gw), ref(B.MxDense(P, B.MX_BF16, 16, 64, 64)), ctypes.c_void_p(P), big, None) == 5
    assert L.mx_gemm_ss_fp4_ws(ref(ga), ref(gw), ref(gc), ctypes.c_void_p(P + 8), big, None) == 4               # misaligned workspace
    assert L.mx_gemm_ss_fp4_ws(ref(ga), ref(gw), ref(gc), ctypes.c_void_p(P), L.mx_gemm_ss_fp4_workspace(64, 256) - 1, None) == 7
    assert L.mx_gemm_ss_fp4_ws(ref(B.MxPacked(None, None, 0, 8)), ref(gw), ref(B.MxDense(None, B.MX_F32, 0, 64, 64)), ctypes.c_void_p(P), big, None) == 0
    # the plan query answers "one slice" for arguments that the entry point would refuse or serve without the workspace
    # the product with a kept W_t: the same checks, no compute
    assert L.mx_gemm_fp8_fp4(None, ref(gw), ref(gc), None) == 1 and L.mx_gemm_fp8_fp4(ref(ga), ref(gw), None, None) == 1
    assert L.mx_gemm_fp8_fp4(ref(ga), ref(gw), ref(B.MxDense(P, B.MX_BF16, 16, 64, 64)), None) == 5
    assert L.mx_gemm_fp8_fp4(ref(ga), ref(B.MxPacked(P, P, 64, 12)), ref(gc), None) == 3
    assert L.mx_gemm_fp8_fp4(ref(B.MxPacked(P, P, 16, 6)), ref(B.MxPacked(P, P, 64, 6)), ref(gc), None) == 5
    assert L.mx_gemm_fp8_fp4(ref(B.MxPacked(None, None, 0, 8)), ref(gw), ref(B.MxDense(None, B.MX_F32, 0, 64, 64)), None) == 0
    assert L.mx_gemm_fp8_fp4_ws(None, ref(gw), ref(gc), ctypes.c_void_p(P), big, None) == 1
    assert L.mx_gemm_fp8_fp4_ws(ref(ga), ref(B.MxPacked(P, P, 64, 12)), ref(gc), ctypes.c_void_p(P), big, None) == 3
    assert L.mx_gemm_fp8_fp4_ws(ref(B.MxPacked(None, None, 0, 8)), ref(gw), ref(B.MxDense(None, B.MX_F32, 0, 64, 64)), ctypes.c_void_p(P), big, None) == 0
    assert L.mx_gemm_fp8_fp4_workspace(0, 64, 256) == 0 and L.mx_gemm_fp8_fp4_workspace(64, 64, 192) == 0
    assert L.mx_gemm_fp8_fp4_ws_slices(64, 64, 192, big) == 1 and L.mx_gemm_fp8_fp4_ws_slices(16, 4096, 14336, big) == 1
    assert L.mx_gemm_ss_fp4_ws_slices(0, 64, 256, big) == 1 and L.mx_gemm_ss_fp4_ws_slices(64, 64, 192, big) == 1
    assert L.mx_gemm_ss_fp4_ws_slices(64, 4096, 14336, 16) == 1                                                  # workspace too small
    for code in range(8):
        assert mx.binding.status_str(code) not in ("", "unknown status")
    assert mx.binding.status_str(42) == "unknown status"


def test_missing_library_fails_loudly(monkeypatch):
    from paper_2604_00529_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", "/nonexistent/libmx.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        binding.lib()
