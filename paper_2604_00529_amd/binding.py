"""ctypes binding of libmx.so: argument marshalling only.  Every step of the path runs in the
HIP kernels behind the C ABI declared in include/mx.h; torch is used for device memory and the
current stream.  There is no CPU fallback: without the built library every call raises."""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmx.so")

MX_OK = 0
STATUS_NAMES = {0: "MX_OK", 1: "MX_ERR_NULL", 2: "MX_ERR_FORMAT", 3: "MX_ERR_SHAPE", 4: "MX_ERR_ALIGN",
                5: "MX_ERR_UNSUPPORTED", 6: "MX_ERR_LAUNCH", 7: "MX_ERR_WORKSPACE"}

# mx_elem_t
ELEMS = {"int8": 0, "int7": 1, "int6": 2, "int5": 3, "int4": 4, "int3": 5, "int2": 6,
         "e4m3": 7, "e3m3": 8, "e3m2": 9, "e2m3": 10, "e2m2": 11, "e2m1": 12}
ROUND = {"default": 0, "away": 1, "even": 2}
MX_F32, MX_BF16 = 0, 1


class MxFormat(ctypes.Structure):
    _fields_ = [("elem", ctypes.c_int), ("scale", ctypes.c_int), ("block", ctypes.c_int32), ("axis", ctypes.c_int32),
                ("round", ctypes.c_int)]


class MxDense(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("dtype", ctypes.c_int), ("rows", ctypes.c_int64), ("cols", ctypes.c_int64),
                ("ld", ctypes.c_int64)]


class MxPacked(ctypes.Structure):
    _fields_ = [("codes", ctypes.c_void_p), ("scales", ctypes.c_void_p), ("outer", ctypes.c_int64),
                ("nblocks", ctypes.c_int64)]


class MxError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__("%s: %s (%s)" % (what, STATUS_NAMES.get(status, status), status_str(status)))


_lib = None


def lib():
    """The loaded C-ABI library; raises if it has not been built (python -m paper_2604_00529_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError("libmx.so is missing: build it with `python -m paper_2604_00529_amd.build` "
                               "(there is no fallback path)")
        # torch first: it brings its own copy of the HIP runtime, and the kernels of libmx.so must be registered
        # with that same runtime (the one that owns the tensors' memory and streams).  Loaded the other way round,
        # libmx.so binds to the system's runtime and its launches fail with "no ROCm-capable device".
        import torch  # noqa: F401
        L = ctypes.CDLL(_LIB_PATH)
        P = ctypes.POINTER
        vp, st = ctypes.c_void_p, ctypes.c_int
        L.mx_elem_bits.argtypes = [ctypes.c_int]
        L.mx_elem_bits.restype = ctypes.c_int
        L.mx_elem_emax.argtypes = [ctypes.c_int]
        L.mx_elem_emax.restype = ctypes.c_int
        L.mx_packed_bytes.argtypes = [P(MxFormat), ctypes.c_int64, ctypes.c_int64, P(ctypes.c_size_t), P(ctypes.c_size_t)]
        L.mx_packed_bytes.restype = st
        L.mx_quantize.argtypes = [P(MxFormat), P(MxDense), P(MxPacked), vp]
        L.mx_quantize.restype = st
        L.mx_slice_and_scale.argtypes = [P(MxFormat), P(MxPacked), P(MxFormat), P(MxPacked), vp]
        L.mx_slice_and_scale.restype = st
        L.mx_slice_and_scale_batched_workspace.argtypes = [ctypes.c_int32, ctypes.c_int64]
        L.mx_slice_and_scale_batched_workspace.restype = ctypes.c_size_t
        L.mx_slice_and_scale_batched.argtypes = [P(MxFormat), P(MxFormat), ctypes.c_int32, P(MxPacked), P(MxPacked), vp,
                                                 ctypes.c_size_t, vp]
        L.mx_slice_and_scale_batched.restype = st
        L.mx_slice_and_scale_batched_noalloc.argtypes = [P(MxFormat), P(MxFormat), ctypes.c_int32, P(MxPacked), P(MxPacked), vp]
        L.mx_slice_and_scale_batched_noalloc.restype = st
        L.mx_slice_and_scale_multi.argtypes = [P(MxFormat), P(MxPacked), ctypes.c_int32, P(MxFormat), P(MxPacked), vp]
        L.mx_slice_and_scale_multi.restype = st
        L.mx_slice_and_scale_multi_batched.argtypes = [P(MxFormat), ctypes.c_int32, P(MxFormat), ctypes.c_int32, P(MxPacked),
                                                       P(MxPacked), vp, ctypes.c_size_t, vp]
        L.mx_slice_and_scale_multi_batched.restype = st
        L.mx_gemm_ss_fp4_workspace.argtypes = [ctypes.c_int64, ctypes.c_int64]
        L.mx_gemm_ss_fp4_workspace.restype = ctypes.c_size_t
        L.mx_gemm_ss_fp4_ws_slices.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_size_t]
        L.mx_gemm_ss_fp4_ws_slices.restype = ctypes.c_int
        L.mx_gemm_ss_fp4_ws.argtypes = [P(MxPacked), P(MxPacked), P(MxDense), vp, ctypes.c_size_t, vp]
        L.mx_gemm_ss_fp4_ws.restype = st
        L.mx_fake_quant.argtypes = [P(MxFormat), P(MxFormat), P(MxDense), P(MxDense), vp]
        L.mx_fake_quant.restype = st
        L.mx_dequant.argtypes = [P(MxFormat), P(MxPacked), P(MxDense), vp]
        L.mx_dequant.restype = st
        L.mx_gemm_ss_fp4.argtypes = [P(MxPacked), P(MxPacked), P(MxDense), vp]
        L.mx_gemm_ss_fp4.restype = st
        L.mx_gemm_fp8_fp4.argtypes = [P(MxPacked), P(MxPacked), P(MxDense), vp]
        L.mx_gemm_fp8_fp4.restype = st
        L.mx_gemm_fp8_fp4_workspace.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int64]
        L.mx_gemm_fp8_fp4_workspace.restype = ctypes.c_size_t
        L.mx_gemm_fp8_fp4_ws_slices.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_size_t]
        L.mx_gemm_fp8_fp4_ws_slices.restype = ctypes.c_int
        L.mx_gemm_fp8_fp4_ws.argtypes = [P(MxPacked), P(MxPacked), P(MxDense), vp, ctypes.c_size_t, vp]
        L.mx_gemm_fp8_fp4_ws.restype = st
        L.mx_status_str.argtypes = [st]
        L.mx_status_str.restype = ctypes.c_char_p
        _lib = L
    return _lib


def status_str(status):
    return lib().mx_status_str(int(status)).decode()


def make_format(elem, axis=1, block=32, round="default"):
    e = ELEMS[elem] if isinstance(elem, str) else int(elem)
    r = ROUND[round] if isinstance(round, str) else int(round)
    return MxFormat(e, 0, block, axis, r)


def check(status, what):
    if status != MX_OK:
        raise MxError(status, what)
