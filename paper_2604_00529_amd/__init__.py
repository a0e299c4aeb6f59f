"""MI355X-native MX quantization, Slice-and-Scale, fake-quant and dequantization.

Thin Python front end over the C-ABI library libmx.so (hand-written HIP kernels for gfx950).
The functions here have the names of the C entry points and only marshal arguments: torch
supplies device memory and the current stream.  bfloat16 / float32 CUDA(HIP) tensors in,
uint8 CUDA tensors for codes and scales.
"""
import ctypes

from . import binding
from .binding import ELEMS, MxError, make_format

__all__ = ["mx_quantize", "mx_slice_and_scale", "mx_slice_and_scale_batched", "mx_slice_and_scale_batched_noalloc",
           "mx_slice_and_scale_multi", "mx_fake_quant", "mx_dequant",
           "mx_gemm_ss_fp4", "mx_gemm_fp8_fp4", "mx_packed_bytes", "mx_elem_bits", "mx_elem_emax", "MxFakeQuantSTE", "ELEMS", "MxError", "make_format",
           "packed_shape", "SsBatch"]


_torch_module = None


def _torch():
    global _torch_module
    if _torch_module is None:
        import torch
        _torch_module = torch
    return _torch_module


def _stream(t):
    """The current HIP stream of t's device as a void pointer (the raw handle: building a torch Stream object for it
    costs 2 us per call, a fifth of what a small call costs on the CPU)."""
    torch = _torch()
    raw = getattr(torch._C, "_cuda_getCurrentRawStream", None)
    if raw is not None:
        return ctypes.c_void_p(raw(t.device.index if t.device.index is not None else torch.cuda.current_device()))
    return ctypes.c_void_p(torch.cuda.current_stream(t.device).cuda_stream)


_ELEM_BITS = {}


def _elem_bits(elem):
    b = _ELEM_BITS.get(elem)
    if b is None:
        b = _ELEM_BITS[elem] = binding.lib().mx_elem_bits(elem)
    return b


def _dense(t):
    torch = _torch()
    if t.dim() != 2:
        raise ValueError("dense tensors are 2-D [rows, cols]")
    if not t.is_cuda:
        raise ValueError("tensors must live on the GPU")
    if t.dtype == torch.float32:
        dt = binding.MX_F32
    elif t.dtype == torch.bfloat16:
        dt = binding.MX_BF16
    else:
        raise TypeError("dense tensors are float32 or bfloat16")
    if t.stride(1) != 1 and t.shape[1] > 1:
        raise ValueError("dense tensors must be row-major (unit stride along columns)")
    ld = t.stride(0) if t.shape[0] > 1 else t.shape[1]
    return binding.MxDense(t.data_ptr(), dt, t.shape[0], t.shape[1], ld)


def _packed(codes, scales, outer, nblocks):
    torch = _torch()
    for x in (codes, scales):
        if x.dtype != torch.uint8 or not x.is_cuda or not x.is_contiguous():
            raise TypeError("codes and scales are contiguous uint8 GPU tensors")
    return binding.MxPacked(codes.data_ptr(), scales.data_ptr(), outer, nblocks)


def mx_elem_bits(elem):
    return binding.lib().mx_elem_bits(ELEMS[elem])


def mx_elem_emax(elem):
    return binding.lib().mx_elem_emax(ELEMS[elem])


def mx_packed_bytes(fmt, rows, cols):
    cb, sb = ctypes.c_size_t(0), ctypes.c_size_t(0)
    binding.check(binding.lib().mx_packed_bytes(ctypes.byref(fmt), rows, cols, ctypes.byref(cb), ctypes.byref(sb)),
                  "mx_packed_bytes")
    return cb.value, sb.value


def packed_shape(fmt, rows, cols):
    """(outer, nblocks, bytes_per_block) of a [rows, cols] tensor in format fmt."""
    outer, ext = (rows, cols) if fmt.axis == 1 else (cols, rows)
    return outer, ext // fmt.block, fmt.block * _elem_bits(fmt.elem) // 8


def _alloc_packed(fmt, rows, cols, device):
    torch = _torch()
    outer, nblocks, bb = packed_shape(fmt, rows, cols)
    codes = torch.empty((outer, nblocks, bb), dtype=torch.uint8, device=device)
    scales = torch.empty((outer, nblocks), dtype=torch.uint8, device=device)
    return codes, scales


def mx_quantize(src, fmt, codes=None, scales=None):
    """Q_f (Eq. (1), (2)): dense [rows, cols] -> (codes[outer, nblocks, bytes], scales[outer, nblocks])."""
    rows, cols = src.shape
    outer, nblocks, bb = packed_shape(fmt, rows, cols)
    if codes is None:
        torch = _torch()
        codes = torch.empty((outer, nblocks, bb), dtype=torch.uint8, device=src.device)
        scales = torch.empty((outer, nblocks), dtype=torch.uint8, device=src.device)
    d = _dense(src)
    p = _packed(codes, scales, outer, nblocks)
    binding.check(binding.lib().mx_quantize(ctypes.byref(fmt), ctypes.byref(d), ctypes.byref(p), _stream(src)), "mx_quantize")
    return codes, scales


def mx_slice_and_scale(codes, scales, fa, ft, out_codes=None, out_scales=None):
    """Q_{A->t} (Eq. (4), (6)) on a packed anchor; returns (codes, scales) of the target format."""
    torch = _torch()
    nb = scales.numel()
    bb = ft.block * _elem_bits(ft.elem) // 8
    if out_codes is None:
        out_codes = torch.empty(tuple(scales.shape) + (bb,), dtype=torch.uint8, device=codes.device)
        out_scales = torch.empty_like(scales)
    a = _packed(codes, scales, 1, nb)
    t = _packed(out_codes, out_scales, 1, nb)
    binding.check(binding.lib().mx_slice_and_scale(ctypes.byref(fa), ctypes.byref(a), ctypes.byref(ft), ctypes.byref(t),
                                                   _stream(codes)), "mx_slice_and_scale")
    return out_codes, out_scales


def mx_slice_and_scale_multi(codes, scales, fa, fts, outs=None):
    """Several targets from one pass over the anchor; returns [(codes, scales)] in the order of fts."""
    torch = _torch()
    L = binding.lib()
    nb = scales.numel()
    if outs is None:
        outs = [(torch.empty(tuple(scales.shape) + (f.block * L.mx_elem_bits(f.elem) // 8,), dtype=torch.uint8,
                             device=codes.device), torch.empty_like(scales)) for f in fts]
    a = _packed(codes, scales, 1, nb)
    F = (binding.MxFormat * len(fts))(*fts)
    T = (binding.MxPacked * len(fts))(*[_packed(c, s, 1, nb) for c, s in outs])
    binding.check(L.mx_slice_and_scale_multi(ctypes.byref(fa), ctypes.byref(a), len(fts), F, T, _stream(codes)),
                  "mx_slice_and_scale_multi")
    return outs


def mx_slice_and_scale_batched(anchors, fa, ft, targets=None, workspace=None):
    """One launch over a list of (codes, scales) anchors (a checkpoint).  Returns the target list."""
    torch = _torch()
    n = len(anchors)
    L = binding.lib()
    bb = ft.block * L.mx_elem_bits(ft.elem) // 8
    if targets is None:
        targets = [(torch.empty(tuple(s.shape) + (bb,), dtype=torch.uint8, device=c.device), torch.empty_like(s))
                   for c, s in anchors]
    if n == 0:
        return targets
    dev = anchors[0][0].device
    need = L.mx_slice_and_scale_batched_workspace(n, sum(s.numel() for _, s in anchors))
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    A = (binding.MxPacked * n)(*[_packed(c, s, 1, s.numel()) for c, s in anchors])
    T = (binding.MxPacked * n)(*[_packed(c, s, 1, s.numel()) for c, s in targets])
    binding.check(L.mx_slice_and_scale_batched(ctypes.byref(fa), ctypes.byref(ft), n, A, T,
                                               ctypes.c_void_p(workspace.data_ptr()), workspace.numel(),
                                               _stream(anchors[0][0])), "mx_slice_and_scale_batched")
    return targets


def mx_slice_and_scale_batched_noalloc(anchors, fa, ft, targets):
    """mx_slice_and_scale_batched with the launch tables in the library's own fixed device array: the call allocates
    nothing (the targets are the caller's).  Calls on one GPU must not overlap in time."""
    n = len(anchors)
    if n == 0:
        return targets
    A = (binding.MxPacked * n)(*[_packed(c, s, 1, s.numel()) for c, s in anchors])
    T = (binding.MxPacked * n)(*[_packed(c, s, 1, s.numel()) for c, s in targets])
    binding.check(binding.lib().mx_slice_and_scale_batched_noalloc(ctypes.byref(fa), ctypes.byref(ft), n, A, T,
                                                                   _stream(anchors[0][0])), "mx_slice_and_scale_batched_noalloc")
    return targets


class SsBatch:
    """A batched Slice-and-Scale call with its descriptor arrays marshalled once (a checkpoint's
    layout is static): `run()` is then a single C call.  `ft` is one target format, or a list of
    formats (increasing element order) that are all produced from one pass over the anchors; `targets`
    is then a list, per anchor tensor, of one (codes, scales) pair per format."""

    def __init__(self, anchors, fa, ft, targets=None, workspace=None):
        torch = _torch()
        L = binding.lib()
        n = len(anchors)
        self.multi = isinstance(ft, (list, tuple))
        fts = list(ft) if self.multi else [ft]
        if targets is None:
            targets = [[(torch.empty(tuple(s.shape) + (f.block * L.mx_elem_bits(f.elem) // 8,), dtype=torch.uint8,
                                     device=c.device), torch.empty_like(s)) for f in fts] for c, s in anchors]
        elif not self.multi:
            targets = [[t] for t in targets]
        if workspace is None:
            need = L.mx_slice_and_scale_batched_workspace(n, sum(s.numel() for _, s in anchors))
            workspace = torch.empty(max(16, need), dtype=torch.uint8, device=anchors[0][0].device)
        self.anchors, self.targets, self.workspace = anchors, targets, workspace     # keep the tensors alive
        self.fa, self.n, self.nt = fa, n, len(fts)
        self._F = (binding.MxFormat * len(fts))(*fts)
        self._A = (binding.MxPacked * n)(*[_packed(c, s, 1, s.numel()) for c, s in anchors])
        self._T = (binding.MxPacked * (n * len(fts)))(*[_packed(c, s, 1, s.numel()) for row in targets for c, s in row])
        self._dev = anchors[0][0].device

    def run(self):
        stream = _stream(self.workspace)
        binding.check(binding.lib().mx_slice_and_scale_multi_batched(
            ctypes.byref(self.fa), self.nt, self._F, self.n, self._A, self._T,
            ctypes.c_void_p(self.workspace.data_ptr()), self.workspace.numel(), stream), "mx_slice_and_scale_multi_batched")
        return self.targets if self.multi else [row[0] for row in self.targets]


def mx_fake_quant(src, target, anchor=None, out=None):
    """DQ(Q_t(src)), or DQ(Q_{A->t}(Q_A(src))) when an anchor format is given (Eq. (7))."""
    torch = _torch()
    if out is None:
        out = torch.empty_like(src)
    s, d = _dense(src), _dense(out)
    a = ctypes.byref(anchor) if anchor is not None else None
    binding.check(binding.lib().mx_fake_quant(ctypes.byref(target), a, ctypes.byref(s), ctypes.byref(d), _stream(src)),
                  "mx_fake_quant")
    return out


def mx_dequant(codes, scales, fmt, rows, cols, dtype=None, out=None):
    """V^ = X * P into a dense [rows, cols] tensor."""
    torch = _torch()
    if out is None:
        out = torch.empty((rows, cols), dtype=dtype or torch.float32, device=codes.device)
    outer, nblocks, _ = packed_shape(fmt, rows, cols)
    p = _packed(codes, scales, outer, nblocks)
    d = _dense(out)
    binding.check(binding.lib().mx_dequant(ctypes.byref(fmt), ctypes.byref(p), ctypes.byref(d), _stream(codes)), "mx_dequant")
    return out


GEMM_HOIST_MIN_ROWS = 512   # MX_GEMM_HOIST_MIN_ROWS of mx.h
GEMM_WORKSPACE_MIN_ROWS = 49   # below, the streaming kernels run whatever the caller lends


def mx_gemm_ss_fp4(a_codes, a_scales, w_codes, w_scales, out=None, workspace=None):
    """C[M, N] = DQ(A) @ DQ(SS(W_anchor -> E2M1)).T (scaled MX MFMA, fp32 out).

    a_*: MXFP8 E4M3 activations [M, K/32, 32] / [M, K/32]; w_*: E4M3 anchor, K-contiguous [N, K/32, 32] / [N, K/32].
    The anchor is sliced in registers on its way into the product, or, from 512 rows on when C has enough tiles, once
    per call into `workspace` (uint8, mx_gemm_ss_fp4_workspace(N, K) bytes; allocated here when not given) and
    multiplied from there, with the same results bit for bit.  From 49 rows on the workspace also lets shapes with few
    tiles split K over several workgroups (partial sums added in a fixed order of their own).  workspace=False keeps
    the on-the-fly kernels without a workspace."""
    torch = _torch()
    L = binding.lib()
    M, KB = a_scales.shape
    N = w_scales.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=a_codes.device)
    a = _packed(a_codes, a_scales, M, KB)
    w = _packed(w_codes, w_scales, N, w_scales.shape[1])
    c = _dense(out)
    if M >= GEMM_WORKSPACE_MIN_ROWS and workspace is not False:
        need = L.mx_gemm_ss_fp4_workspace(N, KB * 32)
        if workspace is None:
            workspace = torch.empty(max(16, need), dtype=torch.uint8, device=a_codes.device)
        binding.check(L.mx_gemm_ss_fp4_ws(ctypes.byref(a), ctypes.byref(w), ctypes.byref(c), ctypes.c_void_p(workspace.data_ptr()),
                                          workspace.numel(), _stream(a_codes)), "mx_gemm_ss_fp4_ws")
        return out
    binding.check(L.mx_gemm_ss_fp4(ctypes.byref(a), ctypes.byref(w), ctypes.byref(c), _stream(a_codes)), "mx_gemm_ss_fp4")
    return out


def mx_gemm_fp8_fp4(a_codes, a_scales, w4_codes, w4_scales, out=None, workspace=None):
    """C[M, N] = DQ(A) @ DQ(W_t).T for MXFP4 E2M1 weights the caller keeps (Sec. 3.5 "Inference": the anchor is converted
    once per precision switch, not per call).

    a_*: MXFP8 E4M3 activations [M, K/32, 32] / [M, K/32]; w4_*: E2M1 codes [N, K/32, 16] / scale bytes [N, K/32], e.g.
    the result of mx_slice_and_scale(anchor -> e2m1).  The results are mx_gemm_ss_fp4's on that anchor bit for bit --
    unless the shape has few tiles and a long K: then, from 49 rows on, K is split over several workgroups per tile
    through `workspace` (uint8; mx_gemm_fp8_fp4_workspace(M, N, K) bytes, allocated here when not given) and the partial
    sums are added in a fixed order of their own.  workspace=False never splits."""
    torch = _torch()
    L = binding.lib()
    M, KB = a_scales.shape
    N = w4_scales.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=a_codes.device)
    a = _packed(a_codes, a_scales, M, KB)
    w = _packed(w4_codes, w4_scales, N, w4_scales.shape[1])
    c = _dense(out)
    if M >= GEMM_WORKSPACE_MIN_ROWS and workspace is not False:
        need = L.mx_gemm_fp8_fp4_workspace(M, N, KB * 32)
        if need:
            if workspace is None:
                workspace = torch.empty(need, dtype=torch.uint8, device=a_codes.device)
            binding.check(L.mx_gemm_fp8_fp4_ws(ctypes.byref(a), ctypes.byref(w), ctypes.byref(c), ctypes.c_void_p(workspace.data_ptr()),
                                               workspace.numel(), _stream(a_codes)), "mx_gemm_fp8_fp4_ws")
            return out
    binding.check(L.mx_gemm_fp8_fp4(ctypes.byref(a), ctypes.byref(w), ctypes.byref(c), _stream(a_codes)), "mx_gemm_fp8_fp4")
    return out


def _ste_class():
    torch = _torch()

    class _MxFakeQuantSTE(torch.autograd.Function):
        """Fake-quant forward; the backward pass is the straight-through estimator of Sec. 3.5:
        the gradient goes through both quantizers unchanged (the same tensor is returned)."""

        @staticmethod
        def forward(ctx, w, target, anchor):
            return mx_fake_quant(w, target, anchor)

        @staticmethod
        def backward(ctx, grad_out):
            return grad_out, None, None

    return _MxFakeQuantSTE


class _Lazy:
    _cls = None

    def apply(self, w, target, anchor=None):
        if _Lazy._cls is None:
            _Lazy._cls = _ste_class()
        return _Lazy._cls.apply(w, target, anchor)


MxFakeQuantSTE = _Lazy()
