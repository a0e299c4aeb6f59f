"""mx_slice_and_scale_batched_noalloc -- the batched Slice-and-Scale call for callers that cannot allocate: its launch
tables live in a fixed device array inside the library.  Through the C ABI, against mx_slice_and_scale_batched (same
kernels, caller's workspace) bit for bit, on two calls in a row of which the second is smaller, and against the oracle."""
import ctypes

import numpy as np
import pytest

from paper_2604_00529_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mx():
    import torch
    assert torch.cuda.is_available()
    import paper_2604_00529_amd as mx
    mx.binding.lib()
    return mx


def _anchors(torch, sizes, seed):
    out = []
    for i, nb in enumerate(sizes):
        c = torch.from_numpy(synth.random_bytes(seed + i, nb * 32).reshape(nb, 32)).cuda()
        s = torch.from_numpy(synth.random_bytes(seed + 500 + i, nb)).cuda()
        out.append((c, s))
    return out


def _targets(torch, anchors, bb, fill):
    return [(torch.full((s.numel(), bb), fill, dtype=torch.uint8, device="cuda"), torch.full_like(s, fill)) for _, s in anchors]


def _call_noalloc(mx, anchors, fa, ft, targets):
    B, L = mx.binding, mx.binding.lib()
    n = len(anchors)
    A = (B.MxPacked * n)(*[mx._packed(c, s, 1, s.numel()) for c, s in anchors])
    T = (B.MxPacked * n)(*[mx._packed(c, s, 1, s.numel()) for c, s in targets])
    return L.mx_slice_and_scale_batched_noalloc(ctypes.byref(fa), ctypes.byref(ft), n, A, T, mx._stream(anchors[0][0]))


@pytest.mark.parametrize("anchor,target", [("e4m3", "e2m1"), ("e4m3", "e3m2"), ("int8", "int4"), ("int8", "int5")])
def test_two_calls_in_a_row_second_smaller(mx, oracle, anchor, target):
    import torch
    fa, ft = mx.make_format(anchor), mx.make_format(target)
    bb = 32 * oracle.elem_bits(target) // 8
    # first call: tensors large enough for the large segments (2^16 pieces each) plus ragged small ones;
    # second call: fewer and smaller tensors (small segments), so most of the table keeps the first call's descriptors
    for sizes, seed in (((300000, 70001, 2, 131072, 4098, 66), 11), ((4098, 34, 2), 77)):
        anchors = _anchors(torch, sizes, seed)
        want = _targets(torch, anchors, bb, 0x5A)
        mx.mx_slice_and_scale_batched(anchors, fa, ft, targets=want)
        got = _targets(torch, anchors, bb, 0xA5)
        assert _call_noalloc(mx, anchors, fa, ft, got) == 0
        torch.cuda.synchronize()
        for i, ((gc, gs), (wc, ws)) in enumerate(zip(got, want)):
            assert torch.equal(gc, wc) and torch.equal(gs, ws), (sizes[i], "differs from mx_slice_and_scale_batched")
        # and against the oracle itself, on the small tensors and a window of the largest
        for i, nb in enumerate(sizes):
            lo, hi = (0, nb) if nb <= 8192 else (nb - 4096, nb)
            oc, os_ = oracle.slice_and_scale(anchors[i][0][lo:hi].cpu().numpy(), anchors[i][1][lo:hi].cpu().numpy(), anchor, target)
            assert np.array_equal(got[i][0][lo:hi].cpu().numpy(), oc) and np.array_equal(got[i][1][lo:hi].cpu().numpy(), os_)


def test_python_front_end_and_empty_batch(mx, oracle):
    import torch
    fa, ft = mx.make_format("e4m3"), mx.make_format("e2m1")
    anchors = _anchors(torch, (1000, 5), 5)
    got = mx.mx_slice_and_scale_batched_noalloc(anchors, fa, ft, _targets(torch, anchors, 16, 0))
    torch.cuda.synchronize()
    for (c, s), (gc, gs) in zip(anchors, got):
        oc, os_ = oracle.slice_and_scale(c.cpu().numpy(), s.cpu().numpy(), "e4m3", "e2m1")
        assert np.array_equal(gc.cpu().numpy(), oc) and np.array_equal(gs.cpu().numpy(), os_)
    L = mx.binding.lib()
    assert L.mx_slice_and_scale_batched_noalloc(ctypes.byref(fa), ctypes.byref(ft), 0, None, None, None) == 0


def test_more_segments_than_the_table_holds_is_an_error_and_writes_nothing(mx):
    # 8200 tensors of one block each need two descriptors apiece (codes, scale bytes): 16400 > 16384
    import torch
    B, L = mx.binding, mx.binding.lib()
    n = 8200
    codes = torch.zeros((n, 32), dtype=torch.uint8, device="cuda")
    scales = torch.zeros((n, 16), dtype=torch.uint8, device="cuda")           # 16 bytes apart: aligned scale pointers
    out_c = torch.full((n, 16), 0xA5, dtype=torch.uint8, device="cuda")
    out_s = torch.full((n, 16), 0xA5, dtype=torch.uint8, device="cuda")
    A = (B.MxPacked * n)(*[B.MxPacked(codes.data_ptr() + 32 * i, scales.data_ptr() + 16 * i, 1, 1) for i in range(n)])
    T = (B.MxPacked * n)(*[B.MxPacked(out_c.data_ptr() + 16 * i, out_s.data_ptr() + 16 * i, 1, 1) for i in range(n)])
    fa, ft = mx.make_format("e4m3"), mx.make_format("e2m1")
    assert L.mx_slice_and_scale_batched_noalloc(ctypes.byref(fa), ctypes.byref(ft), n, A, T, None) == 7   # MX_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((out_c == 0xA5).all()) and bool((out_s == 0xA5).all())
    # 8000 such tensors fit
    assert L.mx_slice_and_scale_batched_noalloc(ctypes.byref(fa), ctypes.byref(ft), 8000, A, T, None) == 0
    torch.cuda.synchronize()
    assert bool((out_c[:8000] == 0).all()) and bool((out_c[8000:] == 0xA5).all())
    assert bool((out_s[:8000, 0] == 6).all()) and bool((out_s[:8000, 1:] == 0xA5).all()) and bool((out_s[8000:] == 0xA5).all())
