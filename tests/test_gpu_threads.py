"""Host threads calling the library at the same time, each on a stream of its own.  The library keeps nothing per call
on the host, and what it memoizes per device (the number of compute units, the kernels whose dynamic LDS size has been
allowed) is safe under concurrent callers: every thread must get the bits that the same calls give one after the other.
(ctypes releases the interpreter lock for the duration of a call, so the launch code really runs concurrently.)"""
import threading

import numpy as np
import pytest

from test_gpu_parity import mx, to_gpu  # noqa: F401  (mx is the module fixture)

pytestmark = pytest.mark.gpu

THREADS, ROUNDS = 4, 12


def _inputs(seed):
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal((96, 1024)) * 0.05).astype(np.float32)        # activations: 96 rows (tiled GEMM), 16 used for decode
    w = (rng.standard_normal((160, 1024)) * 0.02).astype(np.float32)       # weights: N = 160
    xc = (rng.standard_normal((256, 96)) * 0.3).astype(np.float32)         # blocks down the columns
    return to_gpu(x), to_gpu(w), to_gpu(xc)


def _sequence(mx, x, w, xc):
    """One pass over every kind of entry point; returns everything it computed."""
    fa, ft, f6 = mx.make_format("e4m3"), mx.make_format("e2m1"), mx.make_format("e3m2")
    f0 = mx.make_format("int4", axis=0)
    xa = mx.mx_quantize(x, fa)
    wa = mx.mx_quantize(w, fa)
    w4 = mx.mx_slice_and_scale(wa[0], wa[1], fa, ft)
    w6 = mx.mx_slice_and_scale(wa[0], wa[1], fa, f6)
    out = [xa[0], xa[1], wa[0], wa[1], w4[0], w4[1], w6[0], w6[1]]
    out.append(mx.mx_dequant(w6[0], w6[1], f6, w.shape[0], w.shape[1]))
    out.append(mx.mx_fake_quant(w, ft, fa))
    out.append(mx.mx_fake_quant(xc, f0))
    qc = mx.mx_quantize(xc, f0)
    out += [qc[0], qc[1]]
    out.append(mx.mx_gemm_ss_fp4(xa[0][:16], xa[1][:16], wa[0], wa[1]))     # decode kernel
    out.append(mx.mx_gemm_ss_fp4(xa[0][:40], xa[1][:40], wa[0], wa[1]))     # 16 < M <= 48
    out.append(mx.mx_gemm_ss_fp4(xa[0], xa[1], wa[0], wa[1], workspace=False))   # tiled kernel
    out.append(mx.mx_gemm_fp8_fp4(xa[0], xa[1], w4[0], w4[1], workspace=False))  # the same from a kept W_t
    return out


def test_concurrent_host_threads_get_the_sequential_bits(mx):
    import torch
    data = [_inputs(400 + t) for t in range(THREADS)]
    want = [_sequence(mx, *d) for d in data]
    torch.cuda.synchronize()
    got = [None] * THREADS
    errors = []
    start = threading.Barrier(THREADS)

    def worker(t):
        try:
            stream = torch.cuda.Stream()                                   # default priority
            with torch.cuda.stream(stream):
                start.wait()
                for _ in range(ROUNDS):
                    res = _sequence(mx, *data[t])
                stream.synchronize()
            got[t] = res
        except Exception as e:                                             # noqa: BLE001  (reported by the main thread)
            errors.append((t, repr(e)))

    threads = [threading.Thread(target=worker, args=(t,)) for t in range(THREADS)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for t in range(THREADS):
        assert len(got[t]) == len(want[t])
        for k, (g, w_) in enumerate(zip(got[t], want[t])):
            assert g.dtype == w_.dtype and g.shape == w_.shape
            same = torch.equal(g.view(torch.uint8), w_.view(torch.uint8)) if g.dtype != torch.uint8 else torch.equal(g, w_)
            assert same, "thread %d, result %d differs from the sequential run" % (t, k)
