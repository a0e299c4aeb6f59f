"""Seeded synthetic inputs shaped like the paper's workloads.

The paper quantizes the linear weights of Llama / Qwen text decoders (Sec. 3.1,
3.2) and, for its tensor-level study, random (1, 1024) tensors (Sec. 4.3).  The
real checkpoints are not available, so these generators stand in for them.

This module holds no arithmetic of the method (no scale, rounding, packing or
format logic): it only draws numbers.  It is the one module that both the CPU
oracle's tests and the HIP path's tests feed from.

Host generators return numpy arrays: float32, or uint16 holding bfloat16 bit
patterns.  `torch_*` generators build the large tensors directly on the GPU.
"""
import numpy as np

# Llama-8B-shaped decoder (weights are [out_features, in_features], blocks run along in_features)
LLAMA8B = dict(layers=32, hidden=4096, ffn=14336, q_heads=32, kv_heads=8, head_dim=128, vocab=128256)


def f32_to_bf16_bits(x):
    """Nearest-even float32 -> bfloat16 bit patterns (uint16). Input preparation only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    nan = (u & 0x7FFFFFFF) > 0x7F800000
    r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)
    r[nan] = 0x7FC0
    return r


def bf16_bits_to_f32(h):
    return (np.ascontiguousarray(h, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def config1_weight(seed=1001, rows=1024, cols=1024):
    """fp32 N(0, 0.02^2) matrix with 1 % of the columns scaled x20 (outlier channels)."""
    rng = np.random.default_rng(seed)
    w = (rng.standard_normal((rows, cols)) * 0.02).astype(np.float32)
    n_out = max(1, cols // 100)
    out_cols = rng.choice(cols, size=n_out, replace=False)
    w[:, out_cols] *= np.float32(20.0)
    return w


def config2_weight(seed=1002, rows=4096, cols=4096):
    """bf16 matrix 0.02 * Student-t(nu = 4): heavy tails reach target underflow and saturation."""
    rng = np.random.default_rng(seed)
    w = (rng.standard_t(4, size=(rows, cols)) * 0.02).astype(np.float32)
    return f32_to_bf16_bits(w)


def llama8b_tensor_list(layers=None):
    """(name, rows, cols) of every decoder linear, lm_head excluded (Sec. 3.2 weight-only recipe)."""
    c = LLAMA8B
    L = c["layers"] if layers is None else layers
    h, f = c["hidden"], c["ffn"]
    kv = c["kv_heads"] * c["head_dim"]
    out = []
    for l in range(L):
        out += [(f"l{l}.q", h, h), (f"l{l}.k", kv, h), (f"l{l}.v", kv, h), (f"l{l}.o", h, h),
                (f"l{l}.gate", f, h), (f"l{l}.up", f, h), (f"l{l}.down", h, f)]
    return out


def config3_seed(index):
    return 3000 + index


def config3_weight_host(index, rows, cols):
    """One decoder tensor on the host (bf16 bits), N(0, 0.02^2); for reduced-size parity cases."""
    rng = np.random.default_rng(config3_seed(index))
    return f32_to_bf16_bits((rng.standard_normal((rows, cols)) * 0.02).astype(np.float32))


def torch_config3_weight(index, rows, cols, device="cuda"):
    """One decoder tensor generated on the GPU (bf16), N(0, 0.02^2), seeded per tensor."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(config3_seed(index))
    w = torch.empty((rows, cols), dtype=torch.float32, device=device)
    w.normal_(0.0, 0.02, generator=g)
    return w.to(torch.bfloat16)


def config4_activations(seed=1004, tokens=8 * 4096, hidden=4096):
    """bf16 N(0,1) activations with 0.1 % of the channels scaled x100."""
    rng = np.random.default_rng(seed)
    a = rng.standard_normal((tokens, hidden), dtype=np.float32)
    n_out = max(1, hidden // 1000)
    ch = rng.choice(hidden, size=n_out, replace=False)
    a[:, ch] *= np.float32(100.0)
    return f32_to_bf16_bits(a)


def config4_weight(seed=1104, rows=4096, cols=14336):
    rng = np.random.default_rng(seed)
    return f32_to_bf16_bits(rng.standard_normal((rows, cols), dtype=np.float32) * np.float32(0.02))


def torch_config4_activations(seed=1004, tokens=8 * 4096, hidden=4096, device="cuda"):
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    a = torch.empty((tokens, hidden), dtype=torch.float32, device=device)
    a.normal_(0.0, 1.0, generator=g)
    n_out = max(1, hidden // 1000)
    ch = np.random.default_rng(seed).choice(hidden, size=n_out, replace=False)
    a[:, torch.as_tensor(ch, device=device)] *= 100.0
    return a.to(torch.bfloat16)


QAT_FORMATS = ("int8", "int6", "int4", "e4m3", "e3m2", "e2m1")


def config4_format_schedule(seed=1004, steps=64):
    """Uniformly sampled target format per QAT step (Sec. 4.4 cycles formats uniformly)."""
    rng = np.random.default_rng(seed)
    return [QAT_FORMATS[i] for i in rng.integers(len(QAT_FORMATS), size=steps)]


def random_bytes(seed, n):
    """Uniform random bytes: every code and every scale byte shows up (adversarial anchors)."""
    return np.random.default_rng(seed).integers(0, 256, size=n, dtype=np.uint8)


def random_tensors_1x1024(seed=4300, count=100):
    """The tensor-level study's inputs (Sec. 4.3, App. C): 100 random (1, 1024) tensors, N(0,1)."""
    rng = np.random.default_rng(seed)
    return [rng.standard_normal((1, 1024)).astype(np.float32) for _ in range(count)]


def edge_case_matrix(seed=77, rows=8, cols=256, dtype="f32"):
    """Rows that hit the degenerate paths: zeros, fp32 subnormals, huge values, powers of two,
    exact ties, negative zero; NaN / Inf rows are separate (`special_matrix`)."""
    rng = np.random.default_rng(seed)
    m = np.zeros((rows, cols), dtype=np.float32)
    m[1] = (rng.standard_normal(cols) * 1e-41).astype(np.float32)          # fp32 subnormals
    m[2] = (rng.standard_normal(cols) * 1e38).astype(np.float32).clip(-3.0e38, 3.0e38)
    m[3] = np.ldexp(np.float32(1.0), rng.integers(-140, 127, size=cols)).astype(np.float32)
    m[4] = (rng.integers(-256, 257, size=cols) / 16.0).astype(np.float32)   # many exact ties
    m[5] = -0.0
    m[5, ::7] = 1.0
    m[6] = (rng.standard_normal(cols) * np.exp(rng.uniform(-40, 40, size=cols))).astype(np.float32)
    m[7] = (rng.integers(-1024, 1025, size=cols) * 0.125).astype(np.float32)
    if rows > 8:
        m[8:] = (rng.standard_normal((rows - 8, cols)) * 0.02).astype(np.float32)
    return m if dtype == "f32" else f32_to_bf16_bits(m)


def special_matrix(cols=128, dtype="f32"):
    """Blocks that hold NaN / +-Inf next to ordinary numbers."""
    m = np.ones((4, cols), dtype=np.float32)
    m[0, 3] = np.nan
    m[1, 40] = np.inf
    m[2, 70] = -np.inf
    m[3, 5] = np.nan
    m[3, 100] = np.inf
    return m if dtype == "f32" else f32_to_bf16_bits(m)
