"""Multi-format QAT plumbing around the fused fake-quant kernel (Sec. 3.2, Sec. 3.5).

What the paper trains is a model whose linear weights pass, in every forward pass, through the
quantizer of the format that the schedule names for that step:

* standard multi-format QAT (Sec. 3.2): ``W_t = DQ(Q_t(W))``, formats visited one after the other in
  order of increasing bit width, one epoch each;
* anchor-storage training (Sec. 3.5, Eq. (7)): ``W_A = Q_A(W)``, ``W_t = Q_{A->t}(W_A)`` -- the weights
  the model will run with after Slice-and-Scale of the stored anchor -- with the target format cycling
  uniformly over the formats (Sec. 4, anchor variant).

Gradients pass both quantizers unchanged (straight-through estimator).  Everything numeric runs in the
HIP kernels (`mx_fake_quant` through `MxFakeQuantSTE`); this module only routes tensors and names
formats.  The paper's models, datasets and optimizer settings are not part of this repository: the
module is exercised on a synthetic toy model.
"""
import itertools

from . import MxFakeQuantSTE, make_format, mx_elem_bits

# formats of the paper's training runs (Sec. 3.2): MXINT 2 / 4 / 6 / 8 bit and MXFP E2M1 / E3M2 / E4M3
MXINT_TRAIN_FORMATS = ("int2", "int4", "int6", "int8")
MXFP_TRAIN_FORMATS = ("e2m1", "e3m2", "e4m3")


def anchor_of(elem):
    """The 8-bit anchor of an element format's family (Sec. 3.5): MXINT8 or MXFP8 (E4M3)."""
    return "int8" if elem.startswith("int") else "e4m3"


def sequential_schedule(formats, steps_per_epoch, epochs_per_format=1):
    """Sec. 3.2: one format at a time, in order of increasing bit width, `epochs_per_format` epochs each.
    Yields one element-format name per optimizer step."""
    ordered = sorted(formats, key=mx_elem_bits)
    for elem in ordered:
        for _ in range(steps_per_epoch * epochs_per_format):
            yield elem


def cycling_schedule(formats, steps):
    """Anchor variant: the target format cycles uniformly over `formats`, one format per step."""
    return itertools.islice(itertools.cycle(formats), steps)


def _torch():
    import torch
    return torch


def mx_linear_class():
    torch = _torch()

    class MxLinear(torch.nn.Linear):
        """A linear layer whose weight goes through the MX quantizer of the current format in the forward
        pass.  `elem` = None runs the layer in full precision; `via_anchor` selects Eq. (7) (quantize to the
        family's 8-bit anchor, then Slice-and-Scale to the target) instead of the direct quantizer.
        Blocks of 32 run along the input (reduction) dimension of the [out, in] weight."""

        def __init__(self, in_features, out_features, bias=True, device=None, dtype=None):
            super().__init__(in_features, out_features, bias=bias, device=device, dtype=dtype)
            self.elem = None
            self.via_anchor = False

        def set_format(self, elem, via_anchor=False):
            self.elem = elem
            self.via_anchor = bool(via_anchor)

        def quantized_weight(self):
            if self.elem is None:
                return self.weight
            anchor = None
            if self.via_anchor and self.elem != anchor_of(self.elem):
                anchor = make_format(anchor_of(self.elem))
            return MxFakeQuantSTE.apply(self.weight, make_format(self.elem), anchor)

        def forward(self, x):
            return torch.nn.functional.linear(x, self.quantized_weight(), self.bias)

    return MxLinear


class _LazyLinear:
    _cls = None

    def __call__(self, *args, **kwargs):
        if _LazyLinear._cls is None:
            _LazyLinear._cls = mx_linear_class()
        return _LazyLinear._cls(*args, **kwargs)


MxLinear = _LazyLinear()


def set_format(model, elem, via_anchor=False):
    """Switch every MxLinear of `model` to one element format (the run-time format selection of Sec. 3.5)."""
    cls = mx_linear_class() if _LazyLinear._cls is None else _LazyLinear._cls
    _LazyLinear._cls = cls
    for m in model.modules():
        if isinstance(m, cls):
            m.set_format(elem, via_anchor)


def train(model, schedule, batches, optimizer, loss_fn, via_anchor=False):
    """One optimizer step per entry of `schedule` (an iterable of element-format names) on the batches
    `batches` yields ((input, target) pairs).  Returns the list of (format, loss) per step."""
    history = []
    for elem, (x, y) in zip(schedule, batches):
        set_format(model, elem, via_anchor)
        optimizer.zero_grad(set_to_none=True)
        loss = loss_fn(model(x), y)
        loss.backward()
        optimizer.step()
        history.append((elem, float(loss.detach())))
    return history
