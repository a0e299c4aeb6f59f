"""Multi-format QAT plumbing (Sec. 3.2, Sec. 3.5) on a synthetic toy model: the forward weights are what the
oracle's fake-quant gives, gradients pass straight through, training under both schedules lowers the loss,
and the weights the model trains with under anchor storage (Eq. (7)) are bit for bit the weights inference gets
by storing the anchor and running Slice-and-Scale (Sec. 3.5 "Inference")."""
import numpy as np
import pytest


def test_schedules_order_and_length():
    from paper_2604_00529_amd import qat
    seq = list(qat.sequential_schedule(("int8", "int2", "int6", "int4"), steps_per_epoch=3))
    assert seq == ["int2"] * 3 + ["int4"] * 3 + ["int6"] * 3 + ["int8"] * 3          # increasing bit width (Sec. 3.2)
    assert list(qat.sequential_schedule(qat.MXFP_TRAIN_FORMATS, 1, 2)) == ["e2m1", "e2m1", "e3m2", "e3m2", "e4m3", "e4m3"]
    cyc = list(qat.cycling_schedule(("e2m1", "e3m2", "e4m3"), 7))
    assert cyc == ["e2m1", "e3m2", "e4m3", "e2m1", "e3m2", "e4m3", "e2m1"]
    assert qat.anchor_of("int4") == "int8" and qat.anchor_of("e3m2") == "e4m3"


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available()
    import paper_2604_00529_amd as mx
    from paper_2604_00529_amd import qat
    mx.binding.lib()
    return torch, mx, qat


def _toy(torch, qat, seed):
    g = torch.Generator(device="cuda").manual_seed(seed)
    model = torch.nn.Sequential(qat.MxLinear(128, 256, device="cuda"), torch.nn.Tanh(), qat.MxLinear(256, 64, device="cuda"))
    with torch.no_grad():
        for p in model.parameters():
            p.copy_(torch.randn(p.shape, device="cuda", generator=g) * 0.1)
    teacher_a = torch.randn((128, 64), device="cuda", generator=g) * 0.2

    def batches():
        while True:
            x = torch.randn((256, 128), device="cuda", generator=g)
            yield x, torch.tanh(x @ teacher_a)
    return model, batches()


@pytest.mark.gpu
@pytest.mark.parametrize("elem,via_anchor", [("int4", False), ("e2m1", False), ("int4", True), ("e3m2", True), ("e4m3", True)])
def test_forward_weights_and_straight_through(env, oracle, elem, via_anchor):
    torch, mx, qat = env
    model, batches = _toy(torch, qat, 7)
    qat.set_format(model, elem, via_anchor)
    x, y = next(batches)
    loss = torch.nn.functional.mse_loss(model(x), y)
    loss.backward()
    for layer in (model[0], model[2]):
        w = layer.weight.detach()
        anchor = qat.anchor_of(elem) if via_anchor and elem != qat.anchor_of(elem) else None
        want = oracle.fake_quant(w.cpu().numpy(), elem, anchor=anchor)
        got = layer.quantized_weight().detach().cpu().numpy()
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), (elem, via_anchor)
    # straight-through: the weight's gradient is the gradient with respect to the quantized weight
    layer = model[2]
    h = torch.tanh(torch.nn.functional.linear(x, model[0].quantized_weight().detach(), model[0].bias.detach()))
    wq = layer.quantized_weight().detach().clone().requires_grad_(True)
    torch.nn.functional.mse_loss(torch.nn.functional.linear(h, wq, layer.bias.detach()), y).backward()
    assert torch.equal(layer.weight.grad, wq.grad)


@pytest.mark.gpu
@pytest.mark.parametrize("family,via_anchor", [("int", False), ("fp", False), ("int", True), ("fp", True)])
def test_training_lowers_the_loss(env, family, via_anchor):
    torch, mx, qat = env
    model, batches = _toy(torch, qat, 11)
    formats = qat.MXINT_TRAIN_FORMATS[1:] if family == "int" else qat.MXFP_TRAIN_FORMATS
    steps = 40
    if via_anchor:
        schedule = qat.cycling_schedule(formats, steps * len(formats))
    else:
        schedule = qat.sequential_schedule(formats, steps)

    def eval_loss(elem):
        qat.set_format(model, elem, via_anchor)
        g = torch.Generator(device="cuda").manual_seed(99)
        x = torch.randn((1024, 128), device="cuda", generator=g)
        with torch.no_grad():
            return float(torch.nn.functional.mse_loss(model(x), torch.tanh(x @ eval_loss.teacher)))
    # the teacher of _toy(seed 11), rebuilt with the same generator sequence
    g = torch.Generator(device="cuda").manual_seed(11)
    for p in model.parameters():
        torch.randn(p.shape, device="cuda", generator=g)
    eval_loss.teacher = torch.randn((128, 64), device="cuda", generator=g) * 0.2
    before = {e: eval_loss(e) for e in formats}
    opt = torch.optim.AdamW(model.parameters(), lr=3e-3)
    hist = qat.train(model, schedule, batches, opt, torch.nn.functional.mse_loss, via_anchor=via_anchor)
    assert len(hist) == steps * len(formats)
    after = {e: eval_loss(e) for e in formats}
    for e in formats:
        assert after[e] < 0.7 * before[e], (e, before[e], after[e])


@pytest.mark.gpu
@pytest.mark.parametrize("anchor,targets", [("int8", ("int6", "int4", "int2")), ("e4m3", ("e3m2", "e2m3", "e2m1"))])
def test_training_weights_equal_inference_weights(env, anchor, targets):
    # Eq. (7) against Sec. 3.5 "Inference": store Q_A(W) once, Slice-and-Scale it to the target, dequantize
    torch, mx, qat = env
    model, _ = _toy(torch, qat, 13)
    fa = mx.make_format(anchor)
    for layer in (model[0], model[2]):
        w = layer.weight.detach()
        a_codes, a_scales = mx.mx_quantize(w, fa)
        for t in targets:
            ft = mx.make_format(t)
            t_codes, t_scales = mx.mx_slice_and_scale(a_codes, a_scales, fa, ft)
            infer = mx.mx_dequant(t_codes, t_scales, ft, w.shape[0], w.shape[1], dtype=torch.float32)
            layer.set_format(t, via_anchor=True)
            train_w = layer.quantized_weight().detach()
            assert torch.equal(train_w.view(torch.int32), infer.view(torch.int32)), (anchor, t)
