"""The torch.optim front end (paper_2307_02047_amd.CAME) inside a small training loop: the
parameters follow the CPU oracle fed with the same gradients, and checkpoints round-trip."""
import io

import numpy as np
import pytest
import torch

import paper_2307_02047_amd as P
from oracle import came_oracle as O
from parity_util import rel_err_signed, to_f64

pytestmark = pytest.mark.gpu


def make_model(seed):
    torch.manual_seed(seed)
    m = torch.nn.Sequential(torch.nn.Linear(96, 520), torch.nn.GELU(), torch.nn.Linear(520, 40)).to("cuda:0")
    return m


def batch(step):
    g = torch.Generator(device="cuda:0").manual_seed(1000 + step)
    x = torch.randn(64, 96, device="cuda:0", generator=g)
    y = torch.randn(64, 40, device="cuda:0", generator=g)
    return x, y


def test_training_loop_follows_the_oracle():
    model = make_model(1)
    params = list(model.parameters())
    opt = P.CAME(params, lr=1e-3, weight_decay=0.01)
    shapes = [tuple(p.shape) for p in params]
    otl = O.TensorList(shapes, [to_f64(p) for p in params])
    oh = O.Hyper(lr=1e-3)
    for t in range(1, 16):
        x, y = batch(t)
        opt.zero_grad(set_to_none=True)
        loss = torch.nn.functional.mse_loss(model(x), y)
        loss.backward()
        grads = [to_f64(p.grad) for p in params]
        opt.step()
        otl.step(grads, oh, weight_decay=0.01)
    torch.cuda.synchronize()
    for p, ref in zip(params, otl.theta):
        assert rel_err_signed(to_f64(p), ref) <= 1e-4
    st = opt.state[params[0]]
    assert st["step"] == 15 and st["M"].shape == params[0].shape and st["R"].shape == (520,)
    assert set(opt.state[params[1]]) == {"step", "M", "v", "s"}
    np.testing.assert_allclose(to_f64(st["R"]), otl.state[0].R, rtol=1e-4)
    opt.close()


def test_it_learns_a_fixed_batch():
    model = make_model(4)
    opt = P.CAME(model.parameters(), lr=2e-3, place_state=True)
    x, y = batch(0)
    losses = []
    for _ in range(60):
        opt.zero_grad()
        loss = torch.nn.functional.mse_loss(model(x), y)
        loss.backward()
        opt.step()
        losses.append(loss.item())
    assert losses[-1] < 0.5 * losses[0], losses[::10]
    opt.close()


def test_checkpoint_round_trip_through_state_dict():
    def run(steps_a, steps_b, reload):
        model = make_model(2)
        opt = P.CAME(model.parameters(), lr=1e-3, momentum_dtype="bf16")
        t = 0
        for _ in range(steps_a):
            t += 1
            x, y = batch(t)
            opt.zero_grad()
            torch.nn.functional.mse_loss(model(x), y).backward()
            opt.step()
        if reload:
            buf = io.BytesIO()
            torch.save({"model": model.state_dict(), "opt": opt.state_dict()}, buf)
            opt.close()
            buf.seek(0)
            ck = torch.load(buf, weights_only=True)
            model = make_model(99)
            model.load_state_dict(ck["model"])
            opt = P.CAME(model.parameters(), lr=1e-3, momentum_dtype="bf16")
            opt.load_state_dict(ck["opt"])
        for _ in range(steps_b):
            t += 1
            x, y = batch(t)
            opt.zero_grad()
            torch.nn.functional.mse_loss(model(x), y).backward()
            opt.step()
        torch.cuda.synchronize()
        out = [p.detach().clone() for p in model.parameters()]
        steps = [opt.state[p]["step"] for p in model.parameters()]
        opt.close()
        return out, steps

    a, sa = run(4, 3, reload=False)
    b, sb = run(4, 3, reload=True)
    assert sa == sb == [7] * 4
    for x, y in zip(a, b):
        assert torch.equal(x, y)


def test_parameter_groups_and_bfloat16_gradients():
    model = make_model(3)
    w = [p for p in model.parameters() if p.dim() == 2]
    b = [p for p in model.parameters() if p.dim() == 1]
    opt = P.CAME([{"params": w, "lr": 2e-3}, {"params": b, "lr": 5e-4, "vector_confidence": False}])
    otw = O.TensorList([tuple(p.shape) for p in w], [to_f64(p) for p in w])
    otb = O.TensorList([tuple(p.shape) for p in b], [to_f64(p) for p in b])
    for t in range(1, 6):
        x, y = batch(t)
        opt.zero_grad()
        torch.nn.functional.mse_loss(model(x), y).backward()
        gw = [p.grad.to(torch.bfloat16) for p in w]   # a bf16 compute copy's gradients, fp32 master parameters
        gb = [p.grad.to(torch.bfloat16) for p in b]
        opt.step(grads=[gw, gb])
        otw.step([to_f64(g) for g in gw], O.Hyper(lr=2e-3))
        otb.step([to_f64(g) for g in gb], O.Hyper(lr=5e-4), vector_confidence=False)
    torch.cuda.synchronize()
    for p, ref in zip(w + b, otw.theta + otb.theta):
        assert rel_err_signed(to_f64(p), ref) <= 1e-4
    with pytest.raises(RuntimeError):
        model[0].weight.grad = None
        opt.step()
    opt.close()
