"""The autograd glue hands autograd exactly what the C-ABI calls return, and a small stack trains."""
import numpy as np
import pytest
import torch

import oracle
from paper_2408_11200_amd import autograd, binding, workloads

pytestmark = pytest.mark.gpu


def dev(a, grad=False):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda().requires_grad_(grad)


def test_kan_stack_gradients_through_autograd_match_oracle():
    """[2,5,1] with the MSE loss: torch chains the two layers, the oracle chains them in fp64."""
    w = workloads.config1()
    S, P = w.layers, w.params
    T = [{n: dev(a, True) for n, a in p.items()} for p in P]
    x = dev(w.x)
    h = autograd.kan_layer(S[0], x, T[0]["coef"], T[0]["w_s"], T[0]["w_b"])
    y = autograd.kan_layer(S[1], h, T[1]["coef"], T[1]["w_s"], T[1]["w_b"])
    loss = ((y - dev(w.target)) ** 2).mean()
    loss.backward()
    ih = [oracle.inv_h_of(s.grid_lo, s.grid_hi, s.G) for s in S]
    hn, yn = h.detach().cpu().numpy(), y.detach().cpu().numpy()
    gy = (2.0 / yn.size) * (yn.astype(np.float64) - w.target)
    r2 = oracle.kan_backward(hn, P[1]["coef"], P[1]["w_s"], P[1]["w_b"], np.float32(gy), 5, 3, -1.0, ih[1])
    r1 = oracle.kan_backward(w.x, P[0]["coef"], P[0]["w_s"], P[0]["w_b"], np.float32(r2["gx"]), 5, 3, -1.0, ih[0])
    for l, r in ((0, r1), (1, r2)):
        for name, key in (("coef", "gcoef"), ("w_s", "gw_s"), ("w_b", "gw_b")):
            got = T[l][name].grad.cpu().numpy().astype(np.float64)
            err = np.abs(got - r[key]) / (1.0 + np.abs(r[key]))
            assert err.max() <= 1e-4, (l, name, err.max())


def test_adam_reduces_the_regression_loss():
    """A few hundred Adam steps on y = sin(pi x0) + x1^2 with the [2,5,1] network."""
    w = workloads.config1()
    S = w.layers
    T = [{n: dev(a, True) for n, a in p.items()} for p in w.params]
    x, target = dev(w.x), dev(w.target)
    opt = torch.optim.Adam([t for layer in T for t in layer.values()], lr=2e-2)
    losses = []
    for _ in range(300):
        opt.zero_grad()
        h = autograd.kan_layer(S[0], x, T[0]["coef"], T[0]["w_s"], T[0]["w_b"])
        y = autograd.kan_layer(S[1], h, T[1]["coef"], T[1]["w_s"], T[1]["w_b"])
        loss = ((y - target) ** 2).mean()
        loss.backward()
        opt.step()
        losses.append(float(loss.detach()))
    assert losses[-1] < 0.05 * losses[0], (losses[0], losses[-1])


def test_ukan_layer_gradients_through_autograd():
    rng = np.random.default_rng(4)
    spec = workloads.UkanLayerSpec(6, 32, 3, 0.25, 8, 8, 16)
    p = workloads.ukan_params(rng, spec)
    x = np.float32(rng.standard_normal((500, 6)) * 2.0)
    gy = np.float32(rng.standard_normal((500, 32)) / np.sqrt(500))
    T = {n: dev(a, True) for n, a in p.items() if n != "w_b"}
    xt = dev(x, True)
    y = autograd.ukan_layer(spec, xt, T, 64)
    y.backward(dev(gy))
    ref = oracle.ukan_backward(x, p, gy, 3, oracle.inv_h_of_spacing(spec.h))
    pairs = [("gx", xt)] + [("g" + n, T[n]) for n in ("E", "W1", "b1", "W2", "b2", "scale")]
    for key, t in pairs:
        got = t.grad.cpu().numpy().astype(np.float64)
        err = np.abs(got - ref[key]) / (1.0 + np.abs(ref[key]))
        assert err.max() <= 1e-4, (key, err.max())
