"""Regression experiments of section "Tasks" (functions I-III) trained on the HIP layers, KAN and UKAN.

A bounded number of Adam steps instead of the section's 200,000: enough to check that (a) the
gradients the training loop receives equal the oracle's, chained through both layers in fp64 from
the fp32 activations the device produced, before the first step and again after the last one (with
the weights training has reached), and (b) the loss falls well below that of the best constant
predictor.  The paper's final errors are not reproduced here (parity unpinned for the figure).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2408_11200_amd import autograd, regression, workloads

pytestmark = pytest.mark.gpu

STEPS = 600


def host(t):
    return t.detach().cpu().numpy()


def close(got, ref, what):
    """|got - ref| <= 2e-4 (|ref| + rms(ref)): relative to the size of the gradient tensor, since the
    gradients of a batch-mean loss are far below the O(1) scale the layer tests' floor assumes."""
    got, ref = host(got).astype(np.float64), np.asarray(ref, dtype=np.float64)
    bound = 2e-4 * (np.abs(ref) + np.sqrt(np.mean(ref ** 2)) + 1e-30)
    err = np.abs(got - ref)
    assert (err <= bound).all(), "%s: worst ratio %.2f" % (what, (err / bound).max())


def check_gradients(net, x, target, model):
    """One forward + backward through autograd; every parameter gradient against the oracle chain."""
    for t in net.tensors():
        t.grad = None
    acts = [x]
    for s, p in zip(net.specs, net.params):
        acts.append(autograd.kan_layer(s, acts[-1], p["coef"], p["w_s"], p["w_b"]) if model == "kan"
                    else autograd.ukan_layer(s, acts[-1], p, regression.UKAN_MAX_GROUPS))
    loss = ((acts[-1] - target) ** 2).mean()
    loss.backward()
    y = host(acts[-1]).astype(np.float64)
    g = np.float32(2.0 / y.size * (y - host(target)))
    for l in (1, 0):
        s = net.specs[l]
        P = {n: host(t) for n, t in net.params[l].items()}
        xin = host(acts[l])
        if model == "kan":
            inv_h = oracle.inv_h_of(s.grid_lo, s.grid_hi, s.G)
            y_ref = oracle.kan_forward(xin, P["coef"], P["w_s"], P["w_b"], s.G, s.k, s.grid_lo, inv_h)
            ref = oracle.kan_backward(xin, P["coef"], P["w_s"], P["w_b"], g, s.G, s.k, s.grid_lo, inv_h)
            names = {"coef": "gcoef", "w_s": "gw_s", "w_b": "gw_b"}
        else:
            inv_h = oracle.inv_h_of_spacing(s.h)
            y_ref = oracle.ukan_forward(xin, P, s.k, inv_h, s.base_act)
            ref = oracle.ukan_backward(xin, P, g, s.k, inv_h, s.base_act)
            names = {n: "g" + n for n in ("E", "W1", "b1", "W2", "b2", "scale", "w_b")}
        got_y = host(acts[l + 1]).astype(np.float64)
        assert (np.abs(got_y - y_ref) <= 1e-5 * (1.0 + np.abs(y_ref))).all(), "layer %d output" % l
        for n, key in names.items():
            close(net.params[l][n].grad, ref[key], "layer %d %s" % (l, key))
        g = np.float32(ref["gx"])
    return float(loss.detach())


@pytest.mark.parametrize("model", ["kan", "ukan"])
@pytest.mark.parametrize("which", ["I", "II", "III"])
def test_regression_training(which, model):
    xh, th = workloads.regression_task(which, B=2048)
    x, target = torch.from_numpy(xh).cuda(), torch.from_numpy(th).cuda()
    net = (regression.KanNet if model == "kan" else regression.UkanNet)(which)
    first = check_gradients(net, x, target, model)
    losses = regression.train(net, x, target, STEPS)
    assert abs(losses[0] - first) <= 1e-5 * (1.0 + first)
    last = check_gradients(net, x, target, model)
    assert abs(losses[-1] - last) <= 1e-5 * (1.0 + last)
    rmse0, rmse = losses[0] ** 0.5, losses[-1] ** 0.5
    assert np.isfinite(losses).all()
    assert rmse < 0.2 * rmse0, (rmse0, rmse)
    assert rmse < 0.8 * float(th.std()), "not better than the constant predictor: %.4f vs std %.4f" % (rmse, th.std())
