"""torch.autograd glue around the C-ABI entry points.

Nothing is computed here: `forward` calls kan_forward / ukan_cg_forward_saved, `backward` calls
kan_backward_saved / ukan_cg_backward_saved with exactly the gradients autograd asks for (the
backward passes reuse what their forward passes kept: the scale-folded table; for UKAN the
coefficient table and the CG activations).  Lets a stack of
layers be trained with a stock PyTorch optimizer (closed-form regression targets of the paper's
experiments section need nothing else).
"""
import torch

from . import binding

_UKAN_NAMES = ("E", "W1", "b1", "W2", "b2", "scale")


class _KanLayer(torch.autograd.Function):
    @staticmethod
    def forward(ctx, spec, x, coef, w_s, w_b):
        ctx.spec = spec
        # the forward pass's workspace (the scale-folded table) is handed to the backward pass
        ws = torch.empty(max(binding.kan_workspace_bytes(spec, x.shape[0], binding.PASS_FORWARD), 256), dtype=torch.uint8,
                         device=x.device)
        ctx.save_for_backward(x, coef, w_s, w_b, ws)
        return binding.kan_forward(spec, x.contiguous(), coef.contiguous(), w_s.contiguous(),
                                   None if w_b is None else w_b.contiguous(), ws=ws)

    @staticmethod
    def backward(ctx, gy):
        x, coef, w_s, w_b, ws = ctx.saved_tensors
        names = ("gx", "gcoef", "gw_s", "gw_b")
        need = ctx.needs_input_grad[1:5]
        want = tuple(n for n, k in zip(names, need) if k and not (n == "gw_b" and w_b is None))
        g = binding.kan_backward_saved(ctx.spec, x.contiguous(), coef.contiguous(), w_s.contiguous(),
                                       None if w_b is None else w_b.contiguous(), gy.contiguous(), ws, want=want) if want else {}
        return (None,) + tuple(g.get(n) for n in names)


class _UkanLayer(torch.autograd.Function):
    @staticmethod
    def forward(ctx, spec, max_groups, x, E, W1, b1, W2, b2, scale, w_b):
        ctx.spec, ctx.max_groups = spec, max_groups
        p = dict(zip(_UKAN_NAMES, (E, W1, b1, W2, b2, scale)))
        if w_b is not None:
            p["w_b"] = w_b
        y, saved, ctx.span = binding.ukan_cg_forward_saved(spec, x.contiguous(), p, max_groups)
        ctx.save_for_backward(x, E, W1, b1, W2, b2, scale, w_b, saved)
        return y

    @staticmethod
    def backward(ctx, gy):
        x, E, W1, b1, W2, b2, scale, w_b, saved = ctx.saved_tensors
        p = dict(zip(_UKAN_NAMES, (E, W1, b1, W2, b2, scale)))
        if w_b is not None:
            p["w_b"] = w_b
        names = ("gx", "gE", "gW1", "gb1", "gW2", "gb2", "gscale", "gw_b")
        need = ctx.needs_input_grad[2:10]
        want = [n for n, k in zip(names, need) if k and not (n == "gw_b" and w_b is None)]
        g = binding.ukan_cg_backward_saved(ctx.spec, x.contiguous(), p, gy.contiguous(), ctx.max_groups, saved,
                                           ctx.span, want=want) if want else {}
        return (None, None) + tuple(g.get(n) for n in names)


def kan_layer(spec, x, coef, w_s, w_b=None):
    """y = KAN layer `spec` applied to x; differentiable in x, coef, w_s, w_b."""
    return _KanLayer.apply(spec, x, coef, w_s, w_b)


def ukan_layer(spec, x, params, max_groups):
    """y = UKAN layer `spec` applied to x; `params` maps E, W1, b1, W2, b2, scale (and w_b) to tensors."""
    return _UkanLayer.apply(spec, max_groups, x, *(params[n] for n in _UKAN_NAMES), params.get("w_b"))
