"""kan_forward_static (the forward pass on the library's built-in scratch array, for callers that cannot
allocate) against kan_forward, through the C ABI.  Same kernels, same arithmetic: outputs must be bit-identical,
on two calls in a row, the second on a smaller layer and batch (the array keeps the first call's contents)."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2408_11200_amd import binding, workloads

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def both_ways(seed, B, n_in, n_out, G, k):
    w = workloads.random_kan_layer(seed, B, n_in, n_out, G, k, outside_frac=0.1)
    s, p = w.layers[0], w.params[0]
    x, coef, w_s, w_b = (dev(a) for a in (w.x, p["coef"], p["w_s"], p["w_b"]))
    y_ref = binding.kan_forward(s, x, coef, w_s, w_b)
    y = torch.full((B, n_out), float("nan"), dtype=torch.float32, device="cuda")
    lib = binding.load()
    d = binding.kan_desc(s)
    rc = lib.kan_forward_static(ctypes.byref(d), B, x.data_ptr(), coef.data_ptr(), w_s.data_ptr(), w_b.data_ptr(),
                                y.data_ptr(), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == binding.KAN_OK, binding.strerror(rc)
    torch.cuda.synchronize()
    assert torch.equal(y, y_ref), "max diff %g" % (y - y_ref).abs().max().item()
    return s


def test_static_scratch_forward_matches_kan_forward_twice():
    assert binding.kan_static_scratch_bytes() == 32 << 20
    # first call: a table of 9.7 MB (LDS-staged kernel); second: smaller layer and batch (row-stream kernel)
    both_ways(11, 1500, 200, 512, 20, 3)
    both_ways(12, 333, 24, 48, 6, 3)
    # and a third on the generic path with a ragged shape
    both_ways(13, 77, 5, 7, 100, 2)


def test_static_scratch_rejects_oversized_layer():
    lib = binding.load()
    big = binding.KanLayerDesc(1024, 1024, 20, 3, -1.0, 1.0, 1)          # table of 100 MB
    assert lib.kan_workspace_bytes(ctypes.byref(big), 64, binding.PASS_FORWARD) > binding.kan_static_scratch_bytes()
    x = torch.zeros((64, 1024), dtype=torch.float32, device="cuda")
    y = torch.full((64, 1024), 7.0, dtype=torch.float32, device="cuda")
    coef = torch.zeros((1024, 23, 1024), dtype=torch.float32, device="cuda")
    w = torch.zeros((1024, 1024), dtype=torch.float32, device="cuda")
    rc = lib.kan_forward_static(ctypes.byref(big), 64, x.data_ptr(), coef.data_ptr(), w.data_ptr(), w.data_ptr(),
                                y.data_ptr(), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == binding.KAN_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((y == 7.0).all())
