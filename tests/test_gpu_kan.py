"""Parity of the HIP KAN layer (through the C ABI) with the CPU oracle on the same seeded inputs.

Bars: interval indices bit-exact; forward |err| <= 1e-5 (1 + |ref|); gradients
|err| <= 1e-4 (1 + |ref|), all in fp32 against the fp64 oracle.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2408_11200_amd import binding, workloads

pytestmark = pytest.mark.gpu

FWD_TOL = 1e-5
GRAD_TOL = 1e-4


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def assert_close(got, ref, tol, what):
    got = got.detach().cpu().numpy().astype(np.float64)
    err = np.abs(got - ref)
    bound = tol * (1.0 + np.abs(ref))
    bad = err > bound
    assert not bad.any(), "%s: %d/%d outside tolerance, worst err %.3e at ref %.3e (ratio %.2f)" % (
        what, bad.sum(), bad.size, err.max(), ref.flat[err.argmax()], (err / bound).max())
    return float((err / bound).max())


def run_layer_parity(w, rows=None, check_grads=True, gx_in_grid_units=False):
    """gx_in_grid_units: compare h * dL/dx (the gradient with respect to the position in cell widths)
    instead of dL/dx.  dL/dx = (1/h) dL/du: on a grid with 1/h in the tens of thousands it is a sum of
    terms that large, whose fp32 rounding error is relative to them, while the tolerance's absolute part
    is meant for O(1) results; in grid units the terms are O(1) again."""
    s, p = w.layers[0], w.params[0]
    inv_h = oracle.inv_h_of(s.grid_lo, s.grid_hi, s.G)
    x, coef, w_s, w_b, gy = (dev(a) for a in (w.x, p["coef"], p["w_s"], p["w_b"], w.gy))
    # interval index: bit-exact
    idx = binding.kan_interval_index(s, x).cpu().numpy()
    np.testing.assert_array_equal(idx, oracle.interval_index(w.x, s.grid_lo, inv_h))
    y = binding.kan_forward(s, x, coef, w_s, w_b)
    g = binding.kan_backward(s, x, coef, w_s, w_b, gy) if check_grads else None
    torch.cuda.synchronize()
    sel = slice(None) if rows is None else rows
    y_ref = oracle.kan_forward(w.x[sel], p["coef"], p["w_s"], p["w_b"], s.G, s.k, s.grid_lo, inv_h, s.base_act)
    assert_close(y[sel], y_ref, FWD_TOL, "y")
    if check_grads:
        if rows is None:
            ref = oracle.kan_backward(w.x, p["coef"], p["w_s"], p["w_b"], w.gy, s.G, s.k, s.grid_lo, inv_h,
                                      s.base_act)
            for name in ("gx", "gcoef", "gw_s", "gw_b"):
                unit = 1.0 / float(inv_h) if (name == "gx" and gx_in_grid_units) else 1.0
                assert_close(g[name].double() * unit, ref[name] * unit, GRAD_TOL, name)
        else:
            ref = oracle.kan_backward(w.x[sel], p["coef"], p["w_s"], p["w_b"], w.gy[sel], s.G, s.k, s.grid_lo,
                                      inv_h, s.base_act, want=("gx",))
            assert_close(g["gx"][sel], ref["gx"], GRAD_TOL, "gx")
    return y, g


SWEEP = [
    # B, n_in, n_out, G, k, outside
    (1, 1, 1, 1, 1, 0.0),
    (7, 2, 5, 5, 3, 0.3),
    (1024, 5, 1, 5, 3, 0.1),
    (333, 3, 64, 4, 2, 0.2),
    (257, 17, 130, 9, 3, 0.25),        # ragged in every dimension, n_out even -> 2 outputs per lane
    (130, 70, 260, 10, 3, 0.1),        # 4 outputs per lane with a ragged last tile
    (96, 33, 512, 20, 3, 0.05),
    (200, 8, 256, 64, 1, 0.2),
    (65, 4, 7, 200, 3, 0.2),           # large grid, odd n_out
    (700, 5, 32, 300, 3, 0.1),         # three ragged chunks, two sort digits, four streams per wave
    (2100, 3, 132, 40, 2, 0.2),        # one stream per wave with a ragged output tile
    (900, 6, 96, 7, 3, 0.3),           # two streams per wave
    (300, 9, 12, 30, 3, 0.1),          # narrow layer, one output per lane
    (700, 5, 32, 3000, 3, 0.1),        # far more rows than samples: pre-zeroed partial slabs, gap jumps
    (1500, 3, 256, 2500, 2, 0.05),     # the same with one stream per wave
    (400, 6, 18, 12, 3, 0.2),          # two outputs per lane in the walk, ragged stream (18 of 32 lanes' outputs)
    (1300, 3, 30, 25, 2, 0.1),         # the same, 30 outputs
    (64, 2, 8, 70000, 3, 0.1),         # 17-bit row numbers in the sorted records (three sort digits)
    (64, 2, 8, 600000, 3, 0.1),        # more rows than the sorted path indexes (2^19): generic kernels
]


@pytest.mark.parametrize("B,n_in,n_out,G,k,outside", SWEEP)
def test_layer_parity_sweep(B, n_in, n_out, G, k, outside):
    w = workloads.random_kan_layer(100 + B + n_in + n_out, B, n_in, n_out, G, k, outside_frac=outside)
    run_layer_parity(w)


@pytest.mark.parametrize("B,n_in,n_out,G,k,outside", [
    (300, 7, 96, 9, 4, 0.2), (513, 5, 33, 12, 5, 0.25), (64, 3, 256, 40, 5, 0.1), (1000, 4, 8, 6, 4, 0.3),
    (96, 33, 512, 20, 5, 0.05), (200, 8, 256, 12, 4, 0.2), (300, 20, 128, 8, 5, 0.1),     # six-row LDS-staged forward
    (130, 7, 260, 10, 4, 0.1),                                                           # ... with a ragged last tile
])
def test_layer_parity_degrees_four_and_five(B, n_in, n_out, G, k, outside):
    """Degrees 4 and 5 (window of 5 and 6 rows)."""
    w = workloads.random_kan_layer(4000 + B, B, n_in, n_out, G, k, outside_frac=outside)
    run_layer_parity(w)


@pytest.mark.parametrize("B,n_in,n_out,G,k,outside", [
    (2100, 3, 132, 40, 4, 0.2),        # one stream per wave, ragged output tile, three ragged chunks
    (900, 6, 96, 7, 5, 0.3),           # two streams per wave
    (300, 9, 12, 30, 4, 0.1),          # four streams per wave
    (300, 9, 10, 30, 5, 0.1),          # narrow layer, one output per lane
    (130, 4, 520, 10, 5, 0.1),         # eight outputs per lane, two output tiles: four partial dL/dx
    (700, 5, 32, 3000, 4, 0.1),        # far more rows than samples: pre-zeroed partial tables, gap jumps
    (9000, 2, 64, 1, 5, 0.5),          # six rows in all: every window is clamped; two chunks of 4096 + a ragged one
    (64, 2, 8, 1, 4, 0.3),             # five rows: fewer than a six-row window, generic kernels
    (9000, 9, 132, 1, 4, 0.3),         # the same with chunks of a thousand samples in one cell (two-level base sums)
])
def test_high_degree_backward_as_two_records_per_pair(B, n_in, n_out, G, k, outside):
    """Degrees 4 and 5 on the sorted walk: each pair's six-row window is walked as two four-row records
    (rows 0..3 with the base term, rows 4..5); dL/dx is the sum of the two partial results.  Also
    bit-reproducible."""
    w = workloads.random_kan_layer(4200 + B + k, B, n_in, n_out, G, k, outside_frac=outside)
    run_layer_parity(w)
    s, p = w.layers[0], w.params[0]
    x, coef, w_s, w_b, gy = (dev(a) for a in (w.x, p["coef"], p["w_s"], p["w_b"], w.gy))
    a = binding.kan_backward(s, x, coef, w_s, w_b, gy)
    b = binding.kan_backward(s, x, coef, w_s, w_b, gy, want=("gx",))
    c = binding.kan_backward(s, x, coef, w_s, w_b, gy, want=("gcoef", "gw_b"))
    assert torch.equal(a["gx"], b["gx"])
    assert torch.equal(a["gcoef"], c["gcoef"]) and torch.equal(a["gw_b"], c["gw_b"])


def test_half_gigabyte_table_wide_layer():
    """A 16003-row table for 16 -> 512: the partial-sum budget forces chunks longer than 1024 samples,
    i.e. the eight-outputs-per-lane walk with two-level sums, pre-zeroed slabs and gap jumps.  The grid
    spans [-2000, 2000) so that the cell width (and with it the scale of dL/dx) stays O(1)."""
    s = workloads.KanLayerSpec(16, 512, 16000, 3, -2000.0, 2000.0, base_act=0)   # silu(x) ~ 2000 would swamp fp32
    rng = np.random.default_rng(77)
    p = workloads.kan_params(rng, s, 0.1, w_s_std=0.3, w_b_std=0.3)
    B = 4096
    x = np.float32(rng.uniform(-2100.0, 2100.0, size=(B, 16)))
    gy = np.float32(rng.standard_normal((B, 512)) / np.sqrt(B))
    inv_h = oracle.inv_h_of(s.grid_lo, s.grid_hi, s.G)
    xd, coef, w_s = dev(x), dev(p["coef"]), dev(p["w_s"])
    y = binding.kan_forward(s, xd, coef, w_s, None)
    g = binding.kan_backward(s, xd, coef, w_s, None, dev(gy), want=("gx", "gcoef", "gw_s"))
    assert_close(y, oracle.kan_forward(x, p["coef"], p["w_s"], p["w_b"], s.G, s.k, s.grid_lo, inv_h, base_act=0),
                 FWD_TOL, "y")
    ref = oracle.kan_backward(x, p["coef"], p["w_s"], p["w_b"], gy, s.G, s.k, s.grid_lo, inv_h, base_act=0)
    for name in ("gx", "gcoef", "gw_s"):
        assert_close(g[name], ref[name], GRAD_TOL, name)


@pytest.mark.parametrize("B", [6000, 70000])
def test_long_run_in_one_cell(B):
    """Every sample of an input in the same cell: the longest possible run for the window sums (B = 6000: chunks of
    512 samples, single-level sums; B = 70000: chunks of 8192, two-level sums)."""
    s = workloads.KanLayerSpec(2, 64, 6, 3, -1.0, 1.0)
    rng = np.random.default_rng(11)
    p = workloads.kan_params(rng, s, 0.1, w_s_std=1.0, w_b_std=1.0)
    x = np.float32(np.stack([0.05 + 0.2 * rng.random(B), np.full(B, -0.4)], axis=1))
    gy = np.float32(rng.standard_normal((B, 64)) * (80.0 / np.sqrt(B)))
    inv_h = oracle.inv_h_of(-1.0, 1.0, 6)
    g = binding.kan_backward(s, dev(x), dev(p["coef"]), dev(p["w_s"]), dev(p["w_b"]), dev(gy))
    ref = oracle.kan_backward(x, p["coef"], p["w_s"], p["w_b"], gy, 6, 3, -1.0, inv_h)
    for name in ref:
        assert_close(g[name], ref[name], GRAD_TOL, name)


def _random_shapes(n, seed):
    rng = np.random.default_rng(seed)
    outs = [1, 3, 8, 16, 20, 32, 48, 64, 100, 128, 200, 256, 260, 512, 520]
    shapes = []
    for _ in range(n):
        shapes.append((int(rng.integers(1, 3000)), int(rng.integers(1, 40)), int(rng.choice(outs)),
                       int(rng.integers(1, 400)), int(rng.integers(1, 4)), float(rng.choice([0.0, 0.1, 0.3]))))
    return shapes


@pytest.mark.parametrize("B,n_in,n_out,G,k,outside", _random_shapes(24, 2024))
def test_layer_parity_random_shapes(B, n_in, n_out, G, k, outside):
    """Seeded random shapes across every dispatch path (narrow, row-stream, LDS-staged, generic, walk variants)."""
    w = workloads.random_kan_layer(7000 + B, B, n_in, n_out, G, k, outside_frac=outside)
    run_layer_parity(w)


@pytest.mark.parametrize("want", [("gx",), ("gcoef",), ("gw_b",), ("gx", "gw_s")])
def test_gradient_subsets(want):
    """Any subset of the gradient outputs may be requested; what is returned does not depend on the rest."""
    w = workloads.random_kan_layer(21, 900, 6, 96, 40, 3, outside_frac=0.2)
    s, p = w.layers[0], w.params[0]
    inv_h = oracle.inv_h_of(s.grid_lo, s.grid_hi, s.G)
    g = binding.kan_backward(s, dev(w.x), dev(p["coef"]), dev(p["w_s"]), dev(p["w_b"]), dev(w.gy), want=want)
    assert set(g) == set(want)
    ref = oracle.kan_backward(w.x, p["coef"], p["w_s"], p["w_b"], w.gy, s.G, s.k, s.grid_lo, inv_h)
    for name in want:
        assert_close(g[name], ref[name], GRAD_TOL, name)


def test_no_base_term():
    w = workloads.random_kan_layer(5, 100, 6, 64, 8, 3, base_act=0, outside_frac=0.3)
    s, p = w.layers[0], w.params[0]
    x, coef, w_s, gy = (dev(a) for a in (w.x, p["coef"], p["w_s"], w.gy))
    inv_h = oracle.inv_h_of(s.grid_lo, s.grid_hi, s.G)
    y = binding.kan_forward(s, x, coef, w_s, None)
    g = binding.kan_backward(s, x, coef, w_s, None, gy, want=("gx", "gcoef", "gw_s"))
    y_ref = oracle.kan_forward(w.x, p["coef"], p["w_s"], p["w_b"], s.G, s.k, s.grid_lo, inv_h, base_act=0)
    ref = oracle.kan_backward(w.x, p["coef"], p["w_s"], p["w_b"], w.gy, s.G, s.k, s.grid_lo, inv_h, base_act=0)
    assert_close(y, y_ref, FWD_TOL, "y")
    for name in ("gx", "gcoef", "gw_s"):
        assert_close(g[name], ref[name], GRAD_TOL, name)


def test_degenerate_inputs():
    """All samples far outside the grid (base only), exactly on knots, and non-finite x."""
    s = workloads.KanLayerSpec(3, 64, 5, 3, -1.0, 1.0)
    rng = np.random.default_rng(3)
    p = workloads.kan_params(rng, s, 0.1, w_s_std=1.0, w_b_std=1.0)
    inv_h = oracle.inv_h_of(-1.0, 1.0, 5)
    knots = np.float32(-1.0 + 0.4 * (np.arange(-4, 11)))
    x = np.float32(np.stack([np.full(15, 50.0), knots, -knots], axis=1))
    gy = np.float32(rng.standard_normal((15, 64)))
    xd, coef, w_s, w_b, gyd = (dev(a) for a in (x, p["coef"], p["w_s"], p["w_b"], gy))
    y = binding.kan_forward(s, xd, coef, w_s, w_b)
    g = binding.kan_backward(s, xd, coef, w_s, w_b, gyd)
    assert_close(y, oracle.kan_forward(x, p["coef"], p["w_s"], p["w_b"], 5, 3, -1.0, inv_h), FWD_TOL, "y")
    ref = oracle.kan_backward(x, p["coef"], p["w_s"], p["w_b"], gy, 5, 3, -1.0, inv_h)
    for name in ref:
        assert_close(g[name], ref[name], GRAD_TOL, name)
    # the first input never touches the spline: its coefficient gradient is exactly zero
    assert (g["gcoef"][0] == 0).all() and (g["gw_s"][0] == 0).all()
    np.testing.assert_array_equal(binding.kan_interval_index(s, xd).cpu().numpy(),
                                  oracle.interval_index(x, -1.0, inv_h))
    # non-finite x: spline term dropped, index saturates like the definition
    bad = np.float32([[np.inf, -np.inf, np.nan]])
    np.testing.assert_array_equal(binding.kan_interval_index(s, dev(bad)).cpu().numpy(),
                                  oracle.interval_index(bad, -1.0, inv_h))


def test_empty_batch_and_argument_errors():
    s = workloads.KanLayerSpec(4, 8, 5, 3, -1.0, 1.0)
    rng = np.random.default_rng(1)
    p = {n: dev(a) for n, a in workloads.kan_params(rng, s, 0.1, w_s_std=1.0, w_b_std=1.0).items()}
    x0 = torch.empty((0, 4), device="cuda")
    y = binding.kan_forward(s, x0, p["coef"], p["w_s"], p["w_b"])
    assert y.shape == (0, 8)
    x = torch.zeros((3, 4), device="cuda")
    lib = binding.load()
    import ctypes
    d = binding.kan_desc(s)
    ws = torch.empty(binding.kan_workspace_bytes(s, 3), dtype=torch.uint8, device="cuda")
    yv = torch.empty((3, 8), device="cuda")
    ok = lambda: lib.kan_forward(ctypes.byref(d), 3, x.data_ptr(), p["coef"].data_ptr(), p["w_s"].data_ptr(),
                                 p["w_b"].data_ptr(), yv.data_ptr(), ws.data_ptr(), ws.numel(), None)
    assert ok() == binding.KAN_OK
    assert lib.kan_forward(ctypes.byref(d), 3, None, p["coef"].data_ptr(), p["w_s"].data_ptr(), p["w_b"].data_ptr(),
                           yv.data_ptr(), ws.data_ptr(), ws.numel(), None) == binding.KAN_ERR_INVALID_ARG
    assert lib.kan_forward(ctypes.byref(d), 3, x.data_ptr(), p["coef"].data_ptr(), p["w_s"].data_ptr(),
                           p["w_b"].data_ptr(), yv.data_ptr(), ws.data_ptr(), 16, None) == binding.KAN_ERR_WORKSPACE
    assert lib.kan_forward(ctypes.byref(d), 3, x.data_ptr(), p["coef"].data_ptr(), p["w_s"].data_ptr(),
                           p["w_b"].data_ptr(), yv.data_ptr(), None, 0, None) == binding.KAN_ERR_WORKSPACE
    for bad in (dict(k=0), dict(k=6), dict(base_act=7)):
        d2 = binding.kan_desc(s)
        for n, v in bad.items():
            setattr(d2, n, v)
        assert lib.kan_workspace_bytes(ctypes.byref(d2), 3, 0) == 0
        assert lib.kan_forward(ctypes.byref(d2), 3, x.data_ptr(), p["coef"].data_ptr(), p["w_s"].data_ptr(),
                               p["w_b"].data_ptr(), yv.data_ptr(), ws.data_ptr(), ws.numel(),
                               None) == binding.KAN_ERR_UNSUPPORTED
    # a pointer that is not 16-byte aligned is refused
    assert lib.kan_forward(ctypes.byref(d), 3, x.data_ptr() + 4, p["coef"].data_ptr(), p["w_s"].data_ptr(),
                           p["w_b"].data_ptr(), yv.data_ptr(), ws.data_ptr(), ws.numel(),
                           None) == binding.KAN_ERR_INVALID_ARG
    d3 = binding.kan_desc(s)
    d3.grid_hi = -1.0
    assert lib.kan_forward(ctypes.byref(d3), 3, x.data_ptr(), p["coef"].data_ptr(), p["w_s"].data_ptr(),
                           p["w_b"].data_ptr(), yv.data_ptr(), ws.data_ptr(), ws.numel(),
                           None) == binding.KAN_ERR_INVALID_ARG
    torch.cuda.synchronize()


def test_backward_is_bit_reproducible_and_partial_outputs():
    w = workloads.random_kan_layer(77, 3000, 24, 128, 12, 3, outside_frac=0.1)
    s, p = w.layers[0], w.params[0]
    x, coef, w_s, w_b, gy = (dev(a) for a in (w.x, p["coef"], p["w_s"], p["w_b"], w.gy))
    a = binding.kan_backward(s, x, coef, w_s, w_b, gy)
    b = binding.kan_backward(s, x, coef, w_s, w_b, gy)
    for name in a:
        assert torch.equal(a[name], b[name]), name
    only = binding.kan_backward(s, x, coef, w_s, w_b, gy, want=("gcoef",))
    assert set(only) == {"gcoef"} and torch.equal(only["gcoef"], a["gcoef"])
    only = binding.kan_backward(s, x, coef, w_s, w_b, gy, want=("gx", "gw_b"))
    assert torch.equal(only["gx"], a["gx"]) and torch.equal(only["gw_b"], a["gw_b"])


def test_config1_two_layer_chain_with_mse():
    """Tiny KAN [2,5,1], batch 1024, MSE against sin(pi x0) + x1^2: forward and the chained backward."""
    w = workloads.config1()
    S, P = w.layers, w.params
    ih = [oracle.inv_h_of(s.grid_lo, s.grid_hi, s.G) for s in S]
    Pd = [{n: dev(a) for n, a in p.items()} for p in P]
    x = dev(w.x)
    h1 = binding.kan_forward(S[0], x, Pd[0]["coef"], Pd[0]["w_s"], Pd[0]["w_b"])
    y = binding.kan_forward(S[1], h1, Pd[1]["coef"], Pd[1]["w_s"], Pd[1]["w_b"])
    gy = (2.0 / w.B) * (y - dev(w.target))          # host-side loss glue, not part of the layer
    g2 = binding.kan_backward(S[1], h1, Pd[1]["coef"], Pd[1]["w_s"], Pd[1]["w_b"], gy)
    g1 = binding.kan_backward(S[0], x, Pd[0]["coef"], Pd[0]["w_s"], Pd[0]["w_b"], g2["gx"])
    # oracle chain in fp64, fed the fp32 activations the device produced at each layer boundary
    h1n = h1.cpu().numpy()
    h1_ref = oracle.kan_forward(w.x, P[0]["coef"], P[0]["w_s"], P[0]["w_b"], 5, 3, -1.0, ih[0])
    assert_close(h1, h1_ref, FWD_TOL, "h1")
    y_ref = oracle.kan_forward(h1n, P[1]["coef"], P[1]["w_s"], P[1]["w_b"], 5, 3, -1.0, ih[1])
    assert_close(y, y_ref, FWD_TOL, "y")
    gyn = gy.cpu().numpy()
    r2 = oracle.kan_backward(h1n, P[1]["coef"], P[1]["w_s"], P[1]["w_b"], gyn, 5, 3, -1.0, ih[1])
    for name in r2:
        assert_close(g2[name], r2[name], GRAD_TOL, "layer2 " + name)
    r1 = oracle.kan_backward(w.x, P[0]["coef"], P[0]["w_s"], P[0]["w_b"], g2["gx"].cpu().numpy(), 5, 3, -1.0, ih[0])
    for name in r1:
        assert_close(g1[name], r1[name], GRAD_TOL, "layer1 " + name)


def test_step_captured_in_a_graph_replays_to_the_eager_result():
    """Forward + backward of the two config-1 layers and of a walk-path layer captured in one HIP graph (the
    calls only enqueue kernels: no allocation, no memset node, no synchronisation).  Every replay must give
    the eager result bit for bit, with eager work and synchronisations between the replays and with the
    inputs changed in place before the last one."""
    w = workloads.random_kan_layer(31, 3000, 24, 128, 12, 3, outside_frac=0.1)
    s, p = w.layers[0], w.params[0]
    x, coef, w_s, w_b, gy = (dev(a) for a in (w.x, p["coef"], p["w_s"], p["w_b"], w.gy))
    y = torch.empty((w.B, s.n_out), device="cuda")
    out = {"gx": torch.empty_like(x), "gcoef": torch.empty_like(coef), "gw_s": torch.empty_like(w_s),
           "gw_b": torch.empty_like(w_b)}
    ws_f = torch.empty(binding.kan_workspace_bytes(s, w.B, binding.PASS_FORWARD), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(binding.kan_workspace_bytes(s, w.B, binding.PASS_BACKWARD), dtype=torch.uint8, device="cuda")

    def step():
        binding.kan_forward(s, x, coef, w_s, w_b, y=y, ws=ws_f)
        binding.kan_backward(s, x, coef, w_s, w_b, gy, out=out, ws=ws_b)

    def snapshot():
        torch.cuda.synchronize()
        return [y.clone()] + [out[n].clone() for n in sorted(out)]

    step()                              # eager warm-up (sets the kernels' LDS limits) and reference
    ref = snapshot()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for _ in range(3):
        y.zero_()
        for t in out.values():
            t.fill_(7.0)
        ws_b.fill_(0x5A)                # scratch contents must not matter
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        for a, b in zip(got, ref):
            assert torch.equal(a, b)
        binding.kan_forward(s, x, coef, w_s, w_b)       # unrelated eager work between replays
    x.mul_(0.5)
    gy.neg_()
    step()
    ref2 = snapshot()
    graph.replay()
    for a, b in zip(snapshot(), ref2):
        assert torch.equal(a, b)
    assert not torch.equal(ref2[0], ref[0])


@pytest.mark.parametrize("B,n_in,n_out,G,k", [(3000, 24, 128, 12, 3), (500, 5, 8, 30, 3), (900, 6, 33, 9, 2), (700, 4, 64, 10, 5)])
def test_backward_on_the_forward_pass_table(B, n_in, n_out, G, k):
    """kan_backward_saved reads the scale-folded table the forward pass left in its workspace: bit for bit the
    gradients of kan_backward (walk, narrow, generic and degree-5 paths)."""
    w = workloads.random_kan_layer(61 + B, B, n_in, n_out, G, k, outside_frac=0.1)
    s, p = w.layers[0], w.params[0]
    x, coef, w_s, w_b, gy = (dev(a) for a in (w.x, p["coef"], p["w_s"], p["w_b"], w.gy))
    ws_f = torch.empty(max(binding.kan_workspace_bytes(s, B, binding.PASS_FORWARD), 256), dtype=torch.uint8, device="cuda")
    binding.kan_forward(s, x, coef, w_s, w_b, ws=ws_f)
    ref = binding.kan_backward(s, x, coef, w_s, w_b, gy)
    got = binding.kan_backward_saved(s, x, coef, w_s, w_b, gy, ws_f)
    for n in ref:
        assert torch.equal(got[n], ref[n]), n
    ws_b = torch.empty(binding.kan_workspace_bytes(s, B, binding.PASS_BACKWARD), dtype=torch.uint8, device="cuda")
    with pytest.raises(binding.KanError) as e:
        binding.kan_backward_saved(s, x, coef, w_s, w_b, gy, ws_b, ws=ws_b)
    assert e.value.status == binding.KAN_ERR_INVALID_ARG


def test_config2_full_size():
    """64->64, G=10, batch 65536 with 5% of the samples outside the grid: every output element."""
    run_layer_parity(workloads.config2())


def test_config3_full_size():
    """512->512, G=20, batch 16384 in the launch configuration the benchmark times: every output and
    every gradient element against the oracle (a few seconds of host time)."""
    w = workloads.config3()
    y, g = run_layer_parity(w)
    s, p = w.layers[0], w.params[0]
    # property that holds at any size: inside the grid the window weights sum to one, so
    # sum_m gcoef[i][m][j] / w_s[i][j] == sum_b gy[b][j] for every input i
    col = torch.from_numpy(w.gy.astype(np.float64).sum(0)).cuda()
    lhs = (g["gcoef"].double() / dev(p["w_s"]).double()[:, None, :]).sum(1)
    assert float((lhs - col[None, :]).abs().max()) < 2e-2 * float(col.abs().max() + 1)


def test_config4_large_grid_full_size():
    run_layer_parity(workloads.config4())


@pytest.mark.parametrize("G", [32, 1024])
def test_paper_shape_full_size(G):
    """32->32, k=3, N=2^17 (the shape of the paper's throughput table), smallest and largest grid."""
    run_layer_parity(workloads.paper_shape(G))


@pytest.mark.parametrize("G", [1 << 16, 1 << 18])
def test_paper_shape_huge_grids(G):
    """The same shape with 2^16 and 2^18 cells (tables of 0.27 and 1.07 GB): per-chunk partial tables no
    longer fit, so the 16 chunks of the batch take turns adding to one shared partial table."""
    run_layer_parity(workloads.paper_shape(G), gx_in_grid_units=True)


@pytest.mark.parametrize("k", [1, 2, 4, 5])
def test_paper_shape_degrees(k):
    """32->32, G=64, N=2^16 at the other degrees of the degree sweep (k = 3 is covered above)."""
    run_layer_parity(workloads.paper_shape(64, B=1 << 16, k=k))


@pytest.mark.parametrize("B,n_in,n_out,G", [(460000, 4, 16, 300000), (458753, 12, 6, 300000)])
def test_shared_partial_table(B, n_in, n_out, G):
    """Long batch x long table: 57 chunks of 8192 samples whose partial tables together would exceed the
    budget, so they share one (four outputs per lane, then one output per lane); ragged last chunk."""
    w = workloads.random_kan_layer(9100 + n_out, B, n_in, n_out, G, 3, outside_frac=0.02)
    run_layer_parity(w, gx_in_grid_units=True)
    # and bit for bit the same on a second run: the chunks add to the shared table in stream order
    s, p = w.layers[0], w.params[0]
    x, coef, w_s, w_b, gy = (dev(a) for a in (w.x, p["coef"], p["w_s"], p["w_b"], w.gy))
    a = binding.kan_backward(s, x, coef, w_s, w_b, gy)
    b = binding.kan_backward(s, x, coef, w_s, w_b, gy)
    for n in a:
        assert torch.equal(a[n], b[n]), n


def test_dense_gemm_baseline_matches_oracle():
    """The comparison baseline (all G+k bases, one rocBLAS GEMM) computes the same forward pass."""
    for B, n_in, n_out, G, k in [(300, 20, 96, 8, 3), (129, 7, 33, 5, 2)]:
        w = workloads.random_kan_layer(900 + B, B, n_in, n_out, G, k, outside_frac=0.2)
        s, p = w.layers[0], w.params[0]
        inv_h = oracle.inv_h_of(s.grid_lo, s.grid_hi, s.G)
        x, coef, w_s, w_b = (dev(a) for a in (w.x, p["coef"], p["w_s"], p["w_b"]))
        y = binding.kan_dense_baseline_forward(s, x, coef, w_s, w_b)
        g = binding.kan_dense_baseline_backward(s, x, coef, w_s, w_b, dev(w.gy))
        torch.cuda.synchronize()
        assert_close(y, oracle.kan_forward(w.x, p["coef"], p["w_s"], p["w_b"], s.G, s.k, s.grid_lo, inv_h), FWD_TOL, "y")
        ref = oracle.kan_backward(w.x, p["coef"], p["w_s"], p["w_b"], w.gy, s.G, s.k, s.grid_lo, inv_h)
        for name in ref:
            assert_close(g[name], ref[name], GRAD_TOL, "dense " + name)
