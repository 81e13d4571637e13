"""Pins for the CPU oracle of the bounded-grid KAN layer.

Each test ties the oracle to something other than itself: the cubic basis
matrix the paper prints, the Cox-de Boor definition evaluated by a library
routine (scipy), closed forms, invariants (partition of unity, reproduction of
constants and of the identity), library matmul special cases, and finite
differences for the gradients.  No GPU is involved.
"""
import math
import os

import numpy as np
import pytest
from scipy.interpolate import BSpline
from scipy.special import expit

import oracle
from paper_2408_11200_amd import workloads


def read_table(path):
    rows = []
    with open(path) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append([float(t) for t in line.split()])
    return np.array(rows)


def knots(G, k, lo, inv_h):
    h = 1.0 / float(inv_h)
    return lo + (np.arange(G + 2 * k + 1) - k) * h


# ------------------------------------------------------------ local basis --

def test_cubic_local_basis_equals_printed_basis_matrix(golden_dir):
    """Appendix, cubic basis matrix: [1 u u^2 u^3] * M/6 gives the four window weights."""
    M = read_table(os.path.join(golden_dir, "cubic_basis_matrix.txt")) / 6.0
    assert M.shape == (4, 4)
    rng = np.random.default_rng(0)
    for u in list(rng.uniform(0, 1, 200)) + [0.0, 0.5, 1.0 - 1e-12]:
        N, low = oracle.local_basis(3, u)
        U = np.array([1.0, u, u * u, u ** 3])
        np.testing.assert_allclose(N, U @ M, rtol=0, atol=2e-15)


def test_cubic_closed_form_pieces():
    """Uniform cubic B-spline pieces: (1-u)^3/6, (3u^3-6u^2+4)/6, (-3u^3+3u^2+3u+1)/6, u^3/6."""
    for u in np.linspace(0, 1, 41):
        N, _ = oracle.local_basis(3, u)
        ref = [(1 - u) ** 3 / 6, (3 * u ** 3 - 6 * u ** 2 + 4) / 6,
               (-3 * u ** 3 + 3 * u ** 2 + 3 * u + 1) / 6, u ** 3 / 6]
        np.testing.assert_allclose(N, ref, rtol=0, atol=2e-15)


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_local_basis_first_weight_and_partition_of_unity(k):
    for u in np.linspace(0, 1, 17, endpoint=False):
        N, low = oracle.local_basis(k, u)
        assert abs(N.sum() - 1.0) < 1e-14
        assert (N >= 0).all()
        assert abs(N[0] - (1 - u) ** k / math.factorial(k)) < 1e-15      # oldest coefficient
        assert abs(N[k] - u ** k / math.factorial(k)) < 1e-15           # newest coefficient
        assert abs(low.sum() - 1.0) < 1e-14                             # degree k-1 values


@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_local_basis_derivative_rule_by_finite_difference(k):
    """d N^k_s/du = N^{k-1}_{s-1} - N^{k-1}_s, checked against central differences."""
    eps = 1e-6
    for u in [0.1, 0.37, 0.5, 0.93]:
        N, low = oracle.local_basis(k, u)
        Np, _ = oracle.local_basis(k, u + eps)
        Nm, _ = oracle.local_basis(k, u - eps)
        fd = (Np - Nm) / (2 * eps)
        lo = np.concatenate([[0.0], low])
        hi = np.concatenate([low, [0.0]])
        np.testing.assert_allclose(lo - hi, fd, rtol=0, atol=1e-8)


# ------------------------------------------------------------ dense basis --

@pytest.mark.parametrize("G,k,lo,hi", [(5, 3, -1.0, 1.0), (7, 2, 0.0, 3.5), (4, 1, -2.0, 2.0),
                                       (6, 4, -1.0, 2.0), (3, 5, -1.0, 0.5)])
def test_dense_basis_matches_library_bspline(G, k, lo, hi):
    """Cox-de Boor on the extended knots vs scipy's B-spline basis elements."""
    inv_h = oracle.inv_h_of(lo, hi, G)
    tau = knots(G, k, lo, inv_h)
    rng = np.random.default_rng(1)
    xs = rng.uniform(tau[0], tau[-1], 60)
    for x in xs:
        got, dgot = oracle.dense_basis(G, k, lo, inv_h, x, want_grad=True)
        for m in range(G + k):
            el = BSpline.basis_element(tau[m:m + k + 2], extrapolate=False)
            ref = np.nan_to_num(el(x))
            dref = np.nan_to_num(el.derivative()(x)) if k >= 1 else 0.0
            assert abs(got[m] - ref) < 1e-12, (x, m)
            assert abs(dgot[m] - dref) < 1e-10, (x, m)


@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_dense_basis_support_and_unity(k):
    """Compact support [t_m, t_{m+k+1}): exactly k+1 non-zeros inside the grid, summing to 1;
    in the padding cells the sum is below 1; outside the extended knots everything is 0."""
    G, lo, hi = 6, -1.0, 1.0
    inv_h = oracle.inv_h_of(lo, hi, G)
    tau = knots(G, k, lo, inv_h)
    rng = np.random.default_rng(2)
    for x in rng.uniform(lo, hi, 50):
        bas = oracle.dense_basis(G, k, lo, inv_h, x)
        assert np.count_nonzero(bas) == k + 1
        assert abs(bas.sum() - 1.0) < 1e-13
        first = np.flatnonzero(bas)[0]
        assert tau[first + k] <= x < tau[first + k + 1]
    for x in [lo - 0.4 / inv_h, hi + 0.6 / inv_h]:
        bas = oracle.dense_basis(G, k, lo, inv_h, x)
        assert 0 < bas.sum() < 1.0
    for x in [tau[0] - 1e-9, tau[-1], tau[-1] + 1.0]:          # half-open: last knot is outside
        assert oracle.dense_basis(G, k, lo, inv_h, x).sum() == 0.0


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_local_equals_dense_basis(k):
    G, lo, hi = 9, -1.0, 2.0
    inv_h = oracle.inv_h_of(lo, hi, G)
    rng = np.random.default_rng(3)
    xs = np.float32(rng.uniform(lo, hi, 100))
    for x in xs:
        idx = int(oracle.interval_index(np.array([x]), lo, inv_h)[0])
        u = (float(x) - lo) * float(inv_h) - idx
        N, _ = oracle.local_basis(k, u)
        bas = oracle.dense_basis(G, k, lo, inv_h, float(x))
        expect = np.zeros(G + k)
        expect[idx:idx + k + 1] = N
        np.testing.assert_allclose(bas, expect, rtol=0, atol=1e-13)


# ---------------------------------------------------------- interval index --

def test_interval_index_definition():
    lo, hi, G, k = -1.0, 1.0, 20, 3
    inv_h = oracle.inv_h_of(lo, hi, G)
    assert float(inv_h) == 10.0
    x = np.float32([-1.0, -0.95, -0.9, 0.0, 0.05, 0.999, 1.0, 1.25, -1.3, -1.31, 5.0, -7.0])
    idx = oracle.interval_index(x, lo, inv_h)
    # the fp32 products here: (-0.95+1)*10 rounds to 0.5000001 -> 0 ; (-0.9+1)*10 -> 1.0000002 -> 1
    assert list(idx) == [0, 0, 1, 10, 10, 19, 20, 22, -3, -4, 60, -60]
    # property: x lies in the cell it is assigned to, up to one fp32 rounding of t
    rng = np.random.default_rng(4)
    xs = np.float32(rng.uniform(-1.5, 1.5, 5000))
    idx = oracle.interval_index(xs, lo, inv_h)
    t = (xs.astype(np.float64) - lo) * 10.0
    assert (np.abs(np.floor(t) - idx) <= 1).all()
    assert (t - idx > -1e-5).all() and (t - idx < 1 + 1e-5).all()
    same = np.floor(t) == idx
    assert same.mean() > 0.999
    # saturates instead of overflowing the cast
    far = oracle.interval_index(np.float32([3e38, -3e38, np.inf, -np.inf]), lo, inv_h)
    assert list(far) == [1 << 30, -(1 << 30), 1 << 30, -(1 << 30)]


def test_interval_index_is_two_roundings_not_fused():
    """Pick x where (x-a)*inv_h rounded twice differs from the exact product's floor."""
    lo, inv_h = np.float32(-1.0), np.float32(10.0)
    found = 0
    rng = np.random.default_rng(5)
    xs = np.float32(np.round(rng.uniform(-1, 1, 200000) * 10) / 10) + np.float32(0)
    xs = np.nextafter(xs, np.float32(-2))       # just below a knot
    got = oracle.interval_index(xs, lo, inv_h)
    d = (xs - lo).astype(np.float32)
    two_step = np.floor((d * inv_h).astype(np.float32)).astype(np.int32)
    assert (got == two_step).all()
    exact = np.floor((xs.astype(np.float64) + 1.0) * 10.0).astype(np.int32)
    found = int((got != exact).sum())
    assert found > 0      # the fp32 rule really differs from exact arithmetic at some knots


# ------------------------------------------------------------------ forward --

def _tiny(seed=7, B=64, n_in=2, n_out=5, G=5, k=3, outside=0.25):
    return workloads.random_kan_layer(seed, B, n_in, n_out, G, k, outside_frac=outside)


@pytest.mark.parametrize("k", [1, 2, 3, 4])
@pytest.mark.parametrize("shape", [(2, 5), (5, 1), (3, 4)])
def test_forward_local_equals_dense_definition(k, shape):
    """Brute force with all G+k bases on tiny layers, including padding cells and far-outside x."""
    w = _tiny(seed=10 + k, n_in=shape[0], n_out=shape[1], k=k, B=96, outside=0.4)
    s, p = w.layers[0], w.params[0]
    inv_h = oracle.inv_h_of(s.grid_lo, s.grid_hi, s.G)
    y_loc = oracle.kan_forward(w.x, p["coef"], p["w_s"], p["w_b"], s.G, k, s.grid_lo, inv_h)
    y_den = oracle.kan_forward(w.x, p["coef"], p["w_s"], p["w_b"], s.G, k, s.grid_lo, inv_h, dense=True)
    np.testing.assert_allclose(y_loc, y_den, rtol=0, atol=1e-12)
    # and some samples really are in padding cells / outside
    idx = oracle.interval_index(w.x, s.grid_lo, inv_h)
    assert ((idx < 0) & (idx >= -k)).any() and ((idx >= s.G) & (idx < s.G + k)).any()
    assert (idx >= s.G + k).any() or (idx < -k).any()


@pytest.mark.parametrize("k,n_in,n_out,G", [(3, 3, 5, 7), (2, 4, 2, 6), (1, 2, 3, 5), (4, 3, 2, 6)])
def test_forward_and_backward_equal_einsum_over_library_basis(k, n_in, n_out, G):
    """The layer written as one contraction over a basis tensor that comes from scipy, not from the oracle:
    Phi[b][i][m] = B_{m,k}(x[b][i]) by BSpline.basis_element on the extended knots, then
    y = einsum(Phi, coef, w_s) + silu(x) w_b with coefficients that differ along every axis and three
    unequal extents (n_in, G + k, n_out), so a swapped or transposed index of coef[i][m][j], w_s[i][j] or
    w_b[i][j] changes the result; the four gradients are the matching contractions with gy."""
    lo, hi = -1.0, 1.5
    assert len({n_in, G + k, n_out}) == 3
    inv_h = oracle.inv_h_of(lo, hi, G)
    tau = knots(G, k, lo, inv_h)
    rng = np.random.default_rng(40 + k)
    B = 37
    x = np.float32(rng.uniform(lo - 0.3, hi + 0.3, (B, n_in)))          # some samples in the padding cells
    coef = rng.standard_normal((n_in, G + k, n_out))
    w_s = rng.standard_normal((n_in, n_out))
    w_b = rng.standard_normal((n_in, n_out))
    gy = rng.standard_normal((B, n_out))
    els = [BSpline.basis_element(tau[m:m + k + 2], extrapolate=False) for m in range(G + k)]
    x64 = x.astype(np.float64)
    Phi = np.stack([np.nan_to_num(el(x64)) for el in els], axis=-1)                     # [B][n_in][G+k]
    dPhi = np.stack([np.nan_to_num(el.derivative()(x64)) for el in els], axis=-1)
    sig = expit(x64)
    silu, dsilu = x64 * sig, sig * (1.0 + x64 * (1.0 - sig))
    y_ref = np.einsum("bim,imj,ij->bj", Phi, coef, w_s) + silu @ w_b
    y = oracle.kan_forward(x, coef, w_s, w_b, G, k, lo, inv_h)
    np.testing.assert_allclose(y, y_ref, rtol=0, atol=1e-11)
    g = oracle.kan_backward(x, coef, w_s, w_b, gy, G, k, lo, inv_h)
    np.testing.assert_allclose(g["gcoef"], np.einsum("bim,bj,ij->imj", Phi, gy, w_s), rtol=0, atol=1e-11)
    np.testing.assert_allclose(g["gw_s"], np.einsum("bim,imj,bj->ij", Phi, coef, gy), rtol=0, atol=1e-11)
    np.testing.assert_allclose(g["gw_b"], silu.T @ gy, rtol=0, atol=1e-11)
    gx_ref = np.einsum("bim,imj,ij,bj->bi", dPhi, coef, w_s, gy) + dsilu * (gy @ w_b.T)
    np.testing.assert_allclose(g["gx"], gx_ref, rtol=0, atol=1e-10)


def test_forward_constant_coefficients_reproduce_constant():
    """coef == c  =>  spline == c inside the grid, so y = sum_i (w_s*c + w_b*silu(x_i))."""
    w = _tiny(seed=21, outside=0.0, B=50, n_in=4, n_out=3, G=8, k=3)
    s, p = w.layers[0], w.params[0]
    inv_h = oracle.inv_h_of(s.grid_lo, s.grid_hi, s.G)
    c = 0.37
    coef = np.full(p["coef"].shape, c)
    y = oracle.kan_forward(w.x, coef, p["w_s"], p["w_b"], s.G, s.k, s.grid_lo, inv_h)
    x64 = w.x.astype(np.float64)
    silu = x64 * expit(x64)
    ref = c * p["w_s"].astype(np.float64).sum(0)[None, :] + silu @ p["w_b"].astype(np.float64)
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-12)


@pytest.mark.parametrize("k", [1, 2, 3])
def test_forward_greville_coefficients_reproduce_identity(k):
    """With c_m = mean of knots tau_{m+1..m+k} the spline is x itself inside the grid.
    A shifted window, a reversed weight order or a wrong u fails this."""
    G, lo, hi = 10, -1.0, 1.0
    inv_h = oracle.inv_h_of(lo, hi, G)
    tau = knots(G, k, lo, inv_h)
    grev = np.array([tau[m + 1:m + k + 1].mean() for m in range(G + k)])
    n_in, n_out = 3, 2
    coef = np.tile(grev[None, :, None], (n_in, 1, n_out))
    rng = np.random.default_rng(8)
    x = np.float32(rng.uniform(lo, hi * 0.999, (40, n_in)))
    w_s = rng.standard_normal((n_in, n_out))
    y = oracle.kan_forward(x, coef, w_s, np.zeros((n_in, n_out)), G, k, lo, inv_h, base_act=0)
    np.testing.assert_allclose(y, x.astype(np.float64) @ w_s, rtol=0, atol=1e-12)


def test_forward_zero_spline_scale_is_a_matmul():
    """w_s = 0  =>  y = silu(X) W_b, a library GEMM."""
    w = _tiny(seed=22, outside=0.3, B=70, n_in=6, n_out=4)
    s, p = w.layers[0], w.params[0]
    inv_h = oracle.inv_h_of(s.grid_lo, s.grid_hi, s.G)
    y = oracle.kan_forward(w.x, p["coef"], np.zeros_like(p["w_s"]), p["w_b"], s.G, s.k, s.grid_lo, inv_h)
    x64 = w.x.astype(np.float64)
    np.testing.assert_allclose(y, (x64 * expit(x64)) @ p["w_b"].astype(np.float64), rtol=0, atol=1e-12)


def test_forward_far_outside_is_base_only_and_no_base_is_zero():
    s = workloads.KanLayerSpec(3, 2, 5, 3, -1.0, 1.0)
    rng = np.random.default_rng(9)
    p = workloads.kan_params(rng, s, 0.1, w_s_std=1.0, w_b_std=1.0)
    inv_h = oracle.inv_h_of(-1.0, 1.0, 5)
    h = 0.4
    x = np.float32([[1.0 + 3 * h, -1.0 - 3 * h - 1e-3, 9.0]])     # at the last extended knot, below the first, far
    y0 = oracle.kan_forward(x, p["coef"], p["w_s"], p["w_b"], 5, 3, -1.0, inv_h, base_act=0)
    assert (y0 == 0).all()
    y1 = oracle.kan_forward(x, p["coef"], p["w_s"], p["w_b"], 5, 3, -1.0, inv_h, base_act=1)
    x64 = x.astype(np.float64)
    np.testing.assert_allclose(y1, (x64 * expit(x64)) @ p["w_b"].astype(np.float64), atol=1e-13)


def test_silu_and_its_derivative():
    xs = np.linspace(-12, 12, 97)
    np.testing.assert_allclose(oracle.silu(xs), xs * expit(xs), rtol=0, atol=1e-14)
    eps = 1e-6
    fd = (oracle.silu(xs + eps) - oracle.silu(xs - eps)) / (2 * eps)
    np.testing.assert_allclose(oracle.silu_grad(xs), fd, rtol=0, atol=1e-8)


# ---------------------------------------------------------------- backward --

def _loss(w, x, p, gy, k, inv_h):
    s = w.layers[0]
    y = oracle.kan_forward(x, p["coef"], p["w_s"], p["w_b"], s.G, k, s.grid_lo, inv_h, idx_fp32=False)
    return float((y * gy).sum())


@pytest.mark.parametrize("k", [2, 3])
def test_backward_by_central_finite_differences(k):
    w = _tiny(seed=30 + k, B=12, n_in=3, n_out=4, G=5, k=k, outside=0.35)
    s = w.layers[0]
    inv_h = oracle.inv_h_of(s.grid_lo, s.grid_hi, s.G)
    p = {n: a.astype(np.float64) for n, a in w.params[0].items()}
    x = w.x.astype(np.float64)
    gy = w.gy.astype(np.float64)
    g = oracle.kan_backward(x, p["coef"], p["w_s"], p["w_b"], gy, s.G, k, s.grid_lo, inv_h, idx_fp32=False)
    eps = 1e-6

    def fd(name, arr):
        out = np.zeros_like(arr)
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            ix = it.multi_index
            keep = arr[ix]
            arr[ix] = keep + eps
            lp = _loss(w, x, p, gy, k, inv_h)
            arr[ix] = keep - eps
            lm = _loss(w, x, p, gy, k, inv_h)
            arr[ix] = keep
            out[ix] = (lp - lm) / (2 * eps)
        return out

    np.testing.assert_allclose(g["gx"], fd("x", x), rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(g["gcoef"], fd("coef", p["coef"]), rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(g["gw_s"], fd("w_s", p["w_s"]), rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(g["gw_b"], fd("w_b", p["w_b"]), rtol=1e-6, atol=1e-8)


def test_backward_identities():
    """gw_s = sum_m coef * gcoef / w_s ; inside the grid sum_m gcoef/w_s = sum_b gy (partition of unity);
    gw_b = silu(X)^T gy (library GEMM)."""
    w = _tiny(seed=41, B=200, n_in=4, n_out=3, G=6, k=3, outside=0.0)
    s, p = w.layers[0], w.params[0]
    inv_h = oracle.inv_h_of(s.grid_lo, s.grid_hi, s.G)
    g = oracle.kan_backward(w.x, p["coef"], p["w_s"], p["w_b"], w.gy, s.G, s.k, s.grid_lo, inv_h)
    ws = p["w_s"].astype(np.float64)
    gcp = g["gcoef"] / ws[:, None, :]
    np.testing.assert_allclose((p["coef"].astype(np.float64) * gcp).sum(1), g["gw_s"], rtol=0, atol=1e-11)
    np.testing.assert_allclose(gcp.sum(1), np.tile(w.gy.astype(np.float64).sum(0), (s.n_in, 1)), atol=1e-11)
    x64 = w.x.astype(np.float64)
    np.testing.assert_allclose(g["gw_b"], (x64 * expit(x64)).T @ w.gy.astype(np.float64), atol=1e-11)


def test_backward_null_outputs_and_overwrite():
    w = _tiny(seed=42, B=20)
    s, p = w.layers[0], w.params[0]
    inv_h = oracle.inv_h_of(s.grid_lo, s.grid_hi, s.G)
    full = oracle.kan_backward(w.x, p["coef"], p["w_s"], p["w_b"], w.gy, s.G, s.k, s.grid_lo, inv_h)
    part = oracle.kan_backward(w.x, p["coef"], p["w_s"], p["w_b"], w.gy, s.G, s.k, s.grid_lo, inv_h,
                               want=("gx", "gw_b"))
    assert set(part) == {"gx", "gw_b"}
    np.testing.assert_array_equal(part["gx"], full["gx"])
    np.testing.assert_array_equal(part["gw_b"], full["gw_b"])


def test_config1_two_layer_mse_chain_by_finite_differences():
    """Tiny KAN [2,5,1] with MSE against sin(pi x0) + x1^2: the chained oracle gradient of the
    first layer's coefficients equals finite differences of the loss."""
    w = workloads.config1()
    B = 64
    x = w.x[:B].astype(np.float64)
    tgt = w.target[:B].astype(np.float64)
    P = [{n: a.astype(np.float64) for n, a in p.items()} for p in w.params]
    S = w.layers
    ih = [oracle.inv_h_of(s.grid_lo, s.grid_hi, s.G) for s in S]

    def fwd():
        h1 = oracle.kan_forward(x, P[0]["coef"], P[0]["w_s"], P[0]["w_b"], S[0].G, 3, -1.0, ih[0], idx_fp32=False)
        y = oracle.kan_forward(h1, P[1]["coef"], P[1]["w_s"], P[1]["w_b"], S[1].G, 3, -1.0, ih[1], idx_fp32=False)
        return h1, y

    h1, y = fwd()
    gy = 2.0 * (y - tgt) / B
    g2 = oracle.kan_backward(h1, P[1]["coef"], P[1]["w_s"], P[1]["w_b"], gy, S[1].G, 3, -1.0, ih[1], idx_fp32=False)
    g1 = oracle.kan_backward(x, P[0]["coef"], P[0]["w_s"], P[0]["w_b"], g2["gx"], S[0].G, 3, -1.0, ih[0], idx_fp32=False)
    eps = 1e-6
    rng = np.random.default_rng(0)
    for _ in range(12):
        ix = tuple(rng.integers(0, d) for d in P[0]["coef"].shape)
        keep = P[0]["coef"][ix]
        P[0]["coef"][ix] = keep + eps
        lp = float(((fwd()[1] - tgt) ** 2).mean())
        P[0]["coef"][ix] = keep - eps
        lm = float(((fwd()[1] - tgt) ** 2).mean())
        P[0]["coef"][ix] = keep
        assert abs((lp - lm) / (2 * eps) - g1["gcoef"][ix]) < 1e-8
