"""Seeded synthetic inputs shaped like the paper's workloads.

This module holds no arithmetic of the method: it only draws random numbers
with numpy and names the shapes.  It is the one module both the CPU oracle's
tests and the HIP path's tests/benchmark take their inputs from, so that both
sides see identical bits.  All arrays are fp32, C-contiguous, on the host.

The paper's own benchmark (section "Performance Benchmarking") is a single
random layer of fixed shape, so these recipes are its workload, not a stand-in
for a dataset.
"""
from dataclasses import dataclass, field

import numpy as np


@dataclass
class KanLayerSpec:
    """One bounded-grid KAN layer: widths, grid size G (cells), degree k, grid range."""
    n_in: int
    n_out: int
    G: int
    k: int
    grid_lo: float
    grid_hi: float
    base_act: int = 1          # 0 none, 1 SiLU

    @property
    def M(self):               # coefficients per edge
        return self.G + self.k


@dataclass
class UkanLayerSpec:
    """One UKAN layer: widths, degree k, grid spacing h and the CG widths."""
    n_in: int
    n_out: int
    k: int
    h: float
    d_pe: int
    d_feat: int
    d_hidden: int
    base_act: int = 0


@dataclass
class Workload:
    name: str
    B: int
    layers: list
    x: np.ndarray
    params: list = field(default_factory=list)   # one dict per layer
    gy: np.ndarray = None                        # dL/dy at the top
    target: np.ndarray = None


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def kan_params(rng, spec, coef_std, w_s=None, w_b_std=None, w_s_std=None):
    """coef ~ N(0, coef_std^2); w_s constant or N(0, w_s_std^2); w_b ~ N(0, w_b_std^2)."""
    coef = _f32(rng.standard_normal((spec.n_in, spec.M, spec.n_out)) * coef_std)
    if w_s is not None:
        ws = _f32(np.full((spec.n_in, spec.n_out), w_s))
    else:
        ws = _f32(rng.standard_normal((spec.n_in, spec.n_out)) * w_s_std)
    wb = _f32(rng.standard_normal((spec.n_in, spec.n_out)) * w_b_std)
    return {"coef": coef, "w_s": ws, "w_b": wb}


def ukan_params(rng, spec):
    """E ~ N(0,1), W ~ N(0, 1/fan_in), biases 0, scale 1 (the paper states no init)."""
    K = spec.k + 1
    dz = spec.d_feat + spec.d_pe
    p = {
        "E": _f32(rng.standard_normal((spec.n_in, spec.d_feat))),
        "W1": _f32(rng.standard_normal((dz, spec.d_hidden)) / np.sqrt(dz)),
        "b1": _f32(np.zeros(spec.d_hidden)),
        "W2": _f32(rng.standard_normal((spec.d_hidden, K * spec.n_out)) / np.sqrt(spec.d_hidden)),
        "b2": _f32(np.zeros(K * spec.n_out)),
        "scale": _f32(np.ones((spec.n_in, spec.n_out))),
    }
    if spec.base_act:
        p["w_b"] = _f32(rng.standard_normal((spec.n_in, spec.n_out)) / np.sqrt(spec.n_in))
    return p


def random_kan_layer(seed, B, n_in, n_out, G, k, grid_lo=-1.0, grid_hi=1.0, base_act=1,
                     outside_frac=0.0, coef_std=0.1):
    """Generic single layer for parity sweeps.  `outside_frac` of the rows are drawn
    from the band of one grid width on either side of the grid, so that padding
    cells and the fully-outside path both occur."""
    rng = np.random.default_rng(seed)
    spec = KanLayerSpec(n_in, n_out, G, k, grid_lo, grid_hi, base_act)
    width = grid_hi - grid_lo
    x = rng.uniform(grid_lo, grid_hi, size=(B, n_in))
    n_outside = int(round(outside_frac * B))
    if n_outside:
        rows = rng.choice(B, size=n_outside, replace=False)
        d = rng.uniform(0.0, width, size=(n_outside, n_in))
        side = rng.integers(0, 2, size=(n_outside, n_in))
        x[rows] = np.where(side == 0, grid_lo - d, grid_hi + d)
    p = kan_params(rng, spec, coef_std, w_s_std=1.0 / np.sqrt(n_in), w_b_std=1.0 / np.sqrt(n_in))
    gy = _f32(rng.standard_normal((B, n_out)))
    return Workload("random", B, [spec], _f32(x), [p], gy)


def config1(seed=1001):
    """Tiny KAN [2,5,1], G=5, k=3 on [-1,1], batch 1024, MSE against sin(pi x0) + x1^2."""
    rng = np.random.default_rng(seed)
    B = 1024
    specs = [KanLayerSpec(2, 5, 5, 3, -1.0, 1.0), KanLayerSpec(5, 1, 5, 3, -1.0, 1.0)]
    x = _f32(rng.uniform(-1.0, 1.0, size=(B, 2)))
    params = [kan_params(rng, s, 0.1, w_s=1.0, w_b_std=0.1) for s in specs]
    target = _f32(np.sin(np.pi * x[:, :1].astype(np.float64)) + x[:, 1:2].astype(np.float64) ** 2)
    return Workload("C1 KAN[2,5,1] G5 k3 B1024", B, specs, x, params, None, target)


def config2(seed=1002, B=65536):
    """64->64, G=10, k=3 on [-1,1]; 5% of the samples lie outside the grid."""
    rng = np.random.default_rng(seed)
    spec = KanLayerSpec(64, 64, 10, 3, -1.0, 1.0)
    x = rng.uniform(-1.0, 1.0, size=(B, 64))
    n_outside = int(round(0.05 * B))
    rows = rng.choice(B, size=n_outside, replace=False)
    mag = rng.uniform(1.0, 2.0, size=(n_outside, 64))
    sign = np.where(rng.integers(0, 2, size=(n_outside, 64)) == 0, -1.0, 1.0)
    x[rows] = sign * mag
    p = kan_params(rng, spec, 0.1, w_s=1.0, w_b_std=0.1)
    gy = _f32(rng.standard_normal((B, 64)))
    return Workload("C2 KAN 64->64 G10 k3 B%d" % B, B, [spec], _f32(x), [p], gy)


def config3(seed=1003, B=16384, n=512):
    """512->512, G=20, k=3 on [-1,1], batch 16384: the configuration the metric is quoted on."""
    rng = np.random.default_rng(seed)
    spec = KanLayerSpec(n, n, 20, 3, -1.0, 1.0)
    x = _f32(rng.uniform(-1.0, 1.0, size=(B, n)))
    p = kan_params(rng, spec, 0.05, w_s_std=1.0 / np.sqrt(n), w_b_std=1.0 / np.sqrt(n))
    gy = _f32(rng.standard_normal((B, n), dtype=np.float32))
    return Workload("C3 KAN %d->%d G20 k3 B%d" % (n, n, B), B, [spec], x, [p], gy)


def config4(seed=1004, B=8192, n=256):
    """256->256, G=200, k=3 on [-4,4], x ~ N(0, 1.5^2): large-grid case."""
    rng = np.random.default_rng(seed)
    spec = KanLayerSpec(n, n, 200, 3, -4.0, 4.0)
    x = _f32(rng.standard_normal((B, n)) * 1.5)
    p = kan_params(rng, spec, 0.1, w_s_std=1.0 / np.sqrt(n), w_b_std=1.0 / np.sqrt(n))
    gy = _f32(rng.standard_normal((B, n)))
    return Workload("C4 KAN %d->%d G200 k3 B%d" % (n, n, B), B, [spec], x, [p], gy)


def config5(seed=1005, B=32768, widths=(128, 256, 256, 1)):
    """UKAN stack on the unbounded grid, h=0.25, k=3, unnormalised x ~ N(0, 10^2)."""
    rng = np.random.default_rng(seed)
    specs = [UkanLayerSpec(widths[l], widths[l + 1], 3, 0.25, 32, 32, 64) for l in range(len(widths) - 1)]
    x = _f32(rng.standard_normal((B, widths[0])) * 10.0)
    params = [ukan_params(rng, s) for s in specs]
    gy = _f32(rng.standard_normal((B, widths[-1])))
    return Workload("C5 UKAN %s h0.25 k3 B%d" % (list(widths), B), B, specs, x, params, gy)


def paper_shape(G, seed=1100, B=1 << 17, k=3):
    """The paper's own benchmark shape (Table 2): 32->32, k=3, N=2^17, x uniform inside the grid."""
    rng = np.random.default_rng(seed + G)
    spec = KanLayerSpec(32, 32, G, k, -1.0, 1.0)
    x = _f32(rng.uniform(-1.0, 1.0, size=(B, 32)))
    x = np.minimum(x, np.float32(np.nextafter(np.float32(1.0), np.float32(0.0))))
    p = kan_params(rng, spec, 0.1, w_s_std=1.0 / np.sqrt(32), w_b_std=1.0 / np.sqrt(32))
    gy = _f32(rng.standard_normal((B, 32)))
    return Workload("P KAN 32->32 G%d k%d B%d" % (G, k, B), B, [spec], x, [p], gy)


def regression_task(which, seed=1200, B=4096):
    """Inputs and closed-form targets of the regression experiments (section "Tasks", functions I-III):
    x uniform on [-1, 1]^d, d = 2 for I and II and 16 for III.  The targets are data for the training
    loop, evaluated here in fp64 with library routines; they are no part of the layer's arithmetic.
      I    exp(J0(20 x0) + x1^2)           (J0: Bessel function of the first kind, order 0)
      II   exp(sin(pi x0) + x1^2)
      III  exp((1/15) sum_{i=0..15} sin((4 i / 15 + 1) pi x_i))"""
    from scipy.special import j0
    rng = np.random.default_rng(seed + {"I": 1, "II": 2, "III": 3}[which])
    d = 16 if which == "III" else 2
    x = rng.uniform(-1.0, 1.0, size=(B, d))
    if which == "I":
        t = np.exp(j0(20.0 * x[:, 0]) + x[:, 1] ** 2)
    elif which == "II":
        t = np.exp(np.sin(np.pi * x[:, 0]) + x[:, 1] ** 2)
    else:
        i = np.arange(16)
        t = np.exp(np.sin((4.0 * i / 15.0 + 1.0) * np.pi * x).sum(1) / 15.0)
    return _f32(x), _f32(t[:, None])
