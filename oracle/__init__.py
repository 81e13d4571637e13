"""CPU oracle for the KAN / UKAN layer: ctypes front end of the plain C files.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this
module; it exists so that the tests, the smoke check and the benchmark's
cpu_baseline leg can compare the HIP library with a slow fp64 reference.

Every function takes numpy arrays (any float dtype; they are widened to
fp64, which is exact for fp32 inputs) and returns fp64 arrays.  `idx_fp32`
selects how the cell index is computed: True = the fp32 rule on the
fp32-rounded input (what the device does), False = the same formula in fp64
(used by finite-difference tests).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_SOURCES = ["kan_oracle.c", "ukan_oracle.c"]


def build(force=True):
    """Compile the C oracle with gcc (no contraction, so the fp32 index rule
    keeps its two roundings)."""
    if not force and os.path.exists(_LIB_PATH):
        return _LIB_PATH
    cmd = ["gcc", "-O2", "-std=c99", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
           "-o", _LIB_PATH] + [os.path.join(_HERE, s) for s in _SOURCES] + ["-lm"]
    subprocess.run(cmd, check=True)
    return _LIB_PATH


_lib = None


def _load():
    global _lib
    if _lib is None:
        newest = max(os.path.getmtime(os.path.join(_HERE, s)) for s in _SOURCES)
        if not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < newest:
            build()
        _lib = ctypes.CDLL(_LIB_PATH)
        _lib.okan_silu.restype = ctypes.c_double
        _lib.okan_silu.argtypes = [ctypes.c_double]
        _lib.okan_silu_grad.restype = ctypes.c_double
        _lib.okan_silu_grad.argtypes = [ctypes.c_double]
        _lib.okan_interval_index_f32.restype = ctypes.c_int32
        _lib.okan_interval_index_f32.argtypes = [ctypes.c_float] * 3
    return _lib


_D = ctypes.POINTER(ctypes.c_double)
_F = ctypes.POINTER(ctypes.c_float)
_I = ctypes.POINTER(ctypes.c_int32)


def _d(a):
    """fp64 C-contiguous copy + pointer (None passes NULL)."""
    if a is None:
        return None, None
    arr = np.ascontiguousarray(np.asarray(a), dtype=np.float64)
    return arr, arr.ctypes.data_as(_D)


def num_threads():
    return int(_load().okan_num_threads())


def set_num_threads(n):
    """Threads the oracle's loops run on from now on (timing aid; results do not depend on it)."""
    _load().okan_set_num_threads(int(n))


def inv_h_of(grid_lo, grid_hi, G):
    """The fp32 reciprocal cell width both sides use: (float)G / (hi - lo)."""
    return np.float32(G) / (np.float32(grid_hi) - np.float32(grid_lo))


def inv_h_of_spacing(h):
    """UKAN: the fp32 reciprocal of the fp32 grid spacing, 1.0f / h."""
    return np.float32(1.0) / np.float32(h)


def silu(x):
    lib = _load()
    return np.vectorize(lambda v: lib.okan_silu(float(v)))(np.asarray(x, dtype=np.float64))


def silu_grad(x):
    lib = _load()
    return np.vectorize(lambda v: lib.okan_silu_grad(float(v)))(np.asarray(x, dtype=np.float64))


def interval_index(x, grid_lo, inv_h):
    """fp32 cell index of every element of x (int32, same shape)."""
    lib = _load()
    xf = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(xf.shape, dtype=np.int32)
    lib.okan_interval_index_batch(ctypes.c_int64(xf.size), xf.ctypes.data_as(_F),
                                  ctypes.c_float(grid_lo), ctypes.c_float(inv_h),
                                  out.ctypes.data_as(_I))
    return out


def dense_basis(G, k, grid_lo, inv_h, x, want_grad=False):
    """All G+k Cox-de Boor basis values (and x-derivatives) at scalar x."""
    lib = _load()
    out = np.zeros(G + k)
    dout = np.zeros(G + k)
    lib.okan_dense_basis(ctypes.c_int(G), ctypes.c_int(k), ctypes.c_double(grid_lo),
                         ctypes.c_float(inv_h), ctypes.c_double(x),
                         out.ctypes.data_as(_D), dout.ctypes.data_as(_D) if want_grad else None)
    return (out, dout) if want_grad else out


def local_basis(k, u):
    """(N[0..k], N_low[0..k-1]) at local coordinate u."""
    lib = _load()
    N = np.zeros(k + 1)
    low = np.zeros(max(k, 1))
    lib.okan_local_basis(ctypes.c_int(k), ctypes.c_double(u), N.ctypes.data_as(_D),
                         low.ctypes.data_as(_D))
    return N, low[:k]


def _kan_common(x, coef, w_s, w_b, G, k):
    x = np.asarray(x)
    B, n_in = x.shape
    n_out = np.asarray(w_s).shape[1]
    assert np.asarray(coef).shape == (n_in, G + k, n_out), (np.asarray(coef).shape, (n_in, G + k, n_out))
    return B, n_in, n_out


def kan_forward(x, coef, w_s, w_b, G, k, grid_lo, inv_h, base_act=1, idx_fp32=True, dense=False):
    lib = _load()
    B, n_in, n_out = _kan_common(x, coef, w_s, w_b, G, k)
    xa, xp = _d(x); ca, cp = _d(coef); sa, sp = _d(w_s); ba, bp = _d(w_b)
    y = np.zeros((B, n_out))
    if dense:
        rc = lib.okan_forward_dense(n_in, n_out, G, k, ctypes.c_double(grid_lo), ctypes.c_float(inv_h),
                                    base_act, ctypes.c_int64(B), xp, cp, sp, bp, y.ctypes.data_as(_D))
    else:
        rc = lib.okan_forward(n_in, n_out, G, k, ctypes.c_double(grid_lo), ctypes.c_float(inv_h),
                              base_act, int(idx_fp32), ctypes.c_int64(B), xp, cp, sp, bp,
                              y.ctypes.data_as(_D))
    if rc:
        raise ValueError("oracle rejected the arguments (rc=%d)" % rc)
    return y


def kan_backward(x, coef, w_s, w_b, gy, G, k, grid_lo, inv_h, base_act=1, idx_fp32=True,
                 want=("gx", "gcoef", "gw_s", "gw_b")):
    lib = _load()
    B, n_in, n_out = _kan_common(x, coef, w_s, w_b, G, k)
    xa, xp = _d(x); ca, cp = _d(coef); sa, sp = _d(w_s); ba, bp = _d(w_b); ga, gp = _d(gy)
    out = {
        "gx": np.zeros((B, n_in)) if "gx" in want else None,
        "gcoef": np.zeros((n_in, G + k, n_out)) if "gcoef" in want else None,
        "gw_s": np.zeros((n_in, n_out)) if "gw_s" in want else None,
        "gw_b": np.zeros((n_in, n_out)) if "gw_b" in want else None,
    }
    ptr = {n: (a.ctypes.data_as(_D) if a is not None else None) for n, a in out.items()}
    rc = lib.okan_backward(n_in, n_out, G, k, ctypes.c_double(grid_lo), ctypes.c_float(inv_h),
                           base_act, int(idx_fp32), ctypes.c_int64(B), xp, cp, sp, bp, gp,
                           ptr["gx"], ptr["gcoef"], ptr["gw_s"], ptr["gw_b"])
    if rc:
        raise ValueError("oracle rejected the arguments (rc=%d)" % rc)
    return {n: a for n, a in out.items() if a is not None}


# ---------------------------------------------------------------- UKAN ----

def group_index(x, inv_h, K):
    """(cell, group, offset) int32 arrays for every element of x."""
    lib = _load()
    xf = np.ascontiguousarray(x, dtype=np.float32)
    cell = np.empty(xf.shape, dtype=np.int32)
    g = np.empty(xf.shape, dtype=np.int32)
    r = np.empty(xf.shape, dtype=np.int32)
    lib.oukan_group_index_batch(ctypes.c_int64(xf.size), xf.ctypes.data_as(_F), ctypes.c_float(inv_h),
                                ctypes.c_int(K), cell.ctypes.data_as(_I), g.ctypes.data_as(_I),
                                r.ctypes.data_as(_I))
    return cell, g, r


def pe(g, d_pe):
    lib = _load()
    out = np.zeros(d_pe)
    lib.oukan_pe(ctypes.c_int32(int(g)), ctypes.c_int(d_pe), out.ctypes.data_as(_D))
    return out


def _ukan_dims(p, k):
    n_in, d_feat = np.asarray(p["E"]).shape
    dz, d_hid = np.asarray(p["W1"]).shape
    n_out = np.asarray(p["scale"]).shape[1]
    assert np.asarray(p["W2"]).shape == (d_hid, (k + 1) * n_out)
    return n_in, n_out, dz - d_feat, d_feat, d_hid


def cg(p, k, i, g):
    """Raw CG output [K][n_out] for feature i and group g."""
    lib = _load()
    n_in, n_out, d_pe, d_feat, d_hid = _ukan_dims(p, k)
    Ea, Ep = _d(p["E"]); W1a, W1p = _d(p["W1"]); b1a, b1p = _d(p["b1"])
    W2a, W2p = _d(p["W2"]); b2a, b2p = _d(p["b2"])
    out = np.zeros(((k + 1), n_out))
    lib.oukan_cg(n_in, n_out, k, d_pe, d_feat, d_hid, Ep, W1p, b1p, W2p, b2p, int(i),
                 ctypes.c_int32(int(g)), out.ctypes.data_as(_D))
    return out


def ukan_forward(x, p, k, inv_h, base_act=0, idx_fp32=True, direct=False):
    """p: dict with E, W1, b1, W2, b2, scale and (if base_act) w_b."""
    lib = _load()
    n_in, n_out, d_pe, d_feat, d_hid = _ukan_dims(p, k)
    x = np.asarray(x)
    B = x.shape[0]
    assert x.shape[1] == n_in
    xa, xp = _d(x)
    Ea, Ep = _d(p["E"]); W1a, W1p = _d(p["W1"]); b1a, b1p = _d(p["b1"])
    W2a, W2p = _d(p["W2"]); b2a, b2p = _d(p["b2"]); sa, sp = _d(p["scale"])
    wa, wp = _d(p.get("w_b"))
    y = np.zeros((B, n_out))
    fn = lib.oukan_forward_direct if direct else lib.oukan_forward
    rc = fn(n_in, n_out, k, ctypes.c_float(inv_h), d_pe, d_feat, d_hid, base_act, int(idx_fp32),
            ctypes.c_int64(B), xp, Ep, W1p, b1p, W2p, b2p, sp, wp, y.ctypes.data_as(_D))
    if rc:
        raise ValueError("oracle rejected the arguments (rc=%d)" % rc)
    return y


def ukan_materialize(p, k, c_lo, c_hi):
    """KAN coefficients [n_in][(c_hi-c_lo+1)+k][n_out] equal to the UKAN on
    cells c_lo..c_hi (scale applied; use w_s = 1, grid_lo = c_lo*h)."""
    lib = _load()
    n_in, n_out, d_pe, d_feat, d_hid = _ukan_dims(p, k)
    Ea, Ep = _d(p["E"]); W1a, W1p = _d(p["W1"]); b1a, b1p = _d(p["b1"])
    W2a, W2p = _d(p["W2"]); b2a, b2p = _d(p["b2"]); sa, sp = _d(p["scale"])
    coef = np.zeros((n_in, (c_hi - c_lo + 1) + k, n_out))
    lib.oukan_materialize(n_in, n_out, k, d_pe, d_feat, d_hid, Ep, W1p, b1p, W2p, b2p, sp,
                          ctypes.c_int32(int(c_lo)), ctypes.c_int32(int(c_hi)), coef.ctypes.data_as(_D))
    return coef


def ukan_backward(x, p, gy, k, inv_h, base_act=0, idx_fp32=True):
    lib = _load()
    n_in, n_out, d_pe, d_feat, d_hid = _ukan_dims(p, k)
    x = np.asarray(x)
    B = x.shape[0]
    xa, xp = _d(x); ga, gp = _d(gy)
    Ea, Ep = _d(p["E"]); W1a, W1p = _d(p["W1"]); b1a, b1p = _d(p["b1"])
    W2a, W2p = _d(p["W2"]); b2a, b2p = _d(p["b2"]); sa, sp = _d(p["scale"])
    wa, wp = _d(p.get("w_b"))
    K = k + 1
    out = {
        "gx": np.zeros((B, n_in)), "gE": np.zeros((n_in, d_feat)),
        "gW1": np.zeros((d_feat + d_pe, d_hid)), "gb1": np.zeros(d_hid),
        "gW2": np.zeros((d_hid, K * n_out)), "gb2": np.zeros(K * n_out),
        "gscale": np.zeros((n_in, n_out)),
        "gw_b": np.zeros((n_in, n_out)) if base_act else None,
    }
    ptr = {n: (a.ctypes.data_as(_D) if a is not None else None) for n, a in out.items()}
    rc = lib.oukan_backward(n_in, n_out, k, ctypes.c_float(inv_h), d_pe, d_feat, d_hid, base_act,
                            int(idx_fp32), ctypes.c_int64(B), xp, Ep, W1p, b1p, W2p, b2p, sp, wp, gp,
                            ptr["gx"], ptr["gE"], ptr["gW1"], ptr["gb1"], ptr["gW2"], ptr["gb2"],
                            ptr["gscale"], ptr["gw_b"])
    if rc:
        raise ValueError("oracle rejected the arguments (rc=%d)" % rc)
    return {n: a for n, a in out.items() if a is not None}
