"""ctypes front end of libkan_hip.so (include/kan.h) and of the benchmark companion libkan_bench.so
(include/kan_bench.h): same entry-point names as the headers.

Argument marshalling only.  PyTorch is used to hold device memory and to name
the stream; every step of the layer runs inside the HIP library.  If the
library has not been built the first call raises: there is no fallback.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkan_hip.so")
BENCH_LIB_PATH = os.path.join(_HERE, "libkan_bench.so")

KAN_OK = 0
KAN_ERR_INVALID_ARG = -1
KAN_ERR_UNSUPPORTED = -2
KAN_ERR_WORKSPACE = -3
KAN_ERR_RANGE = -4
KAN_ERR_HIP = -5
PASS_FORWARD, PASS_BACKWARD = 0, 1

EXPORTS = ["kan_strerror", "kan_workspace_bytes", "kan_forward", "kan_backward", "kan_backward_saved", "kan_interval_index",
           "kan_static_scratch_bytes", "kan_forward_static", "kan_set_launch_observer",
           "ukan_workspace_bytes", "ukan_cg_forward", "ukan_cg_backward", "ukan_saved_bytes",
           "ukan_cg_forward_saved", "ukan_cg_forward_saved_async", "ukan_cg_backward_saved", "ukan_materialize_workspace_bytes",
           "ukan_materialize", "ukan_group_index"]


BENCH_EXPORTS = ["kan_profile_before", "kan_profile_after", "kan_profile_enable", "kan_profile_read",
                 "kan_dense_baseline_workspace_bytes", "kan_dense_baseline_forward",
                 "kan_dense_baseline_backward_workspace_bytes", "kan_dense_baseline_backward",
                 "kan_bench_ceiling_count", "kan_bench_ceiling"]


class KanLayerDesc(ctypes.Structure):
    _fields_ = [("n_in", ctypes.c_int32), ("n_out", ctypes.c_int32), ("G", ctypes.c_int32),
                ("k", ctypes.c_int32), ("grid_lo", ctypes.c_float), ("grid_hi", ctypes.c_float),
                ("base_act", ctypes.c_int32)]


class UkanLayerDesc(ctypes.Structure):
    _fields_ = [("n_in", ctypes.c_int32), ("n_out", ctypes.c_int32), ("k", ctypes.c_int32),
                ("h", ctypes.c_float), ("d_pe", ctypes.c_int32), ("d_feat", ctypes.c_int32),
                ("d_hidden", ctypes.c_int32), ("base_act", ctypes.c_int32)]


class UkanParams(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("E", "W1", "b1", "W2", "b2", "scale", "w_b")]


class UkanGrads(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("gE", "gW1", "gb1", "gW2", "gb2", "gscale", "gw_b")]


class KanKernelTime(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char_p), ("total_ms", ctypes.c_double), ("launches", ctypes.c_int64)]


class KanError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (where, strerror(status), status))


_lib = None


def load():
    """Load the built library; raise if it is missing (no CPU fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("%s is missing: build it with `python -m paper_2408_11200_amd.build`" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, sz, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t, ctypes.c_int32
    lib.kan_strerror.restype = ctypes.c_char_p
    lib.kan_strerror.argtypes = [ctypes.c_int]
    lib.kan_workspace_bytes.restype = sz
    lib.kan_workspace_bytes.argtypes = [ctypes.POINTER(KanLayerDesc), i64, ctypes.c_int]
    lib.kan_forward.restype = ctypes.c_int
    lib.kan_forward.argtypes = [ctypes.POINTER(KanLayerDesc), i64, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.kan_static_scratch_bytes.restype = sz
    lib.kan_static_scratch_bytes.argtypes = []
    lib.kan_forward_static.restype = ctypes.c_int
    lib.kan_forward_static.argtypes = [ctypes.POINTER(KanLayerDesc), i64, vp, vp, vp, vp, vp, vp]
    lib.kan_backward.restype = ctypes.c_int
    lib.kan_backward.argtypes = [ctypes.POINTER(KanLayerDesc), i64, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.kan_backward_saved.restype = ctypes.c_int
    lib.kan_backward_saved.argtypes = [ctypes.POINTER(KanLayerDesc), i64, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.kan_interval_index.restype = ctypes.c_int
    lib.kan_interval_index.argtypes = [ctypes.POINTER(KanLayerDesc), i64, vp, vp, vp]
    lib.kan_set_launch_observer.restype = ctypes.c_int
    lib.kan_set_launch_observer.argtypes = [vp, vp]
    lib.ukan_workspace_bytes.restype = sz
    lib.ukan_workspace_bytes.argtypes = [ctypes.POINTER(UkanLayerDesc), i64, i32, ctypes.c_int]
    lib.ukan_cg_forward.restype = ctypes.c_int
    lib.ukan_cg_forward.argtypes = [ctypes.POINTER(UkanLayerDesc), i64, vp, ctypes.POINTER(UkanParams), vp, i32,
                                    vp, sz, vp]
    lib.ukan_cg_backward.restype = ctypes.c_int
    lib.ukan_cg_backward.argtypes = [ctypes.POINTER(UkanLayerDesc), i64, vp, ctypes.POINTER(UkanParams), vp, vp,
                                     ctypes.POINTER(UkanGrads), i32, vp, sz, vp]
    lib.ukan_saved_bytes.restype = sz
    lib.ukan_saved_bytes.argtypes = [ctypes.POINTER(UkanLayerDesc), i32]
    lib.ukan_cg_forward_saved.restype = ctypes.c_int
    lib.ukan_cg_forward_saved.argtypes = [ctypes.POINTER(UkanLayerDesc), i64, vp, ctypes.POINTER(UkanParams), vp, i32,
                                          vp, sz, ctypes.POINTER(i32), vp, sz, vp]
    lib.ukan_cg_forward_saved_async.restype = ctypes.c_int
    lib.ukan_cg_forward_saved_async.argtypes = [ctypes.POINTER(UkanLayerDesc), i64, vp, ctypes.POINTER(UkanParams), vp, i32,
                                                i32, vp, sz, vp, vp, sz, vp]
    lib.ukan_cg_backward_saved.restype = ctypes.c_int
    lib.ukan_cg_backward_saved.argtypes = [ctypes.POINTER(UkanLayerDesc), i64, vp, ctypes.POINTER(UkanParams), vp, vp,
                                           ctypes.POINTER(UkanGrads), i32, vp, sz, i32, vp, sz, vp]
    lib.ukan_materialize_workspace_bytes.restype = ctypes.c_size_t
    lib.ukan_materialize_workspace_bytes.argtypes = [ctypes.POINTER(UkanLayerDesc), i64, i64]
    lib.ukan_materialize.restype = ctypes.c_int
    lib.ukan_materialize.argtypes = [ctypes.POINTER(UkanLayerDesc), ctypes.POINTER(UkanParams), i64, i64, vp, vp, sz, vp]
    lib.ukan_group_index.restype = ctypes.c_int
    lib.ukan_group_index.argtypes = [ctypes.POINTER(UkanLayerDesc), i64, vp, vp, vp, vp, vp]
    _lib = lib
    return lib


_bench = None


def load_bench():
    """Load the benchmark companion library (event timing, dense baseline); raise if it is missing."""
    global _bench
    if _bench is not None:
        return _bench
    if not os.path.exists(BENCH_LIB_PATH):
        raise RuntimeError("%s is missing: build it with `python -m paper_2408_11200_amd.build`" % BENCH_LIB_PATH)
    lib = ctypes.CDLL(BENCH_LIB_PATH)
    vp, i64, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t
    lib.kan_profile_enable.restype = ctypes.c_int
    lib.kan_profile_enable.argtypes = [ctypes.c_int]
    lib.kan_profile_read.restype = ctypes.c_int
    lib.kan_profile_read.argtypes = [ctypes.POINTER(KanKernelTime), ctypes.c_int]
    lib.kan_dense_baseline_workspace_bytes.restype = sz
    lib.kan_dense_baseline_workspace_bytes.argtypes = [ctypes.POINTER(KanLayerDesc), i64]
    lib.kan_dense_baseline_backward_workspace_bytes.restype = ctypes.c_size_t
    lib.kan_dense_baseline_backward_workspace_bytes.argtypes = [ctypes.POINTER(KanLayerDesc), i64]
    lib.kan_dense_baseline_backward.restype = ctypes.c_int
    lib.kan_dense_baseline_backward.argtypes = [ctypes.POINTER(KanLayerDesc), i64, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                                vp, sz, vp]
    lib.kan_dense_baseline_forward.restype = ctypes.c_int
    lib.kan_dense_baseline_forward.argtypes = [ctypes.POINTER(KanLayerDesc), i64, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.kan_bench_ceiling_count.restype = ctypes.c_int
    lib.kan_bench_ceiling_count.argtypes = []
    lib.kan_bench_ceiling.restype = ctypes.c_int
    lib.kan_bench_ceiling.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_char_p),
                                      ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(ctypes.c_double),
                                      ctypes.POINTER(ctypes.c_double)]
    _bench = lib
    return lib


def strerror(status):
    return load().kan_strerror(int(status)).decode()


def kan_desc(spec):
    """KanLayerDesc from anything with n_in, n_out, G, k, grid_lo, grid_hi, base_act."""
    return KanLayerDesc(spec.n_in, spec.n_out, spec.G, spec.k, spec.grid_lo, spec.grid_hi, spec.base_act)


def ukan_desc(spec):
    return UkanLayerDesc(spec.n_in, spec.n_out, spec.k, spec.h, spec.d_pe, spec.d_feat, spec.d_hidden,
                         spec.base_act)


def _ptr(t):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensors only"
    return ctypes.c_void_p(t.data_ptr())


def _f32(t):
    assert t is None or t.dtype == torch.float32
    return _ptr(t)


def _stream(stream):
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def _on_stream(t, stream):
    """A tensor allocated here (on torch's current stream) but used by work enqueued on another
    stream: tell the caching allocator, so the block is not handed out again, once the Python
    object is gone, before that work has finished."""
    if stream is not None and t.numel():
        t.record_stream(stream)
    return t


def _workspace(nbytes, device, stream=None):
    # torch's allocator hands out 512-byte aligned blocks
    return _on_stream(torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device), stream)


def kan_workspace_bytes(spec, B, which=PASS_FORWARD):
    d = kan_desc(spec)
    return int(load().kan_workspace_bytes(ctypes.byref(d), B, which))


def kan_forward(spec, x, coef, w_s, w_b, y=None, ws=None, stream=None):
    lib = load()
    d = kan_desc(spec)
    B = x.shape[0]
    if y is None:
        y = _on_stream(torch.empty((B, spec.n_out), dtype=torch.float32, device=x.device), stream)
    if ws is None:
        ws = _workspace(lib.kan_workspace_bytes(ctypes.byref(d), B, PASS_FORWARD), x.device, stream)
    rc = lib.kan_forward(ctypes.byref(d), B, _f32(x), _f32(coef), _f32(w_s), _f32(w_b), _f32(y),
                         _ptr(ws), ws.numel(), _stream(stream))
    if rc != KAN_OK:
        raise KanError(rc, "kan_forward")
    return y


def kan_static_scratch_bytes():
    return int(load().kan_static_scratch_bytes())


def kan_forward_static(spec, x, coef, w_s, w_b, y, stream=None):
    """kan_forward on the library's built-in scratch array: allocates nothing, so y is required."""
    d = kan_desc(spec)
    rc = load().kan_forward_static(ctypes.byref(d), x.shape[0], _f32(x), _f32(coef), _f32(w_s), _f32(w_b), _f32(y),
                                   _stream(stream))
    if rc != KAN_OK:
        raise KanError(rc, "kan_forward_static")
    return y


def kan_backward(spec, x, coef, w_s, w_b, gy, want=("gx", "gcoef", "gw_s", "gw_b"), out=None, ws=None,
                 stream=None, forward_ws=None):
    """All (or the wanted) gradients of one layer.  forward_ws: the workspace tensor a kan_forward call on the same
    layer and parameters used (kan_backward_saved: the scale-folded table is read from it, not rebuilt)."""
    lib = load()
    d = kan_desc(spec)
    B = x.shape[0]
    shapes = {"gx": (B, spec.n_in), "gcoef": (spec.n_in, spec.G + spec.k, spec.n_out),
              "gw_s": (spec.n_in, spec.n_out), "gw_b": (spec.n_in, spec.n_out)}
    out = dict(out or {})
    for name in want:
        if name not in out:
            out[name] = _on_stream(torch.empty(shapes[name], dtype=torch.float32, device=x.device), stream)
    if ws is None:
        ws = _workspace(lib.kan_workspace_bytes(ctypes.byref(d), B, PASS_BACKWARD), x.device, stream)
    if forward_ws is not None:
        rc = lib.kan_backward_saved(ctypes.byref(d), B, _f32(x), _f32(coef), _f32(w_s), _f32(w_b), _f32(gy),
                                    _ptr(forward_ws), _f32(out.get("gx")), _f32(out.get("gcoef")), _f32(out.get("gw_s")),
                                    _f32(out.get("gw_b")), _ptr(ws), ws.numel(), _stream(stream))
    else:
        rc = lib.kan_backward(ctypes.byref(d), B, _f32(x), _f32(coef), _f32(w_s), _f32(w_b), _f32(gy),
                              _f32(out.get("gx")), _f32(out.get("gcoef")), _f32(out.get("gw_s")),
                              _f32(out.get("gw_b")), _ptr(ws), ws.numel(), _stream(stream))
    if rc != KAN_OK:
        raise KanError(rc, "kan_backward_saved" if forward_ws is not None else "kan_backward")
    return out


def kan_backward_saved(spec, x, coef, w_s, w_b, gy, forward_ws, want=("gx", "gcoef", "gw_s", "gw_b"), out=None, ws=None,
                       stream=None):
    return kan_backward(spec, x, coef, w_s, w_b, gy, want=want, out=out, ws=ws, stream=stream, forward_ws=forward_ws)


def kan_interval_index(spec, x, stream=None):
    lib = load()
    d = kan_desc(spec)
    idx = _on_stream(torch.empty(x.shape, dtype=torch.int32, device=x.device), stream)
    rc = lib.kan_interval_index(ctypes.byref(d), x.numel(), _f32(x), _ptr(idx), _stream(stream))
    if rc != KAN_OK:
        raise KanError(rc, "kan_interval_index")
    return idx


def kan_dense_baseline_workspace_bytes(spec, B, which=PASS_FORWARD):
    d = kan_desc(spec)
    lib = load_bench()
    return int(lib.kan_dense_baseline_workspace_bytes(ctypes.byref(d), B) if which == PASS_FORWARD
               else lib.kan_dense_baseline_backward_workspace_bytes(ctypes.byref(d), B))


def kan_dense_baseline_forward(spec, x, coef, w_s, w_b, y=None, ws=None, stream=None):
    """Comparison baseline: the same forward pass as one dense GEMM over all basis functions."""
    lib = load_bench()
    d = kan_desc(spec)
    B = x.shape[0]
    if y is None:
        y = _on_stream(torch.empty((B, spec.n_out), dtype=torch.float32, device=x.device), stream)
    if ws is None:
        ws = _workspace(lib.kan_dense_baseline_workspace_bytes(ctypes.byref(d), B), x.device, stream)
    rc = lib.kan_dense_baseline_forward(ctypes.byref(d), B, _f32(x), _f32(coef), _f32(w_s), _f32(w_b), _f32(y),
                                        _ptr(ws), ws.numel(), _stream(stream))
    if rc != KAN_OK:
        raise KanError(rc, "kan_dense_baseline_forward")
    return y


def kan_dense_baseline_backward(spec, x, coef, w_s, w_b, gy, out=None, ws=None, stream=None):
    """Comparison baseline: the backward pass as two dense GEMMs over all basis functions."""
    lib = load_bench()
    d = kan_desc(spec)
    B = x.shape[0]
    shapes = {"gx": (B, spec.n_in), "gcoef": (spec.n_in, spec.G + spec.k, spec.n_out),
              "gw_s": (spec.n_in, spec.n_out), "gw_b": (spec.n_in, spec.n_out)}
    out = dict(out or {})
    for name in shapes:
        if name not in out:
            out[name] = _on_stream(torch.empty(shapes[name], dtype=torch.float32, device=x.device), stream)
    if ws is None:
        ws = _workspace(lib.kan_dense_baseline_backward_workspace_bytes(ctypes.byref(d), B), x.device, stream)
    rc = lib.kan_dense_baseline_backward(ctypes.byref(d), B, _f32(x), _f32(coef), _f32(w_s), _f32(w_b), _f32(gy),
                                         _f32(out["gx"]), _f32(out["gcoef"]), _f32(out["gw_s"]), _f32(out["gw_b"]),
                                         _ptr(ws), ws.numel(), _stream(stream))
    if rc != KAN_OK:
        raise KanError(rc, "kan_dense_baseline_backward")
    return out


def kan_set_launch_observer(before, after):
    """Install two C function pointers (or None) as the layer library's launch observer."""
    as_vp = lambda f: None if f is None else ctypes.cast(f, ctypes.c_void_p)
    rc = load().kan_set_launch_observer(as_vp(before), as_vp(after))
    if rc != KAN_OK:
        raise KanError(rc, "kan_set_launch_observer")


def kan_bench_ceilings(threads_per_cu=1024, iters=20000):
    """[(name, unit, units per CU per second, kernel ms)] of the benchmark library's instruction-rate microbenchmarks."""
    lib = load_bench()
    rows = []
    for q in range(lib.kan_bench_ceiling_count()):
        name, unit, rate, ms = ctypes.c_char_p(), ctypes.c_char_p(), ctypes.c_double(), ctypes.c_double()
        rc = lib.kan_bench_ceiling(q, threads_per_cu, iters, ctypes.byref(name), ctypes.byref(unit), ctypes.byref(rate),
                                   ctypes.byref(ms))
        if rc != KAN_OK:
            raise KanError(rc, "kan_bench_ceiling")
        rows.append((name.value.decode(), unit.value.decode(), rate.value, ms.value))
    return rows


def kan_profile_enable(on):
    """Start (clearing earlier records) or stop per-kernel event timing: installs the benchmark library's
    hooks as the layer library's launch observer, or removes them."""
    bench = load_bench()
    if on:
        kan_set_launch_observer(bench.kan_profile_before, bench.kan_profile_after)
    else:
        kan_set_launch_observer(None, None)
    bench.kan_profile_enable(1 if on else 0)


def kan_profile_read():
    """{kernel family: (total_ms, launches)} of the launches recorded since kan_profile_enable(True)."""
    arr = (KanKernelTime * 64)()
    n = load_bench().kan_profile_read(arr, 64)
    if n < 0:
        raise KanError(n, "kan_profile_read")
    return {arr[q].name.decode(): (arr[q].total_ms, int(arr[q].launches)) for q in range(min(n, 64))}


# ------------------------------------------------------------------ UKAN ----

_P_NAMES = ("E", "W1", "b1", "W2", "b2", "scale", "w_b")


def _ukan_params(p):
    return UkanParams(*[(_f32(p.get(n)).value if p.get(n) is not None else None) for n in _P_NAMES])


def ukan_workspace_bytes(spec, B, max_groups, which=PASS_FORWARD):
    d = ukan_desc(spec)
    return int(load().ukan_workspace_bytes(ctypes.byref(d), B, max_groups, which))


def ukan_cg_forward(spec, x, p, max_groups, y=None, ws=None, stream=None):
    lib = load()
    d = ukan_desc(spec)
    B = x.shape[0]
    if y is None:
        y = _on_stream(torch.empty((B, spec.n_out), dtype=torch.float32, device=x.device), stream)
    if ws is None:
        ws = _workspace(lib.ukan_workspace_bytes(ctypes.byref(d), B, max_groups, PASS_FORWARD), x.device, stream)
    pp = _ukan_params(p)
    rc = lib.ukan_cg_forward(ctypes.byref(d), B, _f32(x), ctypes.byref(pp), _f32(y), max_groups, _ptr(ws),
                             ws.numel(), _stream(stream))
    if rc != KAN_OK:
        raise KanError(rc, "ukan_cg_forward")
    return y


def ukan_saved_bytes(spec, max_groups):
    d = ukan_desc(spec)
    return int(load().ukan_saved_bytes(ctypes.byref(d), max_groups))


def ukan_cg_forward_saved(spec, x, p, max_groups, saved=None, y=None, ws=None, stream=None):
    """ukan_cg_forward that keeps its intermediates for ukan_cg_backward_saved: returns (y, saved, span)."""
    lib = load()
    d = ukan_desc(spec)
    B = x.shape[0]
    if y is None:
        y = _on_stream(torch.empty((B, spec.n_out), dtype=torch.float32, device=x.device), stream)
    if saved is None:
        saved = _workspace(lib.ukan_saved_bytes(ctypes.byref(d), max_groups), x.device, stream)
    if ws is None:
        ws = _workspace(lib.ukan_workspace_bytes(ctypes.byref(d), B, max_groups, PASS_FORWARD), x.device, stream)
    pp = _ukan_params(p)
    span = ctypes.c_int32(0)
    rc = lib.ukan_cg_forward_saved(ctypes.byref(d), B, _f32(x), ctypes.byref(pp), _f32(y), max_groups, _ptr(saved),
                                   saved.numel(), ctypes.byref(span), _ptr(ws), ws.numel(), _stream(stream))
    if rc != KAN_OK:
        raise KanError(rc, "ukan_cg_forward_saved")
    return y, saved, int(span.value)


def ukan_cg_forward_saved_async(spec, x, p, max_groups, n_groups, saved, overflow, y, ws, stream=None):
    """ukan_cg_forward_saved for a caller-stated span: no read-back, no allocation (every buffer is passed
    in); overflow is a device int32 tensor of one element that receives 1 when n_groups was too small."""
    d = ukan_desc(spec)
    pp = _ukan_params(p)
    assert overflow.dtype == torch.int32 and overflow.numel() >= 1
    rc = load().ukan_cg_forward_saved_async(ctypes.byref(d), x.shape[0], _f32(x), ctypes.byref(pp), _f32(y), max_groups,
                                            int(n_groups), _ptr(saved), saved.numel(), _ptr(overflow), _ptr(ws),
                                            ws.numel(), _stream(stream))
    if rc != KAN_OK:
        raise KanError(rc, "ukan_cg_forward_saved_async")
    return y


def ukan_cg_backward(spec, x, p, gy, max_groups, want=None, out=None, ws=None, stream=None, saved=None, span=None):
    """All gradients of one UKAN layer.  With `saved` and `span` from ukan_cg_forward_saved the call is
    ukan_cg_backward_saved (no recomputation of the coefficient table, no synchronisation)."""
    lib = load()
    d = ukan_desc(spec)
    B = x.shape[0]
    K = spec.k + 1
    shapes = {"gx": (B, spec.n_in), "gE": (spec.n_in, spec.d_feat),
              "gW1": (spec.d_feat + spec.d_pe, spec.d_hidden), "gb1": (spec.d_hidden,),
              "gW2": (spec.d_hidden, K * spec.n_out), "gb2": (K * spec.n_out,),
              "gscale": (spec.n_in, spec.n_out), "gw_b": (spec.n_in, spec.n_out)}
    if want is None:
        want = [n for n in shapes if n != "gw_b" or spec.base_act]
    if out is None:
        out = {n: _on_stream(torch.empty(shapes[n], dtype=torch.float32, device=x.device), stream) for n in want}
    if ws is None:
        ws = _workspace(lib.ukan_workspace_bytes(ctypes.byref(d), B, max_groups, PASS_BACKWARD), x.device, stream)
    pp = _ukan_params(p)
    gg = UkanGrads(*[(out[n].data_ptr() if n in out else None)
                     for n in ("gE", "gW1", "gb1", "gW2", "gb2", "gscale", "gw_b")])
    if saved is not None:
        rc = lib.ukan_cg_backward_saved(ctypes.byref(d), B, _f32(x), ctypes.byref(pp), _f32(gy), _f32(out.get("gx")),
                                        ctypes.byref(gg), max_groups, _ptr(saved), saved.numel(), int(span), _ptr(ws),
                                        ws.numel(), _stream(stream))
    else:
        rc = lib.ukan_cg_backward(ctypes.byref(d), B, _f32(x), ctypes.byref(pp), _f32(gy), _f32(out.get("gx")),
                                  ctypes.byref(gg), max_groups, _ptr(ws), ws.numel(), _stream(stream))
    if rc != KAN_OK:
        raise KanError(rc, "ukan_cg_backward_saved" if saved is not None else "ukan_cg_backward")
    return out


def ukan_cg_backward_saved(spec, x, p, gy, max_groups, saved, span, want=None, out=None, ws=None, stream=None):
    return ukan_cg_backward(spec, x, p, gy, max_groups, want=want, out=out, ws=ws, stream=stream, saved=saved,
                            span=span)


def ukan_materialize(spec, p, cell_lo, cell_hi, coef=None, ws=None, stream=None):
    """Coefficients [n_in][cell_hi - cell_lo + 1 + k][n_out] of the KAN layer equal to this UKAN layer on the cells."""
    lib = load()
    d = ukan_desc(spec)
    dev = p["E"].device
    if coef is None:
        coef = _on_stream(torch.empty((spec.n_in, int(cell_hi) - int(cell_lo) + 1 + spec.k, spec.n_out),
                                      dtype=torch.float32, device=dev), stream)
    if ws is None:
        ws = _workspace(lib.ukan_materialize_workspace_bytes(ctypes.byref(d), int(cell_lo), int(cell_hi)), dev, stream)
    pp = _ukan_params(p)
    rc = lib.ukan_materialize(ctypes.byref(d), ctypes.byref(pp), int(cell_lo), int(cell_hi), _f32(coef), _ptr(ws),
                              ws.numel(), _stream(stream))
    if rc != KAN_OK:
        raise KanError(rc, "ukan_materialize")
    return coef


def ukan_group_index(spec, x, stream=None):
    lib = load()
    d = ukan_desc(spec)
    outs = [_on_stream(torch.empty(x.shape, dtype=torch.int32, device=x.device), stream) for _ in range(3)]
    rc = lib.ukan_group_index(ctypes.byref(d), x.numel(), _f32(x), _ptr(outs[0]), _ptr(outs[1]), _ptr(outs[2]),
                              _stream(stream))
    if rc != KAN_OK:
        raise KanError(rc, "ukan_group_index")
    return tuple(outs)
