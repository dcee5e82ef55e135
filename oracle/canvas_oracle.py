"""ctypes loader for the fp64 CPU oracle (test infrastructure, not product code).

`build()` compiles `canvas_oracle.c` with gcc; `run()` marshals numpy arrays in
and out.  All arithmetic lives in the C file; this module only moves data.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "canvas_oracle.c")
_LIB = os.path.join(_HERE, "libcanvas_oracle.so")
CFLAGS = ["-O2", "-fopenmp", "-std=c99", "-fPIC", "-shared", "-Wall", "-Wextra"]
_lib = None


def build(force=False):
    """Compile the oracle (gcc -O2 -fopenmp).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", *CFLAGS, "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.canvas_oracle_infer.restype = ctypes.c_int
        lib.canvas_oracle_run.restype = ctypes.c_int
        lib.canvas_oracle_set_tie_margin.restype = None
        lib.canvas_oracle_set_tie_rule.restype = None
        _lib = lib
    return _lib


class OracleError(ValueError):
    pass


def infer(blob, in_shape):
    """Shape inference.  Returns (node_shapes [[C,T,H,W]...], out_node, weight_shapes [[G,Og,K]...])."""
    lib = _load()
    b = blob.encode() if isinstance(blob, str) else bytes(blob)
    shp = (ctypes.c_int64 * 4)(*[int(v) for v in in_shape])
    shapes = (ctypes.c_int64 * (4 * 64))()
    wshapes = (ctypes.c_int64 * (3 * 64))()
    n_nodes, out_node, n_w = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    err = ctypes.create_string_buffer(256)
    rc = lib.canvas_oracle_infer(b, ctypes.c_size_t(len(b)), shp, 64, shapes, ctypes.byref(n_nodes),
                                 ctypes.byref(out_node), 64, wshapes, ctypes.byref(n_w), err, ctypes.c_size_t(256))
    if rc != 0:
        raise OracleError(err.value.decode())
    ns = [[int(shapes[4 * k + j]) for j in range(4)] for k in range(n_nodes.value)]
    ws = [[int(wshapes[3 * k + j]) for j in range(3)] for k in range(n_w.value)]
    return ns, out_node.value, ws


def run(blob, x, weights, dy=None, n_threads=0, tie_margin=0.0, tie_rule=0):
    """Run the DAG on fp64 copies of the inputs.

    tie_margin: 0 = the definitions; a non-zero value moves every backward decision point (relu, abs, clip
    bounds, min / max, arg-max of a max fold) by that fraction of the deciding tensor's largest magnitude
    (see the C file), which the comparison rule of the tests uses to bracket near-ties; tie_rule selects which
    decisions move (0 all, 1 / 2 even / odd element index, 3 runner-up of a max fold).

    x: [N,C,H,W]; weights: list of [G,Og,K]; dy: like the output or None.
    Returns dict(y=[N,C,T,H,W] squeezed to [N,C,H,W] when T==1, dx, dw=list, threads).
    """
    lib = _load()
    b = blob.encode() if isinstance(blob, str) else bytes(blob)
    x = np.ascontiguousarray(x, dtype=np.float64)
    assert x.ndim == 4
    ns, out_node, ws = infer(b, x.shape)
    assert len(weights) == len(ws), "wrong number of weight tensors"
    wl = []
    for w, s in zip(weights, ws):
        w = np.ascontiguousarray(w, dtype=np.float64)
        assert w.size == s[0] * s[1] * s[2], f"weight has {w.size} elements, expected shape {s}"
        wl.append(w.reshape(s))
    N = x.shape[0]
    C, T, H, W = ns[out_node]
    y = np.empty((N, C, T, H, W), dtype=np.float64)
    dbl_p = ctypes.POINTER(ctypes.c_double)
    warr = (dbl_p * max(1, len(wl)))(*[w.ctypes.data_as(dbl_p) for w in wl])
    dx = None
    dwl = []
    dy_p = None
    dx_p = None
    dwarr = (dbl_p * max(1, len(wl)))()
    if dy is not None:
        dy = np.ascontiguousarray(dy, dtype=np.float64).reshape(y.shape)
        dx = np.empty_like(x)
        dwl = [np.empty_like(w) for w in wl]
        dy_p = dy.ctypes.data_as(dbl_p)
        dx_p = dx.ctypes.data_as(dbl_p)
        for k, d in enumerate(dwl):
            dwarr[k] = d.ctypes.data_as(dbl_p)
    shp = (ctypes.c_int64 * 4)(*x.shape)
    err = ctypes.create_string_buffer(256)
    lib.canvas_oracle_set_tie_margin(ctypes.c_double(float(tie_margin)))
    lib.canvas_oracle_set_tie_rule(ctypes.c_int(int(tie_rule)))
    try:
        rc = _call_run(lib, b, shp, x, warr, wl, dy_p, y, dx_p, dwarr, n_threads, err, dbl_p)
    finally:
        lib.canvas_oracle_set_tie_margin(ctypes.c_double(0.0))
        lib.canvas_oracle_set_tie_rule(ctypes.c_int(0))
    if rc < 0:
        raise OracleError(err.value.decode())
    if T == 1:
        y = y.reshape(N, C, H, W)
    return {"y": y, "dx": dx, "dw": dwl, "threads": rc}


def _call_run(lib, b, shp, x, warr, wl, dy_p, y, dx_p, dwarr, n_threads, err, dbl_p):
    return lib.canvas_oracle_run(b, ctypes.c_size_t(len(b)), shp, x.ctypes.data_as(dbl_p), warr, len(wl), dy_p,
                               y.ctypes.data_as(dbl_p), dx_p, dwarr, int(n_threads), err, ctypes.c_size_t(256))
