"""Thin ctypes binding of the C-ABI library (argument marshalling only).

Function names mirror include/canvas_dag.h.  Tensors are torch tensors used
purely as device memory; the stream is torch's current HIP stream.  Nothing
here computes: every step of forward and backward runs in the library's kernels.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcanvas_dag.so")

CANVAS_F32, CANVAS_BF16 = 0, 1
CANVAS_OPT_NO_FUSION = 1
CANVAS_OPT_INFERENCE = 2
CANVAS_MAX_NODES = 64
STATUS = {0: "OK", -1: "INVALID_BLOB", -2: "UNKNOWN_OP", -3: "SHAPE_MISMATCH", -4: "BAD_ARG",
          -5: "WORKSPACE_TOO_SMALL", -6: "UNSUPPORTED", -7: "HIP_ERROR"}
CANVAS_STATIC_WORKSPACE_BYTES = 64 << 20
EXPORTS = ["canvas_dag_compile", "canvas_dag_query", "canvas_dag_launch_desc", "canvas_dag_forward", "canvas_dag_forward_static",
           "canvas_dag_backward", "canvas_dag_prepare", "canvas_dag_set_timing", "canvas_dag_get_timing", "canvas_dag_destroy",
           "canvas_last_error"]
# include/canvas_template.h (host only)
TEMPLATE_EXPORTS = ["canvas_template_parse", "canvas_template_query", "canvas_template_node_shape", "canvas_template_substitutions",
                    "canvas_template_substitute", "canvas_group_candidates", "canvas_template_solve",
                    "canvas_template_instantiate", "canvas_template_destroy"]
CANVAS_MAX_VARS = 8
# include/canvas_block.h
BLOCK_EXPORTS = ["canvas_block_compile", "canvas_block_query", "canvas_block_forward", "canvas_block_backward", "canvas_block_destroy"]


class CanvasOptions(ctypes.Structure):
    _fields_ = [("flags", ctypes.c_uint32), ("reserved", ctypes.c_uint32 * 7)]


class CanvasDagInfo(ctypes.Structure):
    _fields_ = [
        ("n_nodes", ctypes.c_int32), ("out_node", ctypes.c_int32), ("n_weights", ctypes.c_int32),
        ("n_launches_fwd", ctypes.c_int32), ("n_launches_bwd", ctypes.c_int32), ("fused", ctypes.c_int32),
        ("n_launches_prepare", ctypes.c_int32), ("n_fused_chains", ctypes.c_int32),
        ("out_shape", ctypes.c_int64 * 5),
        ("node_shape", (ctypes.c_int64 * 5) * CANVAS_MAX_NODES),
        ("weight_shape", (ctypes.c_int64 * 3) * CANVAS_MAX_NODES),
        ("weight_node", ctypes.c_int32 * CANVAS_MAX_NODES),
        ("workspace_bytes", ctypes.c_uint64),
        ("fc_flops_fwd", ctypes.c_double), ("min_bytes_fwd", ctypes.c_double), ("min_bytes_bwd", ctypes.c_double),
        ("n_fused_nodes", ctypes.c_int32), ("reserved1", ctypes.c_int32),
    ]


class CanvasBlockInfo(ctypes.Structure):
    _fields_ = [("instances", ctypes.c_int32), ("expand", ctypes.c_int32), ("template_channels", ctypes.c_int64),
                ("n_weights", ctypes.c_int32), ("reserved0", ctypes.c_int32), ("workspace_bytes", ctypes.c_uint64),
                ("plan", CanvasDagInfo)]


class CanvasTarget(ctypes.Structure):
    _fields_ = [("C", ctypes.c_int64), ("KH", ctypes.c_int64), ("KW", ctypes.c_int64), ("H", ctypes.c_int64), ("W", ctypes.c_int64)]


class CanvasTemplateInfo(ctypes.Structure):
    _fields_ = [("n_nodes", ctypes.c_int32), ("out_node", ctypes.c_int32), ("n_fc", ctypes.c_int32), ("n_free", ctypes.c_int32),
                ("free_var", ctypes.c_int32 * CANVAS_MAX_VARS), ("uses_G", ctypes.c_int32), ("reserved", ctypes.c_int32 * 5)]


class CanvasSolveResult(ctypes.Structure):
    _fields_ = [("flops", ctypes.c_double), ("params", ctypes.c_double), ("rounds", ctypes.c_int32), ("reserved", ctypes.c_int32 * 7)]


class CanvasLaunchDesc(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char * 64), ("bytes", ctypes.c_double), ("flops", ctypes.c_double)]


class CanvasError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"{STATUS.get(status, status)}: {message}")
        self.status = status


_lib = None


def load():
    """Load the HIP library; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` first")
        lib = ctypes.CDLL(LIB_PATH)
        vp, sz = ctypes.c_void_p, ctypes.c_size_t
        lib.canvas_dag_compile.argtypes = [ctypes.c_char_p, sz, ctypes.POINTER(ctypes.c_int64), ctypes.c_int,
                                           ctypes.POINTER(CanvasOptions), ctypes.POINTER(vp)]
        lib.canvas_dag_query.argtypes = [vp, ctypes.POINTER(CanvasDagInfo)]
        lib.canvas_dag_launch_desc.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.POINTER(CanvasLaunchDesc)]
        lib.canvas_dag_forward.argtypes = [vp, vp, ctypes.POINTER(vp), vp, vp, sz, vp]
        lib.canvas_dag_forward_static.argtypes = [vp, vp, ctypes.POINTER(vp), vp, vp]
        lib.canvas_dag_backward.argtypes = [vp, vp, ctypes.POINTER(vp), vp, vp, ctypes.POINTER(vp), vp, sz, vp]
        lib.canvas_dag_prepare.argtypes = [vp, ctypes.POINTER(vp), vp, sz, vp]
        lib.canvas_dag_set_timing.argtypes = [vp, ctypes.c_int]
        lib.canvas_dag_get_timing.argtypes = [vp, ctypes.c_int, ctypes.POINTER(ctypes.c_float), ctypes.c_int]
        lib.canvas_dag_destroy.argtypes = [vp]
        lib.canvas_dag_destroy.restype = None
        lib.canvas_last_error.restype = ctypes.c_char_p
        ip, szp = ctypes.POINTER(ctypes.c_int), ctypes.POINTER(sz)
        lib.canvas_template_parse.argtypes = [ctypes.c_char_p, sz, ctypes.POINTER(vp)]
        lib.canvas_template_query.argtypes = [vp, ctypes.POINTER(CanvasTemplateInfo)]
        lib.canvas_template_node_shape.argtypes = [vp, ctypes.c_int, ctypes.c_char_p, sz, szp]
        lib.canvas_template_substitutions.argtypes = [vp, ctypes.c_int, ip, ip, ctypes.c_char_p, sz, szp]
        lib.canvas_template_substitute.argtypes = [vp, ctypes.c_int, ctypes.c_char_p]
        lib.canvas_group_candidates.argtypes = [ctypes.POINTER(ctypes.c_int64), ctypes.c_int, ctypes.POINTER(ctypes.c_int64), ctypes.c_int, ip]
        lib.canvas_template_solve.argtypes = [vp, ctypes.POINTER(CanvasTarget), ctypes.c_int, ctypes.c_int64, ctypes.c_double,
                                              ctypes.c_double, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(CanvasSolveResult)]
        lib.canvas_template_instantiate.argtypes = [vp, ctypes.POINTER(CanvasTarget), ctypes.c_int64, ctypes.POINTER(ctypes.c_int64),
                                                    ctypes.c_char_p, sz, szp]
        lib.canvas_template_destroy.argtypes = [vp]
        lib.canvas_template_destroy.restype = None
        lib.canvas_block_compile.argtypes = [ctypes.c_char_p, sz, ctypes.POINTER(ctypes.c_int64), ctypes.c_int64, ctypes.c_int,
                                             ctypes.POINTER(CanvasOptions), ctypes.POINTER(vp)]
        lib.canvas_block_query.argtypes = [vp, ctypes.POINTER(CanvasBlockInfo)]
        lib.canvas_block_forward.argtypes = [vp, vp, ctypes.POINTER(vp), vp, vp, sz, vp]
        lib.canvas_block_backward.argtypes = [vp, vp, ctypes.POINTER(vp), vp, vp, ctypes.POINTER(vp), vp, sz, vp]
        lib.canvas_block_destroy.argtypes = [vp]
        lib.canvas_block_destroy.restype = None
        _lib = lib
    return _lib


def _check(rc):
    if rc != 0:
        raise CanvasError(rc, load().canvas_last_error().decode())


def canvas_dag_compile(blob, in_shape, dtype, flags=0):
    """Returns an opaque handle (int).  dtype: CANVAS_F32 or CANVAS_BF16."""
    lib = load()
    b = blob.encode() if isinstance(blob, str) else bytes(blob)
    shp = (ctypes.c_int64 * 4)(*[int(v) for v in in_shape])
    opt = CanvasOptions(flags=flags)
    h = ctypes.c_void_p()
    _check(lib.canvas_dag_compile(b, len(b), shp, int(dtype), ctypes.byref(opt), ctypes.byref(h)))
    return h


def canvas_dag_query(handle):
    info = CanvasDagInfo()
    _check(load().canvas_dag_query(handle, ctypes.byref(info)))
    return info


def canvas_dag_launch_desc(handle, backward, idx):
    d = CanvasLaunchDesc()
    _check(load().canvas_dag_launch_desc(handle, int(backward), int(idx), ctypes.byref(d)))
    return {"name": d.name.decode(), "bytes": d.bytes, "flops": d.flops}


def _ptrs(tensors):
    arr = (ctypes.c_void_p * max(1, len(tensors)))()
    for i, t in enumerate(tensors):
        arr[i] = t.data_ptr()
    return arr


def _stream():
    import torch

    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def canvas_dag_forward(handle, x, weights, y, workspace):
    _check(load().canvas_dag_forward(handle, x.data_ptr(), _ptrs(weights), y.data_ptr(), workspace.data_ptr(),
                                     workspace.numel() * workspace.element_size(), _stream()))


def canvas_dag_forward_static(handle, x, weights, y):
    """canvas_dag_forward on the library's static workspace (no allocation anywhere)."""
    _check(load().canvas_dag_forward_static(handle, x.data_ptr(), _ptrs(weights), y.data_ptr(), _stream()))


def canvas_dag_backward(handle, x, weights, dy, dx, dweights, workspace):
    _check(load().canvas_dag_backward(handle, x.data_ptr(), _ptrs(weights), dy.data_ptr(), dx.data_ptr(),
                                      _ptrs(dweights), workspace.data_ptr(),
                                      workspace.numel() * workspace.element_size(), _stream()))


def canvas_dag_prepare(handle, weights, workspace):
    """Inference plans only: derive what depends on the weights alone (packed / widened copies) into the workspace."""
    _check(load().canvas_dag_prepare(handle, _ptrs(weights), workspace.data_ptr(),
                                     workspace.numel() * workspace.element_size(), _stream()))


def canvas_dag_set_timing(handle, enable):
    _check(load().canvas_dag_set_timing(handle, int(enable)))


def canvas_dag_get_timing(handle, backward, n):
    """Per-launch durations (ms) of the last timed forward or backward call."""
    ms = (ctypes.c_float * max(1, n))()
    _check(load().canvas_dag_get_timing(handle, int(backward), ms, int(n)))
    return [float(ms[i]) for i in range(n)]


def canvas_dag_destroy(handle):
    load().canvas_dag_destroy(handle)


# ---------------------------------------------------------------- blocks with C_in != C_out (include/canvas_block.h)

def canvas_block_compile(blob, in_shape, c_out, dtype, flags=0):
    lib = load()
    b = blob.encode() if isinstance(blob, str) else bytes(blob)
    shp = (ctypes.c_int64 * 4)(*[int(v) for v in in_shape])
    opt = CanvasOptions(flags=flags)
    h = ctypes.c_void_p()
    _check(lib.canvas_block_compile(b, len(b), shp, int(c_out), int(dtype), ctypes.byref(opt), ctypes.byref(h)))
    return h


def canvas_block_query(handle):
    info = CanvasBlockInfo()
    _check(load().canvas_block_query(handle, ctypes.byref(info)))
    return info


def canvas_block_forward(handle, x, weights, y, workspace):
    """weights: flat list, instance-major (all weight tensors of instance 0 first)."""
    _check(load().canvas_block_forward(handle, x.data_ptr(), _ptrs(weights), y.data_ptr(), workspace.data_ptr(),
                                       workspace.numel() * workspace.element_size(), _stream()))


def canvas_block_backward(handle, x, weights, dy, dx, dweights, workspace):
    _check(load().canvas_block_backward(handle, x.data_ptr(), _ptrs(weights), dy.data_ptr(), dx.data_ptr(), _ptrs(dweights),
                                        workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream()))


def canvas_block_destroy(handle):
    load().canvas_block_destroy(handle)


# ---------------------------------------------------------------- templates (include/canvas_template.h), host only

def _text(call):
    """Run call(buf, len, needed_ptr) with a buffer that is grown once if the library asks for more."""
    n = 4096
    for _ in range(2):
        buf = ctypes.create_string_buffer(n)
        needed = ctypes.c_size_t(0)
        rc = call(buf, n, ctypes.byref(needed))
        if rc == 0:
            return buf.value.decode()
        if needed.value <= n:
            break
        n = needed.value
    _check(rc)


def canvas_template_parse(blob):
    b = blob.encode() if isinstance(blob, str) else bytes(blob)
    h = ctypes.c_void_p()
    _check(load().canvas_template_parse(b, len(b), ctypes.byref(h)))
    return h


def canvas_template_query(handle):
    info = CanvasTemplateInfo()
    _check(load().canvas_template_query(handle, ctypes.byref(info)))
    return info


def canvas_template_node_shape(handle, node):
    return _text(lambda buf, n, need: load().canvas_template_node_shape(handle, int(node), buf, n, need))


def canvas_template_substitutions(handle, node):
    """Returns (j of the LHS variable x_j, list of substitution expressions)."""
    var, count = ctypes.c_int(0), ctypes.c_int(0)
    text = _text(lambda buf, n, need: load().canvas_template_substitutions(handle, int(node), ctypes.byref(var), ctypes.byref(count), buf, n, need))
    subs = text.split("\n")[:-1] if text else []
    assert len(subs) == count.value
    return var.value, subs


def canvas_template_substitute(handle, var, expr):
    _check(load().canvas_template_substitute(handle, int(var), expr.encode()))


def canvas_group_candidates(channels):
    c = (ctypes.c_int64 * len(channels))(*[int(v) for v in channels])
    out = (ctypes.c_int64 * 4096)()
    n = ctypes.c_int(0)
    _check(load().canvas_group_candidates(c, len(channels), out, 4096, ctypes.byref(n)))
    return [int(out[i]) for i in range(n.value)]


def _targets(targets):
    arr = (CanvasTarget * len(targets))()
    for i, t in enumerate(targets):
        arr[i] = CanvasTarget(*[int(t[k]) for k in ("C", "KH", "KW", "H", "W")])
    return arr


def canvas_template_solve(handle, targets, G, flops_budget=0.0, params_budget=0.0):
    """targets: list of dicts with C, KH, KW, H, W.  Returns (x[i] = {j: x_ij}, flops, params, rounds)."""
    arr = _targets(targets)
    x = (ctypes.c_int64 * (len(targets) * CANVAS_MAX_VARS))()
    res = CanvasSolveResult()
    _check(load().canvas_template_solve(handle, arr, len(targets), int(G), float(flops_budget), float(params_budget), x, ctypes.byref(res)))
    xs = [{j + 1: int(x[i * CANVAS_MAX_VARS + j]) for j in range(CANVAS_MAX_VARS) if x[i * CANVAS_MAX_VARS + j]} for i in range(len(targets))]
    return xs, res.flops, res.params, res.rounds


def canvas_template_instantiate(handle, target, G, x):
    arr = _targets([target])
    xv = (ctypes.c_int64 * CANVAS_MAX_VARS)(*[int(x.get(j + 1, 0)) for j in range(CANVAS_MAX_VARS)])
    return _text(lambda buf, n, need: load().canvas_template_instantiate(handle, arr, int(G), xv, buf, n, need))


def canvas_template_destroy(handle):
    load().canvas_template_destroy(handle)
