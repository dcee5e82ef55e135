"""Device-memory plumbing around the C-ABI binding: allocates torch tensors, uploads a workload,
calls forward/backward and downloads results.  No arithmetic of the method happens here."""
import numpy as np
import torch

from . import binding as B


class DagRunner:
    """Owns one compiled micro-DAG plus the device buffers of one workload."""

    def __init__(self, blob, shape, dtype, flags=0, device="cuda:0"):
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the micro-DAG executor has no CPU path")
        self.device = torch.device(device)
        self.bf16 = dtype == "bf16"
        self.tdtype = torch.bfloat16 if self.bf16 else torch.float32
        self.handle = B.canvas_dag_compile(blob, shape, B.CANVAS_BF16 if self.bf16 else B.CANVAS_F32, flags)
        self.info = B.canvas_dag_query(self.handle)
        self.shape = tuple(int(v) for v in shape)
        self.out_shape = tuple(int(v) for v in self.info.out_shape)
        self.wshapes = [tuple(int(v) for v in self.info.weight_shape[k]) for k in range(self.info.n_weights)]
        self.ws = torch.empty(max(16, int(self.info.workspace_bytes)), dtype=torch.uint8, device=self.device)
        self.x = torch.empty(self.shape, dtype=self.tdtype, device=self.device)
        self.y = torch.empty(self.out_shape, dtype=self.tdtype, device=self.device)
        self.dy = torch.empty(self.out_shape, dtype=self.tdtype, device=self.device)
        self.dx = torch.empty(self.shape, dtype=self.tdtype, device=self.device)
        self.w = [torch.empty(s, dtype=self.tdtype, device=self.device) for s in self.wshapes]
        self.dw = [torch.empty(s, dtype=torch.float32, device=self.device) for s in self.wshapes]

    def close(self):
        if self.handle is not None:
            B.canvas_dag_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _up(self, dst, a):
        dst.copy_(torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).reshape(dst.shape).to(self.tdtype))

    def load(self, x, weights, dy=None):
        self._up(self.x, x)
        for t, a in zip(self.w, weights):
            self._up(t, a)
        if dy is not None:
            self._up(self.dy, dy)

    def prepare(self):
        B.canvas_dag_prepare(self.handle, self.w, self.ws)

    def forward(self):
        B.canvas_dag_forward(self.handle, self.x, self.w, self.y, self.ws)

    def backward(self):
        B.canvas_dag_backward(self.handle, self.x, self.w, self.dy, self.dx, self.dw, self.ws)

    def poison_outputs(self):
        """Fill outputs with NaN so that an element no kernel writes is caught."""
        for t in [self.y, self.dx, *self.dw]:
            t.fill_(float("nan"))

    def results(self):
        torch.cuda.synchronize()
        out = {"y": self.y.float().cpu().numpy(), "dx": self.dx.float().cpu().numpy(),
               "dw": [t.cpu().numpy() for t in self.dw]}
        if out["y"].shape[2] == 1:
            out["y"] = out["y"].reshape(out["y"].shape[0], out["y"].shape[1], *out["y"].shape[3:])
        return out

    def launches(self, backward):
        n = self.info.n_launches_bwd if backward else self.info.n_launches_fwd
        return [B.canvas_dag_launch_desc(self.handle, backward, i) for i in range(n)]


class BlockRunner:
    """Owns one compiled block (a template composed for C_in != C_out) plus the device buffers of one workload."""

    def __init__(self, blob, shape, c_out, dtype, flags=0, device="cuda:0"):
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the micro-DAG executor has no CPU path")
        self.device = torch.device(device)
        self.bf16 = dtype == "bf16"
        self.tdtype = torch.bfloat16 if self.bf16 else torch.float32
        self.handle = B.canvas_block_compile(blob, shape, c_out, B.CANVAS_BF16 if self.bf16 else B.CANVAS_F32, flags)
        self.info = B.canvas_block_query(self.handle)
        n, _, h, w = (int(v) for v in shape)
        self.m = int(self.info.instances)
        wshapes = [tuple(int(v) for v in self.info.plan.weight_shape[k]) for k in range(self.info.n_weights)]
        self.ws = torch.empty(max(16, int(self.info.workspace_bytes)), dtype=torch.uint8, device=self.device)
        self.x = torch.empty(tuple(int(v) for v in shape), dtype=self.tdtype, device=self.device)
        self.y = torch.empty((n, int(c_out), h, w), dtype=self.tdtype, device=self.device)
        self.dy = torch.empty_like(self.y)
        self.dx = torch.empty_like(self.x)
        self.w = [torch.empty(s, dtype=self.tdtype, device=self.device) for _ in range(self.m) for s in wshapes]
        self.dw = [torch.empty(s, dtype=torch.float32, device=self.device) for _ in range(self.m) for s in wshapes]

    def close(self):
        if self.handle is not None:
            B.canvas_block_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _up(self, dst, a):
        dst.copy_(torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).reshape(dst.shape).to(self.tdtype))

    def load(self, x, weights, dy):
        """weights: m lists (one per instance) of arrays."""
        self._up(self.x, x)
        flat = [a for inst in weights for a in inst]
        for t, a in zip(self.w, flat):
            self._up(t, a)
        self._up(self.dy, dy)

    def run(self):
        for t in [self.y, self.dx, *self.dw]:
            t.fill_(float("nan"))
        self.ws.fill_(0xFF)  # (bf16 / fp32 NaN patterns: nothing may be read before it is written)
        B.canvas_block_forward(self.handle, self.x, self.w, self.y, self.ws)
        B.canvas_block_backward(self.handle, self.x, self.w, self.dy, self.dx, self.dw, self.ws)
        torch.cuda.synchronize()
        nw = int(self.info.n_weights)
        dw = [t.cpu().numpy() for t in self.dw]
        return {"y": self.y.float().cpu().numpy(), "dx": self.dx.float().cpu().numpy(),
                "dw": [dw[j * nw:(j + 1) * nw] for j in range(self.m)]}


def run_case(case, flags=0, dy=None):
    """Upload a workload (see workloads.py), run forward + backward, return (results, runner)."""
    from . import workloads as wl

    r = DagRunner(case["blob"], case["shape"], case["dtype"], flags)
    if dy is None:
        shp = r.out_shape if r.out_shape[2] != 1 else (r.out_shape[0], r.out_shape[1], *r.out_shape[3:])
        dy = wl.make_dy(case, shp)
    r.load(case["x"], case["weights"], dy)
    r.poison_outputs()
    r.forward()
    r.backward()
    return r.results(), r, dy
