"""canvas_dag_forward_static (the forward pass on the library's static workspace, for callers that cannot
allocate device memory) against canvas_dag_forward on a caller's workspace: the same kernels, so the results
must be identical bit for bit.  Two calls in a row, the second with a smaller input; then an inference plan."""
import pytest

from paper_2304_07741_amd import binding as B
from paper_2304_07741_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _both_ways(h, case, flags=0):
    import torch

    r = h.DagRunner(case["blob"], case["shape"], case["dtype"], flags)
    assert int(r.info.workspace_bytes) <= B.CANVAS_STATIC_WORKSPACE_BYTES
    r.load(case["x"], case["weights"])
    r.y.fill_(float("nan"))
    if flags & B.CANVAS_OPT_INFERENCE:
        r.prepare()
    r.forward()
    torch.cuda.synchronize()
    want = r.y.clone()
    r.y.fill_(float("nan"))
    B.canvas_dag_forward_static(r.handle, r.x, r.w, r.y)
    torch.cuda.synchronize()
    assert torch.isfinite(r.y.float()).all()
    assert torch.equal(r.y.view(torch.int16 if r.bf16 else torch.int32), want.view(torch.int16 if r.bf16 else torch.int32))
    r.close()


def test_forward_on_the_static_workspace_equals_forward_on_a_caller_workspace():
    import torch

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2304_07741_amd import harness as h

    _both_ways(h, wl.config3(N=3, C=64, H=14))           # FC, softmax, window weights, FC: intermediates and packed weights in the workspace
    _both_ways(h, wl.config3(N=1, C=32, H=6))            # a smaller input right after: the array still holds the first call's contents
    _both_ways(h, wl.config4(64, 12, N=2))
    _both_ways(h, wl.config5(104, N=2, C=96, H=8), B.CANVAS_OPT_NO_FUSION)
    _both_ways(h, wl.config4(64, 8, N=1), B.CANVAS_OPT_INFERENCE)   # weight-only launches run inside the call
    _both_ways(h, wl.config1())


def test_a_plan_beyond_the_static_workspace_is_rejected_without_a_launch():
    case = wl.config4(64, 56, N=128)
    hd = B.canvas_dag_compile(case["blob"], case["shape"], B.CANVAS_BF16)
    assert int(B.canvas_dag_query(hd).workspace_bytes) > B.CANVAS_STATIC_WORKSPACE_BYTES
    rc = B.load().canvas_dag_forward_static(hd, None, None, None, None)
    assert rc == -5 and b"static workspace" in B.load().canvas_last_error()
    B.canvas_dag_destroy(hd)
