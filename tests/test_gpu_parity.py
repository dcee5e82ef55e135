"""GPU parity: the HIP library (through the C ABI) against the CPU oracle, element by element.

Tolerances: 1e-5 relative for fp32, 2e-2 relative for bf16 (max-norm and l2-norm, see helpers.py)."""
import numpy as np
import pytest

from helpers import TOL, assert_close, check_against_oracle, has_kinks
from paper_2304_07741_amd import binding as B
from paper_2304_07741_amd import workloads as wl

pytestmark = pytest.mark.gpu

H_ = wl.HEADER


@pytest.fixture(scope="module")
def harness():
    import torch

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2304_07741_amd import harness as h

    return h


def _mk(body, shape, dtype, seed, wshapes, name="case"):
    import math

    return wl._case(name, H_ + body, shape, dtype, seed, wshapes, [1.0 / math.sqrt(s[2]) for s in wshapes])


PRIMS = [
    ("%1 = unfold %0 kh=3 kw=3\noutput %1\n", []),
    ("%1 = unfold %0 kh=5 kw=3\noutput %1\n", []),
    ("%1 = unfold %0 kh=3 kw=1\n%2 = unfold %1 kh=1 kw=3\noutput %2\n", []),
    ("%1 = shift %0 dh=1 dw=-2 c0=2 c1=9\noutput %1\n", []),
    ("%1 = shift %0 dh=0 dw=0\noutput %1\n", []),
    ("%1 = fc %0 groups=4 out=8\noutput %1\n", [(4, 2, 3)]),
    ("%1 = unfold %0 kh=3 kw=3\n%2 = fc %1 groups=3 out=6\noutput %2\n", [(3, 2, 36)]),
    ("%1 = unary %0 op=relu\noutput %1\n", []),
    ("%1 = unary %0 op=abs\noutput %1\n", []),
    ("%1 = unary %0 op=gelu\noutput %1\n", []),
    ("%1 = unary %0 op=expclip lo=-1.5 hi=0.75\noutput %1\n", []),
    ("%1 = softmax %0 axis=C\noutput %1\n", []),
    ("%1 = unfold %0 kh=3 kw=3\n%2 = softmax %1 axis=T\noutput %2\n", []),
    ("%1 = unfold %0 kh=3 kw=3\n%2 = softmax %1 axis=C\noutput %2\n", []),
    ("%1 = unfold %0 kh=3 kw=3\n%2 = fold %1 op=sum\noutput %2\n", []),
    ("%1 = unfold %0 kh=3 kw=3\n%2 = fold %1 op=avg\noutput %2\n", []),
    ("%1 = unfold %0 kh=3 kw=3\n%2 = fold %1 op=max\noutput %2\n", []),
    ("%1 = fold %0 op=max\noutput %1\n", []),
    ("%1 = unfold %0 kh=3 kw=3\n%2 = binary %0 %1 op=mul\noutput %2\n", []),
    ("%1 = fc %0 groups=1 out=6\n%2 = binary %1 %0 op=add\noutput %2\n", [(1, 6, 12)]),
    ("%1 = fc %0 groups=1 out=9\n%2 = unfold %0 kh=3 kw=3\n%3 = binary %1 %2 op=mul\noutput %3\n", [(1, 9, 12)]),
    ("%1 = fc %0 groups=1 out=18\n%2 = unfold %0 kh=3 kw=3\n%3 = binary %1 %2 op=add\noutput %3\n", [(1, 18, 12)]),
    ("%1 = binary %0 %0 op=mul\n%2 = binary %1 %0 op=add\noutput %2\n", []),
    ("output %0\n", []),
    ("%1 = unary %0 op=relu\n%2 = fc %0 groups=1 out=12\noutput %1\n", [(1, 12, 12)]),  # dead fc: zero dW
    ("%1 = unary %0 op=sin\noutput %1\n", []),
    ("%1 = fold %0 op=avg axis=HW\noutput %1\n", []),
    ("%1 = fold %0 op=max axis=C groups=3\noutput %1\n", []),
    ("%1 = unfold %0 kh=3 kw=3\n%2 = fold %1 op=avg axis=C groups=4\n%3 = fold %2 op=sum\n%4 = fc %3 groups=2 out=12\n%5 = binary %4 %0 op=add\noutput %5\n", [(2, 6, 2)]),
    ("%1 = fold %0 op=sum axis=C\n%2 = unary %1 op=gelu\n%3 = binary %2 %0 op=mul\noutput %3\n", []),
    ("%1 = fold %0 op=max axis=HW\n%2 = binary %1 %0 op=sub\noutput %2\n", []),
    ("%1 = unfold %0 kh=3 kw=1\n%2 = fold %1 op=sum axis=HW\n%3 = softmax %2 axis=T\n%4 = binary %3 %1 op=mul\n%5 = fold %4 op=sum\noutput %5\n", []),
    # squeeze-and-excite: pooled descriptor -> FC -> gelu -> FC -> softmax over channels -> gate on x
    ("%1 = fold %0 op=avg axis=HW\n%2 = fc %1 groups=1 out=4\n%3 = unary %2 op=gelu\n%4 = fc %3 groups=2 out=12\n"
     "%5 = softmax %4 axis=C\n%6 = binary %5 %0 op=mul\noutput %6\n", [(1, 4, 12), (2, 6, 2)]),
    ("%1 = unfold %0 kh=3 kw=3\n%2 = softmax %1 axis=CT\noutput %2\n", []),
    ("%1 = softmax %0 axis=CT\n%2 = binary %1 %0 op=mul\noutput %2\n", []),
    ("%1 = shift %0 dh=1 dw=0\n%2 = binary %0 %1 op=sub\noutput %2\n", []),
    ("%1 = unfold %0 kh=3 kw=3\n%2 = binary %0 %1 op=max\noutput %2\n", []),
    ("%1 = unfold %0 kh=3 kw=1\n%2 = fc %0 groups=3 out=6\n%3 = binary %2 %1 op=min\n%4 = fold %3 op=avg\noutput %4\n", [(3, 2, 4)]),
    ("%1 = unary %0 op=gelu\n%2 = binary %1 %0 op=min\n%3 = binary %0 %2 op=sub\noutput %3\n", []),
    # pooled vector laid over the pixels (spatial aggregation and kernel spanning, Section 8); 9 x 11 = 99 pixels
    ("%1 = fold %0 op=avg axis=HW\n%2 = fc %1 groups=1 out=99\n%3 = binary %2 %0 op=mul lhs=pixels\noutput %3\n", [(1, 99, 12)]),
    ("%1 = unfold %0 kh=1 kw=3\n%2 = fold %0 op=max axis=HW\n%3 = fc %2 groups=3 out=99\n%4 = unary %3 op=gelu\n"
     "%5 = binary %4 %1 op=sub lhs=pixels\n%6 = fold %5 op=avg\n%7 = binary %0 %6 op=min\noutput %7\n", [(3, 33, 4)]),
    # folds over one spatial dim and replication along it
    ("%1 = fold %0 op=max axis=H\noutput %1\n", []),
    ("%1 = fold %0 op=avg axis=W\noutput %1\n", []),
    ("%1 = fold %0 op=avg axis=H\n%2 = unary %1 op=gelu\n%3 = binary %2 %0 op=mul\n%4 = fold %0 op=max axis=W\n%5 = binary %4 %3 op=sub\noutput %5\n", []),
    ("%1 = unfold %0 kh=3 kw=1\n%2 = fold %1 op=max axis=W\n%3 = fc %2 groups=3 out=6\n%4 = fold %3 op=sum axis=H\n%5 = softmax %4 axis=C\n"
     "%6 = fc %0 groups=1 out=6\n%7 = binary %5 %6 op=mul\n%8 = binary %3 %7 op=add\noutput %8\n", [(3, 2, 12), (1, 6, 12)]),
    ("%1 = fold %0 op=sum axis=HW\n%2 = fold %0 op=max axis=W\n%3 = binary %1 %2 op=max\n%4 = fold %3 op=avg axis=H\n%5 = binary %4 %0 op=add\noutput %5\n", []),
    # Group as a node: the view alone, depth-wise 3x3, grouped Involution, a grouped blend with fan-out, mixed views
    ("%1 = group %0 groups=3\noutput %1\n", []),
    ("%1 = group %0 groups=12\n%2 = unfold %1 kh=3 kw=3\n%3 = fc %2 out=12\noutput %3\n", [(12, 1, 9)]),
    ("%1 = group %0 groups=3\n%2 = fc %1 out=27\n%3 = softmax %2 axis=C\n%4 = unfold %1 kh=3 kw=3\n%5 = binary %3 %4 op=mul\n"
     "%6 = fold %5 op=sum\n%7 = fc %6 out=6\noutput %7\n", [(3, 9, 4), (3, 2, 4)]),
    ("%1 = group %0 groups=2\n%2 = fc %1 out=4\n%3 = unary %2 op=gelu\n%4 = unfold %1 kh=1 kw=3\n%5 = binary %3 %4 op=sub\n"
     "%6 = binary %2 %5 op=max\n%7 = fold %6 op=avg\n%8 = binary %7 %0 op=add\noutput %8\n", [(2, 2, 6)]),
    ("%1 = group %0 groups=4\n%2 = fc %1 out=8\n%3 = group %2 groups=2\n%4 = fc %3 out=6\n%5 = binary %4 %1 op=mul\n%6 = group %5 groups=6\noutput %6\n",
     [(4, 2, 3), (2, 3, 4)]),
    # softmax over the spatial dims: along H, along W, jointly; of an unfolded tensor; of a tensor with one dim folded
    ("%1 = softmax %0 axis=H\noutput %1\n", []),
    ("%1 = softmax %0 axis=W\noutput %1\n", []),
    ("%1 = softmax %0 axis=HW\noutput %1\n", []),
    ("%1 = unfold %0 kh=1 kw=3\n%2 = softmax %1 axis=HW\n%3 = binary %0 %2 op=mul\n%4 = fold %3 op=sum\noutput %4\n", []),
    ("%1 = fold %0 op=avg axis=H\n%2 = softmax %1 axis=W\n%3 = binary %2 %0 op=mul\n%4 = softmax %3 axis=H\noutput %4\n", []),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("idx", range(len(PRIMS)))
def test_single_primitives(harness, oracle, idx, dtype):
    body, wshapes = PRIMS[idx]
    case = _mk(body, (3, 12, 9, 11), dtype, 40 + idx, wshapes, f"prim{idx}_{dtype}")
    res, r, dy = harness.run_case(case)
    check_against_oracle(oracle, case, res, dy)
    r.close()


def test_config1_conv_fp32(harness, oracle):
    """Unfold(3x3) -> FC on fp32 [1,16,8,8] equals a direct convolution (forward, dX, dW) within 1e-5."""
    import torch

    case = wl.config1()
    res, r, dy = harness.run_case(case)
    check_against_oracle(oracle, case, res, dy)
    xt = torch.tensor(case["x"].astype(np.float64), requires_grad=True)
    wt = torch.tensor(case["weights"][0].astype(np.float64).reshape(16, 16, 3, 3), requires_grad=True)
    yt = torch.nn.functional.conv2d(xt, wt, padding=1)
    yt.backward(torch.tensor(dy.astype(np.float64)))
    assert_close(res["y"], yt.detach().numpy(), 1e-5, "conv:y")
    assert_close(res["dx"], xt.grad.numpy(), 1e-5, "conv:dx")
    assert_close(res["dw"][0].reshape(16, 16, 3, 3), wt.grad.numpy(), 1e-5, "conv:dw")
    r.close()


@pytest.mark.parametrize("flags", [0, B.CANVAS_OPT_NO_FUSION])
@pytest.mark.parametrize("N,H", [(2, 56), (3, 13), (1, 8), (64, 56)])
def test_config2_shift_residual(harness, oracle, N, H, flags):
    case = wl.config2(N=N, H=H)
    res, r, dy = harness.run_case(case, flags)
    assert r.info.fused == (1 if flags == 0 and H in (56, 8) else 0)
    check_against_oracle(oracle, case, res, dy)
    r.close()


@pytest.mark.parametrize("N,C,H", [(64, 128, 56), (16, 128, 28), (5, 128, 12)])
def test_shift_residual_with_groups_of_32_at_full_size(harness, oracle, N, C, H):
    """The same DAG with C / 4 = 32 channels per FC group, in the launch configuration the bench times (N=64, 56x56)."""
    case = wl.config2(N=N, C=C, H=H)
    res, r, dy = harness.run_case(case)
    assert r.info.fused == 1 and [d["name"] for d in r.launches(1)] == ["sgfc_bwd", "sgfc_dw_reduce"]
    check_against_oracle(oracle, case, res, dy)
    r.close()


SGFC_VARIANTS = [
    # (offsets per 16-channel group, unary, residual, N, H, W)
    ([(0, 1), (0, -1), (1, 0), (-1, 0)], "relu", True, 2, 28, 28),     # 8-pixel units straddle rows
    ([(0, 2), (-2, 0), (1, 0), (0, 0)], "gelu", True, 2, 16, 24),      # larger shifts, H != W
    ([(0, 1), (0, -1), (1, 0), (-1, 0)], None, False, 1, 8, 8),         # plain shift convolution
    ([(0, 0), (0, 0), (0, 0), (0, 0)], "abs", True, 3, 12, 10),         # no shift at all
    ([(1, 1), (-1, -1), (1, -1), (-1, 1)], "expclip lo=-1 hi=1", False, 2, 8, 16),
    ([(0, 1), (0, -1), (1, 0), (-1, 0)], "relu", True, 1, 4, 8),        # one half-empty tile
    ([(0, 9), (0, -9), (5, 0), (-5, 0)], "relu", True, 1, 4, 8),        # shifts larger than the image
]


@pytest.mark.parametrize("idx", range(len(SGFC_VARIANTS)))
def test_fused_shift_fc_variants(harness, oracle, idx):
    """The fused shift -> grouped FC -> unary -> (+x) kernels over their parameter space."""
    offs, unary, res, N, H, W = SGFC_VARIANTS[idx]
    lines, k = [], 0
    for g, (dh, dw) in enumerate(offs):
        lines.append(f"%{k + 1} = shift %{k} dh={dh} dw={dw} c0={16 * g} c1={16 * g + 16}\n")
        k += 1
    lines.append(f"%{k + 1} = fc %{k} groups=4 out=64\n")
    k += 1
    if unary:
        lines.append(f"%{k + 1} = unary %{k} op={unary}\n")
        k += 1
    if res:
        lines.append(f"%{k + 1} = binary %{k} %0 op=add\n")
        k += 1
    lines.append(f"output %{k}\n")
    case = _mk("".join(lines), (N, 64, H, W), "bf16", 70 + idx, [(4, 16, 16)], f"sgfc{idx}")
    res_, r, dy = harness.run_case(case)
    assert r.info.fused == 1, "the fused lowering was not selected"
    check_against_oracle(oracle, case, res_, dy)
    r.close()


@pytest.mark.parametrize("idx", range(len(SGFC_VARIANTS)))
def test_fused_shift_fc_groups_of_32(harness, oracle, idx):
    """The same family with 32 channels per FC group (two 16-channel blocks per group and side of the contraction)."""
    offs, unary, res, N, H, W = SGFC_VARIANTS[idx]
    lines, k = [], 0
    for g, (dh, dw) in enumerate(offs):
        lines.append(f"%{k + 1} = shift %{k} dh={dh} dw={dw} c0={32 * g} c1={32 * g + 32}\n")
        k += 1
    lines.append(f"%{k + 1} = fc %{k} groups=4 out=128\n")
    k += 1
    if unary:
        lines.append(f"%{k + 1} = unary %{k} op={unary}\n")
        k += 1
    if res:
        lines.append(f"%{k + 1} = binary %{k} %0 op=add\n")
        k += 1
    lines.append(f"output %{k}\n")
    case = _mk("".join(lines), (N, 128, H, W), "bf16", 170 + idx, [(4, 32, 32)], f"sgfc32_{idx}")
    res_, r, dy = harness.run_case(case)
    assert r.info.fused == 1 and [d["name"] for d in r.launches(0)] == ["sgfc_fwd"], "the fused lowering was not selected"
    check_against_oracle(oracle, case, res_, dy)
    r.close()


GFC_CASES = [
    # (body, weight shapes, input shape): the MFMA grouped-FC kernels on awkward sizes
    ("%1 = unfold %0 kh=3 kw=3\n%2 = fc %1 groups=1 out=40\noutput %2\n", [(1, 40, 180)], (5, 20, 7, 7)),      # 7x7 planes, odd K
    ("%1 = unfold %0 kh=5 kw=5\n%2 = fc %1 groups=2 out=6\noutput %2\n", [(2, 3, 250)], (2, 20, 9, 5)),        # W=5, 5x5 window
    ("%1 = unfold %0 kh=7 kw=3\n%2 = fc %1 groups=4 out=36\noutput %2\n", [(4, 9, 105)], (3, 20, 6, 13)),      # 7x3 window
    ("%1 = unfold %0 kh=3 kw=1\n%2 = unfold %1 kh=1 kw=3\n%3 = fc %2 groups=5 out=10\noutput %3\n", [(5, 2, 36)], (2, 20, 5, 9)),  # taps on taps
    ("%1 = unfold %0 kh=3 kw=3\n%2 = unary %1 op=gelu\n%3 = fc %2 groups=1 out=17\noutput %3\n", [(1, 17, 180)], (2, 20, 4, 11)),  # materialised taps
    ("%1 = fc %0 groups=1 out=130\n%2 = fc %1 groups=13 out=26\n%3 = fc %2 groups=2 out=20\noutput %3\n",
     [(1, 130, 20), (13, 2, 10), (2, 10, 13)], (3, 20, 3, 4)),                                                      # chained, tiny planes (W=4)
    ("%1 = unfold %0 kh=3 kw=3\n%2 = fc %1 groups=1 out=10\n%3 = fc %1 groups=20 out=20\n%4 = binary %2 %3 op=add\noutput %4\n",
     [(1, 10, 180), (20, 1, 9)], (2, 20, 6, 6)),                                                                     # one unfold, two FCs
    ("%1 = fc %0 groups=1 out=70\noutput %1\n", [(1, 70, 20)], (1, 20, 1, 130)),                                  # single row image
]


@pytest.mark.parametrize("idx", range(len(GFC_CASES)))
def test_mfma_grouped_fc_shapes(harness, oracle, idx):
    body, wshapes, shape = GFC_CASES[idx]
    case = _mk(body, shape, "bf16", 90 + idx, wshapes, f"gfc{idx}")
    res, r, dy = harness.run_case(case)
    names = [d["name"] for d in r.launches(0)] + [d["name"] for d in r.launches(1)]
    assert any(n.startswith("gfc_") for n in names), names
    check_against_oracle(oracle, case, res, dy)
    r.close()


@pytest.mark.parametrize("flags", [0, B.CANVAS_OPT_NO_FUSION])
@pytest.mark.parametrize("N,H", [(2, 28), (3, 9), (32, 28), (1, 4)])
def test_config3_involution(harness, oracle, N, H, flags):
    case = wl.config3(N=N, H=H)
    res, r, dy = harness.run_case(case, flags)
    assert r.info.fused == (1 if flags == 0 else 0)
    check_against_oracle(oracle, case, res, dy)
    r.close()


DYN_VARIANTS = [
    # (window, groups of FC1, softmax, fold, groups of FC2, out of FC2, N, C, H, W, unfold first)
    (3, 1, True, "sum", 1, 24, 2, 24, 9, 11, False),     # ragged 8-pixel tail, odd width
    (5, 1, True, "avg", 2, 32, 2, 16, 7, 7, True),       # 5x5 window, average over the taps, unfold listed first
    (3, 3, False, "sum", 1, 12, 3, 12, 6, 10, False),    # no softmax, grouped FC1 (3 groups of 3 taps)
    (3, 1, True, "avg", 4, 64, 1, 32, 4, 12, False),     # image of four rows
    (5, 5, False, "sum", 1, 40, 2, 40, 5, 4, True),      # window larger than the image width
]


@pytest.mark.parametrize("idx", range(len(DYN_VARIANTS)))
def test_fused_dynamic_window_weights_variants(harness, oracle, idx):
    """The lowering of FC -> [softmax] -> broadcast-mul onto Unfold(x) -> Fold over taps -> FC over its parameter space."""
    k, g1, soft, fold, g2, o2, N, C, H, W, unfold_first = DYN_VARIANTS[idx]
    lines, cur = [], 0

    def emit(text):
        nonlocal cur
        cur += 1
        lines.append(f"%{cur} = {text}")
        return cur

    if unfold_first:
        u = emit(f"unfold %0 kh={k} kw={k}")
    a = emit(f"fc %0 groups={g1} out={k * k}")
    if soft:
        a = emit(f"softmax %{a} axis=C")
    if not unfold_first:
        u = emit(f"unfold %0 kh={k} kw={k}")
    emit(f"binary %{a} %{u} op=mul")
    emit(f"fold %{cur} op={fold}")
    emit(f"fc %{cur} groups={g2} out={o2}")
    body = "\n".join(lines) + f"\noutput %{cur}\n"
    wshapes = [(g1, k * k // g1, C // g1), (g2, o2 // g2, C // g2)]
    case = _mk(body, (N, C, H, W), "bf16", 400 + idx, wshapes, f"dyn{idx}")
    res, r, dy = harness.run_case(case)
    assert r.info.fused == 1, "the fused lowering was not selected"
    check_against_oracle(oracle, case, res, dy)
    r.close()


GROUPED_DYN = [
    # (window, G, softmax, fold, out of FC2, N, C, H, W): the Involution of Section 5 with G groups of per-pixel window weights
    (3, 4, True, "sum", 32, 2, 32, 9, 11),
    (3, 16, False, "avg", 64, 3, 64, 14, 14),   # many small groups (4 channels each)
    (5, 2, True, "sum", 24, 2, 24, 7, 6),
    (3, 8, True, "sum", 8, 1, 8, 5, 8),         # one channel per group
    (7, 3, False, "sum", 12, 2, 12, 6, 9),      # window outside the fused family: per-node lowering
]


@pytest.mark.parametrize("flags", [0, B.CANVAS_OPT_NO_FUSION])
@pytest.mark.parametrize("idx", range(len(GROUPED_DYN)))
def test_grouped_involution(harness, oracle, idx, flags):
    k, G, soft, fold, o2, N, C, H, W = GROUPED_DYN[idx]
    body = f"%1 = group %0 groups={G}\n%2 = fc %1 out={G * k * k}\n"
    a = 2
    if soft:
        body += "%3 = softmax %2 axis=C\n"
        a = 3
    body += (f"%{a + 1} = unfold %1 kh={k} kw={k}\n%{a + 2} = binary %{a} %{a + 1} op=mul\n%{a + 3} = fold %{a + 2} op={fold}\n"
             f"%{a + 4} = fc %{a + 3} out={o2}\noutput %{a + 4}\n")
    wshapes = [(G, k * k, C // G), (G, o2 // G, C // G)]
    case = _mk(body, (N, C, H, W), "bf16", 450 + idx, wshapes, f"gdyn{idx}")
    res, r, dy = harness.run_case(case, flags)
    tiny = min(G * k * k * (C // G), o2 * (C // G)) < 16  # weight tensors of a few scalars keep fp32 intermediates
    assert r.info.fused == (1 if flags == 0 and k <= 5 and C // G != k * k and not tiny else 0)
    check_against_oracle(oracle, case, res, dy)
    r.close()


@pytest.mark.parametrize("flags", [0, B.CANVAS_OPT_NO_FUSION])
@pytest.mark.parametrize("C,H,N", [(64, 56, 2), (128, 28, 2), (256, 14, 3), (512, 7, 5), (64, 11, 2), (64, 4, 1), (1024, 7, 2), (8, 5, 3)])
def test_config4_sampled_small_batch(harness, oracle, C, H, N, flags):
    case = wl.config4(C, H, N=N)
    res, r, dy = harness.run_case(case, flags)
    assert r.info.fused == (1 if flags == 0 else 0)
    check_against_oracle(oracle, case, res, dy)
    r.close()


@pytest.mark.parametrize("C,H", wl.CONFIG4_SHAPES)
def test_config4_sampled_full_batch(harness, oracle, C, H):
    case = wl.config4(C, H, N=128)
    res, r, dy = harness.run_case(case)
    assert r.info.fused == 1
    check_against_oracle(oracle, case, res, dy)
    r.close()


UFC_VARIANTS = [
    # (window, groups of FC1, unary, shifts [(dh, dw, c0, c1)], binary, identity fold, groups of FC2, out of FC2, N, C, H, W)
    (3, 8, "gelu", [(0, 1, 24, 48)], "mul", True, 1, 48, 2, 48, 9, 11),          # ragged 8-pixel tail, odd width
    (3, 4, "relu", [(1, 0, 0, 16), (-1, 0, 16, 32)], "add", False, 2, 64, 3, 32, 8, 8),
    (5, 2, None, [], "mul", False, 1, 16, 2, 16, 7, 7),                            # no unary, no shift, 5x5 window
    (1, 1, "abs", [(0, -1, 0, 8), (2, 0, 8, 12), (0, 3, 20, 24)], "mul", True, 4, 24, 1, 24, 6, 10),  # no unfold
    (3, 8, "gelu", [(5, 0, 0, 32)], "add", False, 1, 96, 2, 64, 4, 12),           # shift beyond the image
    (3, 1, "gelu", [(0, 1, 4, 8)], "mul", False, 1, 8, 5, 8, 5, 4),                # tiny channel counts
    (3, 8, "expclip lo=-1 hi=1", [(0, 1, 0, 32)], "add", False, 1, 96, 2, 64, 4, 12),  # clip bounds: not fused
    (3, 3, "relu", [(0, -1, 0, 12)], "mul", False, 3, 48, 2, 24, 8, 16),           # 3 groups of 8 rows: the last merged pair is half empty
    (5, 5, "abs", [], "add", True, 1, 20, 1, 20, 9, 9),                             # groups of 4 rows: four merged, one left over
    (3, 2, "sin", [(0, 1, 0, 8)], "mul", False, 2, 16, 2, 16, 8, 8),                # a smooth unary outside the first four
    # rows of 24 pixels and more: the 3x3 weight gradient walks down the image rows (one or two 32-column chunks)
    (3, 2, "relu", [(0, 1, 0, 8)], "mul", False, 1, 16, 3, 16, 5, 25),              # odd width, one chunk, ragged 16-byte pieces at the row ends
    (3, 8, "gelu", [], "add", False, 1, 32, 2, 64, 7, 48),                          # two chunks, groups of 8 rows merged in pairs
    (3, 1, None, [(1, 0, 0, 40)], "mul", False, 2, 24, 2, 40, 3, 64),               # rows of exactly two chunks, 40 rows: 16 + 16 + 8
    (3, 4, "abs", [], "add", False, 1, 8, 1, 32, 30, 31),                           # one image, odd width, more rows than steps per wavefront
    # weight tiles too large for LDS (> 72 KB per workgroup): the MFMA operands are read from memory directly
    (5, 1, "relu", [], "add", False, 1, 32, 2, 64, 9, 9),                           # 5x5 window on 64 rows: 32 x 25 x 64 weights per tile
    (1, 1, "abs", [(0, 1, 0, 512)], "mul", False, 1, 64, 1, 1024, 4, 8),            # 1024 channels: 64 x 1024 weights per tile
]


@pytest.mark.parametrize("idx", range(len(UFC_VARIANTS)))
def test_fused_unfold_fc_gate_fc_variants(harness, oracle, idx):
    """The lowering of [Unfold] -> FC -> [unary] -> Shift* -> add|mul with x -> FC over its parameter space."""
    k, g1, act, shifts, bop, fold, g2, o2, N, C, H, W = UFC_VARIANTS[idx]
    lines, cur = [], 0

    def emit(text):
        nonlocal cur
        cur += 1
        lines.append(f"%{cur} = {text}")
        return cur

    if k > 1:
        emit(f"unfold %0 kh={k} kw={k}")
    emit(f"fc %{cur} groups={g1} out={C}")
    if act:
        emit(f"unary %{cur} op={act}")
    for dh, dw, c0, c1 in shifts:
        emit(f"shift %{cur} dh={dh} dw={dw} c0={c0} c1={c1}")
    emit(f"binary %0 %{cur} op={bop}" if idx % 2 == 0 else f"binary %{cur} %0 op={bop}")
    if fold:
        emit(f"fold %{cur} op=avg")
    emit(f"fc %{cur} groups={g2} out={o2}")
    body = "\n".join(lines) + f"\noutput %{cur}\n"
    wshapes = [(g1, C // g1, (C // g1) * k * k), (g2, o2 // g2, C // g2)]
    case = _mk(body, (N, C, H, W), "bf16", 300 + idx, wshapes, f"ufc{idx}")
    res, r, dy = harness.run_case(case)
    # bf16 intermediates would move values across the clip bounds of expclip: that unary keeps the per-node lowering
    assert r.info.fused == (0 if act and act.startswith("expclip") else 1), "unexpected choice of lowering"
    check_against_oracle(oracle, case, res, dy)
    r.close()


def _fuzz_case(oracle, seed):
    """Seeds whose oracle result is not finite are re-drawn with the next attempt number."""
    for attempt in range(5):
        case = wl.config5(seed, attempt)
        ref = oracle.run(case["blob"], case["x"], case["weights"])
        if np.isfinite(ref["y"]).all():
            return case
    raise AssertionError(f"seed {seed}: no finite DAG in 5 attempts")


@pytest.mark.parametrize("block", range(20))
def test_config5_fuzz(harness, oracle, block):
    """200 random micro-DAGs (seeds 100-299), 10 per test."""
    for seed in range(100 + 10 * block, 110 + 10 * block):
        case = _fuzz_case(oracle, seed)
        res, r, dy = harness.run_case(case)
        try:
            check_against_oracle(oracle, case, res, dy, what=f"fuzz seed {seed}\n{case['blob']}")
        finally:
            r.close()


# The primitives beyond the five configurations at planes larger than one workgroup pass (56 x 56 = 3136 pixels) and
# at many channels with few pixels: folds over HW / H / W / C, a pooled LHS replicated over the pixels, lhs=pixels,
# softmax over C and T jointly and over the spatial dims.
BIG_PLANE_BODIES = [
    ("%1 = fold %0 op=avg axis=HW\n%2 = binary %1 %0 op=mul\noutput %2\n", []),
    ("%1 = fold %0 op=max axis=HW\n%2 = binary %1 %0 op=sub\noutput %2\n", []),
    ("%1 = fold %0 op=sum axis=H\n%2 = fold %0 op=max axis=W\n%3 = binary %1 %0 op=add\n%4 = binary %2 %3 op=mul\noutput %4\n", []),
    ("%1 = fold %0 op=avg axis=C groups=4\n%2 = fold %1 op=max axis=HW\noutput %2\n", []),
    ("%1 = unfold %0 kh=3 kw=1\n%2 = softmax %1 axis=CT\n%3 = fold %2 op=sum\noutput %3\n", []),
    ("%1 = softmax %0 axis=HW\n%2 = binary %1 %0 op=mul\noutput %2\n", []),
    ("%1 = softmax %0 axis=H\n%2 = softmax %0 axis=W\n%3 = binary %1 %2 op=add\noutput %3\n", []),
]


@pytest.mark.parametrize("N,C,H", [(4, 64, 56), (4, 512, 7)])
@pytest.mark.parametrize("idx", range(len(BIG_PLANE_BODIES)))
def test_primitives_at_full_size_planes(harness, oracle, idx, N, C, H):
    body, wshapes = BIG_PLANE_BODIES[idx]
    case = _mk(body, (N, C, H, H), "bf16", 70 + idx, wshapes, name=f"big_plane_{idx}")
    res, r, dy = harness.run_case(case)
    try:
        check_against_oracle(oracle, case, res, dy, what=f"{case['name']} {case['shape']}")
    finally:
        r.close()


def test_pixel_aligned_lhs_at_a_full_size_plane(harness, oracle):
    """The kernel with spatial aggregation and kernel spanning (Section 8): pool to [C], FC to H*W, lay it over the pixels."""
    C, H = 64, 28
    body = f"%1 = fold %0 op=avg axis=HW\n%2 = fc %1 groups=1 out={H * H}\n%3 = binary %2 %0 op=mul lhs=pixels\noutput %3\n"
    case = _mk(body, (4, C, H, H), "bf16", 77, [(1, H * H, C)], name="spatial_aggregation")
    res, r, dy = harness.run_case(case)
    try:
        check_against_oracle(oracle, case, res, dy, what="spatial aggregation 28x28")
    finally:
        r.close()


# FC-free chains (one fused kernel each way) at the shapes bench.py times them on, and at planes that leave a ragged
# tail for every vector width the kernels have (7x7: one pixel per thread and 16 channels side by side; 14x14: four
# pixels; 13x11: odd sizes; 28x28 and 56x56: sixteen pixels, a vector may straddle two image rows), both dtypes
CHAIN_SHAPES = [(128, 64, 56), (8, 128, 28), (4, 256, 14), (5, 40, 7), (3, 24, 13), (2, 6, 20)]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("N,C,H", CHAIN_SHAPES)
@pytest.mark.parametrize("body", sorted(wl.CHAIN_BODIES))
def test_fused_chain_workloads(harness, oracle, body, N, C, H, dtype):
    if dtype == "f32" and N > 8:
        pytest.skip("the full batch is checked in bf16, the dtype it is timed in")
    case = wl.chain(body, N=N, C=C, H=H, dtype=dtype)
    res, r, dy = harness.run_case(case)
    try:
        assert r.info.n_fused_chains == 1 and r.info.n_launches_fwd == 1 and r.info.n_launches_bwd == 1
        check_against_oracle(oracle, case, res, dy, what=f"{case['name']} {case['shape']} {dtype}")
    finally:
        r.close()


# Windows whose taps reach across the first and last rows of the whole tensor (one image or few, few channels), on planes
# for every pixels-per-thread width of the window instances: rows that are whole vectors (W = 8, 12, 16, 6 with two
# pixels), vectors that straddle two rows (6x6 and 10x6 with four pixels), single pixels (odd sizes); after a shift, so
# that the window load itself is displaced; 5x5; max, whose ties at the zero border go to the first tap
WINDOW_END_BODIES = [
    "%1 = unfold %0 kh=3 kw=3\n%2 = fold %1 op=sum\noutput %2\n",
    "%1 = shift %0 dh=2 dw=-3\n%2 = unfold %1 kh=3 kw=3\n%3 = fold %2 op=max\noutput %3\n",
    "%1 = unfold %0 kh=5 kw=5\n%2 = unary %1 op=abs\n%3 = fold %2 op=avg\noutput %3\n",
    "%1 = unfold %0 kh=3 kw=3\n%2 = unary %1 op=gelu\n%3 = fold %2 op=avg\n%4 = shift %3 dh=-1 dw=1\n%5 = binary %0 %4 op=add\noutput %5\n",
    "%1 = shift %0 dh=-1 dw=2\n%2 = unfold %1 kh=1 kw=3\n%3 = binary %0 %2 op=mul\n%4 = fold %3 op=sum\noutput %4\n",
]
WINDOW_END_SHAPES = [(1, 1, 4, 8), (2, 3, 5, 12), (1, 2, 6, 6), (1, 1, 3, 16), (2, 2, 9, 7), (1, 3, 10, 6), (1, 1, 1, 4), (3, 1, 2, 2)]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("shape", WINDOW_END_SHAPES)
@pytest.mark.parametrize("idx", range(len(WINDOW_END_BODIES)))
def test_window_chains_at_the_ends_of_the_tensor(harness, oracle, idx, shape, dtype):
    case = _mk(WINDOW_END_BODIES[idx], shape, dtype, 900 + idx, [], f"window_ends{idx}")
    res, r, dy = harness.run_case(case)
    try:
        assert r.info.n_fused_chains >= 1
        check_against_oracle(oracle, case, res, dy, what=f"window chain {idx} at {shape} {dtype}")
    finally:
        r.close()


DETERMINISM_CASES = [lambda: wl.config4(64, 14, N=4), lambda: wl.config4(64, 56, N=2), lambda: wl.config4(128, 28, N=3),
                     lambda: wl.config4(512, 7, N=8), lambda: wl.config3(N=2, H=28), lambda: wl.config2(N=2, H=56),
                     lambda: wl.config5(157), lambda: wl.config5(130), lambda: wl.chain("shift_residual", N=8, C=64, H=28),
                     lambda: wl.config2(N=3, C=128, H=28), lambda: wl.config3(N=4, H=28)]


@pytest.mark.parametrize("idx", range(len(DETERMINISM_CASES)))
def test_backward_is_deterministic(harness, idx):
    """Two runs give the same bits: every reduction (split K, weight-gradient partials, their sums) has a fixed order."""
    case = DETERMINISM_CASES[idx]()
    a, r1, dy = harness.run_case(case)
    b, r2, _ = harness.run_case(case, dy=dy)
    assert np.array_equal(a["dx"], b["dx"]) and np.array_equal(a["y"], b["y"])
    for u, v in zip(a["dw"], b["dw"]):
        assert np.array_equal(u, v)
    r1.close()
    r2.close()


INFER_CASES = [lambda o: wl.config2(N=2, H=24), lambda o: wl.config2(N=1, H=56), lambda o: wl.config3(N=2, H=14), lambda o: wl.config3(N=8, H=28),
               lambda o: wl.config4(64, 28, N=1), lambda o: wl.config4(256, 14, N=8), lambda o: wl.config4(512, 7, N=4),
               lambda o: _fuzz_case(o, 123), lambda o: _fuzz_case(o, 207)]


@pytest.mark.parametrize("flags", [0, B.CANVAS_OPT_NO_FUSION])
@pytest.mark.parametrize("idx", range(len(INFER_CASES)))
def test_inference_plan_matches_training_forward(harness, oracle, idx, flags):
    """The inference plan (weight-only work hoisted into canvas_dag_prepare, batch 1-8) runs the same
    kernels on the same operands, so its forward equals the training plan's bit for bit, also on repeated
    calls and after the weights change; the training forward itself is checked against the oracle."""
    import torch

    case = INFER_CASES[idx](oracle)
    res, rt, dy = harness.run_case(case, flags)
    check_against_oracle(oracle, case, res, dy, what=f"{case['name']} flags={flags}")
    ri = harness.DagRunner(case["blob"], case["shape"], case["dtype"], flags | B.CANVAS_OPT_INFERENCE)
    try:
        assert ri.info.n_launches_bwd == 0 and ri.info.fused == rt.info.fused
        ri.load(case["x"], case["weights"])
        ri.ws.fill_(0xFF)
        ri.prepare()
        for _ in range(3):
            ri.y.fill_(float("nan"))
            ri.forward()
            assert np.array_equal(ri.results()["y"], res["y"])
        with pytest.raises(B.CanvasError) as e:
            ri.backward()
        assert e.value.status == -6
        # new weights: prepare again, compare with the training plan on the same weights
        w2 = [np.ascontiguousarray(w[..., ::-1]) * 0.5 for w in case["weights"]]
        rt.load(case["x"], w2)
        rt.forward()
        ri.load(case["x"], w2)
        ri.prepare()
        ri.forward()
        assert np.array_equal(ri.results()["y"], rt.results()["y"])
        assert not np.array_equal(ri.results()["y"], res["y"]) or not case["weights"]
    finally:
        ri.close()
        rt.close()


@pytest.mark.parametrize("which", ["config2", "config3", "config4"])
def test_inference_forward_replays_from_a_hip_graph(harness, which):
    """The forward of an inference plan is a fixed list of kernel launches (no allocation, no memset, no
    synchronisation), so a captured HIP graph of it gives the eager result on every replay, with other
    work and new inputs between the replays."""
    import torch

    case = {"config2": lambda: wl.config2(N=4, H=28), "config3": lambda: wl.config3(N=2, H=14),
            "config4": lambda: wl.config4(128, 14, N=4)}[which]()
    r = harness.DagRunner(case["blob"], case["shape"], case["dtype"], B.CANVAS_OPT_INFERENCE)
    try:
        r.load(case["x"], case["weights"])
        r.prepare()
        r.forward()
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            r.forward()
            with torch.cuda.graph(g, stream=side):
                r.forward()
        torch.cuda.synchronize()
        for rep in range(4):
            r.x.copy_(torch.roll(r.x, rep + 1, dims=0) * (1.0 + 0.25 * rep))  # eager work on new inputs
            r.forward()
            want = r.y.clone()
            r.y.fill_(float("nan"))
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(r.y, want), f"replay {rep}"
    finally:
        r.close()


@pytest.mark.parametrize("which", ["config2", "config3", "config4", "config4_rows", "chains_and_fcs", "chain_with_passes", "chain_gate"])
def test_training_step_replays_from_a_hip_graph(harness, which):
    """Forward and backward of a training plan are fixed lists of kernel launches too: a captured HIP graph of the
    step gives the eager y, dx and dW (bit for bit: every reduction has a fixed order) on every replay, with
    other work and new inputs between the replays."""
    import torch

    case = {"config2": lambda: wl.config2(N=4, H=28), "config3": lambda: wl.config3(N=2, H=14),
            "config4": lambda: wl.config4(256, 14, N=4), "config4_rows": lambda: wl.config4(64, 28, N=2),
            # fused chains (the program travels in the kernel arguments), with FC nodes between them; a chain whose
            # softmax over channels runs in passes and hands gradients over through LDS; a chain alone
            "chains_and_fcs": lambda: wl.config5(135), "chain_with_passes": lambda: wl.config5(157),
            "chain_gate": lambda: wl.chain("gate", N=4, C=32, H=28)}[which]()
    r = harness.DagRunner(case["blob"], case["shape"], case["dtype"])
    try:
        rng = np.random.default_rng(5)
        dy = rng.standard_normal(tuple(r.dy.shape)).astype(np.float32)
        r.load(case["x"], case["weights"], dy)
        r.forward()
        r.backward()
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            r.forward()
            r.backward()
            with torch.cuda.graph(g, stream=side):
                r.forward()
                r.backward()
        torch.cuda.synchronize()
        for rep in range(3):
            r.x.copy_(torch.roll(r.x, rep + 1, dims=0) * (1.0 + 0.25 * rep))  # eager work on new inputs
            r.dy.copy_(torch.roll(r.dy, rep + 1, dims=1))
            r.forward()
            r.backward()
            want = [r.y.clone(), r.dx.clone()] + [t.clone() for t in r.dw]
            r.poison_outputs()
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            for k, (got, w) in enumerate(zip([r.y, r.dx, *r.dw], want)):
                assert torch.equal(got, w), f"replay {rep}, tensor {k}"
    finally:
        r.close()


@pytest.mark.parametrize("which", ["shape_matching", "constraints"])
def test_template_to_executor_end_to_end(harness, oracle, which):
    """A kernel template goes through the two solvers, is instantiated for two replacement targets and each
    concrete micro-DAG runs forward and backward on the GPU against the DAG oracle (the paper's pipeline from a
    sampled template to a trained kernel, Sections 6 and 7, without the sampler)."""
    import math

    if which == "shape_matching":
        t = B.canvas_template_parse(wl.TEMPLATE_SHAPE_MATCHING)
        var, subs = B.canvas_template_substitutions(t, 7)
        assert "KW*x2" in subs
        B.canvas_template_substitute(t, var, "KW*x2")
        targets, G = [dict(C=32, KH=3, KW=3, H=14, W=14), dict(C=64, KH=3, KW=3, H=9, W=11)], 4
    else:
        t = B.canvas_template_parse(wl.TEMPLATE_CONSTRAINTS)
        targets, G = [dict(C=64, KH=3, KW=3, H=14, W=14), dict(C=256, KH=5, KW=5, H=7, W=7)], 4
    xs, flops, params, rounds = B.canvas_template_solve(t, targets, G, flops_budget=6.0e7)
    assert rounds >= 1
    for tg, x in zip(targets, xs):
        blob = B.canvas_template_instantiate(t, tg, G, x)
        shape = (3, tg["C"], tg["H"], tg["W"])
        _, _, wshapes = oracle.infer(blob, shape)
        wshapes = [tuple(s_) for s_ in wshapes]
        case = wl._case(f"tmpl_{which}_{tg['C']}", blob, shape, "bf16", 900 + tg["C"], wshapes, [1.0 / math.sqrt(s_[2]) for s_ in wshapes])
        res, r, dy = harness.run_case(case)
        check_against_oracle(oracle, case, res, dy, what=blob)
        assert list(r.out_shape) == [3, tg["C"], 1, tg["H"], tg["W"]]   # a template maps [C, H, W] to [C, H, W]
        r.close()
    B.canvas_template_destroy(t)


def test_runtime_argument_checks(harness):
    import torch

    case = wl.config2(N=1, H=8)
    r = harness.DagRunner(case["blob"], case["shape"], "bf16")
    small = torch.empty(max(0, int(r.info.workspace_bytes) - 1), dtype=torch.uint8, device="cuda")
    if r.info.workspace_bytes > 0:
        with pytest.raises(B.CanvasError) as e:
            B.canvas_dag_forward(r.handle, r.x, r.w, r.y, small)
        assert e.value.status == -5
    r.close()
