"""Pins of the block-composition oracle (oracle/block_oracle.py) to its stated rule: with a convolution as the
template a block is the convolution C_in => C_out whose weight is cut into square blocks (Canvas, Section 4)."""
import numpy as np
import pytest
import torch

from oracle import block_oracle, canvas_oracle

HEADER = "canvas-dag 1\n"
CONV3 = HEADER + "%1 = unfold %0 kh=3 kw=3\n%2 = fc %1 groups=1 out={C}\noutput %2\n"
FC1 = HEADER + "%1 = fc %0 groups=1 out={C}\noutput %1\n"
GATED = (HEADER + "%1 = shift %0 dh=0 dw=1 c0=0 c1={H2}\n%2 = fc %1 groups=2 out={C}\n%3 = unary %2 op=gelu\n"
         "%4 = binary %0 %3 op=mul\noutput %4\n")


def _rng(seed):
    return np.random.default_rng(seed)


@pytest.mark.parametrize("c_in,c_out", [(4, 12), (12, 4), (6, 6)])
def test_a_convolution_template_composes_to_the_full_convolution(c_in, c_out):
    """Instance j's [C, C, 3, 3] weight is block j of the [C_out, C_in, 3, 3] weight: rows when expanding, columns
    when reducing.  torch's conv2d on the assembled weight is the reference, forward and both gradients."""
    g = _rng(1)
    n, h, w = 2, 5, 6
    c = min(c_in, c_out)
    m, mode = block_oracle.multiple_and_mode(c_in, c_out)
    x = g.standard_normal((n, c_in, h, w))
    dy = g.standard_normal((n, c_out, h, w))
    blocks = [g.standard_normal((c, c, 3, 3)) for _ in range(m)]
    r = block_oracle.run_block(CONV3.format(C=c), x, [[b.reshape(1, c, c * 9)] for b in blocks], c_out, dy)
    assert (r["m"], r["mode"]) == (m, mode)
    full = np.concatenate(blocks, axis=0 if mode == "expand" else 1)   # [C_out, C_in, 3, 3]
    assert full.shape == (c_out, c_in, 3, 3)
    xt = torch.tensor(x, requires_grad=True)
    wt = torch.tensor(full, requires_grad=True)
    yt = torch.nn.functional.conv2d(xt, wt, padding=1)
    yt.backward(torch.tensor(dy))
    np.testing.assert_allclose(r["y"], yt.detach().numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(r["dx"], xt.grad.numpy(), rtol=1e-12, atol=1e-12)
    gw = wt.grad.numpy()
    for j in range(m):
        ref = gw[j * c:(j + 1) * c] if mode == "expand" else gw[:, j * c:(j + 1) * c]
        np.testing.assert_allclose(r["dw"][j][0].reshape(c, c, 3, 3), ref, rtol=1e-12, atol=1e-12)


def test_a_pointwise_template_is_a_matrix_product_with_stacked_blocks():
    g = _rng(2)
    n, c, h, w, m = 3, 5, 2, 3, 3
    x = g.standard_normal((n, c, h, w))
    ws = [g.standard_normal((c, c)) for _ in range(m)]
    r = block_oracle.run_block(FC1.format(C=c), x, [[v.reshape(1, c, c)] for v in ws], m * c)
    np.testing.assert_allclose(r["y"], np.einsum("oi,nihw->nohw", np.vstack(ws), x), rtol=1e-12, atol=1e-12)
    xr = g.standard_normal((n, m * c, h, w))
    r = block_oracle.run_block(FC1.format(C=c), xr, [[v.reshape(1, c, c)] for v in ws], c)
    np.testing.assert_allclose(r["y"], np.einsum("oi,nihw->nohw", np.hstack(ws), xr), rtol=1e-12, atol=1e-12)


def test_one_instance_is_the_template_itself():
    g = _rng(3)
    c = 8
    x = g.standard_normal((2, c, 4, 4))
    dy = g.standard_normal((2, c, 4, 4))
    wts = [g.standard_normal((2, c // 2, c // 2))]
    blob = GATED.format(C=c, H2=c // 2)
    a = block_oracle.run_block(blob, x, [wts], c, dy)
    b = canvas_oracle.run(blob, x, wts, dy)
    assert np.array_equal(a["y"], b["y"]) and np.array_equal(a["dx"], b["dx"]) and np.array_equal(a["dw"][0][0], b["dw"][0])


@pytest.mark.parametrize("c_in,c_out", [(4, 8), (8, 4)])
def test_gradients_of_a_nonlinear_block_match_central_differences(c_in, c_out):
    g = _rng(4)
    n, h, w = 1, 3, 4
    c = min(c_in, c_out)
    m, _ = block_oracle.multiple_and_mode(c_in, c_out)
    blob = GATED.format(C=c, H2=c // 2)
    x = g.standard_normal((n, c_in, h, w))
    dy = g.standard_normal((n, c_out, h, w))
    wts = [[g.standard_normal((2, c // 2, c // 2))] for _ in range(m)]
    r = block_oracle.run_block(blob, x, wts, c_out, dy)

    def loss(xv, wv):
        return float((block_oracle.run_block(blob, xv, wv, c_out)["y"] * dy).sum())

    eps = 1e-6
    for idx in [(0, 0, 0, 0), (0, c_in - 1, 2, 3), (0, c_in // 2, 1, 1)]:
        xp, xm = x.copy(), x.copy()
        xp[idx] += eps
        xm[idx] -= eps
        assert abs((loss(xp, wts) - loss(xm, wts)) / (2 * eps) - r["dx"][idx]) < 1e-6
    for j in range(m):
        for idx in [(0, 0, 0), (1, c // 2 - 1, c // 2 - 1)]:
            wp = [[v.copy() for v in s] for s in wts]
            wm = [[v.copy() for v in s] for s in wts]
            wp[j][0][idx] += eps
            wm[j][0][idx] -= eps
            assert abs((loss(x, wp) - loss(x, wm)) / (2 * eps) - r["dw"][j][0][idx]) < 1e-6


def test_channel_counts_that_do_not_divide_are_refused():
    with pytest.raises(ValueError):
        block_oracle.multiple_and_mode(6, 4)
