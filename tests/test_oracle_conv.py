"""Pins the oracle's Unfold, grouped FC and their gradients to direct convolution.

Section 5 of the paper: a convolution is Unfold (U(c,kh,kw,h,w) = I(c,h+kh,w+kw))
followed by a multiplication with the weights (im2col); group convolution is the
same with channels split as g*GROUP_SIZE + c.  The reference here is a 7-loop
direct grouped convolution and its gradients, written independently below, plus
torch's CPU conv2d as a third opinion.
"""
import numpy as np
import pytest

from paper_2304_07741_amd import workloads as wl


def direct_conv(x, w, groups):
    """y[n,co,h,w] = sum_{ci,kh,kw} w[co,ci,kh,kw] * x[n, g*Cg+ci, h+kh-ph, w+kw-pw], zero padded."""
    N, C, H, W = x.shape
    Co, Cg, KH, KW = w.shape
    Og = Co // groups
    y = np.zeros((N, Co, H, W))
    for n in range(N):
        for co in range(Co):
            g = co // Og
            for ci in range(Cg):
                for kh in range(KH):
                    for kw in range(KW):
                        for h in range(H):
                            hs = h + kh - KH // 2
                            if hs < 0 or hs >= H:
                                continue
                            for ww in range(W):
                                ws = ww + kw - KW // 2
                                if 0 <= ws < W:
                                    y[n, co, h, ww] += w[co, ci, kh, kw] * x[n, g * Cg + ci, hs, ws]
    return y


def direct_conv_grads(x, w, dy, groups):
    N, C, H, W = x.shape
    Co, Cg, KH, KW = w.shape
    Og = Co // groups
    dx = np.zeros_like(x)
    dw = np.zeros_like(w)
    for n in range(N):
        for co in range(Co):
            g = co // Og
            for ci in range(Cg):
                for kh in range(KH):
                    for kw in range(KW):
                        for h in range(H):
                            hs = h + kh - KH // 2
                            if hs < 0 or hs >= H:
                                continue
                            for ww in range(W):
                                ws = ww + kw - KW // 2
                                if 0 <= ws < W:
                                    dx[n, g * Cg + ci, hs, ws] += w[co, ci, kh, kw] * dy[n, co, h, ww]
                                    dw[co, ci, kh, kw] += dy[n, co, h, ww] * x[n, g * Cg + ci, hs, ws]
    return dx, dw


CASES = [
    # N, C, H, W, K, groups, Cout
    (1, 16, 8, 8, 3, 1, 16),   # the tiny conv-equivalent configuration
    (2, 8, 5, 7, 3, 2, 4),
    (1, 8, 6, 4, 5, 4, 16),
    (2, 16, 4, 5, 3, 8, 8),
    (1, 4, 7, 3, 5, 1, 6),
]


@pytest.mark.parametrize("N,C,H,W,K,G,Co", CASES)
def test_unfold_fc_equals_direct_conv(oracle, N, C, H, W, K, G, Co):
    rng = np.random.default_rng(N * 1000 + C * 10 + K)
    x = rng.standard_normal((N, C, H, W))
    w = rng.standard_normal((Co, C // G, K, K))
    dy = rng.standard_normal((N, Co, H, W))
    blob = wl.blob_conv(K, G, Co)
    # FC weight [G, Co/G, (C/G)*K*K] is the conv weight [Co, C/G, K, K] reshaped.
    r = oracle.run(blob, x, [w.reshape(G, Co // G, (C // G) * K * K)], dy)
    y = direct_conv(x, w, G)
    dx, dw = direct_conv_grads(x, w, dy, G)
    np.testing.assert_allclose(r["y"], y, rtol=0, atol=1e-12)
    np.testing.assert_allclose(r["dx"], dx, rtol=0, atol=1e-12)
    np.testing.assert_allclose(r["dw"][0].reshape(w.shape), dw, rtol=0, atol=1e-12)


def test_config1_against_direct_conv_and_torch(oracle):
    import torch

    case = wl.config1()
    x = case["x"].astype(np.float64)
    w = case["weights"][0].astype(np.float64).reshape(16, 16, 3, 3)
    dy = wl.make_dy(case, (1, 16, 8, 8)).astype(np.float64)
    r = oracle.run(case["blob"], x, [case["weights"][0]], dy)
    y = direct_conv(x, w, 1)
    dx, dw = direct_conv_grads(x, w, dy, 1)
    np.testing.assert_allclose(r["y"], y, atol=1e-12)
    np.testing.assert_allclose(r["dx"], dx, atol=1e-12)
    np.testing.assert_allclose(r["dw"][0].reshape(w.shape), dw, atol=1e-12)
    xt = torch.tensor(x, requires_grad=True)
    wt = torch.tensor(w, requires_grad=True)
    yt = torch.nn.functional.conv2d(xt, wt, padding=1)
    yt.backward(torch.tensor(dy))
    np.testing.assert_allclose(r["y"], yt.detach().numpy(), atol=1e-12)
    np.testing.assert_allclose(r["dx"], xt.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(r["dw"][0].reshape(w.shape), wt.grad.numpy(), atol=1e-12)


@pytest.mark.parametrize("G", [1, 2, 4, 8])
def test_grouped_conv_matches_torch(oracle, G):
    import torch

    rng = np.random.default_rng(G)
    x = rng.standard_normal((2, 16, 6, 5))
    w = rng.standard_normal((24 if G != 8 else 16, 16 // G, 5, 5))
    Co = w.shape[0]
    dy = rng.standard_normal((2, Co, 6, 5))
    r = oracle.run(wl.blob_conv(5, G, Co), x, [w.reshape(G, Co // G, -1)], dy)
    xt = torch.tensor(x, requires_grad=True)
    wt = torch.tensor(w, requires_grad=True)
    yt = torch.nn.functional.conv2d(xt, wt, padding=2, groups=G)
    yt.backward(torch.tensor(dy))
    np.testing.assert_allclose(r["y"], yt.detach().numpy(), atol=1e-11)
    np.testing.assert_allclose(r["dx"], xt.grad.numpy(), atol=1e-11)
    np.testing.assert_allclose(r["dw"][0].reshape(w.shape), wt.grad.numpy(), atol=1e-11)


def test_grouped_fc_is_block_diagonal_dense_fc(oracle):
    rng = np.random.default_rng(5)
    G, C, Co = 4, 8, 12
    x = rng.standard_normal((2, C, 3, 4))
    w = rng.standard_normal((G, Co // G, C // G))
    dense = np.zeros((1, Co, C))
    for g in range(G):
        dense[0, g * 3:(g + 1) * 3, g * 2:(g + 1) * 2] = w[g]
    dy = rng.standard_normal((2, Co, 3, 4))
    a = oracle.run(wl.HEADER + f"%1 = fc %0 groups={G} out={Co}\noutput %1\n", x, [w], dy)
    b = oracle.run(wl.HEADER + f"%1 = fc %0 groups=1 out={Co}\noutput %1\n", x, [dense], dy)
    np.testing.assert_allclose(a["y"], b["y"], atol=1e-13)
    np.testing.assert_allclose(a["dx"], b["dx"], atol=1e-13)
    for g in range(G):
        np.testing.assert_allclose(a["dw"][0][g], b["dw"][0][0, g * 3:(g + 1) * 3, g * 2:(g + 1) * 2], atol=1e-13)
    # plain definition of a per-pixel matrix product
    np.testing.assert_allclose(b["y"], np.einsum("oc,nchw->nohw", dense[0], x), atol=1e-13)


def test_depthwise_is_fc_with_one_channel_per_group(oracle):
    """Depth-wise convolution = FC within each channel separately (Section 8, ResNet-34 analysis)."""
    import torch

    rng = np.random.default_rng(6)
    C = 6
    x = rng.standard_normal((1, C, 5, 5))
    w = rng.standard_normal((C, 1, 3, 3))
    r = oracle.run(wl.blob_conv(3, C, C), x, [w.reshape(C, 1, 9)])
    yt = torch.nn.functional.conv2d(torch.tensor(x), torch.tensor(w), padding=1, groups=C)
    np.testing.assert_allclose(r["y"], yt.numpy(), atol=1e-13)


def test_two_1d_unfolds_equal_one_2d_unfold(oracle):
    """Unfolding H then W covers the same 9 neighbours in the same tap order (Section 8 case study)."""
    rng = np.random.default_rng(7)
    x = rng.standard_normal((1, 3, 5, 6))
    a = oracle.run(wl.HEADER + "%1 = unfold %0 kh=3 kw=1\n%2 = unfold %1 kh=1 kw=3\noutput %2\n", x, [])
    b = oracle.run(wl.HEADER + "%1 = unfold %0 kh=3 kw=3\noutput %1\n", x, [])
    assert a["y"].shape == (1, 3, 9, 5, 6)
    np.testing.assert_array_equal(a["y"], b["y"])
