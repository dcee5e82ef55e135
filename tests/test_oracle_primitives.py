"""Pins every primitive of the oracle (forward and backward) to identities,
closed forms, adjoint dot-products and central finite differences.

Primitive definitions: Section 5 of the paper (table of fine-grained primitives).
"""
import math

import numpy as np
import pytest

from paper_2304_07741_amd import workloads as wl

H_ = wl.HEADER


def run1(oracle, body, x, weights=(), dy=None):
    return oracle.run(H_ + body, x, list(weights), dy)


# ------------------------------------------------------------------- shift

def test_zero_shift_is_identity(oracle):
    x = np.random.default_rng(0).standard_normal((2, 4, 5, 6))
    r = run1(oracle, "%1 = shift %0 dh=0 dw=0\noutput %1\n", x)
    np.testing.assert_array_equal(r["y"], x)


@pytest.mark.parametrize("dh,dw", [(1, 0), (-1, 0), (0, 1), (0, -1), (2, 0), (0, -2)])
def test_shift_direction_and_zero_fill(oracle, dh, dw):
    """S(c,h,w) = I(c,h+dh,w+dw): the output at (h,w) reads the input at (h+dh,w+dw)."""
    x = np.random.default_rng(1).standard_normal((1, 3, 6, 7))
    r = run1(oracle, f"%1 = shift %0 dh={dh} dw={dw}\noutput %1\n", x)
    exp = np.zeros_like(x)
    for h in range(6):
        for w in range(7):
            if 0 <= h + dh < 6 and 0 <= w + dw < 7:
                exp[:, :, h, w] = x[:, :, h + dh, w + dw]
    np.testing.assert_array_equal(r["y"], exp)


def test_shift_then_back_zeroes_a_border_band(oracle):
    x = np.random.default_rng(2).standard_normal((1, 2, 5, 5))
    r = run1(oracle, "%1 = shift %0 dh=0 dw=1\n%2 = shift %1 dh=0 dw=-1\noutput %2\n", x)
    exp = x.copy()
    exp[:, :, :, 0] = 0.0  # column 0 reads column -1 of the shifted tensor
    np.testing.assert_array_equal(r["y"], exp)


def test_shift_channel_slice(oracle):
    x = np.random.default_rng(3).standard_normal((1, 6, 4, 4))
    r = run1(oracle, "%1 = shift %0 dh=1 dw=0 c0=2 c1=4\noutput %1\n", x)
    np.testing.assert_array_equal(r["y"][:, :2], x[:, :2])
    np.testing.assert_array_equal(r["y"][:, 4:], x[:, 4:])
    np.testing.assert_array_equal(r["y"][:, 2:4, :3], x[:, 2:4, 1:])
    np.testing.assert_array_equal(r["y"][:, 2:4, 3], 0 * x[:, 2:4, 3])


@pytest.mark.parametrize("k", [3, 5])
def test_unfold_tap_equals_shift(oracle, k):
    """Tap (kh,kw) of Unfold is the tensor shifted by (kh-K/2, kw-K/2)."""
    x = np.random.default_rng(4).standard_normal((1, 2, 6, 5))
    u = run1(oracle, f"%1 = unfold %0 kh={k} kw={k}\noutput %1\n", x)["y"]
    assert u.shape == (1, 2, k * k, 6, 5)
    for kh in range(k):
        for kw in range(k):
            s = run1(oracle, f"%1 = shift %0 dh={kh - k // 2} dw={kw - k // 2}\noutput %1\n", x)["y"]
            np.testing.assert_array_equal(u[:, :, kh * k + kw], s)


# ------------------------------------------- adjoints of the linear primitives

LINEAR_BODIES = [
    ("%1 = unfold %0 kh=3 kw=3\noutput %1\n", []),
    ("%1 = unfold %0 kh=5 kw=3\noutput %1\n", []),
    ("%1 = shift %0 dh=1 dw=-2 c0=1 c1=3\noutput %1\n", []),
    ("%1 = unfold %0 kh=3 kw=3\n%2 = shift %1 dh=0 dw=1\n%3 = fold %2 op=sum\noutput %3\n", []),
    ("%1 = unfold %0 kh=3 kw=3\n%2 = fold %1 op=avg\noutput %2\n", []),
    ("%1 = unfold %0 kh=3 kw=3\n%2 = binary %0 %1 op=add\noutput %2\n", []),
    ("%1 = fc %0 groups=2 out=6\noutput %1\n", [(2, 3, 2)]),
    ("%1 = unfold %0 kh=3 kw=3\n%2 = fc %1 groups=4 out=12\n%3 = binary %2 %1 op=add\noutput %3\n", [(4, 3, 9)]),
]


@pytest.mark.parametrize("body,wshapes", LINEAR_BODIES)
def test_adjoint_dot_product(oracle, body, wshapes):
    """<A x, y> == <x, A^T y> for DAGs that are linear in x."""
    rng = np.random.default_rng(10)
    x = rng.standard_normal((2, 4, 5, 6))
    ws = [rng.standard_normal(s) for s in wshapes]
    y0 = run1(oracle, body, x, ws)["y"]
    dy = rng.standard_normal(y0.shape)
    r = run1(oracle, body, x, ws, dy)
    lhs = float(np.sum(r["y"] * dy))
    rhs = float(np.sum(x * r["dx"]))
    assert abs(lhs - rhs) <= 1e-12 * max(1.0, abs(lhs))
    # linear in the weights as well: <dW, W> == <y, dy>
    for w, dw in zip(ws, r["dw"]):
        if len(ws) == 1 and "binary" not in body:
            assert abs(float(np.sum(w * dw)) - lhs) <= 1e-12 * max(1.0, abs(lhs))


# ----------------------------------------------------- finite differences

def fd_check(oracle, body, x, ws, h=1e-6, tol=2e-6, n_probe=25, seed=0):
    rng = np.random.default_rng(seed)
    y0 = run1(oracle, body, x, ws)["y"]
    dy = rng.standard_normal(y0.shape)
    r = run1(oracle, body, x, ws, dy)

    def loss(xx, wws):
        return float(np.sum(run1(oracle, body, xx, wws)["y"] * dy))

    for _ in range(n_probe):
        idx = tuple(rng.integers(0, s) for s in x.shape)
        xp, xm = x.copy(), x.copy()
        xp[idx] += h
        xm[idx] -= h
        num = (loss(xp, ws) - loss(xm, ws)) / (2 * h)
        assert abs(num - r["dx"][idx]) <= tol * max(1.0, abs(num)), (body, idx, num, r["dx"][idx])
    for k, w in enumerate(ws):
        for _ in range(min(n_probe, w.size)):
            idx = tuple(rng.integers(0, s) for s in w.shape)
            wp = [a.copy() for a in ws]
            wm = [a.copy() for a in ws]
            wp[k][idx] += h
            wm[k][idx] -= h
            num = (loss(x, wp) - loss(x, wm)) / (2 * h)
            assert abs(num - r["dw"][k][idx]) <= tol * max(1.0, abs(num)), (body, k, idx)


def away_from_kinks(x, margin=1e-2):
    return np.where(np.abs(x) < margin, margin * np.where(x < 0, -1.0, 1.0), x)


FD_BODIES = [
    ("%1 = unary %0 op=relu\noutput %1\n", []),
    ("%1 = unary %0 op=abs\noutput %1\n", []),
    ("%1 = unary %0 op=gelu\noutput %1\n", []),
    ("%1 = unary %0 op=expclip lo=-1.5 hi=0.75\noutput %1\n", []),
    ("%1 = softmax %0 axis=C\noutput %1\n", []),
    ("%1 = unfold %0 kh=3 kw=3\n%2 = softmax %1 axis=T\noutput %2\n", []),
    ("%1 = unfold %0 kh=3 kw=3\n%2 = softmax %1 axis=C\n%3 = fold %2 op=max\noutput %3\n", []),
    ("%1 = unfold %0 kh=3 kw=3\n%2 = binary %0 %1 op=mul\n%3 = fold %2 op=avg\noutput %3\n", []),
    ("%1 = unfold %0 kh=3 kw=3\n%2 = fold %1 op=max\noutput %2\n", []),
    ("%1 = fc %0 groups=2 out=8\n%2 = unary %1 op=gelu\n%3 = binary %0 %2 op=mul\noutput %3\n", [(2, 4, 2)]),
    ("%1 = fc %0 groups=1 out=9\n%2 = softmax %1 axis=C\n%3 = unfold %0 kh=3 kw=3\n%4 = binary %2 %3 op=mul\n"
     "%5 = fold %4 op=sum\n%6 = fc %5 groups=1 out=4\noutput %6\n", [(1, 9, 4), (1, 4, 4)]),
    ("%1 = shift %0 dh=0 dw=1 c0=0 c1=2\n%2 = fc %1 groups=2 out=4\n%3 = unary %2 op=relu\n%4 = binary %0 %3 op=add\n"
     "output %4\n", [(2, 2, 2)]),
    ("%1 = unfold %0 kh=3 kw=3\n%2 = fc %1 groups=2 out=4\n%3 = unary %2 op=gelu\n%4 = shift %3 dh=0 dw=1 c0=2 c1=4\n"
     "%5 = binary %0 %4 op=mul\n%6 = fold %5 op=avg\n%7 = fc %6 groups=1 out=4\noutput %7\n", [(2, 2, 18), (1, 4, 4)]),
    ("%1 = unfold %0 kh=3 kw=3\n%2 = unary %1 op=abs\n%3 = binary %0 %2 op=mul\n%4 = softmax %3 axis=T\noutput %4\n", []),
    ("%1 = unfold %0 kh=1 kw=3\n%2 = softmax %1 axis=CT\n%3 = fold %2 op=max\noutput %3\n", []),
    # squeeze-and-excite: pooled descriptor -> FC -> gelu -> FC -> softmax -> gate on x
    ("%1 = fold %0 op=avg axis=HW\n%2 = fc %1 groups=1 out=2\n%3 = unary %2 op=gelu\n%4 = fc %3 groups=1 out=4\n"
     "%5 = softmax %4 axis=C\n%6 = binary %5 %0 op=mul\noutput %6\n", [(1, 2, 4), (1, 4, 2)]),
    ("%1 = unfold %0 kh=3 kw=3\n%2 = fold %1 op=max axis=HW\n%3 = binary %2 %1 op=sub\n%4 = fold %3 op=avg\noutput %4\n", []),
    ("%1 = unfold %0 kh=3 kw=3\n%2 = fold %1 op=max axis=C groups=2\n%3 = fold %2 op=avg\n%4 = binary %3 %0 op=mul\noutput %4\n", []),
    ("%1 = unary %0 op=sin\noutput %1\n", []),
    ("%1 = unfold %0 kh=3 kw=3\n%2 = unary %1 op=sin\n%3 = binary %0 %2 op=sub\n%4 = fold %3 op=sum\noutput %4\n", []),
    ("%1 = shift %0 dh=1 dw=0\n%2 = unary %1 op=gelu\n%3 = binary %2 %0 op=max\noutput %3\n", []),
    ("%1 = unfold %0 kh=3 kw=1\n%2 = fc %0 groups=1 out=2\n%3 = binary %2 %1 op=min\n%4 = fold %3 op=avg\noutput %4\n", [(1, 2, 4)]),
    # grouped Involution: per-group window weights, replicated inside each group
    ("%1 = group %0 groups=2\n%2 = fc %1 out=6\n%3 = softmax %2 axis=C\n%4 = unfold %1 kh=3 kw=1\n%5 = binary %3 %4 op=mul\n"
     "%6 = fold %5 op=sum\n%7 = fc %6 out=4\noutput %7\n", [(2, 3, 2), (2, 2, 2)]),
    ("%1 = group %0 groups=4\n%2 = unfold %1 kh=3 kw=3\n%3 = fc %2 out=8\n%4 = unary %3 op=gelu\n%5 = binary %1 %4 op=mul\noutput %5\n", [(4, 2, 9)]),
    # folds over one spatial dim: a row profile gates the columns, a column profile is subtracted
    ("%1 = fold %0 op=avg axis=H\n%2 = unary %1 op=gelu\n%3 = binary %2 %0 op=mul\n%4 = fold %0 op=max axis=W\n%5 = binary %4 %3 op=sub\noutput %5\n", []),
    ("%1 = unfold %0 kh=3 kw=1\n%2 = fold %1 op=max axis=W\n%3 = fold %2 op=sum axis=H\n%4 = softmax %3 axis=T\n%5 = binary %4 %1 op=mul\n%6 = fold %5 op=sum\noutput %6\n", []),
    # spatial aggregation and kernel spanning: pool to [C], FC to H*W (= 20 here), laid over the pixels of x
    ("%1 = fold %0 op=avg axis=HW\n%2 = fc %1 groups=1 out=20\n%3 = unary %2 op=gelu\n%4 = binary %3 %0 op=mul lhs=pixels\noutput %4\n", [(1, 20, 4)]),
    ("%1 = unfold %0 kh=1 kw=3\n%2 = fold %0 op=max axis=HW\n%3 = fc %2 groups=2 out=20\n%4 = binary %3 %1 op=max lhs=pixels\n%5 = fold %4 op=sum\noutput %5\n", [(2, 10, 2)]),
]


@pytest.mark.parametrize("body,wshapes", FD_BODIES)
def test_finite_differences(oracle, body, wshapes):
    rng = np.random.default_rng(20)
    x = away_from_kinks(rng.standard_normal((2, 4, 4, 5)))
    ws = [rng.standard_normal(s) * 0.5 for s in wshapes]
    fd_check(oracle, body, x, ws)


# ------------------------------------------------------------------ unary

def test_unary_closed_forms(oracle):
    x = np.array([-3.0, -1.0, -0.25, 0.0, 0.5, 1.0, 2.5, 7.0]).reshape(1, 8, 1, 1)
    dy = np.ones_like(x)
    v = x.ravel()
    r = run1(oracle, "%1 = unary %0 op=relu\noutput %1\n", x, (), dy)
    np.testing.assert_array_equal(r["y"].ravel(), np.maximum(v, 0))
    np.testing.assert_array_equal(r["dx"].ravel(), (v > 0).astype(float))  # derivative 0 at 0
    r = run1(oracle, "%1 = unary %0 op=abs\noutput %1\n", x, (), dy)
    np.testing.assert_array_equal(r["y"].ravel(), np.abs(v))
    np.testing.assert_array_equal(r["dx"].ravel(), np.sign(v))  # sign(0) = 0
    r = run1(oracle, "%1 = unary %0 op=gelu\noutput %1\n", x, (), dy)
    exp = np.array([t * 0.5 * (1 + math.erf(t / math.sqrt(2))) for t in v])
    np.testing.assert_allclose(r["y"].ravel(), exp, atol=1e-15)
    assert r["y"].ravel()[3] == 0.0 and r["dx"].ravel()[3] == 0.5  # gelu(0) = 0, gelu'(0) = 1/2
    r = run1(oracle, "%1 = unary %0 op=expclip lo=-1 hi=2\noutput %1\n", x, (), dy)
    np.testing.assert_allclose(r["y"].ravel(), np.exp(np.clip(v, -1, 2)), atol=1e-15)
    inside = (v > -1) & (v < 2)
    np.testing.assert_allclose(r["dx"].ravel(), np.where(inside, np.exp(v), 0.0), atol=1e-15)
    # the boundary itself has zero gradient (open interval)
    assert r["dx"].ravel()[1] == 0.0


def test_sin_closed_form(oracle):
    x = np.array([-math.pi, -0.5 * math.pi, -0.3, 0.0, 0.3, 0.5 * math.pi, 2.0, 9.0]).reshape(1, 8, 1, 1)
    r = run1(oracle, "%1 = unary %0 op=sin\noutput %1\n", x, (), np.ones_like(x))
    np.testing.assert_allclose(r["y"].ravel(), np.sin(x.ravel()), atol=1e-15)
    np.testing.assert_allclose(r["dx"].ravel(), np.cos(x.ravel()), atol=1e-15)
    assert r["y"].ravel()[3] == 0.0 and r["dx"].ravel()[3] == 1.0
    # sin(x)^2 + (d/dx sin x)^2 = 1
    np.testing.assert_allclose(r["y"] ** 2 + r["dx"] ** 2, 1.0, atol=1e-15)


# ------------------------------------------------- blends other than add/mul

def test_sub_min_max_definitions_and_operand_order(oracle):
    """out = op(tile(LHS), RHS): sub is LHS - RHS; min + max = LHS + RHS; max - min = |LHS - RHS|."""
    rng = np.random.default_rng(30)
    x = rng.standard_normal((2, 3, 4, 5))
    body = "%1 = shift %0 dh=0 dw=1\n%2 = binary %0 %1 op={op}\noutput %2\n"
    a = x
    b = np.zeros_like(x)
    b[..., :-1] = x[..., 1:]
    got = {op: run1(oracle, body.format(op=op), x)["y"] for op in ("sub", "min", "max", "add")}
    np.testing.assert_array_equal(got["sub"], a - b)
    np.testing.assert_array_equal(got["min"], np.minimum(a, b))
    np.testing.assert_array_equal(got["max"], np.maximum(a, b))
    np.testing.assert_array_equal(got["min"] + got["max"], got["add"])
    np.testing.assert_array_equal(got["max"] - got["min"], np.abs(got["sub"]))
    # swapping the operands negates sub and leaves min / max alone
    swapped = "%1 = shift %0 dh=0 dw=1\n%2 = binary %1 %0 op={op}\noutput %2\n"
    np.testing.assert_array_equal(run1(oracle, swapped.format(op="sub"), x)["y"], b - a)
    np.testing.assert_array_equal(run1(oracle, swapped.format(op="max"), x)["y"], got["max"])


def test_sub_min_max_gradients(oracle):
    """sub: +g to the LHS, -g to the RHS.  min / max: all of g to the selected side; a tie goes to the LHS."""
    # two weight-free routes from x: LHS = relu(x) (gradient 1 where x > 0), RHS = |x| (gradient sign x)
    x = np.array([-2.0, -0.5, 0.0, 0.5, 3.0]).reshape(1, 5, 1, 1)
    g = np.array([1.0, 2.0, 3.0, 4.0, 5.0]).reshape(1, 5, 1, 1)
    body = "%1 = unary %0 op=relu\n%2 = unary %0 op=abs\n%3 = binary %1 %2 op={op}\noutput %3\n"
    v = x.ravel()
    relu_g, abs_g = (v > 0).astype(float), np.sign(v)
    r = run1(oracle, body.format(op="sub"), x, (), g)
    np.testing.assert_array_equal(r["y"].ravel(), np.maximum(v, 0) - np.abs(v))
    np.testing.assert_array_equal(r["dx"].ravel(), g.ravel() * (relu_g - abs_g))
    # relu(x) <= |x| everywhere, equal for x >= 0: min picks the LHS on ties, max picks the LHS only on ties
    r = run1(oracle, body.format(op="min"), x, (), g)
    np.testing.assert_array_equal(r["y"].ravel(), np.maximum(v, 0))
    np.testing.assert_array_equal(r["dx"].ravel(), g.ravel() * relu_g)
    r = run1(oracle, body.format(op="max"), x, (), g)
    np.testing.assert_array_equal(r["y"].ravel(), np.abs(v))
    np.testing.assert_array_equal(r["dx"].ravel(), g.ravel() * np.where(v >= 0, relu_g, abs_g))


def test_min_max_broadcast_sums_over_replicas(oracle):
    """LHS [C,1] against RHS [C,9]: the LHS gradient is the sum over the taps that selected it."""
    rng = np.random.default_rng(31)
    x = rng.standard_normal((1, 2, 4, 4))
    g = rng.standard_normal((1, 2, 9, 4, 4))
    r = run1(oracle, "%1 = unfold %0 kh=3 kw=3\n%2 = binary %0 %1 op=max\noutput %2\n", x, (), g)
    u = run1(oracle, "%1 = unfold %0 kh=3 kw=3\noutput %1\n", x)["y"]
    a = np.broadcast_to(x[:, :, None], u.shape)
    np.testing.assert_array_equal(r["y"], np.maximum(a, u))
    lhs_wins = a >= u
    # route through the unfold adjoint for the RHS part: reuse the oracle's own (separately pinned) unfold backward
    rhs_part = run1(oracle, "%1 = unfold %0 kh=3 kw=3\noutput %1\n", x, (), np.where(lhs_wins, 0.0, g))["dx"]
    np.testing.assert_allclose(r["dx"], np.where(lhs_wins, g, 0.0).sum(axis=2) + rhs_part, atol=1e-14)


# ------------------------------------------- fold over the spatial dims

def test_spatial_fold_definitions(oracle):
    """fold axis=HW: sum / mean / max over the pixels of every (channel, tap) plane; the result is [C, T, 1, 1]."""
    rng = np.random.default_rng(40)
    x = rng.standard_normal((2, 3, 4, 5))
    for op, fn in (("sum", np.sum), ("avg", np.mean), ("max", np.max)):
        y = run1(oracle, f"%1 = fold %0 op={op} axis=HW\noutput %1\n", x)["y"]
        assert y.shape == (2, 3, 1, 1)
        np.testing.assert_allclose(y[:, :, 0, 0], fn(x, axis=(2, 3)), atol=1e-14)
    u = run1(oracle, "%1 = unfold %0 kh=3 kw=1\noutput %1\n", x)["y"]
    y = run1(oracle, "%1 = unfold %0 kh=3 kw=1\n%2 = fold %1 op=avg axis=HW\noutput %2\n", x)["y"]
    assert y.shape == (2, 3, 3, 1, 1)
    np.testing.assert_allclose(y[..., 0, 0], u.mean(axis=(3, 4)), atol=1e-14)
    # folding the taps and the pixels commutes for sum / avg
    a = run1(oracle, "%1 = unfold %0 kh=3 kw=1\n%2 = fold %1 op=avg axis=HW\n%3 = fold %2 op=avg\noutput %3\n", x)["y"]
    b = run1(oracle, "%1 = unfold %0 kh=3 kw=1\n%2 = fold %1 op=avg\n%3 = fold %2 op=avg axis=HW\noutput %3\n", x)["y"]
    np.testing.assert_allclose(a, b, atol=1e-14)


def test_spatial_fold_gradients(oracle):
    x = np.arange(24, dtype=float).reshape(1, 2, 3, 4)
    x[0, 1] = 5.0            # a plane of ties: max takes the first pixel
    x[0, 0, 1, 2] = 100.0    # a unique maximum
    g = np.array([2.0, -3.0]).reshape(1, 2, 1, 1)
    r = run1(oracle, "%1 = fold %0 op=sum axis=HW\noutput %1\n", x, (), g)
    np.testing.assert_array_equal(r["dx"], np.broadcast_to(g, x.shape))
    r = run1(oracle, "%1 = fold %0 op=avg axis=HW\noutput %1\n", x, (), g)
    np.testing.assert_allclose(r["dx"], np.broadcast_to(g / 12.0, x.shape), atol=1e-16)
    r = run1(oracle, "%1 = fold %0 op=max axis=HW\noutput %1\n", x, (), g)
    exp = np.zeros_like(x)
    exp[0, 0, 1, 2] = 2.0
    exp[0, 1, 0, 0] = -3.0
    np.testing.assert_array_equal(r["dx"], exp)


def test_pooled_tensor_is_replicated_over_pixels(oracle):
    """y = x * mean_hw(x): closed-form value and gradient; an FC of a pooled tensor is a matrix-vector product."""
    rng = np.random.default_rng(41)
    x = rng.standard_normal((2, 3, 4, 5))
    g = rng.standard_normal(x.shape)
    r = run1(oracle, "%1 = fold %0 op=avg axis=HW\n%2 = binary %1 %0 op=mul\noutput %2\n", x, (), g)
    m = x.mean(axis=(2, 3), keepdims=True)
    np.testing.assert_allclose(r["y"], x * m, atol=1e-14)
    np.testing.assert_allclose(r["dx"], g * m + (g * x).sum(axis=(2, 3), keepdims=True) / 20.0, atol=1e-14)
    w = rng.standard_normal((1, 4, 3))
    gy = rng.standard_normal((2, 4, 1, 1))
    r = run1(oracle, "%1 = fold %0 op=avg axis=HW\n%2 = fc %1 groups=1 out=4\noutput %2\n", x, [w], gy)
    np.testing.assert_allclose(r["y"][:, :, 0, 0], m[:, :, 0, 0] @ w[0].T, atol=1e-14)
    np.testing.assert_allclose(r["dw"][0][0], gy[:, :, 0, 0].T @ m[:, :, 0, 0], atol=1e-14)
    np.testing.assert_allclose(r["dx"], np.broadcast_to(((gy[:, :, 0, 0] @ w[0]) / 20.0)[:, :, None, None], x.shape), atol=1e-14)


def test_channel_group_fold(oracle):
    """fold axis=C groups=G: sum / mean / max over the C/G channels of each group; G channels remain."""
    rng = np.random.default_rng(42)
    x = rng.standard_normal((2, 6, 3, 4))
    xg = x.reshape(2, 3, 2, 3, 4)
    for op, fn in (("sum", np.sum), ("avg", np.mean), ("max", np.max)):
        y = run1(oracle, f"%1 = fold %0 op={op} axis=C groups=3\noutput %1\n", x)["y"]
        assert y.shape == (2, 3, 3, 4)
        np.testing.assert_allclose(y, fn(xg, axis=2), atol=1e-15)
        y1 = run1(oracle, f"%1 = fold %0 op={op} axis=C\noutput %1\n", x)["y"]  # one group: all channels
        np.testing.assert_allclose(y1[:, 0], fn(x, axis=1), atol=1e-15)
        # as many groups as channels: the identity
        np.testing.assert_array_equal(run1(oracle, f"%1 = fold %0 op={op} axis=C groups=6\noutput %1\n", x)["y"], x)
    # with taps: every tap is folded on its own
    u = run1(oracle, "%1 = unfold %0 kh=1 kw=3\noutput %1\n", x)["y"]
    y = run1(oracle, "%1 = unfold %0 kh=1 kw=3\n%2 = fold %1 op=avg axis=C groups=2\noutput %2\n", x)["y"]
    np.testing.assert_allclose(y, u.reshape(2, 2, 3, 3, 3, 4).mean(axis=2), atol=1e-15)
    # gradients: sum replicates, avg divides by the group size, max goes to the first maximal channel
    g = rng.standard_normal((2, 3, 3, 4))
    r = run1(oracle, "%1 = fold %0 op=sum axis=C groups=3\noutput %1\n", x, (), g)
    np.testing.assert_array_equal(r["dx"], np.repeat(g, 2, axis=1))
    r = run1(oracle, "%1 = fold %0 op=avg axis=C groups=3\noutput %1\n", x, (), g)
    np.testing.assert_allclose(r["dx"], np.repeat(g, 2, axis=1) / 2.0, atol=1e-16)
    xt = x.copy()
    xt[:, 1] = xt[:, 0]  # a tie inside group 0: the first channel takes it
    r = run1(oracle, "%1 = fold %0 op=max axis=C groups=3\noutput %1\n", xt, (), g)
    first = np.argmax(xt.reshape(2, 3, 2, 3, 4), axis=2)
    exp = np.zeros((2, 3, 2, 3, 4))
    for c in range(2):
        exp[:, :, c] = np.where(first == c, g, 0.0)
    np.testing.assert_array_equal(r["dx"], exp.reshape(2, 6, 3, 4))
    assert (r["dx"][:, 1] == 0).all()
    with pytest.raises(Exception):
        run1(oracle, "%1 = fold %0 op=avg axis=C groups=4\noutput %1\n", x)


def test_spatial_fold_legality(oracle):
    x = np.zeros((1, 4, 3, 3))
    for body in ("%1 = fold %0 op=avg axis=HW\n%2 = unfold %1 kh=3 kw=3\noutput %2\n",      # no window without pixels
                 "%1 = fold %0 op=avg axis=HW\n%2 = shift %1 dh=0 dw=1\noutput %2\n",
                 "%1 = fold %0 op=avg axis=HW\n%2 = fold %1 op=max axis=HW\noutput %2\n",       # already folded
                 "%1 = fold %0 op=avg axis=HW\n%2 = binary %0 %1 op=add\noutput %2\n",          # LHS larger than RHS
                 "%1 = fold %0 op=avg axis=X\noutput %1\n"):
        with pytest.raises(Exception):
            run1(oracle, body, x)


# ---------------------------------------------------------------- softmax

@pytest.mark.parametrize("axis", ["C", "T"])
def test_softmax_invariants(oracle, axis):
    rng = np.random.default_rng(30)
    x = rng.standard_normal((2, 5, 4, 3))
    body = f"%1 = unfold %0 kh=3 kw=3\n%2 = softmax %1 axis={axis}\noutput %2\n"
    y = run1(oracle, body, x)["y"]  # [N, C, T, H, W]
    ax = 1 if axis == "C" else 2
    np.testing.assert_allclose(y.sum(axis=ax), 1.0, atol=1e-14)
    assert (y > 0).all()
    dy = rng.standard_normal(y.shape)
    # gradient w.r.t. the softmax input sums to zero along the axis: check on a DAG without unfold
    if axis == "C":
        r = run1(oracle, "%1 = softmax %0 axis=C\noutput %1\n", x, (), dy[:, :, 0])
        np.testing.assert_allclose(r["dx"].sum(axis=1), 0.0, atol=1e-14)
        y1 = run1(oracle, "%1 = softmax %0 axis=C\noutput %1\n", x + 3.25)["y"]
        np.testing.assert_allclose(y1, r["y"], atol=1e-14)  # shift invariance
        e = np.exp(x)
        np.testing.assert_allclose(r["y"], e / e.sum(axis=1, keepdims=True), atol=1e-14)


def test_joint_softmax_over_channels_and_taps(oracle):
    """axis=CT: one distribution over all (channel, tap) pairs of a pixel."""
    rng = np.random.default_rng(33)
    x = rng.standard_normal((2, 3, 4, 5))
    body = "%1 = unfold %0 kh=3 kw=1\n%2 = softmax %1 axis=CT\noutput %2\n"
    u = run1(oracle, "%1 = unfold %0 kh=3 kw=1\noutput %1\n", x)["y"]  # [N, C, T, H, W]
    y = run1(oracle, body, x)["y"]
    e = np.exp(u - u.max(axis=(1, 2), keepdims=True))
    np.testing.assert_allclose(y, e / e.sum(axis=(1, 2), keepdims=True), atol=1e-15)
    np.testing.assert_allclose(y.sum(axis=(1, 2)), 1.0, atol=1e-14)
    # with one tap it is the channel softmax, with one channel the tap softmax
    np.testing.assert_array_equal(run1(oracle, "%1 = softmax %0 axis=CT\noutput %1\n", x)["y"],
                                  run1(oracle, "%1 = softmax %0 axis=C\noutput %1\n", x)["y"])
    x1 = x[:, :1]
    np.testing.assert_array_equal(run1(oracle, "%1 = unfold %0 kh=3 kw=3\n%2 = softmax %1 axis=CT\noutput %2\n", x1)["y"],
                                  run1(oracle, "%1 = unfold %0 kh=3 kw=3\n%2 = softmax %1 axis=T\noutput %2\n", x1)["y"])
    # Jacobian-vector product: dx_j = y_j (g_j - sum_k g_k y_k) over the joint index, through the unfold adjoint
    g = rng.standard_normal(y.shape)
    r = run1(oracle, body, x, (), g)
    gu = y * (g - (g * y).sum(axis=(1, 2), keepdims=True))
    np.testing.assert_allclose(r["dx"], run1(oracle, "%1 = unfold %0 kh=3 kw=1\noutput %1\n", x, (), gu)["dx"], atol=1e-14)


@pytest.mark.parametrize("axis", ["H", "W", "HW"])
def test_softmax_over_spatial_dims(oracle, axis):
    """Softmax "at any continuous dims" (table of primitives): along H, along W, or over both jointly, of every
    (channel, tap) plane.  Pinned by the closed form on a non-square plane with taps (a swapped h / w or a softmax that
    ran across taps or channels fails), by the normalisation and shift invariance, by the closed-form Jacobian-vector
    product through the unfold adjoint, by finite differences, and by the transposed image."""
    rng = np.random.default_rng(41)
    x = rng.standard_normal((2, 3, 4, 5))
    dims = {"H": (3,), "W": (4,), "HW": (3, 4)}[axis]
    body = f"%1 = unfold %0 kh=1 kw=3\n%2 = softmax %1 axis={axis}\noutput %2\n"
    u = run1(oracle, "%1 = unfold %0 kh=1 kw=3\noutput %1\n", x)["y"]  # [N, C, T, H, W]
    y = run1(oracle, body, x)["y"]
    e = np.exp(u - u.max(axis=dims, keepdims=True))
    np.testing.assert_allclose(y, e / e.sum(axis=dims, keepdims=True), atol=1e-15)
    np.testing.assert_allclose(y.sum(axis=dims), 1.0, atol=1e-14)
    # no unfold: plain [N, C, H, W]; adding a constant per plane changes nothing
    plain = f"%1 = softmax %0 axis={axis}\noutput %1\n"
    y0 = run1(oracle, plain, x)["y"]
    d0 = tuple(d - 1 for d in dims)
    e0 = np.exp(x)
    np.testing.assert_allclose(y0, e0 / e0.sum(axis=d0, keepdims=True), atol=1e-14)
    np.testing.assert_allclose(run1(oracle, plain, x + rng.standard_normal((2, 3, 1, 1)))["y"], y0, atol=1e-14)
    # backward: dx_j = y_j (g_j - sum_k g_k y_k) along the axis; its sum along the axis is zero
    g = rng.standard_normal(y.shape)
    r = run1(oracle, body, x, (), g)
    gu = y * (g - (g * y).sum(axis=dims, keepdims=True))
    np.testing.assert_allclose(r["dx"], run1(oracle, "%1 = unfold %0 kh=1 kw=3\noutput %1\n", x, (), gu)["dx"], atol=1e-14)
    g0 = rng.standard_normal(x.shape)
    np.testing.assert_allclose(run1(oracle, plain, x, (), g0)["dx"].sum(axis=d0), 0.0, atol=1e-14)
    fd_check(oracle, body, x, ())
    # the transposed image: softmax along H of x equals softmax along W of x^T, transposed back
    if axis != "HW":
        other = "W" if axis == "H" else "H"
        yt = run1(oracle, f"%1 = softmax %0 axis={other}\noutput %1\n", np.ascontiguousarray(x.transpose(0, 1, 3, 2)))["y"]
        np.testing.assert_allclose(y0, yt.transpose(0, 1, 3, 2), atol=1e-15)
    else:
        # jointly over H and W is not H then W
        hw = run1(oracle, "%1 = softmax %0 axis=H\n%2 = softmax %1 axis=W\noutput %2\n", x)["y"]
        assert np.abs(hw - y0).max() > 1e-3
        # but on a one-row image it is the softmax along W (and along H it is all ones)
        x1 = x[:, :, :1]
        np.testing.assert_array_equal(run1(oracle, plain, x1)["y"], run1(oracle, "%1 = softmax %0 axis=W\noutput %1\n", x1)["y"])
        np.testing.assert_array_equal(run1(oracle, "%1 = softmax %0 axis=H\noutput %1\n", x1)["y"], np.ones_like(x1))


def test_softmax_over_single_tap_is_all_ones_with_zero_gradient(oracle):
    x = np.random.default_rng(31).standard_normal((1, 3, 2, 2))
    r = run1(oracle, "%1 = softmax %0 axis=T\noutput %1\n", x, (), np.ones((1, 3, 2, 2)))
    np.testing.assert_array_equal(r["y"], np.ones_like(x))
    np.testing.assert_array_equal(r["dx"], np.zeros_like(x))


def test_softmax_large_inputs_do_not_overflow(oracle):
    x = np.array([1000.0, 1001.0, 999.0, -1000.0]).reshape(1, 4, 1, 1)
    y = run1(oracle, "%1 = softmax %0 axis=C\noutput %1\n", x)["y"].ravel()
    e = np.exp(np.array([0.0, 1.0, -1.0]))
    np.testing.assert_allclose(y[:3], e / e.sum(), atol=1e-15)
    assert y[3] == 0.0


# ------------------------------------------------------------------- fold

def test_fold_relations(oracle):
    rng = np.random.default_rng(40)
    x = rng.standard_normal((2, 3, 5, 4))
    pre = "%1 = unfold %0 kh=3 kw=3\n"
    s = run1(oracle, pre + "%2 = fold %1 op=sum\noutput %2\n", x)["y"]
    a = run1(oracle, pre + "%2 = fold %1 op=avg\noutput %2\n", x)["y"]
    m = run1(oracle, pre + "%2 = fold %1 op=max\noutput %2\n", x)["y"]
    u = run1(oracle, pre + "output %1\n", x)["y"]
    np.testing.assert_allclose(s, u.sum(axis=2), atol=1e-14)
    np.testing.assert_allclose(a, s / 9.0, atol=1e-15)
    np.testing.assert_array_equal(m, u.max(axis=2))
    assert (m >= a - 1e-15).all()
    # sum-pool of a 3x3 unfold is a box filter; check against scipy's zero-padded correlate
    from scipy.ndimage import correlate

    box = np.stack([[correlate(x[n, c], np.ones((3, 3)), mode="constant") for c in range(3)] for n in range(2)])
    np.testing.assert_allclose(s, box, atol=1e-13)


def test_fold_over_one_tap_is_identity(oracle):
    x = np.random.default_rng(41).standard_normal((1, 3, 2, 2))
    dy = np.random.default_rng(42).standard_normal((1, 3, 2, 2))
    for op in ("sum", "avg", "max"):
        r = run1(oracle, f"%1 = fold %0 op={op}\noutput %1\n", x, (), dy)
        np.testing.assert_array_equal(r["y"], x)
        np.testing.assert_array_equal(r["dx"], dy)


def test_fold_max_ties_take_first_tap(oracle):
    """Constant input: every interior pixel has 9 equal taps; the gradient goes to tap 0 only."""
    x = np.ones((1, 1, 4, 4))
    dy = np.arange(16, dtype=float).reshape(1, 1, 4, 4) + 1
    # dU via a DAG whose dx is unfold^T of the routed gradient; inspect through a per-tap mul by one-hot weights
    r = run1(oracle, "%1 = unfold %0 kh=3 kw=3\n%2 = fold %1 op=max\noutput %2\n", x, (), dy)
    # pixel (h,w) routes dy to its first maximal tap.  Interior pixels: tap 0 = neighbour (h-1,w-1).
    exp = np.zeros((4, 4))
    for h in range(4):
        for w in range(4):
            taps = [(kh, kw) for kh in range(3) for kw in range(3)]
            vals = [1.0 if (0 <= h + kh - 1 < 4 and 0 <= w + kw - 1 < 4) else 0.0 for kh, kw in taps]
            t = int(np.argmax(vals))  # numpy argmax returns the first maximum
            kh, kw = taps[t]
            exp[h + kh - 1, w + kw - 1] += dy[0, 0, h, w]
    np.testing.assert_array_equal(r["dx"][0, 0], exp)


# -------------------------------------------------------------- broadcast

def test_broadcast_equal_shapes_is_elementwise(oracle):
    rng = np.random.default_rng(50)
    x = rng.standard_normal((2, 3, 4, 4))
    r = run1(oracle, "%1 = unary %0 op=abs\n%2 = binary %1 %0 op=mul\noutput %2\n", x)
    np.testing.assert_allclose(r["y"], np.abs(x) * x, atol=1e-15)


def test_broadcast_common_channel_prefix_is_per_channel(oracle):
    """[C,H,W] onto [C,T,H,W]: the channel dim is a common prefix, so each channel meets its own taps."""
    rng = np.random.default_rng(51)
    x = rng.standard_normal((1, 4, 3, 3))
    r = run1(oracle, "%1 = unfold %0 kh=3 kw=3\n%2 = binary %0 %1 op=mul\noutput %2\n", x)
    u = run1(oracle, "%1 = unfold %0 kh=3 kw=3\noutput %1\n", x)["y"]
    np.testing.assert_allclose(r["y"], x[:, :, None] * u, atol=1e-15)


def test_broadcast_channel_tiling(oracle):
    """[C/2,H,W] onto [C,H,W]: the LHS is replicated, lhs channel = c mod (C/2)."""
    rng = np.random.default_rng(52)
    x = rng.standard_normal((2, 4, 3, 3))
    w = rng.standard_normal((1, 2, 4))
    dy = rng.standard_normal((2, 4, 3, 3))
    r = run1(oracle, "%1 = fc %0 groups=1 out=2\n%2 = binary %1 %0 op=add\noutput %2\n", x, [w], dy)
    f = np.einsum("oc,nchw->nohw", w[0], x)
    np.testing.assert_allclose(r["y"], np.concatenate([f, f], axis=1) + x, atol=1e-14)
    # gradient to the LHS sums over its replicas
    gf = dy[:, :2] + dy[:, 2:]
    np.testing.assert_allclose(r["dw"][0][0], np.einsum("nohw,nchw->oc", gf, x), atol=1e-13)


def test_broadcast_tiling_of_an_lhs_with_taps_of_its_own(oracle):
    """C_L != C_R and T_L > 1 (Section 5, Blending): the LHS [C_L, T_L] is replicated along the flattened
    (c*T_R + t) index of the RHS [C_R, T_R] modulo C_L*T_L, innermost dims aligned.  Here [6, 3] onto [4, 9]
    (36 = 2 * 18): checked against a loop over the flattened index on plain reshapes, forward and the
    gradient that reaches the LHS (seen through the weights of the FC that produces it)."""
    rng = np.random.default_rng(54)
    N, C, H, W, CL, TL, TR = 2, 4, 3, 5, 6, 3, 9
    x = rng.standard_normal((N, C, H, W))
    w = rng.standard_normal((1, CL, C))
    dy = rng.standard_normal((N, C, TR, H, W))
    body = ("%1 = fc %0 groups=1 out=6\n%2 = unfold %1 kh=3 kw=1\n%3 = unfold %0 kh=3 kw=3\n"
            "%4 = binary %2 %3 op=mul\noutput %4\n")
    r = run1(oracle, body, x, [w], dy)
    lhs = run1(oracle, "%1 = fc %0 groups=1 out=6\n%2 = unfold %1 kh=3 kw=1\noutput %2\n", x, [w])["y"]
    rhs = run1(oracle, "%1 = unfold %0 kh=3 kw=3\noutput %1\n", x)["y"]
    assert lhs.shape == (N, CL, TL, H, W) and rhs.shape == (N, C, TR, H, W)
    lflat = lhs.reshape(N, CL * TL, H, W)
    exp = np.empty_like(rhs)
    glflat = np.zeros_like(lflat)
    for c in range(C):
        for t in range(TR):
            j = (c * TR + t) % (CL * TL)
            exp[:, c, t] = lflat[:, j] * rhs[:, c, t]
            glflat[:, j] += dy[:, c, t] * rhs[:, c, t]
    np.testing.assert_allclose(r["y"], exp, atol=1e-14)
    # the gradient of the LHS goes back through the 3 x 1 unfold (tap kh reads row h + kh - 1) and the FC
    gl = glflat.reshape(N, CL, TL, H, W)
    g1 = np.zeros((N, CL, H, W))
    for kh in range(3):
        for h in range(H):
            if 0 <= h + kh - 1 < H:
                g1[:, :, h + kh - 1] += gl[:, :, kh, h]
    np.testing.assert_allclose(r["dw"][0][0], np.einsum("nohw,nchw->oc", g1, x), atol=1e-12)


def test_tie_margin_moves_only_decisions_next_to_a_kink(oracle):
    """The comparison rule's bracketing runs: margin 0 is the definition; a margin m moves the backward
    decision points by |m| * max|operand| and leaves the forward pass and every element away from a kink alone."""
    x = np.array([-2.0, -1e-7, 0.0, 1e-7, 0.5, 2.0]).reshape(1, 1, 1, 6)
    dy = np.ones_like(x)
    for op, d0, dlo, dhi in [("relu", [0, 0, 0, 1, 1, 1], [0, 1, 1, 1, 1, 1], [0, 0, 0, 0, 1, 1]),
                             ("abs", [-1, -1, 0, 1, 1, 1], [-1, 1, 1, 1, 1, 1], [-1, -1, -1, -1, 1, 1])]:
        body = f"%1 = unary %0 op={op}\noutput %1\n"
        r0 = oracle.run(H_ + body, x, [], dy)
        rl = oracle.run(H_ + body, x, [], dy, tie_margin=-1e-6)
        rh = oracle.run(H_ + body, x, [], dy, tie_margin=1e-6)
        again = oracle.run(H_ + body, x, [], dy)
        np.testing.assert_array_equal(r0["dx"].ravel(), d0)
        np.testing.assert_array_equal(rl["dx"].ravel(), dlo)
        np.testing.assert_array_equal(rh["dx"].ravel(), dhi)
        np.testing.assert_array_equal(again["dx"], r0["dx"])  # the margin does not outlive its run
        np.testing.assert_array_equal(rl["y"], r0["y"])
        np.testing.assert_array_equal(rh["y"], r0["y"])
    # arg-max of a max fold: taps within the margin of the maximum; the first of them (m < 0) or the last (m > 0)
    xm = np.zeros((1, 1, 1, 3))
    xm[0, 0, 0] = [1.0, 1.0 + 1e-6, 0.2]
    body = "%1 = unfold %0 kh=1 kw=3\n%2 = fold %1 op=max\noutput %2\n"
    dyo = np.array([0.0, 1.0, 0.0]).reshape(1, 1, 1, 3)  # only the middle pixel, whose taps are (1, 1 + 1e-6, 0.2)
    g0 = oracle.run(H_ + body, xm, [], dyo)["dx"].ravel()
    gl = oracle.run(H_ + body, xm, [], dyo, tie_margin=-1e-5)["dx"].ravel()
    gh = oracle.run(H_ + body, xm, [], dyo, tie_margin=1e-5)["dx"].ravel()
    np.testing.assert_array_equal(g0, [0, 1, 0])
    np.testing.assert_array_equal(gl, [1, 0, 0])
    np.testing.assert_array_equal(gh, [0, 1, 0])
    # decisions look at the operands in fp32, the kernels' precision: what differs only beyond that is a tie, first tap wins
    xm[0, 0, 0] = [1.0, 1.0 + 1e-12, 0.2]
    np.testing.assert_array_equal(oracle.run(H_ + body, xm, [], dyo)["dx"].ravel(), [1, 0, 0])
    np.testing.assert_array_equal(oracle.run(H_ + body, xm, [])["y"].ravel()[1], 1.0 + 1e-12)  # values are not rounded
    # min / max blends: the definition sends a tie to the LHS
    a = np.array([1.0, 1.0, 3.0]).reshape(1, 1, 1, 3)
    body = "%1 = unary %0 op=sin\n%2 = binary %1 %1 op=max\noutput %2\n"
    assert oracle.run(H_ + body, a, [], np.ones_like(a), tie_margin=1e-6)["dx"].shape == a.shape


def test_involution_core_against_explicit_dynamic_kernel(oracle):
    """Section 5: [K*K,H,W] broadcast-multiplied onto [C,K,K,H,W], then summed over taps, is a
    per-pixel dynamic KxK filter: out(c,h,w) = sum_t k(t,h,w) * x(c,h+dh_t,w+dw_t)."""
    rng = np.random.default_rng(53)
    C, H, W = 5, 4, 6
    x = rng.standard_normal((1, C, H, W))
    w1 = rng.standard_normal((1, 9, C))
    body = ("%1 = fc %0 groups=1 out=9\n%2 = unfold %0 kh=3 kw=3\n%3 = binary %1 %2 op=mul\n%4 = fold %3 op=sum\n"
            "output %4\n")
    r = run1(oracle, body, x, [w1])
    ker = np.einsum("tc,nchw->nthw", w1[0], x)
    exp = np.zeros((1, C, H, W))
    for c in range(C):
        for h in range(H):
            for w in range(W):
                for t in range(9):
                    hs, ws = h + t // 3 - 1, w + t % 3 - 1
                    if 0 <= hs < H and 0 <= ws < W:
                        exp[0, c, h, w] += ker[0, t, h, w] * x[0, c, hs, ws]
    np.testing.assert_allclose(r["y"], exp, atol=1e-13)


# ------------------------------------------------------- Group as a node of its own

def test_group_is_a_view_and_fc_inherits_it(oracle):
    """Section 5, Group: a rearrangement without copies; a following FC works inside each group, so
    group + fc equals the fc with the groups written on it, values and gradients alike."""
    rng = np.random.default_rng(70)
    x = rng.standard_normal((2, 6, 4, 5))
    r = run1(oracle, "%1 = group %0 groups=3\noutput %1\n", x, [], x * 2.0)
    np.testing.assert_array_equal(r["y"], x)
    np.testing.assert_array_equal(r["dx"], x * 2.0)
    w = rng.standard_normal((3, 2, 18))
    a = "%1 = group %0 groups=3\n%2 = unfold %1 kh=3 kw=3\n%3 = unary %2 op=abs\n%4 = fc %3 out=6\noutput %4\n"
    b = "%1 = unfold %0 kh=3 kw=3\n%2 = unary %1 op=abs\n%3 = fc %2 groups=3 out=6\noutput %3\n"
    dy = rng.standard_normal((2, 6, 4, 5))
    ra, rb = run1(oracle, a, x, [w], dy), run1(oracle, b, x, [w], dy)
    for k in ("y", "dx"):
        np.testing.assert_array_equal(ra[k], rb[k])
    np.testing.assert_array_equal(ra["dw"][0], rb["dw"][0])
    # stating the same groups again is allowed, contradicting the view is not
    run1(oracle, "%1 = group %0 groups=3\n%2 = fc %1 groups=3 out=6\noutput %2\n", x, [rng.standard_normal((3, 2, 2))])
    for bad in ("%1 = group %0 groups=3\n%2 = fc %1 groups=2 out=6\noutput %2\n", "%1 = group %0 groups=4\noutput %1\n",
                "%1 = group %0\noutput %1\n", "%1 = group %0 groups=0\noutput %1\n"):
        with pytest.raises(Exception):
            run1(oracle, bad, x, [rng.standard_normal((2, 3, 3))])


def test_depthwise_group_is_a_per_channel_filter(oracle):
    """[X] => [X, 1]: every channel its own group; Unfold + FC is then a depth-wise convolution."""
    rng = np.random.default_rng(71)
    C, H, W = 5, 6, 4
    x = rng.standard_normal((1, C, H, W))
    w = rng.standard_normal((C, 1, 9))
    y = run1(oracle, f"%1 = group %0 groups={C}\n%2 = unfold %1 kh=3 kw=3\n%3 = fc %2 out={C}\noutput %3\n", x, [w])["y"]
    exp = np.zeros_like(x)
    xp = np.pad(x, ((0, 0), (0, 0), (1, 1), (1, 1)))
    for c in range(C):
        for kh in range(3):
            for kw in range(3):
                exp[0, c] += w[c, 0, kh * 3 + kw] * xp[0, c, kh:kh + H, kw:kw + W]
    np.testing.assert_allclose(y, exp, atol=1e-13)


def test_grouped_broadcast_equals_the_groups_run_one_by_one(oracle):
    """With the same Group view on both sides G is a common leading dim (Section 5: [G, x/G, H, W] onto
    [G, C/G, K_H, H, W]): the blend of group g involves only the channels of group g, i.e. the result is
    what the ungrouped DAG gives on each group's channel slice, concatenated."""
    rng = np.random.default_rng(72)
    G, C, H, W = 2, 8, 4, 5
    x = rng.standard_normal((2, C, H, W))
    w = rng.standard_normal((G, 3, C // G))          # fc to 3 channels per group = one per tap of a 3x1 window
    dy = rng.standard_normal((2, C, 3, H, W))
    for op in ("mul", "sub", "max"):
        body = (f"%1 = group %0 groups={G}\n%2 = fc %1 out={3 * G}\n%3 = unfold %1 kh=3 kw=1\n"
                f"%4 = binary %2 %3 op={op}\noutput %4\n")
        r = run1(oracle, body, x, [w], dy)
        one = f"%1 = fc %0 groups=1 out=3\n%2 = unfold %0 kh=3 kw=1\n%3 = binary %1 %2 op={op}\noutput %3\n"
        cg = C // G
        for g in range(G):
            sl = slice(g * cg, (g + 1) * cg)
            rg = run1(oracle, one, np.ascontiguousarray(x[:, sl]), [w[g:g + 1]], np.ascontiguousarray(dy[:, sl]))
            np.testing.assert_array_equal(r["y"][:, sl], rg["y"])
            np.testing.assert_allclose(r["dx"][:, sl], rg["dx"], atol=1e-13)
            np.testing.assert_allclose(r["dw"][0][g], rg["dw"][0][0], atol=1e-12)
        # and it differs from the blend without the common group dim (flat replication pairs other channels)
        flat = f"%1 = fc %0 groups={G} out={3 * G}\n%2 = unfold %0 kh=3 kw=1\n%3 = binary %1 %2 op={op}\noutput %3\n"
        assert not np.allclose(run1(oracle, flat, x, [w])["y"], r["y"])


def test_grouped_involution_against_explicit_per_group_kernel(oracle):
    """Section 5's Involution: [G, K, K, H, W] times [G, C/G, K, K, H, W], summed over the window:
    out(g, c, h, w) = sum_t ker(g, t, h, w) * x(g, c, h + dh_t, w + dw_t)."""
    rng = np.random.default_rng(73)
    G, C, H, W = 3, 6, 4, 5
    cg = C // G
    x = rng.standard_normal((1, C, H, W))
    w1 = rng.standard_normal((G, 9, cg))
    body = (f"%1 = group %0 groups={G}\n%2 = fc %1 out={9 * G}\n%3 = unfold %1 kh=3 kw=3\n%4 = binary %2 %3 op=mul\n"
            "%5 = fold %4 op=sum\noutput %5\n")
    y = run1(oracle, body, x, [w1])["y"]
    xg = x.reshape(1, G, cg, H, W)
    ker = np.einsum("gtc,ngchw->ngthw", w1, xg)
    xp = np.pad(xg, ((0, 0), (0, 0), (0, 0), (1, 1), (1, 1)))
    exp = np.zeros_like(xg)
    for t in range(9):
        exp += ker[:, :, t][:, :, None] * xp[:, :, :, t // 3:t // 3 + H, t % 3:t % 3 + W]
    np.testing.assert_allclose(y, exp.reshape(1, C, H, W), atol=1e-13)


def test_group_view_legality_and_propagation(oracle):
    x = np.zeros((1, 8, 3, 3))
    # LHS [G=2, 3 per group] onto RHS [G=2, 4 per group]: 3 does not divide 4 (flat 6 | 8 fails as well)
    with pytest.raises(Exception):
        run1(oracle, "%1 = group %0 groups=2\n%2 = fc %1 out=6\n%3 = binary %2 %1 op=add\noutput %3\n", x, [np.zeros((2, 3, 4))])
    # per group 2 | 4 holds, while flat replication of 4 onto 8 would hold too; views differ -> flat rule
    run1(oracle, "%1 = group %0 groups=2\n%2 = fc %1 out=4\n%3 = binary %2 %0 op=add\noutput %3\n", x, [np.zeros((2, 2, 4))])
    # a channel fold drops the view: the following fc is an ordinary one
    _, _, ws = oracle.infer(H_ + "%1 = group %0 groups=2\n%2 = fold %1 op=sum axis=C groups=4\n%3 = fc %2 out=4\noutput %3\n", (1, 8, 3, 3))
    assert ws == [[1, 4, 4]]
    ns, _, ws = oracle.infer(H_ + "%1 = group %0 groups=4\n%2 = unfold %1 kh=3 kw=3\n%3 = fold %2 op=max axis=HW\n%4 = fc %3 out=12\noutput %4\n", (1, 8, 3, 3))
    assert ws == [[4, 3, 18]] and ns[4] == [12, 1, 1, 1]


def test_folds_over_one_spatial_dim(oracle):
    """Section 5, Folding removes any one dim: axis=H and axis=W against numpy reductions, their gradients in
    closed form, the first-maximum rule, H then W equals HW, and replication of the folded result along the dim
    it lost (numpy broadcasting)."""
    rng = np.random.default_rng(90)
    N, C, H, W = 2, 3, 4, 5
    x = rng.standard_normal((N, C, H, W))
    for axis, ax in (("H", 2), ("W", 3)):
        shape = (N, C, 1, W) if axis == "H" else (N, C, H, 1)
        dy = rng.standard_normal(shape)
        for op, fn in (("sum", np.sum), ("avg", np.mean), ("max", np.max)):
            r = run1(oracle, f"%1 = fold %0 op={op} axis={axis}\noutput %1\n", x, [], dy)
            np.testing.assert_allclose(r["y"], fn(x, axis=ax, keepdims=True), atol=1e-14)
            if op == "max":
                g = np.zeros_like(x)
                idx = np.argmax(x, axis=ax)      # numpy's argmax is the first maximum as well
                if axis == "H":
                    for n in range(N):
                        for c in range(C):
                            for w in range(W):
                                g[n, c, idx[n, c, w], w] = dy[n, c, 0, w]
                else:
                    for n in range(N):
                        for c in range(C):
                            for h in range(H):
                                g[n, c, h, idx[n, c, h]] = dy[n, c, h, 0]
            else:
                g = np.broadcast_to(dy, x.shape) / (1 if op == "sum" else x.shape[ax])
            np.testing.assert_allclose(r["dx"], g, atol=1e-14)
    # ties: constant input, the gradient goes to index 0 of the folded dim
    r = run1(oracle, "%1 = fold %0 op=max axis=W\noutput %1\n", np.ones((1, 1, 2, 3)), [], np.array([[[[5.0], [7.0]]]]))
    np.testing.assert_array_equal(r["dx"][0, 0], [[5, 0, 0], [7, 0, 0]])
    # H then W (and W then H) is the fold over both
    for op in ("sum", "avg", "max"):
        both = run1(oracle, f"%1 = fold %0 op={op} axis=HW\noutput %1\n", x)["y"]
        for a, b in (("H", "W"), ("W", "H")):
            two = run1(oracle, f"%1 = fold %0 op={op} axis={a}\n%2 = fold %1 op={op} axis={b}\noutput %2\n", x)["y"]
            np.testing.assert_allclose(two, both, atol=1e-13)
    # replication along the folded dim: a row profile [C, 1, W] onto [C, H, W]; its gradient sums over H
    dy = rng.standard_normal((N, C, H, W))
    r = run1(oracle, "%1 = fold %0 op=avg axis=H\n%2 = binary %1 %0 op=mul\noutput %2\n", x, [], dy)
    prof = x.mean(axis=2, keepdims=True)
    np.testing.assert_allclose(r["y"], prof * x, atol=1e-14)
    np.testing.assert_allclose(r["dx"], dy * prof + (dy * x).sum(axis=2, keepdims=True) / H, atol=1e-13)
    # a column profile [C, H, 1] minus an unfolded tensor [C, 3, H, W]
    u = run1(oracle, "%1 = unfold %0 kh=1 kw=3\noutput %1\n", x)["y"]
    got = run1(oracle, "%1 = unfold %0 kh=1 kw=3\n%2 = fold %0 op=max axis=W\n%3 = binary %2 %1 op=sub\noutput %3\n", x)["y"]
    np.testing.assert_allclose(got, x.max(axis=3, keepdims=True)[:, :, None] - u, atol=1e-14)
    # shapes and legality
    ns, _, _ = oracle.infer(H_ + "%1 = fold %0 op=sum axis=W\n%2 = fc %1 groups=1 out=7\n%3 = fold %2 op=max axis=H\noutput %3\n", (1, C, H, W))
    assert ns[1] == [C, 1, H, 1] and ns[2] == [7, 1, H, 1] and ns[3] == [7, 1, 1, 1]
    for bad in ("%1 = fold %0 op=sum axis=H\n%2 = fold %1 op=sum axis=H\noutput %2\n",
                "%1 = fold %0 op=sum axis=H\n%2 = fold %1 op=sum axis=HW\noutput %2\n",
                "%1 = fold %0 op=sum axis=H\n%2 = fold %0 op=sum axis=W\n%3 = binary %1 %2 op=add\noutput %3\n",   # [C,1,W] onto [C,H,1]
                "%1 = fold %0 op=sum axis=W\n%2 = binary %0 %1 op=add\noutput %2\n",                               # full-size onto folded
                "%1 = fold %0 op=sum axis=W\n%2 = unfold %1 kh=3 kw=1\noutput %2\n",
                "%1 = fold %0 op=sum axis=H\n%2 = shift %1 dh=0 dw=1\noutput %2\n",
                "%1 = fold %0 op=sum axis=X\noutput %1\n"):
        with pytest.raises(Exception):
            run1(oracle, bad, x)
    # a tensor folded over both dims is an LHS for one folded over one
    run1(oracle, "%1 = fold %0 op=sum axis=HW\n%2 = fold %0 op=sum axis=W\n%3 = binary %1 %2 op=add\noutput %3\n", x)


def test_pooled_vector_laid_over_the_pixels(oracle):
    """Section 8, the kernel with spatial aggregation and kernel spanning: pool [C,H,W] to [C], an FC to H*W
    outputs, multiplied with the input: y(c,h,w) = x(c,h,w) * (W mean_hw x)(h*W+w); the gradient of the
    vector sums over channels (and taps)."""
    rng = np.random.default_rng(80)
    N, C, H, W = 2, 3, 4, 5
    x = rng.standard_normal((N, C, H, W))
    w = rng.standard_normal((1, H * W, C))
    body = f"%1 = fold %0 op=avg axis=HW\n%2 = fc %1 groups=1 out={H * W}\n%3 = binary %2 %0 op=mul lhs=pixels\noutput %3\n"
    dy = rng.standard_normal((N, C, H, W))
    r = run1(oracle, body, x, [w], dy)
    v = np.einsum("oc,nc->no", w[0], x.mean(axis=(2, 3))).reshape(N, 1, H, W)
    np.testing.assert_allclose(r["y"], x * v, atol=1e-14)
    dv = (dy * x).sum(axis=1).reshape(N, H * W)                     # gradient of the vector
    np.testing.assert_allclose(r["dw"][0][0], np.einsum("no,nc->oc", dv, x.mean(axis=(2, 3))), atol=1e-12)
    dx = dy * v + np.einsum("no,oc->nc", dv, w[0])[:, :, None, None] / (H * W)
    np.testing.assert_allclose(r["dx"], dx, atol=1e-12)
    # operand order and taps: tile(LHS) - RHS on an unfolded RHS
    u = run1(oracle, "%1 = unfold %0 kh=3 kw=1\noutput %1\n", x)["y"]
    got = run1(oracle, f"%1 = unfold %0 kh=3 kw=1\n%2 = fold %0 op=sum axis=HW\n%3 = fc %2 groups=1 out={H * W}\n"
                       "%4 = binary %3 %1 op=sub lhs=pixels\noutput %4\n", x, [w])["y"]
    vec = np.einsum("oc,nc->no", w[0], x.sum(axis=(2, 3))).reshape(N, 1, 1, H, W)
    np.testing.assert_allclose(got, vec - u, atol=1e-12)
    # legality: the LHS must be pooled and have exactly H*W elements, the RHS must have its pixels
    for bad in (f"%1 = fold %0 op=avg axis=HW\n%2 = fc %1 groups=1 out={H * W + 1}\n%3 = binary %2 %0 op=mul lhs=pixels\noutput %3\n",
                f"%1 = fc %0 groups=1 out={H * W}\n%2 = binary %1 %0 op=mul lhs=pixels\noutput %2\n",
                f"%1 = fold %0 op=avg axis=HW\n%2 = fc %1 groups=1 out={H * W}\n%3 = binary %2 %1 op=mul lhs=pixels\noutput %3\n",
                f"%1 = fold %0 op=avg axis=HW\n%2 = fc %1 groups=1 out={H * W}\n%3 = binary %2 %0 op=mul lhs=channels\noutput %3\n"):
        with pytest.raises(Exception):
            run1(oracle, bad, x, [rng.standard_normal((1, H * W + 1, C))])


def test_fan_out_gradients_add(oracle):
    rng = np.random.default_rng(54)
    x = rng.standard_normal((1, 3, 3, 3))
    dy = rng.standard_normal((1, 3, 3, 3))
    r = run1(oracle, "%1 = binary %0 %0 op=add\n%2 = binary %1 %0 op=add\noutput %2\n", x, (), dy)
    np.testing.assert_allclose(r["y"], 3 * x, atol=1e-15)
    np.testing.assert_allclose(r["dx"], 3 * dy, atol=1e-15)
    r = run1(oracle, "%1 = binary %0 %0 op=mul\noutput %1\n", x, (), dy)
    np.testing.assert_allclose(r["dx"], 2 * x * dy, atol=1e-15)


def test_output_can_be_the_input(oracle):
    x = np.random.default_rng(55).standard_normal((1, 2, 2, 2))
    r = run1(oracle, "output %0\n", x, (), 2 * x)
    np.testing.assert_array_equal(r["y"], x)
    np.testing.assert_array_equal(r["dx"], 2 * x)


def test_batch_images_are_independent_and_dw_sums_over_batch(oracle):
    rng = np.random.default_rng(56)
    case_body = "%1 = unfold %0 kh=3 kw=3\n%2 = fc %1 groups=1 out=3\n%3 = unary %2 op=gelu\noutput %3\n"
    x = rng.standard_normal((5, 2, 4, 4))
    w = rng.standard_normal((1, 3, 18))
    dy = rng.standard_normal((5, 3, 4, 4))
    full = run1(oracle, case_body, x, [w], dy)
    acc = np.zeros_like(w)
    for n in range(5):
        one = run1(oracle, case_body, x[n:n + 1], [w], dy[n:n + 1])
        np.testing.assert_array_equal(one["y"][0], full["y"][n])
        np.testing.assert_array_equal(one["dx"][0], full["dx"][n])
        acc += one["dw"][0]
    np.testing.assert_allclose(full["dw"][0], acc, atol=1e-13)
    one_thread = oracle.run(H_ + case_body, x, [w], dy, n_threads=1)
    np.testing.assert_allclose(one_thread["dw"][0], full["dw"][0], atol=1e-13)
