"""Comparison rule shared by the GPU parity tests."""
import numpy as np

TOL = {"f32": 1e-5, "bf16": 2e-2}


def rel_errors(got, ref, floor=1e-30):
    """(max-norm relative error, l2 relative error, |got-ref|); norms of ref below `floor` count as floor."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0, 0.0, 0
    d = np.abs(got - ref)
    scale = max(np.abs(ref).max(), floor)
    l2 = np.sqrt((d * d).sum()) / max(np.sqrt((ref * ref).sum()), floor * np.sqrt(ref.size))
    return d.max() / scale, l2, d


def assert_close(got, ref, tol, what, kinks=False, floor=1e-30):
    """||got-ref||_inf <= tol*||ref||_inf and ||got-ref||_2 <= tol*||ref||_2.

    `floor` guards tensors that are mathematically zero (e.g. the gradient through the mean of a
    softmax): there both sides hold only cancellation noise, a relative error means nothing, and the
    norms of ref are taken as at least floor (per element), which turns the test into an absolute one.

    DAGs with decision points (relu, abs, max, clip) can hold exact mathematical ties that rounding
    resolves differently in fp32 and fp64 (e.g. exp(a)*exp(b) against exp(c)*exp(d) with a+b == c+d);
    either decision is a valid subgradient; and where values are squeezed into a narrow range (softmax of
    softmax) fp32 cannot order neighbours that fp64 can.  For such DAGs up to max(8, 1e-4*numel) elements may
    exceed the max-norm bound; they are counted, and both bounds must hold on all the others.
    """
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert np.isfinite(got).all(), f"{what}: non-finite values in the GPU result"
    einf, el2, d = rel_errors(got, ref, floor)
    if ref.size == 0:
        return 0.0, 0.0
    scale = max(np.abs(ref).max(), floor)
    if kinks:
        bad = d > tol * scale
        nbad = int(bad.sum())
        allowed = max(8, int(1e-4 * ref.size))
        assert nbad <= allowed, f"{what}: {nbad} elements beyond {tol} (allowed {allowed}), max rel {einf:.3e}"
        if nbad:
            keep = ~bad
            el2 = np.sqrt((d[keep] ** 2).sum()) / max(np.sqrt((ref[keep] ** 2).sum()), floor * np.sqrt(ref.size))
            einf = d[keep].max() / scale
    else:
        assert einf <= tol, f"{what}: max-norm relative error {einf:.3e} > {tol}"
    assert el2 <= tol, f"{what}: l2 relative error {el2:.3e} > {tol}"
    return einf, el2


def has_kinks(blob):
    return any(k in blob for k in ("relu", "abs", "op=max", "op=min", "expclip"))


def check_against_oracle(oracle, case, res, dy, what=None):
    ref = oracle.run(case["blob"], case["x"], case["weights"], dy)
    tol = TOL[case["dtype"]]
    what = what or case["name"]
    kinks = has_kinks(case["blob"])
    # gradients below 1e-5 of the incoming gradient's magnitude are cancellation noise on both sides
    gfloor = 1e-5 * float(np.abs(dy).max())
    out = {"y": assert_close(res["y"], ref["y"], tol, what + ":y", kinks),
           "dx": assert_close(res["dx"], ref["dx"], tol, what + ":dx", kinks, gfloor)}
    for k, (g, r) in enumerate(zip(res["dw"], ref["dw"])):
        out[f"dw{k}"] = assert_close(g, r, tol, what + f":dw{k}", kinks, gfloor)
    return out, ref
