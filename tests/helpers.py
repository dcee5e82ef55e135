"""Comparison rule shared by the GPU parity tests."""
import numpy as np

TOL = {"f32": 1e-5, "bf16": 2e-2}


def rel_errors(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0, 0.0, 0
    d = np.abs(got - ref)
    scale = max(np.abs(ref).max(), 1e-30)
    l2 = np.sqrt((d * d).sum()) / max(np.sqrt((ref * ref).sum()), 1e-30)
    return d.max() / scale, l2, d


def assert_close(got, ref, tol, what, kinks=False):
    """||got-ref||_inf <= tol*||ref||_inf and ||got-ref||_2 <= tol*||ref||_2.

    For DAGs with decision points (relu, abs, max, clip) a near-tie can be decided differently in fp32
    and fp64; then up to max(1, 1e-5*numel) elements may exceed the max-norm bound while the l2 bound
    must still hold.
    """
    assert np.isfinite(got).all(), f"{what}: non-finite values in the GPU result"
    einf, el2, d = rel_errors(got, ref)
    scale = max(np.abs(np.asarray(ref)).max(), 1e-30)
    if kinks:
        bad = int((d > tol * scale).sum()) if np.ndim(d) else 0
        allowed = max(1, int(1e-5 * np.asarray(ref).size))
        assert bad <= allowed, f"{what}: {bad} elements beyond {tol} (allowed {allowed}), max rel {einf:.3e}"
    else:
        assert einf <= tol, f"{what}: max-norm relative error {einf:.3e} > {tol}"
    assert el2 <= tol, f"{what}: l2 relative error {el2:.3e} > {tol}"
    return einf, el2


def has_kinks(blob):
    return any(k in blob for k in ("relu", "abs", "op=max", "expclip"))


def check_against_oracle(oracle, case, res, dy, what=None):
    ref = oracle.run(case["blob"], case["x"], case["weights"], dy)
    tol = TOL[case["dtype"]]
    what = what or case["name"]
    kinks = has_kinks(case["blob"])
    out = {"y": assert_close(res["y"], ref["y"], tol, what + ":y", kinks),
           "dx": assert_close(res["dx"], ref["dx"], tol, what + ":dx", kinks)}
    for k, (g, r) in enumerate(zip(res["dw"], ref["dw"])):
        out[f"dw{k}"] = assert_close(g, r, tol, what + f":dw{k}", kinks)
    return out, ref
