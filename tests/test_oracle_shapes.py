"""Pins the oracle's shape inference, legality rules and parameter counts to what the paper states
(Section 5 table of primitives, Broadcast divisibility rule, Involution shapes, Section 8 case study)."""
import os

import numpy as np
import pytest

from paper_2304_07741_amd import workloads as wl

H_ = wl.HEADER


def golden():
    facts = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "paper_facts.txt")) as f:
        for line in f:
            line = line.split("#")[0].split()
            if len(line) == 2:
                facts[line[0]] = line[1]
    return facts


def test_primitive_table_shapes(oracle):
    ns, out, ws = oracle.infer(H_ + "%1 = unfold %0 kh=3 kw=5\n%2 = shift %1 dh=1 dw=0\n%3 = unary %2 op=abs\n"
                               "%4 = softmax %3 axis=T\n%5 = fold %4 op=max\n%6 = fc %5 groups=4 out=24\noutput %6\n",
                               (2, 8, 6, 7))
    assert ns == [[8, 1, 6, 7], [8, 15, 6, 7], [8, 15, 6, 7], [8, 15, 6, 7], [8, 15, 6, 7], [8, 1, 6, 7], [24, 1, 6, 7]]
    assert out == 6 and ws == [[4, 6, 2]]
    assert golden()["conv_unfold_shape"] == "C,KH,KW,H,W"  # [C, K_H*K_W, H, W] with taps kh-major


def test_parameter_counts_of_the_case_study(oracle):
    """Single channel: unfold on both dims then FC has 9 weights; 1-D unfold then FC has 3 (no bias)."""
    g = golden()
    _, _, ws = oracle.infer(H_ + "%1 = unfold %0 kh=3 kw=3\n%2 = fc %1 groups=1 out=1\noutput %2\n", (1, 1, 4, 4))
    assert int(np.prod(ws[0])) == int(g["unfold2d_single_channel_params"])
    body = "%1 = unfold %0 kh=3 kw=1\n%2 = fc %1 groups=1 out=1\n%3 = shift %0 dh=0 dw=1\n%4 = binary %3 %2 op=add\noutput %4\n"
    _, _, ws = oracle.infer(H_ + body, (1, 1, 4, 4))
    assert int(np.prod(ws[0])) == int(g["unfold1d_shift_residual_params"])
    # 3 multiply-adds for the FC plus 1 add for the residual = 4 operations per pixel
    assert int(np.prod(ws[0])) + 1 == int(g["unfold1d_shift_residual_flops"])


def test_involution_shapes(oracle):
    """[G,x2/G,H,W] with x2 = G*K*K blends onto [G,C/G,K,K,H,W]; here G = 1 and G = 2."""
    ns, _, ws = oracle.infer(wl.blob_involution(128, 3), (1, 128, 28, 28))
    assert ns[1] == [9, 1, 28, 28] and ns[3] == [128, 9, 28, 28] and ns[4] == [128, 9, 28, 28]
    assert ws == [[1, 9, 128], [1, 128, 128]]
    # grouped: 2 groups of 9 dynamic weights each, tiled over the 64 channels of each group
    body = "%1 = fc %0 groups=2 out=18\n%2 = unfold %0 kh=3 kw=3\n%3 = binary %1 %2 op=mul\noutput %3\n"
    ns, _, ws = oracle.infer(H_ + body, (1, 128, 4, 4))
    assert ns[3] == [128, 9, 4, 4] and ws == [[2, 9, 64]]


def test_broadcast_divisibility(oracle):
    """The LHS size must be a factor of the RHS size after stripping common dims."""
    ok = "%1 = fc %0 groups=1 out=6\n%2 = unfold %0 kh=3 kw=1\n%3 = binary %1 %2 op=add\noutput %3\n"  # 6 | 4*3
    oracle.infer(H_ + ok, (1, 4, 4, 4))
    bad = "%1 = fc %0 groups=1 out=5\n%2 = unfold %0 kh=3 kw=1\n%3 = binary %1 %2 op=add\noutput %3\n"  # 5 !| 12
    with pytest.raises(oracle.OracleError):
        oracle.infer(H_ + bad, (1, 4, 4, 4))
    # taps cannot be broadcast onto a tensor without taps
    bad2 = "%1 = unfold %0 kh=3 kw=3\n%2 = binary %1 %0 op=add\noutput %2\n"
    with pytest.raises(oracle.OracleError):
        oracle.infer(H_ + bad2, (1, 4, 4, 4))


def test_grouped_broadcast_alignment(oracle):
    """LHS [G*K*K] onto RHS [C, K*K] with G=2: channel c of group g meets the K*K weights of group g...
    only when the flattened sizes line up, i.e. lhs index = (c*T + t) mod (G*K*K)."""
    rng = np.random.default_rng(3)
    x = rng.standard_normal((1, 4, 3, 3))
    lhs_w = rng.standard_normal((1, 6, 4))
    body = "%1 = fc %0 groups=1 out=6\n%2 = unfold %0 kh=3 kw=1\n%3 = binary %1 %2 op=mul\noutput %3\n"
    r = oracle.run(H_ + body, x, [lhs_w])
    lhs = np.einsum("oc,nchw->nohw", lhs_w[0], x)
    u = oracle.run(H_ + "%1 = unfold %0 kh=3 kw=1\noutput %1\n", x, [])["y"]
    exp = np.empty_like(u)
    for c in range(4):
        for t in range(3):
            exp[:, c, t] = lhs[:, (c * 3 + t) % 6] * u[:, c, t]
    np.testing.assert_allclose(r["y"], exp, atol=1e-14)


@pytest.mark.parametrize("body", [
    "%1 = fc %0 groups=3 out=6\noutput %1\n",            # groups must divide C
    "%1 = fc %0 groups=2 out=5\noutput %1\n",            # and the output width
    "%1 = unfold %0 kh=2 kw=3\noutput %1\n",             # even window
    "%1 = shift %0 dh=0 dw=1 c0=3 c1=9\noutput %1\n",    # slice outside the channels
    "%2 = unary %0 op=relu\noutput %2\n",                # ids must be consecutive
    "%1 = unary %1 op=relu\noutput %1\n",                # operand must precede
    "%1 = unary %0 op=tanh\noutput %1\n",
    "%1 = softmax %0 axis=X\noutput %1\n",
    "%1 = unary %0 op=expclip lo=1 hi=1\noutput %1\n",
    "%1 = unary %0 op=relu\n",                           # no output
])
def test_illegal_blobs_are_rejected(oracle, body):
    with pytest.raises(oracle.OracleError):
        oracle.infer(H_ + body, (1, 4, 4, 4))


def test_missing_header_is_rejected(oracle):
    with pytest.raises(oracle.OracleError):
        oracle.infer("%1 = unary %0 op=relu\noutput %1\n", (1, 4, 4, 4))


# ------------------------------------------------------------- workloads

def test_config_blobs_are_legal_and_weight_shapes_match(oracle):
    cases = [wl.config1(), wl.config2(N=1, H=8), wl.config3(N=1, H=6)] + [wl.config4(C, 4, N=1) for C, _ in wl.CONFIG4_SHAPES]
    for case in cases:
        ns, out, ws = oracle.infer(case["blob"], case["shape"])
        assert [tuple(s) for s in ws] == case["wshapes"], case["name"]
        assert ns[out][:2] == [case["shape"][1], 1]


def test_fuzz_generator_emits_legal_dags(oracle):
    depths = set()
    for seed in range(100, 300):
        blob, wshapes = wl.fuzz_dag(seed)
        ns, out, ws = oracle.infer(blob, (16, 96, 32, 32))
        assert ns[out] == [96, 1, 32, 32]
        assert [tuple(s) for s in ws] == wshapes
        d = len(ns) - 1
        assert 2 <= d <= 8
        depths.add(d)
        assert out == d  # chain structure: the last node is the output
        assert blob == wl.fuzz_dag(seed)[0]  # deterministic
    assert depths == set(range(2, 9))


def test_normal_generator_statistics_and_bf16_rounding():
    a = wl.normal(7, 3, (200000,))
    assert abs(a.mean()) < 0.01 and abs(a.std() - 1.0) < 0.01
    assert np.array_equal(a, wl.normal(7, 3, (200000,)))
    assert not np.array_equal(a, wl.normal(7, 4, (200000,)))
    import torch

    f = a.astype(np.float32)
    ours = wl.round_to_bf16(f)
    theirs = torch.tensor(f).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(ours, theirs)
    np.testing.assert_array_equal(wl.bf16_bits_to_f32(wl.bf16_bits(ours)), ours)
