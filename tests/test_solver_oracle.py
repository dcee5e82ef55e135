"""Pins of the solver oracle (oracle/solver_oracle.py): the numbers the paper prints, Theorem 1, brute force."""
import itertools
from fractions import Fraction

import numpy as np
import pytest

from oracle import solver_oracle as S
from paper_2304_07741_amd import workloads as wl

T_ = wl.TEMPLATE_HEADER


def test_paper_example_x1_onto_C_KH():
    """Section 6.2: [x1, H, W] broadcast to [C, K_H, H, W] with G | C: x1 is one of
    {C, K_H, G, C/G, C K_H, G K_H, (C/G) K_H} (and, as in the section's second example, 1)."""
    t = S.Template(T_ + "%1 = unfold %0 kh=KH kw=1\n%2 = fc %0 groups=1 out=x1\n%3 = binary %2 %1 op=mul\noutput %3\n")
    var, subs = t.substitutions(3)
    assert var == 1
    assert set(subs) == {"1", "C", "KH", "G", "C/G", "C*KH", "G*KH", "C*KH/G"}


def test_paper_example_x1_KH_onto_G_x2_KH_KW():
    """Section 6.2: [x1, K_H, H, W] and [G, x2/G, K_H, K_W, H, W]: common suffix {H, W}; the substitutions of x1
    are the factors of x2 K_W: {1, x2, K_W, x2 K_W}; choosing x1 = x2 K_W makes the LHS [x2 K_W, K_H, H, W]."""
    t = S.Template(wl.TEMPLATE_SHAPE_MATCHING)
    assert t.node_shape(3) == "[x1 | KH | H, W]" and t.node_shape(6) == "[G, x2/G | KH, KW | H, W]"
    var, subs = t.substitutions(7)
    assert var == 1 and set(subs) == {"1", "x2", "KW", "KW*x2"}
    t.substitute(1, "x2*KW")
    assert t.node_shape(3) == "[KW*x2 | KH | H, W]" and t.free_vars() == [2]
    assert t.integers[[w for _, _, w in t.integers].index("M")][0] == S.mono()   # M = 1 now


def test_paper_example_group_number():
    """Section 6.3: C1 = 32, C2 = 48: G is sampled from {2, 4, 8, 16}."""
    assert S.group_candidates([32, 48]) == [2, 4, 8, 16]
    assert S.group_candidates([64, 128, 256, 512]) == [2, 4, 8, 16, 32, 64]
    assert S.group_candidates([7, 9]) == []


def _example_targets():
    # G K_1H = 12 and G K_iH = 20 with G = 4; C_i / C_1 = 4 makes ceil(C_i lcm_1 / (C_1 lcm_i)) = ceil(2.4) = 3
    return [dict(C=64, KH=3, KW=3, H=56, W=56), dict(C=256, KH=5, KW=5, H=14, W=14)], 4


def test_paper_example_base_values_12_and_60():
    """Section 6.3, the figure's example: [G K_H, H, W] onto [x1, H, W] needs G K_H | x1; lcm_11 = 12, lcm_i1 = 20,
    x_11 = 12, x_i1 = ceil(C_i lcm_11 / (C_1 lcm_i1)) * lcm_i1 = 60."""
    t = S.Template(wl.TEMPLATE_CONSTRAINTS)
    targets, G = _example_targets()
    X, flops, params, rounds = t.solve(targets, G)
    assert X == [{1: 12}, {1: 60}] and rounds == 0
    # weights: target 1: 12*64 + 12*64 + 64*12, target i: 20*256 + 60*256 + 256*60
    assert params == 3 * 12 * 64 + 20 * 256 + 2 * 60 * 256
    assert flops == 3 * 12 * 64 * 56 * 56 + (20 * 256 + 2 * 60 * 256) * 14 * 14


def test_paper_example_doubling_twice_gives_48_and_240():
    """... 'to fully utilize the budget, we double the values two times and get x_11 = 48 and x_i1 = 240': any budget
    between the cost at (48, 240) and the cost of the cheapest further doubling."""
    t = S.Template(wl.TEMPLATE_CONSTRAINTS)
    targets, G = _example_targets()

    def flops_at(x1, xi):
        return (12 * 64 + 2 * x1 * 64) * 56 * 56 + (20 * 256 + 2 * xi * 256) * 14 * 14

    lo, nxt = flops_at(48, 240), min(flops_at(96, 240), flops_at(48, 480))
    assert lo < nxt
    for budget in (lo, (lo + nxt) // 2, nxt - 1):
        X, flops, params, rounds = t.solve(targets, G, flops_budget=budget)
        assert X == [{1: 48}, {1: 240}] and rounds == 2 and flops == lo
    # one unit below the cost at (48, 240): one of the two last doublings does not fit
    X, _, _, _ = t.solve(targets, G, flops_budget=lo - 1)
    assert X != [{1: 48}, {1: 240}] and X[0][1] in (24, 48) and X[1][1] in (120, 240)
    with pytest.raises(OverflowError):
        t.solve(targets, G, flops_budget=flops_at(12, 60) - 1)


def test_doubling_order_is_ascending_delta():
    """A budget that admits exactly one doubling: the one with the smaller Delta wins (hand-computed)."""
    t = S.Template(T_ + "%1 = fc %0 groups=1 out=x1\n%2 = fc %1 groups=1 out=x2\n%3 = fc %2 groups=1 out=C\noutput %3\n")
    tg = [dict(C=8, KH=3, KW=3, H=2, W=2)]
    # params = 8 x1 + x1 x2 + 8 x2; base x1 = x2 = 1 -> 17; doubling either: 26, i.e. equal Deltas: lowest (i, j) first
    X, _, params, rounds = t.solve(tg, 1, params_budget=26)
    assert X == [{1: 2, 2: 1}] and params == 26 and rounds == 1
    # now x1 = 2, x2 = 1: Delta_1 = 16 + 2 = 18, Delta_2 = 2 + 8 = 10: with room for 10 more, x2 doubles, x1 cannot
    X, _, params, _ = t.solve(tg, 1, params_budget=36)
    assert X == [{1: 2, 2: 2}] and params == 16 + 4 + 16


def _primes_binding():
    # (primes other than the 2 and 3 that occur as literal coefficients in the templates)
    return {"G": 47, "Cg": 53, "KH": 5, "KW": 7, "H": 11, "W": 13, **{f"x{j}": p for j, p in zip(range(1, 9), (17, 19, 23, 29, 31, 37, 41, 43))}}


def _divisors(n):
    small = [d for d in range(1, int(n ** 0.5) + 1) if n % d == 0]
    return sorted(set(small + [n // d for d in small]))


def test_substitutions_are_exactly_the_divisors_brute_force():
    """With distinct primes bound to the symbols, a symbolic factor is a numeric divisor and vice versa: the
    substitution set, evaluated, must be the set of all x for which M = #RHS / #LHS is an integer, x | numerator."""
    b = _primes_binding()
    checked = 0
    for seed in range(1500):
        try:
            t = S.Template(wl.fuzz_template(seed))
        except ValueError:
            continue
        for k, nd in enumerate(t.nodes):
            if nd["op"] != "binary" or not S.variables(t.nodes[nd["a"]]["C"]) or S.Template.attr(nd, "lhs"):
                continue
            var, subs = t.substitutions(k)
            A, B = t.nodes[nd["a"]], t.nodes[nd["b"]]
            rhs = S.evaluate(S.mul(B["C"], S.prod(B["taps"])), b)
            lhs_rest = S.evaluate(S.div(S.mul(A["C"], S.prod(A["taps"])), S.mono(**{f"x{var}": 1})), b)
            got = sorted(S.evaluate(S.parse_mono(s), b) for s in subs)
            top = rhs / lhs_rest
            if f"x{var}" in B["C"][1]:
                assert got == []       # x on both sides: nothing to choose
                continue
            want = sorted(Fraction(x) for x in _divisors(top.numerator)) if top.denominator == 1 else []
            assert got == want, (seed, k, subs)
            checked += 1
    assert checked > 50


def test_theorem_1_on_random_templates():
    """Section 6.2, Theorem 1: no variable in spatial dims or denominators, at most one per tensor -- for every
    tensor of every accepted template, before and after substitutions."""
    accepted = 0
    for seed in range(400):
        try:
            t = S.Template(wl.fuzz_template(seed))
        except ValueError:
            continue
        accepted += 1
        for _ in range(3):
            for nd in t.nodes:
                vs = S.variables(nd["C"])
                assert len(vs) <= 1 and all(nd["C"][1][f"x{v}"] == 1 for v in vs)
                assert not any(S.variables(m) for m in nd["taps"]) and not S.variables(nd["grp"])
            todo = [k for k, nd in enumerate(t.nodes) if nd["op"] == "binary" and S.variables(t.nodes[nd["a"]]["C"])]
            if not todo:
                break
            var, subs = t.substitutions(todo[0])
            if not subs:
                break
            try:
                t.substitute(var, subs[seed % len(subs)])
            except ValueError:
                break
    assert accepted > 100


def test_base_value_is_the_least_legal_width_brute_force(oracle):
    """x_1j = lcm_1j is the least width for which the instantiated micro-DAG is legal, and exactly its multiples
    are legal -- checked with the DAG oracle's own shape inference on the instantiated blobs."""
    body = ("%1 = group %0 groups=G\n%2 = fc %1 out=x1\n%3 = fc %0 groups=1 out=G*KH\n%4 = binary %3 %2 op=mul\n"
            "%5 = unfold %4 kh=KH kw=1\n%6 = fold %5 op=max\n%7 = fc %6 out=C\noutput %7\n")
    t = S.Template(T_ + body)
    for tg, G, want in ((dict(C=24, KH=3, KW=3, H=4, W=4), 4, 12), (dict(C=40, KH=5, KW=1, H=3, W=5), 4, 20),
                        (dict(C=18, KH=3, KW=3, H=4, W=4), 6, 18), (dict(C=16, KH=1, KW=1, H=4, W=4), 8, 8)):
        X, _, _, _ = t.solve([tg], G)
        assert X == [{1: want}]
        for x in range(1, 3 * want + 1):
            blob = t.instantiate(tg, G, {1: x})
            try:
                oracle.infer(blob, (1, tg["C"], tg["H"], tg["W"]))
                legal = True
            except Exception:
                legal = False
            assert legal == (x % want == 0), (tg, x)


def test_free_variable_in_a_denominator_is_refused():
    """An LHS variable that shape matching has not substituted leaves M = .../x: the constraint solver cannot
    give it a value (Section 6.3 solves the *remaining* variables, which sit in numerators only)."""
    t = S.Template(T_ + "%1 = fc %0 groups=1 out=x1\n%2 = unfold %0 kh=KH kw=KW\n%3 = binary %1 %2 op=mul\n%4 = fold %3 op=avg\noutput %4\n")
    with pytest.raises(ValueError):
        t.solve([dict(C=16, KH=3, KW=3, H=4, W=4)], 2)
    t.substitute(1, "C/G")
    assert t.solve([dict(C=16, KH=3, KW=3, H=4, W=4)], 2)[0] == [{}]
    assert "out=8" in t.instantiate(dict(C=16, KH=3, KW=3, H=4, W=4), 2, {})


def test_proportional_base_values():
    """k_ij = ceil(C_i lcm_1j / (C_1 lcm_ij)) with the target of least C as target 1, wherever it is listed."""
    t = S.Template(T_ + "%1 = group %0 groups=G\n%2 = fc %1 out=x1\n%3 = fc %2 out=C\noutput %3\n")
    tg = [dict(C=96, KH=3, KW=3, H=8, W=8), dict(C=32, KH=3, KW=3, H=8, W=8), dict(C=80, KH=3, KW=3, H=8, W=8)]
    X, _, _, _ = t.solve(tg, 16)          # lcm = G = 16 everywhere: x = 16 * ceil(C_i / 32)
    assert X == [{1: 48}, {1: 16}, {1: 48}]
