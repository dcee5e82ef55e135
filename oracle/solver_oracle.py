"""solver_oracle.py -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

A plain Python rendering of the two dynamic-variable solvers of "Canvas: End-to-End Kernel Architecture
Search" (Section 6.2, shape matching; Section 6.3, analytical constraints) on kernel templates, written
from the paper's definitions with exact rational arithmetic.  It shares nothing with the C++ library
(paper_2304_07741_amd/csrc/template.cpp); tests compare the two.  Pins (tests/test_solver_oracle.py): the
numbers the paper prints (the substitution sets of Section 6.2, the group-number set and the lcm 12/20 ->
x = 12/60 -> 48/240 example of Section 6.3), Theorem 1 as a property of random templates, brute force over
divisors with distinct primes bound to the symbols, brute force over x against the legality of the
instantiated micro-DAG.  No function here is "parity unpinned".

A size is a monomial: Fraction coefficient times symbols to integer powers, kept as (Fraction, {symbol: exponent}).
Symbols: G, Cg (= C/G: Section 6.2 takes the group number to be a factor of C, so C = G*Cg), KH, KW, H, W, x1..x8.
"""
from fractions import Fraction
from itertools import product as cartesian
from math import gcd, lcm

SYMBOL_ORDER = ["C", "G", "KH", "KW", "H", "W"] + [f"x{j}" for j in range(1, 9)]


def mono(coeff=1, **exps):
    return (Fraction(coeff), {k: v for k, v in exps.items() if v})


def mul(a, b, sign=1):
    e = dict(a[1])
    for k, v in b[1].items():
        e[k] = e.get(k, 0) + sign * v
        if e[k] == 0:
            del e[k]
    return (a[0] * b[0] if sign > 0 else a[0] / b[0], e)


def div(a, b):
    return mul(a, b, -1)


def prod(ms):
    r = mono()
    for m in ms:
        r = mul(r, m)
    return r


def parse_mono(text):
    """'x2*KW/G', 'C/2', '3': products and quotients, `/` applies to the one factor after it."""
    r, op, tok = mono(), "*", ""
    for ch in text + "*":
        if ch in "*/":
            if not tok:
                raise ValueError(f"bad size expression {text!r}")
            if tok == "C":
                f = mono(G=1, Cg=1)
            elif tok in ("G", "KH", "KW", "H", "W"):
                f = mono(**{tok: 1})
            elif tok[0] == "x" and tok[1:].isdigit() and 1 <= int(tok[1:]) <= 8:
                f = mono(**{f"x{int(tok[1:])}": 1})
            elif tok.isdigit() and int(tok) >= 1:
                f = mono(int(tok))
            else:
                raise ValueError(f"bad size expression {text!r}")
            r = mul(r, f) if op == "*" else div(r, f)
            op, tok = ch, ""
        else:
            tok += ch
    return r


def to_text(m):
    """Canonical text in terms of C and G (Cg = C/G): integer first, then C G KH KW H W x1.., then '/factor' each."""
    e = dict(m[1])
    ec = e.pop("Cg", 0)
    eg = e.pop("G", 0) - ec
    e["C"], e["G"] = ec, eg
    up, down = [], []
    if m[0].numerator != 1:
        up.append(str(m[0].numerator))
    if m[0].denominator != 1:
        down.append(str(m[0].denominator))
    for s in SYMBOL_ORDER:
        up += [s] * max(e.get(s, 0), 0)
        down += [s] * max(-e.get(s, 0), 0)
    return ("*".join(up) or "1") + "".join("/" + d for d in down)


def variables(m):
    return sorted(int(k[1:]) for k in m[1] if k[0] == "x")


def evaluate(m, binding):
    v = m[0]
    for k, ex in m[1].items():
        v *= Fraction(binding[k]) ** ex
    return v


SYMBOLIC_KEYS = {"unfold": ("kh", "kw"), "shift": ("c0", "c1"), "fc": ("groups", "out"), "group": ("groups",), "fold": ("groups",)}


class Template:
    """nodes[k] = dict(op, a, b, attrs=[(key, raw or monomial, symbolic)]) plus the inferred C, taps, pooled, grp."""

    def __init__(self, blob):
        lines = [l.split() for l in blob.splitlines() if l.split() and not l.lstrip().startswith("#")]
        if not lines or lines[0] != ["canvas-template", "1"]:
            raise ValueError("expected header 'canvas-template 1'")
        self.nodes = [dict(op="input", a=-1, b=-1, attrs=[])]
        self.out = None
        for tok in lines[1:]:
            if self.out is not None:
                raise ValueError("text after the output line")
            if tok[0] == "output":
                self.out = int(tok[1][1:])
                if not 0 <= self.out < len(self.nodes):
                    raise ValueError("bad output reference")
                continue
            if len(tok) < 4 or tok[1] != "=" or int(tok[0][1:]) != len(self.nodes):
                raise ValueError("expected '%k = op %operand ...' with consecutive ids")
            op = tok[2]
            if op not in ("unfold", "shift", "fc", "unary", "binary", "softmax", "fold", "group"):
                raise ValueError(f"unknown op {op}")
            nd = dict(op=op, a=int(tok[3][1:]), b=-1, attrs=[])
            rest = tok[4:]
            if op == "binary":
                nd["b"] = int(tok[4][1:])
                rest = tok[5:]
            if not (0 <= nd["a"] < len(self.nodes) and nd["b"] < len(self.nodes)):
                raise ValueError("operand must be an earlier node")
            for kv in rest:
                key, _, raw = kv.partition("=")
                if not key or not raw:
                    raise ValueError(f"expected key=value, got {kv!r}")
                symbolic = key in SYMBOLIC_KEYS.get(op, ())
                nd["attrs"].append([key, parse_mono(raw) if symbolic else raw, symbolic])
            self.nodes.append(nd)
        if self.out is None:
            raise ValueError("no output line")
        self.infer()

    @staticmethod
    def attr(nd, key):
        for k, v, _ in nd["attrs"]:
            if k == key:
                return v
        return None

    def infer(self):
        """Symbolic shapes (Section 5 shape rules with symbols) and every size that has to be an integer."""
        self.integers = []   # (monomial, node, what)
        self.ones = []       # (monomial that must equal 1, node)
        for k, nd in enumerate(self.nodes):
            if nd["op"] == "input":
                nd.update(C=mono(G=1, Cg=1), taps=[], pooled=0, grp=mono())   # pooled: mask of folded spatial dims, 1 = H, 2 = W
                continue
            A = self.nodes[nd["a"]]
            C, taps, pooled, grp = A["C"], list(A["taps"]), A["pooled"], A["grp"]
            op = nd["op"]
            if op == "unfold":
                kh, kw = self.attr(nd, "kh"), self.attr(nd, "kw")
                if kh is None or kw is None or variables(kh) or variables(kw) or pooled:
                    raise ValueError(f"node {k}: bad unfold")
                taps += [m for m in (kh, kw) if m != mono()]
                self.integers += [(kh, k, "kh"), (kw, k, "kw")]
            elif op == "shift":
                if pooled:
                    raise ValueError(f"node {k}: shift without spatial dims")
                self.integers += [(self.attr(nd, c), k, c) for c in ("c0", "c1") if self.attr(nd, c) is not None]
            elif op == "group":
                g = self.attr(nd, "groups")
                if g is None or variables(g):
                    raise ValueError(f"node {k}: bad group")
                grp = g
                nd["groups_used"] = g
                self.integers += [(g, k, "groups"), (div(C, g), k, "channels per group")]
            elif op == "fc":
                out, stated = self.attr(nd, "out"), self.attr(nd, "groups")
                if out is None:
                    raise ValueError(f"node {k}: fc needs out=")
                g = grp
                if stated is not None:
                    if grp != mono() and stated != grp:
                        raise ValueError(f"node {k}: fc groups= contradicts the view")
                    g = stated
                if variables(g):
                    raise ValueError(f"node {k}: variable group number")
                nd["groups_used"] = g
                self.integers += [(g, k, "groups"), (div(C, g), k, "in per group"), (div(out, g), k, "out per group")]
                C, taps = out, []
            elif op == "binary":
                B = self.nodes[nd["b"]]
                if (pooled & B["pooled"]) != B["pooled"]:
                    raise ValueError(f"node {k}: the RHS has folded a spatial dim that the LHS keeps")
                lhs, rhs = mul(C, prod(taps)), mul(B["C"], prod(B["taps"]))
                al = self.attr(nd, "lhs")
                if al is not None:
                    if al != "pixels" or pooled != 3 or B["pooled"]:
                        raise ValueError(f"node {k}: bad lhs=")
                    self.ones.append((div(mono(H=1, W=1), lhs), k))
                else:
                    self.integers.append((div(rhs, lhs), k, "M"))   # M = #RHS / #LHS (Section 6.2)
                C, taps, pooled, grp = B["C"], list(B["taps"]), B["pooled"], B["grp"]
            elif op == "fold":
                axis = self.attr(nd, "axis") or "T"
                if axis == "T":
                    taps = []
                elif axis in ("HW", "H", "W"):
                    m = {"HW": 3, "H": 1, "W": 2}[axis]
                    if pooled & m:
                        raise ValueError(f"node {k}: already folded")
                    pooled |= m
                elif axis == "C":
                    g = self.attr(nd, "groups") or mono()
                    if variables(g):
                        raise ValueError(f"node {k}: variable group number")
                    nd["groups_used"] = g
                    self.integers += [(g, k, "groups"), (div(C, g), k, "folded per group")]
                    C, grp = g, mono()
                else:
                    raise ValueError(f"node {k}: bad fold axis")
            # Theorem 1: one variable at most, first power, numerator of the channel dim only
            vs = variables(C)
            if len(vs) > 1 or (vs and C[1][f"x{vs[0]}"] != 1):
                raise ValueError(f"node {k}: {to_text(C)} breaks Theorem 1")
            nd.update(C=C, taps=taps, pooled=pooled, grp=grp)
            self.integers.append((C, k, "channels"))
            if grp != mono():
                self.integers.append((div(C, grp), k, "channels per group of the view"))
        for m, k, what in self.integers:
            if not m[1] and m[0].denominator != 1:
                raise ValueError(f"node {k}: {what} is no integer")

    def free_vars(self):
        vs = set()
        for nd in self.nodes:
            for _, v, symbolic in nd["attrs"]:
                if symbolic:
                    vs.update(variables(v))
        return sorted(vs)

    def node_shape(self, k):
        nd = self.nodes[k]
        c = to_text(nd["C"]) if nd["grp"] == mono() else to_text(nd["grp"]) + ", " + to_text(div(nd["C"], nd["grp"]))
        t = (" " + ", ".join(to_text(m) for m in nd["taps"]) + " |") if nd["taps"] else ""
        return f"[{c} |{t} " + ("1" if nd["pooled"] & 1 else "H") + ", " + ("1" if nd["pooled"] & 2 else "W") + "]"

    # ------------------------------------------------------------ Section 6.2: shape matching

    def substitutions(self, k):
        """Valid substitutions of the LHS variable of binary node k: all factors of x_R^k * R_RHS (over R_LHS)."""
        nd = self.nodes[k]
        if nd["op"] != "binary":
            raise ValueError("not a binary node")
        A, B = self.nodes[nd["a"]], self.nodes[nd["b"]]
        vs = variables(A["C"])
        if not vs:
            raise ValueError("no free variable on the LHS")
        x = mono(**{f"x{vs[0]}": 1})
        r_lhs = div(mul(A["C"], prod(A["taps"])), x)
        if self.attr(nd, "lhs") is not None:
            only = div(mono(H=1, W=1), r_lhs)
            ok = only[0].denominator == 1 and all(e > 0 for e in only[1].values())
            return vs[0], sorted([to_text(only)] if ok else [])
        numer = div(mul(B["C"], prod(B["taps"])), r_lhs)
        if numer[0].denominator != 1 or any(e < 0 for e in numer[1].values()) or f"x{vs[0]}" in numer[1]:
            return vs[0], []
        n = numer[0].numerator
        syms = sorted(numer[1])
        out = []
        for d in [d for d in range(1, n + 1) if n % d == 0]:
            for exps in cartesian(*[range(numer[1][s] + 1) for s in syms]):
                out.append(to_text(mono(d, **dict(zip(syms, exps)))))
        return vs[0], sorted(out)

    def substitute(self, var, expr):
        e = parse_mono(expr)
        if var in variables(e) or var not in self.free_vars():
            raise ValueError("bad substitution")
        x = mono(**{f"x{var}": 1})
        saved = [[list(a) for a in nd["attrs"]] for nd in self.nodes]
        for nd in self.nodes:
            for a in nd["attrs"]:
                if a[2]:
                    p = a[1][1].get(f"x{var}", 0)
                    for _ in range(abs(p)):
                        a[1] = mul(div(a[1], x), e) if p > 0 else div(mul(a[1], x), e)
        try:
            self.infer()
        except ValueError:
            for nd, old in zip(self.nodes, saved):
                nd["attrs"] = old
            self.infer()
            raise

    # ------------------------------------------------------------ Section 6.3: analytical constraints

    @staticmethod
    def binding(target, G):
        if target["C"] % G:
            raise ValueError("G does not divide C")
        return {"G": G, "Cg": target["C"] // G, "KH": target["KH"], "KW": target["KW"], "H": target["H"], "W": target["W"]}

    def cost(self, b):
        """(multiply-accumulates, weights) of the fc nodes: out * (C_in / G) * taps [* H * W]."""
        flops = params = Fraction(0)
        for nd in self.nodes:
            if nd["op"] == "fc":
                A = self.nodes[nd["a"]]
                w = evaluate(div(mul(mul(nd["C"], A["C"]), prod(A["taps"])), nd["groups_used"]), b)
                if w.denominator != 1:
                    raise ValueError("weight shape is no integer")
                params += w
                flops += w * (1 if A["pooled"] & 1 else b["H"]) * (1 if A["pooled"] & 2 else b["W"])
        return flops, params

    def solve(self, targets, G, flops_budget=0, params_budget=0):
        """x_ij = k_ij * lcm_ij with k_1j = 1 at the target of least C and k_ij = ceil(C_i lcm_1j / (C_1 lcm_ij));
        then doublings in ascending order of Delta_ij, iteration after iteration, while a budget allows."""
        fv = self.free_vars()
        binds = [self.binding(t, G) for t in targets]
        for m, k in self.ones:
            if m != mono():
                raise ValueError(f"node {k}: the LHS laid over the pixels is not H*W long")
        lcms = []
        for i, b in enumerate(binds):
            l = {j: 1 for j in fv}
            for m, k, what in self.integers:
                vs = variables(m)
                if len(vs) > 1:
                    raise ValueError(f"node {k}: two variables in {what}")
                if vs and m[1][f"x{vs[0]}"] < 0:
                    raise ValueError(f"node {k}: free variable in a denominator")
                rest = div(m, mono(**{f"x{vs[0]}": 1})) if vs else m
                v = evaluate(rest, b)            # the size is p * x / q with v = p / q reduced
                if not vs:
                    if v.denominator != 1:
                        raise ValueError(f"target {i}, node {k}: {what} is no integer")
                else:
                    l[vs[0]] = lcm(l[vs[0]], v.denominator)
            lcms.append(l)
        i1 = min(range(len(targets)), key=lambda i: (targets[i]["C"], i))
        X = [{j: (1 if i == i1 else -((-targets[i]["C"] * lcms[i1][j]) // (targets[i1]["C"] * lcms[i][j]))) * lcms[i][j] for j in fv}
             for i in range(len(targets))]

        def net():
            f = p = Fraction(0)
            for b, x in zip(binds, X):
                fi, pi = self.cost({**b, **{f"x{j}": v for j, v in x.items()}})
                f, p = f + fi, p + pi
            return f, p

        def within(f, p):
            return (flops_budget <= 0 or f <= flops_budget) and (params_budget <= 0 or p <= params_budget)

        f, p = net()
        if not within(f, p):
            raise OverflowError("the base values already exceed a budget")
        rounds = 0
        while flops_budget > 0 or params_budget > 0:
            deltas = []
            for i in range(len(targets)):
                for j in fv:
                    X[i][j] *= 2
                    f2, p2 = net()
                    X[i][j] //= 2
                    d = (f2 - f) if flops_budget > 0 else (p2 - p)
                    if d > 0:
                        deltas.append((d, i, j))
            changed = False
            for d, i, j in sorted(deltas):
                X[i][j] *= 2
                f2, p2 = net()
                if within(f2, p2):
                    f, p, changed = f2, p2, True
                else:
                    X[i][j] //= 2
            if not changed:
                break
            rounds += 1
        return X, float(f), float(p), rounds

    def instantiate(self, target, G, x):
        b = {**self.binding(target, G), **{f"x{j}": v for j, v in x.items()}}
        lines = ["canvas-dag 1"]
        for k, nd in enumerate(self.nodes[1:], 1):
            s = f"%{k} = {nd['op']} %{nd['a']}" + (f" %{nd['b']}" if nd["op"] == "binary" else "")
            for key, v, symbolic in nd["attrs"]:
                if symbolic:
                    val = evaluate(v, b)
                    if val.denominator != 1:
                        raise ValueError(f"node {k}: {key} is no integer")
                    s += f" {key}={val.numerator}"
                else:
                    s += f" {key}={v}"
            lines.append(s)
        lines.append(f"output %{self.out}")
        return "\n".join(lines) + "\n"


def group_candidates(channels):
    """Section 6.3: the global G is a factor of gcd(C_i); 1 would mean no grouping and is not a candidate."""
    g = 0
    for c in channels:
        g = gcd(g, c)
    return [d for d in range(2, g + 1) if g % d == 0]
