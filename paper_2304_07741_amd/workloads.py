"""Seeded synthetic workloads: serialized micro-DAGs and their input tensors.

This module only *generates inputs* (DAG text, random tensors, bf16 rounding of
those tensors).  It contains none of the primitives' arithmetic, and both the
GPU library's tests and the CPU oracle's tests draw their inputs from here so
that the two sides see identical bytes.

The DAG shapes follow the examples of the paper: convolution as Unfold then FC
(Section 5), shift plus residual addition (Section 8, kernel-level analysis),
Involution (Section 5, expressibility paragraph) and random DAGs grown one
primitive at a time (Section 6.1).  Tensor sizes are ResNet layer shapes.

Random numbers: splitmix64 keyed by (seed, tensor id, element index), turned
into N(0,1) by Box-Muller.
"""
import math

import numpy as np

_M64 = (1 << 64) - 1


def _splitmix64(z):
    """Vectorised splitmix64 finaliser on uint64 arrays."""
    z = (z + np.uint64(0x9E3779B97F4A7C15)).astype(np.uint64)
    z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
    z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
    return z ^ (z >> np.uint64(31))


def _mix_int(z):
    z = (z + 0x9E3779B97F4A7C15) & _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def normal(seed, tensor_id, shape, std=1.0):
    """N(0, std^2) samples as float64, a pure function of (seed, tensor_id, index)."""
    n = int(np.prod(shape))
    key = _mix_int(_mix_int(int(seed)) ^ (int(tensor_id) * 0xD1342543DE82EF95 & _M64))
    out = np.empty(n, dtype=np.float64)
    chunk = 1 << 22
    with np.errstate(over="ignore"):
        for s in range(0, n, chunk):
            e = min(n, s + chunk)
            idx = np.arange(s, e, dtype=np.uint64)
            a = _splitmix64(np.uint64(key) ^ (idx * np.uint64(2)))
            b = _splitmix64(np.uint64(key) ^ (idx * np.uint64(2) + np.uint64(1)))
            u1 = ((a >> np.uint64(11)).astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)  # (0, 1]
            u2 = (b >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)  # [0, 1)
            out[s:e] = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * math.pi * u2)
    return (out * std).reshape(shape)


def round_to_bf16(a):
    """Round to the nearest bf16 (ties to even); result as float32 holding bf16-exact values."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    r = ((u + np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))) >> np.uint64(16)) << np.uint64(16)
    return r.astype(np.uint32).view(np.float32).reshape(f.shape)


def bf16_bits(a):
    """uint16 bit patterns of an array that already holds bf16-exact float32 values."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    return (f.view(np.uint32) >> np.uint32(16)).astype(np.uint16).reshape(f.shape)


def bf16_bits_to_f32(bits):
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


class IntRng:
    """Small counter-based integer generator for structural choices."""

    def __init__(self, seed):
        self.key = _mix_int(int(seed) ^ 0xA5A5A5A5DEADBEEF)
        self.ctr = 0

    def below(self, n):
        self.ctr += 1
        return _mix_int(self.key ^ (self.ctr * 0x2545F4914F6CDD1D & _M64)) % n

    def choice(self, seq):
        return seq[self.below(len(seq))]


HEADER = "canvas-dag 1\n"


def blob_conv(k=3, groups=1, out=16):
    return HEADER + f"%1 = unfold %0 kh={k} kw={k}\n%2 = fc %1 groups={groups} out={out}\noutput %2\n"


def blob_shift_residual(C=64):
    """Four channel slices shifted by (0,+1), (0,-1), (+1,0), (-1,0); grouped FC; ReLU; + input."""
    q = C // 4
    offs = [(0, 1), (0, -1), (1, 0), (-1, 0)]
    lines = [HEADER]
    for k, (dh, dw) in enumerate(offs):
        lines.append(f"%{k + 1} = shift %{k} dh={dh} dw={dw} c0={k * q} c1={(k + 1) * q}\n")
    lines.append(f"%5 = fc %4 groups=4 out={C}\n%6 = unary %5 op=relu\n%7 = binary %0 %6 op=add\noutput %7\n")
    return "".join(lines)


def blob_involution(C=128, k=3):
    """FC to k*k per-pixel weights, softmax over them, applied to the unfolded input, tap sum, FC."""
    return (HEADER + f"%1 = fc %0 groups=1 out={k * k}\n%2 = softmax %1 axis=C\n%3 = unfold %0 kh={k} kw={k}\n"
            f"%4 = binary %2 %3 op=mul\n%5 = fold %4 op=sum\n%6 = fc %5 groups=1 out={C}\noutput %6\n")


def blob_sampled(C):
    """Unfold 3x3, grouped FC, GELU, shift of the upper half of the channels, times input, fold, FC."""
    return (HEADER + f"%1 = unfold %0 kh=3 kw=3\n%2 = fc %1 groups=8 out={C}\n%3 = unary %2 op=gelu\n"
            f"%4 = shift %3 dh=0 dw=1 c0={C // 2} c1={C}\n%5 = binary %0 %4 op=mul\n%6 = fold %5 op=avg\n"
            f"%7 = fc %6 groups=1 out={C}\noutput %7\n")


def _case(name, blob, shape, dtype, seed, wshapes, wstds):
    """Tensors for one workload.  Values are float32; bf16-exact when dtype == 'bf16'."""
    rnd = round_to_bf16 if dtype == "bf16" else (lambda a: np.ascontiguousarray(a, dtype=np.float32))
    x = rnd(normal(seed, 0, shape))
    weights = [rnd(normal(seed, 100 + k, s, std)) for k, (s, std) in enumerate(zip(wshapes, wstds))]
    return {"name": name, "blob": blob, "shape": tuple(shape), "dtype": dtype, "seed": seed, "x": x,
            "weights": weights, "wshapes": [tuple(s) for s in wshapes]}


def make_dy(case, out_shape):
    rnd = round_to_bf16 if case["dtype"] == "bf16" else (lambda a: np.ascontiguousarray(a, dtype=np.float32))
    return rnd(normal(case["seed"], 1, out_shape))


def block_case(name, blob, shape, c_out, dtype, seed, wshapes, wstds):
    """Tensors for a block [C_in, H, W] => [C_out, H, W] composed of m = max / min instances of one template: x, dy
    and one weight set per instance (inputs only; the composition itself is the library's and the oracle's business)."""
    rnd = round_to_bf16 if dtype == "bf16" else (lambda a: np.ascontiguousarray(a, dtype=np.float32))
    n, c_in, h, w = shape
    m = max(c_in, c_out) // min(c_in, c_out)
    weights = [[rnd(normal(seed, 100 + 16 * j + k, s, std)) for k, (s, std) in enumerate(zip(wshapes, wstds))] for j in range(m)]
    return {"name": name, "blob": blob, "shape": tuple(shape), "c_out": int(c_out), "dtype": dtype, "seed": seed,
            "x": rnd(normal(seed, 0, shape)), "dy": rnd(normal(seed, 1, (n, c_out, h, w))), "weights": weights}


def config1():
    return _case("conv3x3_fp32", blob_conv(3, 1, 16), (1, 16, 8, 8), "f32", 0, [(1, 16, 144)], [1.0 / 12.0])


def config2(N=64, C=64, H=56):
    return _case("shift_residual", blob_shift_residual(C), (N, C, H, H), "bf16", 1, [(4, C // 4, C // 4)],
                 [1.0 / math.sqrt(C // 4)])


def config3(N=32, C=128, H=28):
    return _case("involution", blob_involution(C, 3), (N, C, H, H), "bf16", 2, [(1, 9, C), (1, C, C)],
                 [0.09, 1.0 / math.sqrt(C)])


CONFIG4_SHAPES = [(64, 56), (128, 28), (256, 14), (512, 7)]


def config4(C, H, N=128):
    k1 = (C // 8) * 9
    return _case(f"sampled_c{C}_h{H}", blob_sampled(C), (N, C, H, H), "bf16", 3, [(8, C // 8, k1), (1, C, C)],
                 [math.sqrt(2.0 / k1), math.sqrt(2.0 / C)])


# ---------------------------------------------------------------- random DAGs

FUZZ_FC_LIMIT = 96 * 25 * 192  # largest (K * C_out) a random FC may have


# FC-free chains of memory-bound primitives at ResNet layer shapes: what the fused-chain kernels are measured on against
# the HBM roof (the gate of config 4 without its two FCs; a shifted residual; an unfold folded again; a channel softmax).
CHAIN_BODIES = {
    "gate": "%1 = unary %0 op=gelu\n%2 = shift %1 dh=0 dw=1 c0={half} c1={C}\n%3 = binary %0 %2 op=mul\noutput %3\n",
    "relu": "%1 = unary %0 op=relu\noutput %1\n",
    "shift_residual": "%1 = shift %0 dh=1 dw=0 c0=0 c1={half}\n%2 = shift %1 dh=0 dw=-1 c0={half} c1={C}\n%3 = unary %2 op=relu\n"
                      "%4 = binary %0 %3 op=add\noutput %4\n",
    "box3": "%1 = unfold %0 kh=3 kw=3\n%2 = fold %1 op=avg\noutput %2\n",
    "softmax_c": "%1 = softmax %0 axis=C\noutput %1\n",
}


def chain(name, N=128, C=64, H=56, dtype="bf16"):
    return _case(f"chain_{name}", HEADER + CHAIN_BODIES[name].format(C=C, half=C // 2), (N, C, H, H), dtype, 6, [], [])


def _bcast_ok(CL, TL, CR, TR):
    if CL == CR:
        return TR % TL == 0
    return (CR * TR) % (CL * TL) == 0


def fuzz_dag(seed, attempt=0, C0=96):
    """A random legal DAG of depth 2..8 that maps [C0,H,W] to [C0,H,W].

    Returns (blob, weight_shapes).  Grown one primitive at a time from the
    current tensor; branches are merged by a broadcast with an earlier tensor.
    """
    rng = IntRng(seed * 1000003 + attempt)
    depth = 2 + rng.below(7)
    nodes = [(C0, 1)]  # (C, T) per node id
    lines = [HEADER]
    wshapes = []
    cur = 0

    def closing(C, T):
        return (1 if T > 1 else 0) + (1 if C != C0 else 0)

    def emit(text, C, T):
        nonlocal cur
        nodes.append((C, T))
        cur = len(nodes) - 1
        lines.append(f"%{cur} = {text}\n")

    def emit_fc(G, out):
        C, T = nodes[cur]
        wshapes.append((G, out // G, (C // G) * T))
        emit(f"fc %{cur} groups={G} out={out}", out, 1)

    count = 0
    while True:
        C, T = nodes[cur]
        remaining = depth - count
        need = closing(C, T)
        if remaining <= need:
            break
        for _ in range(200):
            kind = rng.choice(["unfold", "shift", "fc", "unary", "binary", "softmax", "fold"])
            if kind == "unfold":
                k = rng.choice([3, 5])
                if T != 1 or closing(C, k * k) > remaining - 1:
                    continue
                emit(f"unfold %{cur} kh={k} kw={k}", C, k * k)
            elif kind == "shift":
                d = rng.choice([1, -1, 2, -2])
                dh, dw = (d, 0) if rng.below(2) == 0 else (0, d)
                c0, c1 = rng.choice([(0, C), (0, C // 2), (C // 2, C)])
                emit(f"shift %{cur} dh={dh} dw={dw} c0={c0} c1={c1}", C, T)
            elif kind == "fc":
                G = rng.choice([1, 2, 4, 8])
                num, den = rng.choice([(1, 2), (1, 1), (2, 1)])
                if (C * num) % den:
                    continue
                out = C * num // den
                if C % G or out % G or out < 24 or out > 384 or (C // G) * T * out > FUZZ_FC_LIMIT:
                    continue
                if closing(out, 1) > remaining - 1:
                    continue
                emit_fc(G, out)
            elif kind == "unary":
                op = rng.choice(["relu", "gelu", "abs", "expclip lo=-4 hi=4"])
                emit(f"unary %{cur} op={op}", C, T)
            elif kind == "binary":
                op = rng.choice(["add", "mul"])
                cands = []
                for j, (Cj, Tj) in enumerate(nodes):
                    if j == cur:
                        continue
                    if _bcast_ok(Cj, Tj, C, T):
                        cands.append((j, cur, C, T))
                    if _bcast_ok(C, T, Cj, Tj) and closing(Cj, Tj) <= remaining - 1:
                        cands.append((cur, j, Cj, Tj))
                if not cands:
                    continue
                lhs, rhs, Cn, Tn = rng.choice(cands)
                emit(f"binary %{lhs} %{rhs} op={op}", Cn, Tn)
            elif kind == "softmax":
                axis = rng.choice(["C", "T"]) if T > 1 else "C"
                emit(f"softmax %{cur} axis={axis}", C, T)
            else:
                if T == 1:
                    continue
                emit(f"fold %{cur} op={rng.choice(['sum', 'avg', 'max'])}", C, 1)
            count += 1
            break
        else:
            raise RuntimeError("fuzz generator could not extend the DAG")
    C, T = nodes[cur]
    if T > 1:
        emit(f"fold %{cur} op={rng.choice(['sum', 'avg', 'max'])}", C, 1)
    C, T = nodes[cur]
    if C != C0:
        Gs = [g for g in (1, 2, 4, 8) if C % g == 0 and C0 % g == 0]
        emit_fc(rng.choice(Gs), C0)
    lines.append(f"output %{cur}\n")
    return "".join(lines), wshapes


def config5(seed, attempt=0, N=16, C=96, H=32):
    blob, wshapes = fuzz_dag(seed, attempt, C)
    stds = [1.0 / math.sqrt(s[2]) for s in wshapes]
    return _case(f"fuzz_{seed}_{attempt}", blob, (N, C, H, H), "bf16", seed * 7919 + attempt, wshapes, stds)


# ----------------------------------------------------------------------------- kernel templates (symbolic sizes)

TEMPLATE_HEADER = "canvas-template 1\n"

# the two worked examples of the paper's solver sections, as templates
TEMPLATE_SHAPE_MATCHING = (TEMPLATE_HEADER + "%1 = unfold %0 kh=KH kw=1\n%2 = fc %1 groups=1 out=x1\n%3 = unfold %2 kh=KH kw=1\n"
                           "%4 = group %0 groups=G\n%5 = fc %4 out=x2\n%6 = unfold %5 kh=KH kw=KW\n%7 = binary %3 %6 op=mul\n"
                           "%8 = fold %7 op=avg\n%9 = fc %8 out=C\noutput %9\n")
TEMPLATE_CONSTRAINTS = (TEMPLATE_HEADER + "%1 = fc %0 groups=1 out=G*KH\n%2 = fc %0 groups=1 out=x1\n%3 = binary %1 %2 op=mul\n"
                        "%4 = fc %3 groups=1 out=C\noutput %4\n")


def fuzz_template(seed):
    """A random kernel template (text).  Structure only: sizes are symbols, FC widths are new dynamic variables
    or expressions; not every draw is legal, which is part of what the tests compare."""
    rng = IntRng(seed * 7777 + 13)
    lines = [TEMPLATE_HEADER]
    n, nvar, cur = 0, 0, 0
    depth = 3 + rng.below(7)

    def emit(text):
        nonlocal n, cur
        n += 1
        cur = n
        lines.append(f"%{n} = {text}\n")

    for _ in range(depth):
        kind = rng.choice(["unfold", "shift", "group", "fc", "fc", "unary", "binary", "binary", "softmax", "fold"])
        if kind == "unfold":
            emit(f"unfold %{cur} kh={rng.choice(['KH', '1', '3'])} kw={rng.choice(['KW', '1', '3', 'KW'])}")
        elif kind == "shift":
            emit(f"shift %{cur} dh={rng.choice([0, 1, -1])} dw={rng.choice([0, 1, -1])}" + rng.choice(["", " c0=0 c1=C/2", ""]))
        elif kind == "group":
            emit(f"group %{cur} groups={rng.choice(['G', 'G', 'C', '2'])}")
        elif kind == "fc":
            if rng.below(2) == 0 and nvar < 8:
                nvar += 1
                out = f"x{nvar}"
            else:
                out = rng.choice(["C", "G*KH", "C/G", "2*C", "KH*KW", "G*KH*KW", "H*W", "C/2"])
            emit(f"fc %{rng.choice([cur, 0])}{rng.choice(['', ' groups=1', ' groups=G', ''])} out={out}")
        elif kind == "unary":
            emit(f"unary %{cur} op={rng.choice(['relu', 'gelu', 'abs', 'sin'])}")
        elif kind == "binary":
            other = rng.below(n + 1)
            a, b = (cur, other) if rng.below(2) else (other, cur)
            emit(f"binary %{a} %{b} op={rng.choice(['add', 'mul', 'sub', 'max'])}" + (" lhs=pixels" if rng.below(12) == 0 else ""))
        elif kind == "softmax":
            emit(f"softmax %{cur} axis={rng.choice(['C', 'T', 'CT'])}")
        else:
            ax = rng.choice(["", "", " axis=HW", " axis=C groups=G", " axis=C", " axis=H", " axis=W"])
            emit(f"fold %{cur} op={rng.choice(['sum', 'avg', 'max'])}{ax}")
    emit(f"fold %{cur} op=avg")
    emit(f"fc %{cur} out=C")
    lines.append(f"output %{cur}\n")
    return "".join(lines)


def fuzz_targets(seed):
    """Replacement targets (C, KH, KW, H, W) at ResNet-like sizes plus a group number dividing every C."""
    rng = IntRng(seed * 31337 + 5)
    nt = 1 + rng.below(4)
    G = rng.choice([1, 2, 4, 8])
    targets = []
    for _ in range(nt):
        k = rng.choice([1, 3, 3, 5, 7])
        side = rng.choice([7, 14, 28, 56])
        targets.append({"C": rng.choice([16, 24, 32, 48, 64, 96, 128, 256]), "KH": k, "KW": rng.choice([k, k, 1, 3]), "H": side, "W": side})
    return targets, G
