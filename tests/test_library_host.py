"""Host-only checks of the C-ABI library: it loads without a GPU, exports every declared symbol,
infers the same shapes as the oracle and rejects illegal blobs with the documented status codes."""
import ctypes
import os
import re

import pytest

from paper_2304_07741_amd import binding as B
from paper_2304_07741_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        import __graft_entry__ as g

        g.build()
    return B.load()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "canvas_dag.h")).read()
    declared = set(re.findall(r"\b(canvas_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_info_struct_matches_header(lib):
    h = B.canvas_dag_compile(wl.blob_conv(3, 1, 16), (1, 16, 8, 8), B.CANVAS_F32)
    info = B.canvas_dag_query(h)
    assert info.n_nodes == 3 and info.out_node == 2 and info.n_weights == 1
    assert list(info.out_shape) == [1, 16, 1, 8, 8]
    assert list(info.weight_shape[0]) == [1, 16, 144] and info.weight_node[0] == 2
    assert info.fc_flops_fwd == 2.0 * 64 * 16 * 144
    assert info.min_bytes_fwd == 4.0 * (1024 + 1024 + 2304)
    assert info.n_launches_fwd >= 1 and info.n_launches_bwd >= 1
    d = B.canvas_dag_launch_desc(h, 0, 0)
    assert d["name"] and d["bytes"] > 0
    with pytest.raises(B.CanvasError):
        B.canvas_dag_launch_desc(h, 0, 10000)
    B.canvas_dag_destroy(h)


def test_shapes_agree_with_the_oracle_bit_exactly(lib, oracle):
    blobs = [wl.blob_conv(5, 2, 8), wl.blob_shift_residual(64), wl.blob_involution(128), wl.blob_sampled(64)]
    blobs += [wl.fuzz_dag(s)[0] for s in range(100, 300)]
    for blob in blobs:
        C = 96 if "fuzz" in blob or blob in blobs[4:] else (128 if blob == blobs[2] else 64)
        shape = (2, C, 6, 5)
        ns, out, ws = oracle.infer(blob, shape)
        for flags in (0, B.CANVAS_OPT_NO_FUSION):
            h = B.canvas_dag_compile(blob, shape, B.CANVAS_BF16, flags)
            info = B.canvas_dag_query(h)
            assert info.n_nodes == len(ns) and info.out_node == out and info.n_weights == len(ws)
            for k, s in enumerate(ns):
                assert list(info.node_shape[k]) == [2] + s
            for k, s in enumerate(ws):
                assert list(info.weight_shape[k]) == s
            B.canvas_dag_destroy(h)


BAD = [
    ("%1 = fc %0 groups=3 out=6\noutput %1\n", -3),
    ("%1 = fc %0 groups=2 out=5\noutput %1\n", -3),
    ("%1 = unfold %0 kh=2 kw=3\noutput %1\n", -3),
    ("%1 = shift %0 dh=0 dw=1 c0=3 c1=9\noutput %1\n", -3),
    ("%1 = fc %0 groups=1 out=5\n%2 = unfold %0 kh=3 kw=1\n%3 = binary %1 %2 op=add\noutput %3\n", -3),
    ("%1 = unfold %0 kh=3 kw=3\n%2 = binary %1 %0 op=add\noutput %2\n", -3),
    ("%2 = unary %0 op=relu\noutput %2\n", -1),
    ("%1 = unary %1 op=relu\noutput %1\n", -1),
    ("%1 = unary %0 op=relu\n", -1),
    ("%1 = unary %0\noutput %1\n", -1),
    ("%1 = unary %0 op=tanh\noutput %1\n", -2),
    ("%1 = softmax %0 axis=X\noutput %1\n", -2),
    ("%1 = conv %0 k=3\noutput %1\n", -2),
    ("%1 = unary %0 op=expclip lo=1 hi=1\noutput %1\n", -3),
    ("foo=bar\noutput %0\n", -1),                      # a line of key=value tokens only
    ("%1 = unary %0 op=relu\nop=relu\noutput %1\n", -1),
]


@pytest.mark.parametrize("body,status", BAD)
def test_illegal_blobs_give_status_codes(lib, body, status):
    with pytest.raises(B.CanvasError) as e:
        B.canvas_dag_compile(wl.HEADER + body, (1, 4, 4, 4), B.CANVAS_F32)
    assert e.value.status == status
    assert str(e.value)


def test_random_dags_are_lowered_to_fused_chains(lib):
    """Lowering by units on the 200 random DAGs of config 5 (host logic only): the runs of memory-bound primitives
    between FC nodes become fused chains, few launches remain, and switching fusion off gives one kernel per node."""
    chains, fwd, bwd, fully = 0, 0, 0, 0
    for seed in range(100, 300):
        case = wl.config5(seed)
        h = B.canvas_dag_compile(case["blob"], case["shape"], B.CANVAS_BF16)
        info = B.canvas_dag_query(h)
        names = [B.canvas_dag_launch_desc(h, 0, i)["name"] for i in range(info.n_launches_fwd)]
        n_nonfc = sum(1 for line in case["blob"].splitlines() if " = " in line and " fc " not in line)
        assert info.n_fused_nodes <= n_nonfc and info.n_fused_chains <= info.n_fused_nodes
        assert names.count("chain_fwd") == info.n_fused_chains
        chains += 1 if info.n_fused_chains else 0
        fully += 1 if info.n_fused_chains and not any(n.startswith("node_") and "fc" not in n for n in names) else 0
        fwd += info.n_launches_fwd
        bwd += info.n_launches_bwd
        B.canvas_dag_destroy(h)
        h = B.canvas_dag_compile(case["blob"], case["shape"], B.CANVAS_BF16, B.CANVAS_OPT_NO_FUSION)
        assert B.canvas_dag_query(h).n_fused_chains == 0
        B.canvas_dag_destroy(h)
    # (a softmax over the channels of a tensor with taps keeps a kernel of its own: 13 of the 200 DAGs have one)
    assert chains >= 185 and fully >= 165, (chains, fully)
    assert fwd / 200 <= 3.1 and bwd / 200 <= 6.0, (fwd / 200, bwd / 200)


def test_chain_boundaries(lib):
    """What ends a fused chain: a stencil above a reduction, an FC, a blend across channel counts."""
    H = wl.HEADER

    def plan(body, shape=(2, 96, 16, 16)):
        h = B.canvas_dag_compile(H + body, shape, B.CANVAS_BF16)
        info = B.canvas_dag_query(h)
        names = [B.canvas_dag_launch_desc(h, 0, i)["name"] for i in range(info.n_launches_fwd)]
        B.canvas_dag_destroy(h)
        return info.n_fused_chains, info.n_fused_nodes, names

    # element-wise work, shifts and an unfold that is folded again: one kernel, x read and y written in place
    assert plan("%1 = unary %0 op=relu\n%2 = unfold %1 kh=3 kw=3\n%3 = softmax %2 axis=T\n%4 = binary %3 %2 op=mul\n"
                "%5 = unary %4 op=gelu\n%6 = fold %5 op=sum\noutput %6\n") == (1, 6, ["chain_fwd"])
    # a softmax over channels inside a chain (statistics in a pass of their own), stencils above element-wise work
    assert plan("%1 = shift %0 dh=0 dw=2 c0=0 c1=96\n%2 = unary %1 op=relu\n%3 = softmax %2 axis=C\noutput %3\n") == (1, 3, ["chain_fwd"])
    # ... but every pass of that softmax computes what precedes it again: behind a dear prefix (two transcendental
    # functions per element here) the chain is cut where the halves together are cheaper than the whole
    assert plan("%1 = shift %0 dh=0 dw=2 c0=0 c1=96\n%2 = unary %1 op=expclip lo=-4 hi=4\n%3 = binary %0 %2 op=add\n"
                "%4 = shift %3 dh=-2 dw=0 c0=0 c1=48\n%5 = softmax %4 axis=C\noutput %5\n") == (2, 5, ["chain_fwd", "chain_fwd"])
    # an unfold of a folded (reduced) tensor starts a new chain: the reduction would be needed at other pixels
    assert plan("%1 = unfold %0 kh=3 kw=3\n%2 = fold %1 op=sum\n%3 = unfold %2 kh=5 kw=5\n%4 = binary %2 %3 op=mul\n"
                "%5 = fold %4 op=avg\noutput %5\n") == (2, 5, ["chain_fwd", "chain_fwd"])
    # FC nodes cut; an unfold that only FCs read is never a node of a chain (the contraction reads it in place)
    assert plan("%1 = unary %0 op=abs\n%2 = unfold %1 kh=3 kw=3\n%3 = fc %2 groups=4 out=96\n%4 = unary %3 op=gelu\noutput %4\n") \
        == (2, 2, ["chain_fwd", "gfc_fwd_unfold", "chain_fwd"])
    # a blend across channel counts keeps a kernel of its own
    n_chains, n_nodes, names = plan("%1 = fc %0 groups=1 out=48\n%2 = binary %1 %0 op=mul\n%3 = unary %2 op=relu\noutput %3\n")
    assert "node_binary_fwd" in names and n_chains == 1 and n_nodes == 1


def test_huge_shift_is_clamped_to_the_image(lib):
    """A shift by the image's extent or more leaves nothing inside: the parser clamps it (the kernels multiply dh by W)."""
    h = B.canvas_dag_compile(wl.HEADER + "%1 = shift %0 dh=1073741824 dw=-1073741824\noutput %1\n", (1, 4, 4, 4), B.CANVAS_F32)
    assert list(B.canvas_dag_query(h).out_shape) == [1, 4, 1, 4, 4]
    B.canvas_dag_destroy(h)


def test_bad_arguments(lib):
    with pytest.raises(B.CanvasError) as e:
        B.canvas_dag_compile("garbage", (1, 4, 4, 4), B.CANVAS_F32)
    assert e.value.status == -1
    with pytest.raises(B.CanvasError) as e:
        B.canvas_dag_compile(wl.blob_conv(), (1, 0, 4, 4), B.CANVAS_F32)
    assert e.value.status == -4
    with pytest.raises(B.CanvasError) as e:
        B.canvas_dag_compile(wl.blob_conv(), (1, 4, 4, 4), 7)
    assert e.value.status == -4
    with pytest.raises(B.CanvasError) as e:
        B.canvas_dag_compile(wl.blob_conv(), (1, 4, 4, 4), B.CANVAS_F32, flags=1 << 9)
    assert e.value.status == -4
    # forward with null pointers must be refused before any launch (no GPU is touched)
    h = B.canvas_dag_compile(wl.blob_conv(3, 1, 4), (1, 4, 4, 4), B.CANVAS_F32)
    rc = lib.canvas_dag_forward(h, None, None, None, None, 0, None)
    assert rc == -4
    arr = (ctypes.c_void_p * 1)(0x1000)
    rc = lib.canvas_dag_forward(h, 0x1000, arr, 0x2000, 0x3000, 0, None)
    assert rc == -5  # workspace too small
    rc = lib.canvas_dag_forward(h, 0x1001, arr, 0x2000, 0x3000, 1 << 30, None)
    assert rc == -4  # misaligned x
    rc = lib.canvas_dag_backward(h, 0x1000, arr, 0x2000, None, arr, 0x3000, 1 << 30, None)
    assert rc == -4
    B.canvas_dag_destroy(h)


def _compile_info(blob, shape, dtype=B.CANVAS_BF16, flags=0):
    h = B.canvas_dag_compile(blob, shape, dtype, flags)
    info = B.canvas_dag_query(h)
    names = ([B.canvas_dag_launch_desc(h, 0, i)["name"] for i in range(info.n_launches_fwd)],
             [B.canvas_dag_launch_desc(h, 1, i)["name"] for i in range(info.n_launches_bwd)])
    out = (info.fused, int(info.workspace_bytes), names)
    B.canvas_dag_destroy(h)
    return out


def test_lowering_selection(lib):
    """Which lowering compile picks (host logic only): the three fused families on their patterns, per node elsewhere."""
    H = wl.HEADER
    # config 2: shift -> grouped FC -> relu -> + x
    fused, ws, (fwd, bwd) = _compile_info(wl.blob_shift_residual(64), (64, 64, 56, 56))
    assert fused == 1 and fwd == ["sgfc_fwd"] and bwd == ["sgfc_bwd", "sgfc_dw_reduce"] and ws < (1 << 20)
    # ... but not in fp32, not with fusion off, not when H*W is no multiple of 8
    assert _compile_info(wl.blob_shift_residual(64), (2, 64, 56, 56), B.CANVAS_F32)[0] == 0
    assert _compile_info(wl.blob_shift_residual(64), (2, 64, 56, 56), B.CANVAS_BF16, B.CANVAS_OPT_NO_FUSION)[0] == 0
    assert _compile_info(wl.blob_shift_residual(64), (2, 64, 13, 13))[0] == 0
    # config 4: unfold -> FC -> gelu -> shift -> * x -> fold(1 tap) -> FC; windowed contractions on the tap-major kernels
    fused, ws, (fwd, bwd) = _compile_info(wl.blob_sampled(64), (128, 64, 56, 56))
    # (all derived weight copies, of forward and backward, in one launch at the head of the forward list)
    assert fused == 1 and fwd == ["weight_prep", "ufc_fc1_unfold", "ufc_mid_fwd", "ufc_fc2"]
    assert not any("pack" in n or "transpose" in n for n in bwd)
    # (the sums of the weight-gradient partials of both FCs: one launch at the end of the backward list)
    assert bwd[-2:] == ["ufc_fc1_dgrad_unfold", "wgrad_reduce"] and "ufc_mid_bwd" in bwd and bwd.count("wgrad_reduce") == 1
    assert not any(n.endswith("_reduce") and n != "wgrad_reduce" for n in bwd)
    assert 4 * 128 * 64 * 56 * 56 * 2 <= ws < 5 * 128 * 64 * 56 * 56 * 2   # z, v, dv, dz + partials and packed weights
    # a unary whose decisions bf16 rounding could change keeps fp32 intermediates
    clip = H + ("%1 = unfold %0 kh=3 kw=3\n%2 = fc %1 groups=8 out=64\n%3 = unary %2 op=expclip lo=-1 hi=1\n"
                "%4 = binary %0 %3 op=mul\n%5 = fc %4 groups=1 out=64\noutput %5\n")
    assert _compile_info(clip, (2, 64, 8, 8))[0] == 0
    assert _compile_info(clip.replace("expclip lo=-1 hi=1", "relu"), (2, 64, 8, 8))[0] == 1
    # config 3: per-pixel window weights
    fused, ws, (fwd, bwd) = _compile_info(wl.blob_involution(128, 3), (32, 128, 28, 28))
    # (the softmax over the 9 window weights is the epilogue of FC1; 25 weights of a 5x5 window exceed one tile of 16)
    assert fused == 1 and fwd == ["weight_prep", "dyn_fc1_softmax", "dyn_apply", "dyn_fc2"] and "dyn_apply_dx_da" in bwd
    assert _compile_info(wl.blob_involution(128, 5), (2, 128, 28, 28))[2][0] == ["weight_prep", "dyn_fc1", "dyn_softmax", "dyn_apply", "dyn_fc2"]
    # 9 softmax channels onto 9 unfolded channels would be the per-channel broadcast, not the tap pairing
    assert _compile_info(wl.blob_involution(9, 3).replace("out=9\noutput", "out=9\noutput"), (2, 9, 8, 8))[0] == 0
    # the config-2 kernels are instantiated for relu / abs / gelu / expclip only
    assert _compile_info(wl.blob_shift_residual(64).replace("relu", "sin"), (2, 64, 8, 8))[0] == 0
    # blends other than add / mul with the input keep the per-node lowering
    assert _compile_info(clip.replace("expclip lo=-1 hi=1", "relu").replace("op=mul", "op=max"), (2, 64, 8, 8))[0] == 0
    # a 7x7 window is outside the fused kernels
    assert _compile_info(wl.blob_involution(128, 7), (2, 128, 8, 8))[0] == 0


def test_spatial_fold_shapes_and_legality(lib, oracle):
    """fold axis=HW gives [N, C, T, 1, 1]; the shapes agree with the oracle; windows and reversed broadcasts are refused."""
    H = wl.HEADER
    se = H + ("%1 = fold %0 op=avg axis=HW\n%2 = fc %1 groups=1 out=4\n%3 = unary %2 op=gelu\n%4 = fc %3 groups=1 out=12\n"
              "%5 = softmax %4 axis=C\n%6 = binary %5 %0 op=mul\noutput %6\n")
    ns, out, ws = oracle.infer(se, (2, 12, 6, 5))
    h = B.canvas_dag_compile(se, (2, 12, 6, 5), B.CANVAS_BF16)
    info = B.canvas_dag_query(h)
    for k, s in enumerate(ns):
        assert list(info.node_shape[k]) == [2] + s
    assert list(info.node_shape[1]) == [2, 12, 1, 1, 1] and list(info.out_shape) == [2, 12, 1, 6, 5] and info.fused == 0
    B.canvas_dag_destroy(h)
    for body in ("%1 = fold %0 op=avg axis=HW\n%2 = unfold %1 kh=3 kw=3\noutput %2\n",
                 "%1 = fold %0 op=avg axis=HW\n%2 = shift %1 dh=0 dw=1\noutput %2\n",
                 "%1 = fold %0 op=avg axis=HW\n%2 = fold %1 op=max axis=HW\noutput %2\n",
                 "%1 = fold %0 op=avg axis=HW\n%2 = binary %0 %1 op=add\noutput %2\n"):
        with pytest.raises(B.CanvasError) as e:
            B.canvas_dag_compile(H + body, (2, 12, 6, 5), B.CANVAS_BF16)
        assert e.value.status == -3
        with pytest.raises(Exception):
            oracle.infer(H + body, (2, 12, 6, 5))


def test_workspace_grows_with_batch_only_where_it_should(lib):
    """The config-2 lowering keeps only weight-gradient partials; the others keep activations."""
    small = _compile_info(wl.blob_shift_residual(64), (8, 64, 56, 56))[1]
    big = _compile_info(wl.blob_shift_residual(64), (64, 64, 56, 56))[1]
    assert big <= 8 * small and big < (1 << 20)
    a = _compile_info(wl.blob_sampled(64), (2, 64, 16, 16))[1]
    b = _compile_info(wl.blob_sampled(64), (4, 64, 16, 16))[1]
    assert 1.5 * a < b < 2.5 * a


def test_inference_plan_moves_weight_only_launches_out_of_forward(lib):
    """An inference plan has the training plan's forward launches minus the weight-only ones, no backward,
    and refuses misuse before any launch (host logic only)."""
    for blob, shape in [(wl.blob_sampled(64), (2, 64, 14, 14)), (wl.blob_involution(128), (2, 128, 12, 12)),
                        (wl.blob_shift_residual(64), (2, 64, 16, 16)), (wl.blob_conv(3, 1, 16), (2, 16, 8, 8))]:
        for flags in (0, B.CANVAS_OPT_NO_FUSION):
            ht = B.canvas_dag_compile(blob, shape, B.CANVAS_BF16, flags)
            hi = B.canvas_dag_compile(blob, shape, B.CANVAS_BF16, flags | B.CANVAS_OPT_INFERENCE)
            it, ii = B.canvas_dag_query(ht), B.canvas_dag_query(hi)
            assert it.n_launches_prepare == 0 and ii.n_launches_bwd == 0
            assert ii.n_launches_fwd + ii.n_launches_prepare == it.n_launches_fwd
            assert ii.fused == it.fused and ii.workspace_bytes == it.workspace_bytes
            tn = [B.canvas_dag_launch_desc(ht, 0, i)["name"] for i in range(it.n_launches_fwd)]
            inn = [B.canvas_dag_launch_desc(hi, 0, i)["name"] for i in range(ii.n_launches_fwd)]
            assert [n for n in tn if n in inn] == inn  # same kernels, same order
            assert all("weight_prep" in n or "widen" in n for n in tn if n not in inn)
            arr = (ctypes.c_void_p * 4)(0x1000, 0x1000, 0x1000, 0x1000)
            assert lib.canvas_dag_backward(hi, 0x1000, arr, 0x2000, 0x4000, arr, 0x3000, 1 << 40, None) == -6
            assert lib.canvas_dag_prepare(ht, arr, 0x3000, 1 << 40, None) == -4  # not an inference plan
            if ii.n_launches_prepare:
                assert lib.canvas_dag_prepare(hi, arr, 0x3000, 0, None) == -5
                assert lib.canvas_dag_prepare(hi, None, 0x3000, 1 << 40, None) == -4
            B.canvas_dag_destroy(ht)
            B.canvas_dag_destroy(hi)
    # the tap-major windows of the sampled kernel do repack their weights: something must have moved
    hi = B.canvas_dag_compile(wl.blob_sampled(64), (2, 64, 14, 14), B.CANVAS_BF16, B.CANVAS_OPT_INFERENCE)
    assert B.canvas_dag_query(hi).n_launches_prepare >= 1
    B.canvas_dag_destroy(hi)


def test_group_views_shapes_and_legality(lib, oracle):
    """Group nodes: shapes and weight shapes equal the oracle's, the same blobs are refused, and a Group node
    costs no launch unless it is the output."""
    H_ = wl.HEADER
    ok = ["%1 = group %0 groups=4\n%2 = unfold %1 kh=3 kw=3\n%3 = fold %2 op=max axis=HW\n%4 = fc %3 out=12\noutput %4\n",
          "%1 = group %0 groups=2\n%2 = fc %1 out=18\n%3 = unfold %1 kh=3 kw=3\n%4 = binary %2 %3 op=mul\n%5 = fold %4 op=sum\noutput %5\n",
          "%1 = group %0 groups=8\n%2 = unfold %1 kh=3 kw=3\n%3 = fc %2 out=8\n%4 = group %3 groups=2\n%5 = fc %4 groups=2 out=4\noutput %5\n",
          "%1 = group %0 groups=2\n%2 = fold %1 op=sum axis=C groups=4\n%3 = fc %2 out=4\noutput %3\n",
          "%1 = group %0 groups=2\noutput %1\n",
          "%1 = group %0 groups=2\n%2 = fc %1 out=4\n%3 = binary %2 %0 op=add\noutput %3\n"]
    for body in ok:
        ns, out, ws = oracle.infer(H_ + body, (2, 8, 5, 6))
        for flags in (0, B.CANVAS_OPT_NO_FUSION):
            h = B.canvas_dag_compile(H_ + body, (2, 8, 5, 6), B.CANVAS_BF16, flags)
            info = B.canvas_dag_query(h)
            assert info.n_nodes == len(ns) and info.out_node == out and info.n_weights == len(ws)
            for k, s_ in enumerate(ns):
                assert list(info.node_shape[k]) == [2] + s_
            for k, s_ in enumerate(ws):
                assert list(info.weight_shape[k]) == s_
            names = [B.canvas_dag_launch_desc(h, 0, i)["name"] for i in range(info.n_launches_fwd)]
            assert ("node_group_fwd" in names) == body.endswith("groups=2\noutput %1\n")
            B.canvas_dag_destroy(h)
    bad = ["%1 = group %0 groups=3\noutput %1\n", "%1 = group %0\noutput %1\n", "%1 = group %0 groups=0\noutput %1\n",
           "%1 = group %0 groups=2\n%2 = fc %1 groups=4 out=8\noutput %2\n",
           "%1 = group %0 groups=2\n%2 = fc %1 out=6\n%3 = binary %2 %1 op=add\noutput %3\n"]
    for body in bad:
        with pytest.raises(Exception):
            oracle.infer(H_ + body, (2, 8, 5, 6))
        with pytest.raises(B.CanvasError) as e:
            B.canvas_dag_compile(H_ + body, (2, 8, 5, 6), B.CANVAS_BF16)
        assert e.value.status in (-1, -3)


def test_pixel_aligned_blend_legality(lib, oracle):
    H_ = wl.HEADER
    good = "%1 = fold %0 op=avg axis=HW\n%2 = fc %1 groups=1 out=30\n%3 = binary %2 %0 op=mul lhs=pixels\noutput %3\n"
    ns, out, ws = oracle.infer(H_ + good, (2, 8, 5, 6))
    h = B.canvas_dag_compile(H_ + good, (2, 8, 5, 6), B.CANVAS_BF16)
    info = B.canvas_dag_query(h)
    assert [list(info.node_shape[k]) for k in range(info.n_nodes)] == [[2] + s_ for s_ in ns] and list(info.out_shape) == [2, 8, 1, 5, 6]
    B.canvas_dag_destroy(h)
    for bad in (good.replace("out=30", "out=15"), good.replace("%2 %0 op=mul", "%2 %1 op=mul"), good.replace("lhs=pixels", "lhs=rows"),
                "%1 = fc %0 groups=1 out=30\n%2 = binary %1 %0 op=mul lhs=pixels\noutput %2\n"):
        with pytest.raises(Exception):
            oracle.infer(H_ + bad, (2, 8, 5, 6))
        with pytest.raises(B.CanvasError):
            B.canvas_dag_compile(H_ + bad, (2, 8, 5, 6), B.CANVAS_BF16)


def test_tensors_beyond_32_bit_offsets_take_the_per_node_lowering(lib):
    """The fused kernels address tensors through 32-bit byte offsets; a batch whose tensors reach 2 GiB compiles
    to the per-node lowering (64-bit indexing), reports its workspace, and smaller batches stay fused."""
    for blob, C, H, n_ok, n_big in ((wl.blob_shift_residual(64), 64, 56, 4096, 8192), (wl.blob_sampled(64), 64, 56, 4096, 8192),
                                    (wl.blob_involution(128), 128, 28, 8192, 20000)):
        h = B.canvas_dag_compile(blob, (n_ok, C, H, H), B.CANVAS_BF16)
        assert B.canvas_dag_query(h).fused == 1
        B.canvas_dag_destroy(h)
        h = B.canvas_dag_compile(blob, (n_big, C, H, H), B.CANVAS_BF16)
        info = B.canvas_dag_query(h)
        assert info.fused == 0 and info.workspace_bytes > 4 * n_big * C * H * H
        assert list(info.out_shape) == [n_big, C, 1, H, H]
        B.canvas_dag_destroy(h)
    with pytest.raises(B.CanvasError) as e:     # more than 2^40 elements in one tensor
        B.canvas_dag_compile(wl.blob_conv(3, 1, 16), (1 << 20, 1 << 10, 64, 64), B.CANVAS_BF16)
    assert e.value.status == -6


def test_single_dim_spatial_folds_shapes_and_legality(lib, oracle):
    H_ = wl.HEADER
    ok = ["%1 = fold %0 op=sum axis=W\n%2 = fc %1 groups=1 out=7\n%3 = fold %2 op=max axis=H\noutput %3\n",
          "%1 = fold %0 op=avg axis=H\n%2 = binary %1 %0 op=mul\noutput %2\n",
          "%1 = fold %0 op=sum axis=HW\n%2 = fold %0 op=sum axis=W\n%3 = binary %1 %2 op=add\noutput %3\n"]
    for body in ok:
        ns, out, ws = oracle.infer(H_ + body, (2, 8, 5, 6))
        h = B.canvas_dag_compile(H_ + body, (2, 8, 5, 6), B.CANVAS_BF16)
        info = B.canvas_dag_query(h)
        assert [list(info.node_shape[k]) for k in range(info.n_nodes)] == [[2] + s_ for s_ in ns]
        B.canvas_dag_destroy(h)
    bad = ["%1 = fold %0 op=sum axis=H\n%2 = fold %1 op=sum axis=H\noutput %2\n", "%1 = fold %0 op=sum axis=H\n%2 = fold %1 op=sum axis=HW\noutput %2\n",
           "%1 = fold %0 op=sum axis=H\n%2 = fold %0 op=sum axis=W\n%3 = binary %1 %2 op=add\noutput %3\n",
           "%1 = fold %0 op=sum axis=W\n%2 = binary %0 %1 op=add\noutput %2\n", "%1 = fold %0 op=sum axis=W\n%2 = unfold %1 kh=3 kw=1\noutput %2\n",
           "%1 = fold %0 op=sum axis=X\noutput %1\n"]
    for body in bad:
        with pytest.raises(Exception):
            oracle.infer(H_ + body, (2, 8, 5, 6))
        with pytest.raises(B.CanvasError):
            B.canvas_dag_compile(H_ + body, (2, 8, 5, 6), B.CANVAS_BF16)
