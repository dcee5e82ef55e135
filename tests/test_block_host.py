"""Host-side checks of include/canvas_block.h: exported symbols, composition rule in the info, error paths (no GPU)."""
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


def test_every_declared_block_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "canvas_block.h")).read()
    declared = set(re.findall(r"^(?:int|void)\s+(canvas_[a-z_]+)\s*\(", header, re.M))
    assert declared == set(B.BLOCK_EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


@pytest.mark.parametrize("c_in,c_out,m,expand", [(16, 64, 4, 1), (64, 16, 4, 0), (32, 32, 1, 1), (16, 48, 3, 1)])
def test_composition_in_the_info(lib, c_in, c_out, m, expand):
    c = min(c_in, c_out)
    h = B.canvas_block_compile(wl.blob_conv(3, 1, c), (2, c_in, 8, 8), c_out, B.CANVAS_BF16)
    info = B.canvas_block_query(h)
    assert (info.instances, info.expand, info.template_channels, info.n_weights) == (m, expand, c, 1)
    assert list(info.plan.out_shape) == [2, c, 1, 8, 8] and list(info.plan.weight_shape[0]) == [1, c, 9 * c]
    dense = 2 * c * 64
    assert info.workspace_bytes >= m * info.plan.workspace_bytes + 2 * m * dense * 2
    B.canvas_block_destroy(h)


def test_illegal_blocks_are_refused(lib):
    with pytest.raises(B.CanvasError) as e:
        B.canvas_block_compile(wl.blob_conv(3, 1, 16), (1, 24, 8, 8), 16, B.CANVAS_F32)   # 24 and 16: no multiple
    assert e.value.status == -3
    with pytest.raises(B.CanvasError) as e:   # the template changes its channel count
        B.canvas_block_compile(wl.blob_conv(3, 1, 8), (1, 16, 8, 8), 32, B.CANVAS_F32)
    assert e.value.status == -3
    with pytest.raises(B.CanvasError) as e:   # taps left on the output
        B.canvas_block_compile(wl.HEADER + "%1 = unfold %0 kh=3 kw=3\noutput %1\n", (1, 16, 8, 8), 32, B.CANVAS_F32)
    assert e.value.status == -3
    with pytest.raises(B.CanvasError) as e:
        B.canvas_block_compile(wl.blob_conv(3, 1, 16), (1, 16, 8, 8), 32, B.CANVAS_F32, B.CANVAS_OPT_INFERENCE)
    assert e.value.status == -6
    with pytest.raises(B.CanvasError):
        B.canvas_block_compile("not a dag", (1, 16, 8, 8), 32, B.CANVAS_F32)
