"""A block with different input and output channel counts, composed from one kernel template (test infrastructure,
not product code; only tests, the smoke check and the benchmark's CPU-baseline leg may import it).

Canvas searches a single template [C, H, W] => [C, H, W] and applies it to a general convolution
[C_in, H, W] => [C_out, H, W] where one channel count is a multiple of the other (Section 4, "Main focus:
convolutions").  The figure that shows the composition is not part of the text, so the rule below is a reading of that
sentence, chosen so that with a convolution as the template the block is exactly the convolution C_in => C_out whose
weight matrix is cut into square blocks:

  * C_out = m * C_in ("expand"): m instances of the template, each with weights of its own, all read the input;
    their outputs are concatenated along the channels, instance j giving channels [j * C_in, (j + 1) * C_in).
  * C_in = m * C_out ("reduce"): the input is cut into m slices of C_out channels, instance j (weights of its own)
    reads slice j; the outputs are summed.

parity unpinned by the paper: the paper prints no value for a composed block.  The pins in tests/test_oracle_block.py
hold this file to its own stated rule (a convolution template against a library convolution with the assembled
weights, m = 1 against the plain DAG, finite differences), not to the paper.

Every instance runs through the fp64 DAG oracle (canvas_oracle.run); this file only slices, concatenates and sums.
"""
import numpy as np

from . import canvas_oracle


def multiple_and_mode(c_in, c_out):
    """(m, 'expand' | 'reduce'); equal channel counts are an expand block of one instance."""
    if c_out % c_in == 0:
        return c_out // c_in, "expand"
    if c_in % c_out == 0:
        return c_in // c_out, "reduce"
    raise ValueError(f"neither of {c_in} and {c_out} is a multiple of the other")


def run_block(blob, x, weights, c_out, dy=None, **kw):
    """x: [N, C_in, H, W]; weights: m lists (one per instance) of the template's weight tensors; dy: [N, C_out, H, W].

    Returns dict(y=[N, C_out, H, W], dx, dw=m lists)."""
    x = np.asarray(x, dtype=np.float64)
    n, c_in, h, w = x.shape
    m, mode = multiple_and_mode(c_in, c_out)
    assert len(weights) == m, "one weight set per instance"
    c = min(c_in, c_out)
    y = np.zeros((n, c_out, h, w))
    dx = None if dy is None else np.zeros_like(x)
    dws = []
    if dy is not None:
        dy = np.asarray(dy, dtype=np.float64).reshape(y.shape)
    for j in range(m):
        sl = slice(j * c, (j + 1) * c)
        if mode == "expand":
            r = canvas_oracle.run(blob, x, weights[j], None if dy is None else dy[:, sl], **kw)
            assert r["y"].shape == (n, c, h, w), "the template must map [C, H, W] to [C, H, W]"
            y[:, sl] = r["y"]
            if dy is not None:
                dx += r["dx"]
        else:
            r = canvas_oracle.run(blob, x[:, sl], weights[j], dy, **kw)
            assert r["y"].shape == (n, c, h, w), "the template must map [C, H, W] to [C, H, W]"
            y += r["y"]
            if dy is not None:
                dx[:, sl] = r["dx"]
        dws.append(r["dw"])
    return {"y": y, "dx": dx, "dw": dws, "m": m, "mode": mode}
