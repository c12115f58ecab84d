"""The entry point that allocates nothing (fg_linear_static: partial sums in a device array the
library owns) against fg_linear with a caller-provided workspace: same kernels, so the outputs must be
bit-identical; two calls in a row, the second smaller, because every call on a GPU shares the one
scratch array and finds the previous call's contents in it."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2303_06865_amd import binding as B

pytestmark = pytest.mark.gpu


def _case(m, n, k, seed, wdtype):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    w = torch.empty((n, k), dtype=torch.float16, device="cuda").normal_(0.0, 0.02, generator=g)
    x = torch.empty((m, k), dtype=torch.float16, device="cuda").normal_(0.0, 1.0, generator=g)
    res = torch.empty((m, n), dtype=torch.float16, device="cuda").normal_(0.0, 1.0, generator=g)
    bias = torch.empty((n,), dtype=torch.float16, device="cuda").normal_(0.0, 0.5, generator=g)
    mat = B.Mat.from_f16(w, wdtype != "f16", tiled=wdtype == "q4t")
    return mat, bias, x, res


@pytest.mark.parametrize("wdtype", ["q4t", "q4", "f16"])
def test_static_scratch_linear_matches_workspace_linear_twice_in_a_row(wdtype):
    # first a projection whose partial sums fill most of the scratch (144 rows, split contraction), then a
    # smaller one with a ragged row count that finds the first call's partial sums still in place
    for (m, n, k, seed) in ((144, 4096, 12288, 1), (37, 1024, 2048, 2)):
        mat, bias, x, res = _case(m, n, k, seed, wdtype)
        need = B.lib().fg_linear_workspace_bytes(C.byref(mat.c), m)
        assert need <= B.lib().fg_linear_static_scratch_bytes()
        want = B.fg_linear(mat, bias, x, res, True)
        out = torch.full((m, n), float("nan"), dtype=torch.float16, device="cuda")
        B.fg_linear_static(mat, bias, x, res, True, out)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(out.float()).all())
        assert np.array_equal(out.cpu().numpy().view(np.uint16), want.cpu().numpy().view(np.uint16)), (wdtype, m, n, k)


def test_static_scratch_linear_refuses_what_does_not_fit():
    """The 256-row-tile shape of the prefill phase needs 128 MiB of partial sums: refused, nothing launched."""
    mat, bias, x, res = _case(1024, 1024, 1024, 3, "q4t")
    assert B.lib().fg_linear_workspace_bytes(C.byref(mat.c), 1024) > B.lib().fg_linear_static_scratch_bytes()
    out = torch.zeros((1024, 1024), dtype=torch.float16, device="cuda")
    with pytest.raises(B.FgError) as e:
        B.fg_linear_static(mat, bias, x, res, False, out)
    assert e.value.status == B.FG_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert float(out.abs().max()) == 0.0
