"""amdp_column_sums_static -- the column sums for callers that cannot allocate --
through the C ABI against amdp_column_sums (the form with a caller workspace):
two calls in a row on one stream, the second on a smaller input, so that the
second call meets the first call's leftovers in the library's fixed scratch
array. With at most 8192 floats of width both forms split the rows alike and the
results must be bit-identical; beyond that the fixed array holds fewer row
chunks and the results agree within fp32 summation error. Also: the size limit
is refused with AMDP_E_TOO_LARGE before anything is enqueued."""
import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu


def _case(rows, cols, with_ln, seed):
    import torch
    rng = np.random.default_rng(seed)
    dy = torch.from_numpy(W.quantize_bf16_grid(1e-3 * rng.standard_normal((rows, cols)))).to("cuda:0").to(torch.bfloat16)
    x = stats = None
    if with_ln:
        x = torch.from_numpy(W.quantize_bf16_grid(rng.standard_normal((rows, cols)))).to("cuda:0").to(torch.bfloat16)
        xf = x.float()
        mean = xf.mean(dim=1)
        rstd = 1.0 / torch.sqrt(xf.var(dim=1, unbiased=False) + 1e-5)
        stats = torch.stack([mean, rstd], dim=1).contiguous()
    return dy, x, stats


def _both(amdp, dy, x, stats):
    import torch
    rows, cols = dy.shape
    width = cols * (2 if x is not None else 1)
    ws = torch.empty(amdp.amdp_column_sums_workspace_bytes(rows, cols, amdp.BF16, x is not None), dtype=torch.uint8,
                     device="cuda:0")
    ref = torch.full((width,), float("nan"), dtype=torch.float32, device="cuda:0")
    got = torch.full((width,), float("nan"), dtype=torch.float32, device="cuda:0")
    amdp.amdp_column_sums(dy, x, stats, ref, ws)
    amdp.amdp_column_sums_static(dy, x, stats, got)
    return ref, got


@pytest.mark.parametrize("with_ln", [False, True])
def test_two_calls_in_a_row_second_one_smaller(with_ln):
    import torch
    import paper_2605_29664_amd as amdp
    big = _case(4096, 4096, with_ln, 1)            # configuration 5's width, 256 row chunks
    small = _case(333, 512, with_ln, 2)            # fewer rows, fewer columns, a ragged last chunk
    r1, g1 = _both(amdp, *big)
    r2, g2 = _both(amdp, *small)                   # no synchronisation in between: stream order alone
    torch.cuda.synchronize()
    assert torch.isfinite(r1).all() and torch.isfinite(r2).all()
    assert torch.equal(g1, r1), "first call differs from amdp_column_sums"
    assert torch.equal(g2, r2), "second, smaller call differs from amdp_column_sums"
    # and the sums are the sums (fp64 on the host from the same inputs)
    dy, x, stats = small
    want = dy.double().sum(dim=0).cpu().numpy()
    tail = g2.cpu().numpy()[-dy.shape[1]:].astype(np.float64)
    assert np.all(np.abs(tail - want) <= 335 * 2.0 ** -24 * dy.double().abs().sum(dim=0).cpu().numpy() + 1e-30)


def test_wide_problem_uses_fewer_chunks_and_limit_is_refused():
    import torch
    import paper_2605_29664_amd as amdp
    dy, _, _ = _case(512, 16384, False, 3)         # width 16384 floats: 128 row chunks fit, the workspace form takes 256
    ref, got = _both(amdp, dy, None, None)
    torch.cuda.synchronize()
    bound = 514 * 2.0 ** -24 * dy.double().abs().sum(dim=0)
    assert bool(((got.double() - ref.double()).abs() <= bound).all())
    assert amdp.amdp_column_sums_static_max_cols(False) == 2 * 1024 * 1024
    assert amdp.amdp_column_sums_static_max_cols(True) == 1024 * 1024
    # one row of one column more than fits: refused, nothing enqueued, `out` untouched
    cols = amdp.amdp_column_sums_static_max_cols(True) + 8
    x = torch.zeros((1, cols), dtype=torch.bfloat16, device="cuda:0")
    stats = torch.zeros((1, 2), dtype=torch.float32, device="cuda:0")
    out = torch.full((2 * cols,), 7.0, dtype=torch.float32, device="cuda:0")
    with pytest.raises(amdp.AmdpError) as ei:
        amdp.amdp_column_sums_static(x, x, stats, out)
    assert ei.value.code == amdp.E_TOO_LARGE
    torch.cuda.synchronize()
    assert float(out.min()) == 7.0 and float(out.max()) == 7.0
    # the largest width that is accepted runs with a single row chunk
    cols = amdp.amdp_column_sums_static_max_cols(False)
    dy = torch.ones((3, cols), dtype=torch.bfloat16, device="cuda:0")
    out = torch.empty(cols, dtype=torch.float32, device="cuda:0")
    amdp.amdp_column_sums_static(dy, None, None, out)
    torch.cuda.synchronize()
    assert float(out.min()) == 3.0 and float(out.max()) == 3.0
