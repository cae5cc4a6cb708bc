"""The block's row operators through their own C entry points, element by
element against the oracle's LayerNorm definitions (fp64 from the same bf16 /
fp32 inputs): forward, backward with and without the fused residual, and the
parameter gradients that are column sums over the tokens. Shapes span one
vector per lane up to configuration 5's widths, ragged row counts (not a
multiple of the rows a workgroup or a row chunk takes), zero rows, and the
widest reduction the stage launches."""
import numpy as np
import pytest

import workloads as W
from oracle import stage as OS

pytestmark = pytest.mark.gpu

SHAPES = [(1, 8), (5, 64), (131, 512), (1000, 1600), (2048, 4096), (777, 12288), (4096, 1024)]


def _inputs(rows, cols, dtype, seed):
    rng = np.random.default_rng(seed)
    q = W.quantize_bf16_grid if dtype == "bf16" else (lambda a: a.astype(np.float32))
    x = q(rng.standard_normal((rows, cols)) * 1.5 + 0.3)
    dy = q(1e-3 * rng.standard_normal((rows, cols)))
    res = q(1e-3 * rng.standard_normal((rows, cols)))
    gamma = q(1.0 + 0.02 * rng.standard_normal(cols))
    beta = q(0.02 * rng.standard_normal(cols))
    return x, dy, res, gamma, beta


def _dev(a, dtype):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def _check(got, ref, dtype, what, out_rounded=True):
    """fp32: 1e-5 of the tensor's rms per element. bf16 outputs carry one rounding
    to 8 bits of their own value on top of fp32-exact arithmetic."""
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    rms = np.sqrt(np.mean(ref * ref)) if ref.size else 0.0
    if dtype == "bf16" and out_rounded:
        bound = 2.0 ** -8 * np.abs(ref) + 1e-4 * rms
    else:
        bound = 2e-5 * np.abs(ref) + 2e-5 * rms
    bad = np.abs(got - ref) > bound
    assert not bad.any(), (what, int(bad.sum()), float(np.abs(got - ref).max()), float(rms))


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("rows,cols", SHAPES)
def test_layernorm_forward_backward_and_parameter_gradients(rows, cols, dtype):
    import torch
    import paper_2605_29664_amd as amdp
    x, dy, res, gamma, beta = _inputs(rows, cols, dtype, rows * 131 + cols)
    eps = 1e-5
    y_ref, (xhat, rstd) = OS.layernorm_fwd(x.astype(np.float64), gamma.astype(np.float64), beta.astype(np.float64), eps)
    dx_ref, dgamma_ref, dbeta_ref = OS.layernorm_bwd(dy.astype(np.float64), (xhat, rstd), gamma.astype(np.float64))

    xd, dyd, resd, gd, bd = (_dev(a, dtype) for a in (x, dy, res, gamma, beta))
    y = torch.full_like(xd, float("nan"))
    stats = torch.full((rows, 2), float("nan"), dtype=torch.float32, device="cuda:0")
    amdp.amdp_layernorm_forward(xd, gd, bd, y, stats, eps)
    torch.cuda.synchronize()
    _check(y.float().cpu().numpy(), y_ref, dtype, "y")
    st = stats.cpu().numpy().astype(np.float64)
    _check(st[:, 0], x.astype(np.float64).mean(axis=1), "fp32", "mean")
    _check(st[:, 1], rstd[:, 0], "fp32", "rstd")

    for with_res in (False, True):
        dx = torch.full_like(xd, float("nan"))
        amdp.amdp_layernorm_backward(dyd, xd, stats, gd, resd if with_res else None, dx)
        torch.cuda.synchronize()
        _check(dx.float().cpu().numpy(), dx_ref + (res.astype(np.float64) if with_res else 0.0), dtype,
               f"dx res={with_res}")

    code = amdp.BF16 if dtype == "bf16" else amdp.FP32
    for ln in (False, True):
        nbytes = amdp.amdp_column_sums_workspace_bytes(rows, cols, code, ln)
        assert nbytes > 0
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0").fill_(255)      # NaN bit patterns
        out = torch.full(((2 if ln else 1) * cols,), float("nan"), dtype=torch.float32, device="cuda:0")
        amdp.amdp_column_sums(dyd, xd if ln else None, stats if ln else None, out, ws)
        torch.cuda.synchronize()
        o = out.cpu().numpy()
        if ln:
            # sums of rows * cols products: fp32 accumulation error grows with the number of rows
            # xhat itself is formed in fp32 from (x - mean) * rstd: absolute error of a few 2^-24 of
            # (|x| + |mean|) * rstd per entry, whatever the size of xhat
            _check_sum(o[:cols], dgamma_ref, dy.astype(np.float64) * xhat, "dgamma",
                       slack=2e-6 * np.abs(dy.astype(np.float64)).sum(axis=0))
            _check_sum(o[cols:], dbeta_ref, dy.astype(np.float64), "dbeta")
        else:
            _check_sum(o, dbeta_ref, dy.astype(np.float64), "column sums")
        out2 = torch.empty_like(out)
        amdp.amdp_column_sums(dyd, xd if ln else None, stats if ln else None, out2, ws)
        torch.cuda.synchronize()
        assert torch.equal(out, out2), "column sums are not run-to-run identical"


def _check_sum(got, ref, terms, what, slack=0.0):
    """A sum of n fp32 terms in any order is within n * 2^-24 * sum|terms| of the exact sum
    (the terms themselves are formed in fp32: one more rounding each)."""
    n = terms.shape[0]
    bound = (n + 2) * 2.0 ** -24 * np.abs(terms).sum(axis=0) + slack + 1e-30
    bad = np.abs(np.asarray(got, dtype=np.float64) - ref) > bound
    assert not bad.any(), (what, int(bad.sum()), float(np.abs(got - ref).max()))


def test_zero_rows_and_rejected_arguments():
    import torch
    import paper_2605_29664_amd as amdp
    x = torch.empty((0, 64), dtype=torch.bfloat16, device="cuda:0")
    g = torch.ones(64, dtype=torch.bfloat16, device="cuda:0")
    stats = torch.empty((0, 2), dtype=torch.float32, device="cuda:0")
    amdp.amdp_layernorm_forward(x, g, g, x, stats, 1e-5)
    ws = torch.empty(amdp.amdp_column_sums_workspace_bytes(0, 64, amdp.BF16, False), dtype=torch.uint8, device="cuda:0")
    out = torch.full((64,), float("nan"), dtype=torch.float32, device="cuda:0")
    amdp.amdp_column_sums(x, None, None, out, ws)
    torch.cuda.synchronize()
    assert float(out.abs().max()) == 0.0
    bad = torch.empty((4, 12), dtype=torch.bfloat16, device="cuda:0")        # 12 columns: not whole 16-byte vectors
    assert amdp.amdp_column_sums_workspace_bytes(4, 12, amdp.BF16, False) == 0
    with pytest.raises(amdp.AmdpError) as ei:
        amdp.amdp_column_sums(bad, None, None, out, ws)
    assert ei.value.code == amdp.E_INVAL
    small = torch.empty(16, dtype=torch.uint8, device="cuda:0")
    ok = torch.empty((4, 64), dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(amdp.AmdpError) as ei:
        amdp.amdp_column_sums(ok, None, None, out, small)                    # workspace too small
    assert ei.value.code == amdp.E_INVAL
