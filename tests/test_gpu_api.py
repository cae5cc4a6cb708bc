"""Entry points around the hot path, through the C ABI on the GPU: the library's
copy kernel, reading a published version back, the option switches, and the
per-kernel timing when the stage's side stream carries part of the work."""
import numpy as np
import pytest

import workloads as W
from tests.parity import GpuStage

pytestmark = pytest.mark.gpu


def _theta(w):
    import paper_2605_29664_amd as amdp
    return W.make_theta(w, amdp.amdp_stage_param_layout(amdp.make_config(**W.stage_config_args(w))))


def test_device_copy_both_paths_and_rejections():
    import torch
    import paper_2605_29664_amd as amdp
    src = torch.arange(0, 1 << 20, dtype=torch.int32, device="cuda:0")
    dst = torch.zeros_like(src)
    amdp.amdp_device_copy(dst, src)                                   # 16-byte vectors
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    dst.zero_()
    amdp.amdp_device_copy(dst[1:], src[1:1001], nbytes=4000)          # 4-byte aligned only: the word path
    torch.cuda.synchronize()
    assert torch.equal(dst[1:1001], src[1:1001]) and int(dst[0]) == 0 and int(dst[1001]) == 0
    b = torch.zeros(64, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(amdp.AmdpError) as ei:
        amdp.amdp_device_copy(b[1:], b[33:], nbytes=8)                # not 4-byte aligned
    assert ei.value.code == amdp.E_INVAL
    with pytest.raises(amdp.AmdpError) as ei:
        amdp.amdp_device_copy(b, b[32:], nbytes=6)                    # not a multiple of 4 bytes
    assert ei.value.code == amdp.E_INVAL
    amdp.amdp_device_copy(b, b[32:], nbytes=0)                        # nothing to do is not an error


def test_read_version_and_options():
    import torch
    import paper_2605_29664_amd as amdp
    from oracle.optim import round_to_bf16
    w = W.TINY["gpt_tile"]
    theta = _theta(w)
    gpu = GpuStage(w, act_slots=2, stash_slots=1)
    gpu.set_state(theta, version=7)
    assert np.array_equal(gpu.read_version(7), round_to_bf16(theta).astype(np.float32))
    buf = torch.empty(gpu.n + 1, dtype=gpu.dt, device="cuda:0")
    with pytest.raises(amdp.AmdpError) as ei:
        gpu.stage.amdp_stage_read_version(6, buf)
    assert ei.value.code == amdp.E_VERSION
    for opt, bad in ((99, 0), (amdp.OPT_GEMM_DIRECT_TO_LDS, 3), (amdp.OPT_SPLIT_K_MIN_TOKENS, 8), (amdp.OPT_LEAF_FORKS, 3)):
        with pytest.raises(amdp.AmdpError) as ei:
            gpu.stage.amdp_stage_set_option(opt, bad)
        assert ei.value.code == amdp.E_INVAL
    # a bad attention form is a bad configuration
    cfg = amdp.make_config(**W.stage_config_args(w, attention=5))
    assert amdp.amdp_stage_workspace_bytes(cfg) == 0 and amdp.amdp_stage_n_params(cfg) == 0
    # the unfused form keeps the probabilities: a larger activation slot
    fused = amdp.amdp_stage_workspace_bytes(amdp.make_config(**W.stage_config_args(w)))
    unfused = amdp.amdp_stage_workspace_bytes(amdp.make_config(**W.stage_config_args(w, attention=amdp.ATTN_UNFUSED)))
    assert unfused > fused
    gpu.stage.close()


def test_profile_counts_every_launch_with_the_side_stream_on():
    """The span ends right after a backward and its accumulation, whose gradient
    leaves and G += g sit on the stage's side stream: the profile must still
    hold every launch (it joins the side stream before reading the events)."""
    import torch
    w = W.TINY["gpt_tile"]
    gpu = GpuStage(w, act_slots=2, stash_slots=1)
    gpu.set_state(_theta(w))
    assert gpu.stage.amdp_stage_get_overlap()
    x, dy = gpu.to_dev(W.make_x(w, 0), gpu.dt), gpu.to_dev(W.make_dy(w, 0), gpu.dt)
    y, dx = torch.empty_like(x), torch.empty_like(x)
    counts = []
    for overlap in (True, False):
        gpu.stage.amdp_stage_set_overlap(overlap)
        gpu.stage.amdp_stage_profile_begin()
        gpu.stage.amdp_stage_forward(overlap, 0, x, None, y)
        gpu.stage.amdp_stage_backward(overlap, 0, dy, dx)
        gpu.stage.amdp_grad_accumulate(overlap)
        prof = gpu.stage.amdp_stage_profile_end()
        counts.append({k: v["launches"] for k, v in prof.items()})
        assert all(v["ms"] > 0 for v in prof.values())
    L = w.n_layers
    assert counts[0] == counts[1]
    assert counts[0]["grad_accumulate"] == 1 and counts[0]["column_sums"] == L
    assert counts[0]["layernorm_fwd"] == 2 * L and counts[0]["layernorm_bwd"] == 2 * L
    gemms = sum(v for k, v in counts[0].items() if k.startswith("gemm_"))
    assert gemms == 12 * L                      # four products forward, four dX and four dW backward, per layer
    gpu.stage.close()
