"""Seeded random inputs, shaped and distributed like the stage's real traffic.

A middle pipeline stage never sees tokens, only activations from its
predecessor and gradients from its successor, so the stand-in for the paper's
text corpora (Section 4.1) is by distribution: activations ~ N(0,1), upstream
gradients ~ N(0, (1e-3)^2), weights ~ N(0, 0.02^2) with LayerNorm gains centred
on one. Everything is drawn from numpy's PCG64 with
seed = 296640 + config number + 1000 * buffer index.
"""
import numpy as np

from .configs import BF16, BERT_POSTLN_BIDIR

SEED_BASE = 29664 * 10


def seed_for(workload, k=0):
    return SEED_BASE + workload.number + 1000 * k


def quantize_bf16_grid(a):
    """Snap fp32 values to the nearest value representable in bfloat16
    (ties to even), returned as fp32. Used so that both consumers of a 16-bit
    workload start from bit-identical inputs."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def _maybe_q(workload, a):
    return quantize_bf16_grid(a) if workload.dtype == BF16 else a.astype(np.float32)


def make_theta(workload, layout):
    """Flat fp32 master parameters. `layout` is a list of
    (name, offset, rows, cols) records supplied by the caller; entries whose
    name starts with 'ln' and ends with 'gamma' are drawn around one."""
    total = max(off + r * c for _, off, r, c in layout)
    rng = np.random.default_rng(seed_for(workload, 0))
    theta = (0.02 * rng.standard_normal(total)).astype(np.float32)
    for name, off, r, c in layout:
        if name.endswith("gamma"):
            theta[off:off + r * c] += 1.0
    return theta


def make_x(workload, mb):
    rng = np.random.default_rng(seed_for(workload, 1 + 2 * mb))
    x = rng.standard_normal((workload.tokens, workload.d_model)).astype(np.float32)
    return _maybe_q(workload, x)


def make_dy(workload, mb):
    rng = np.random.default_rng(seed_for(workload, 2 + 2 * mb))
    dy = (1e-3 * rng.standard_normal((workload.tokens, workload.d_model))).astype(np.float32)
    return _maybe_q(workload, dy)


def make_valid_len(workload, mb):
    """Per-sequence number of valid (unpadded) key positions, uniform on
    [seq/4, seq] inclusive (128..512 at sequence length 512)."""
    rng = np.random.default_rng(seed_for(workload, 500000 + mb))
    lo = max(1, workload.seq_len // 4)
    return rng.integers(lo, workload.seq_len + 1, size=workload.microbatch).astype(np.int32)


def make_targets(workload, mb):
    rng = np.random.default_rng(seed_for(workload, 700000 + mb))
    return rng.integers(0, workload.vocab, size=workload.tokens).astype(np.int32)


def make_tokens(workload, mb):
    """Token ids of a first-stage minibatch, uniform over the vocabulary."""
    rng = np.random.default_rng(seed_for(workload, 900000 + mb))
    return rng.integers(0, workload.vocab, size=workload.tokens).astype(np.int32)


def make_aux(workload, mb):
    """The int32 side input of a forward: targets on an LM-head stage; token
    ids (then the padding mask of a bidirectional block) on a first stage; the
    padding mask alone for other bidirectional stages; else None."""
    if workload.has_lm_head:
        return make_targets(workload, mb)
    if workload.has_embedding:
        t = make_tokens(workload, mb)
        return np.concatenate([t, make_valid_len(workload, mb)]) if workload.block_kind == BERT_POSTLN_BIDIR else t
    if workload.block_kind == BERT_POSTLN_BIDIR:
        return make_valid_len(workload, mb)
    return None


def stage_config_args(workload, **overrides):
    """Keyword arguments that describe `workload` as a stage configuration
    (field names of the library's configuration record), as a plain dict."""
    args = dict(block_kind=workload.block_kind, n_layers=workload.n_layers, d_model=workload.d_model,
                n_heads=workload.n_heads, d_ffn=workload.d_ffn, seq_len=workload.seq_len,
                microbatch=workload.microbatch, dtype=workload.dtype, has_lm_head=workload.has_lm_head,
                vocab=workload.vocab, ln_eps=workload.ln_eps, act_slots=workload.act_slots,
                stash_slots=workload.stash_slots, has_embedding=workload.has_embedding)
    args.update(overrides)
    return args
