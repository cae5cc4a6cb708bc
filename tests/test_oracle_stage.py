"""Pins for oracle/stage.py (no GPU): library reference ops in fp64, central
finite differences, torch.autograd as a second opinion, structural properties,
and Table 2's parameter counts."""
import json
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as TF

import workloads as W
from oracle import stage as OS
from oracle.stage import Stage

F64 = torch.float64


def _setup(key, mb=0):
    w = W.TINY[key]
    st = Stage.from_workload(w)
    theta = W.make_theta(w, st.layout).astype(np.float64)
    x = W.make_x(w, mb).astype(np.float64)
    aux = None
    if w.has_lm_head:
        aux = W.make_targets(w, mb)
    elif w.block_kind == W.configs.BERT_POSTLN_BIDIR:
        aux = np.array([5, 8], dtype=np.int32)[: w.microbatch]
    dy = None if w.has_lm_head else W.make_dy(w, mb).astype(np.float64) * 1e3
    return w, st, theta, x, aux, dy


# ------------------------------------------------ an independent torch model
def torch_stage(w, theta_t, x_t, aux):
    """The same stage written with torch.nn.functional building blocks."""
    lay = OS.param_layout(w.n_layers, w.d_model, w.d_ffn, w.has_lm_head, w.vocab)
    p = {}
    for name, off, r, c in lay:
        v = theta_t[off:off + r * c]
        p[name] = v if r == 1 else v.view(r, c)
    D, H, s, b = w.d_model, w.n_heads, w.seq_len, w.microbatch
    dh = D // H
    causal = w.block_kind == W.configs.GPT_PRELN_CAUSAL

    def attn(a, l):
        qkv = TF.linear(a, p[f"l{l}.w_qkv"].T, p[f"l{l}.b_qkv"])
        q, k, v = (t.view(b, s, H, dh).transpose(1, 2) for t in qkv.split(D, dim=1))
        if causal:
            o = TF.scaled_dot_product_attention(q, k, v, is_causal=True)
        else:
            keep = torch.arange(s)[None, :] < torch.as_tensor(np.asarray(aux))[:, None]   # [b, s]
            o = TF.scaled_dot_product_attention(q, k, v, attn_mask=keep[:, None, None, :])
        o = o.transpose(1, 2).reshape(b * s, D)
        return TF.linear(o, p[f"l{l}.w_o"].T, p[f"l{l}.b_o"])

    def mlp(c, l):
        return TF.linear(TF.gelu(TF.linear(c, p[f"l{l}.w_1"].T, p[f"l{l}.b_1"])),
                         p[f"l{l}.w_2"].T, p[f"l{l}.b_2"])

    def ln(t, name):
        return TF.layer_norm(t, (D,), p[name + "_gamma"], p[name + "_beta"], w.ln_eps)

    h = x_t
    for l in range(w.n_layers):
        if causal:
            h = h + attn(ln(h, f"l{l}.ln1"), l)
            h = h + mlp(ln(h, f"l{l}.ln2"), l)
        else:
            h = ln(h + attn(h, l), f"l{l}.ln1")
            h = ln(h + mlp(h, l), f"l{l}.ln2")
    if not w.has_lm_head:
        return h
    z = ln(h, "lnf")
    return TF.cross_entropy(z @ p["embed"].T, torch.as_tensor(np.asarray(aux), dtype=torch.long))


@pytest.mark.parametrize("key", ["gpt", "bert", "lmhead"])
def test_forward_matches_library_ops(key):
    w, st, theta, x, aux, _ = _setup(key)
    out, _ = st.forward(theta, x, aux)
    ref = torch_stage(w, torch.tensor(theta, dtype=F64), torch.tensor(x, dtype=F64), aux).detach().numpy()
    assert np.allclose(out, ref, rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("key", ["gpt", "bert", "lmhead"])
def test_backward_matches_autograd(key):
    w, st, theta, x, aux, dy = _setup(key)
    _, saved = st.forward(theta, x, aux)
    dx, g = st.backward(theta, saved, dy)
    tt = torch.tensor(theta, dtype=F64, requires_grad=True)
    xt = torch.tensor(x, dtype=F64, requires_grad=True)
    out = torch_stage(w, tt, xt, aux)
    if w.has_lm_head:
        out.backward()
    else:
        out.backward(torch.tensor(dy, dtype=F64))
    assert np.allclose(dx, xt.grad.numpy(), rtol=1e-9, atol=1e-12)
    assert np.allclose(g, tt.grad.numpy(), rtol=1e-9, atol=1e-12)


@pytest.mark.parametrize("key", ["gpt", "bert", "lmhead"])
def test_backward_finite_differences(key):
    """Every parameter tensor and dX, central differences in fp64."""
    w, st, theta, x, aux, dy = _setup(key)
    _, saved = st.forward(theta, x, aux)
    dx, g = st.backward(theta, saved, dy)

    def scalar(th, xx):
        out, _ = st.forward(th, xx, aux)
        return float(out) if w.has_lm_head else float((out * dy).sum())

    rng = np.random.default_rng(5)
    h = 1e-5
    for name, off, r, c in st.layout:
        for j in rng.choice(r * c, size=min(3, r * c), replace=False):
            tp, tm = theta.copy(), theta.copy()
            tp[off + j] += h
            tm[off + j] -= h
            fd = (scalar(tp, x) - scalar(tm, x)) / (2 * h)
            assert abs(fd - g[off + j]) <= 1e-6 * max(1.0, abs(fd)) + 1e-9, (name, j, fd, g[off + j])
    for j in rng.choice(x.size, size=12, replace=False):
        xp, xm = x.copy().reshape(-1), x.copy().reshape(-1)
        xp[j] += h
        xm[j] -= h
        fd = (scalar(theta, xp.reshape(x.shape)) - scalar(theta, xm.reshape(x.shape))) / (2 * h)
        assert abs(fd - dx.reshape(-1)[j]) <= 1e-6 * max(1.0, abs(fd)) + 1e-9


def _two_version_backward_by_local_autograd(w, theta1, theta2, x, aux, dy):
    """The backward with a parameter version other than the forward's, built
    from torch.autograd alone: the forward runs with theta1 and records the
    INPUT of every primitive (LayerNorm, linear, attention core, GELU, loss);
    the reverse sweep then takes, primitive by primitive, the vector-Jacobian
    product of that primitive evaluated at its recorded input -- a detached
    constant -- with the parameters of theta2. Returns (dX, flat gradient)."""
    lay = OS.param_layout(w.n_layers, w.d_model, w.d_ffn, w.has_lm_head, w.vocab)

    def params(theta):
        t = torch.tensor(theta, dtype=F64)
        return {name: (t[off:off + r * c] if r == 1 else t[off:off + r * c].view(r, c)) for name, off, r, c in lay}

    p1, p2 = params(theta1), params(theta2)
    D, H, s, b = w.d_model, w.n_heads, w.seq_len, w.microbatch
    dh = D // H
    causal = w.block_kind == W.configs.GPT_PRELN_CAUSAL
    keep = None if causal else (torch.arange(s)[None, :] < torch.as_tensor(np.asarray(aux))[:, None])[:, None, None, :]

    def f_ln(t, g, be):
        return TF.layer_norm(t, (D,), g, be, w.ln_eps)

    def f_lin(t, W_, b_):
        return t @ W_ + b_

    def f_core(qkv):
        q, k, v = (t.view(b, s, H, dh).transpose(1, 2) for t in qkv.split(D, dim=1))
        o = TF.scaled_dot_product_attention(q, k, v, is_causal=True) if causal else \
            TF.scaled_dot_product_attention(q, k, v, attn_mask=keep)
        return o.transpose(1, 2).reshape(b * s, D)

    tape = []          # (function, recorded input, parameter names, kind)

    def run(fn, t, names=()):
        tape.append((fn, t.detach().clone(), names))
        return fn(t, *[p1[n] for n in names])

    # forward with theta1; residual structure kept beside the tape
    h = torch.tensor(x, dtype=F64)
    plan = []
    for l in range(w.n_layers):
        L = f"l{l}."
        if causal:
            i0 = len(tape)
            a = run(f_ln, h, (L + "ln1_gamma", L + "ln1_beta"))
            qkv = run(f_lin, a, (L + "w_qkv", L + "b_qkv"))
            o = run(f_core, qkv)
            y1 = h + run(f_lin, o, (L + "w_o", L + "b_o"))
            i1 = len(tape)
            c = run(f_ln, y1, (L + "ln2_gamma", L + "ln2_beta"))
            u = run(f_lin, c, (L + "w_1", L + "b_1"))
            g_ = run(TF.gelu, u)
            h = y1 + run(f_lin, g_, (L + "w_2", L + "b_2"))
            plan += [("res", i0, i1), ("res", i1, len(tape))]
        else:
            i0 = len(tape)
            qkv = run(f_lin, h, (L + "w_qkv", L + "b_qkv"))
            o = run(f_core, qkv)
            r1 = h + run(f_lin, o, (L + "w_o", L + "b_o"))
            i1 = len(tape)
            y1 = run(f_ln, r1, (L + "ln1_gamma", L + "ln1_beta"))
            i2 = len(tape)
            u = run(f_lin, y1, (L + "w_1", L + "b_1"))
            g_ = run(TF.gelu, u)
            r2 = y1 + run(f_lin, g_, (L + "w_2", L + "b_2"))
            i3 = len(tape)
            h = run(f_ln, r2, (L + "ln2_gamma", L + "ln2_beta"))
            plan += [("res", i0, i1), ("seq", i1, i2), ("res", i2, i3), ("seq", i3, len(tape))]
    if w.has_lm_head:
        i0 = len(tape)
        z = run(f_ln, h, ("lnf_gamma", "lnf_beta"))
        tgt = torch.as_tensor(np.asarray(aux), dtype=torch.long)
        logits = run(lambda t, E: t @ E.T, z, ("embed",))      # the logits are a saved activation like any other
        run(lambda t: TF.cross_entropy(t, tgt), logits)
        plan += [("seq", i0, len(tape))]

    grads = {name: torch.zeros_like(v) for name, v in p2.items()}

    def vjp_chain(lo, hi, gout):
        for k in range(hi - 1, lo - 1, -1):
            fn, t_in, names = tape[k]
            t_in = t_in.clone().requires_grad_(True)
            ps = [p2[n].detach().clone().requires_grad_(True) for n in names]
            out = fn(t_in, *ps)
            got = torch.autograd.grad(out, [t_in] + ps, gout)
            gout = got[0]
            for n, gp in zip(names, got[1:]):
                grads[n] += gp
        return gout

    gout = torch.tensor(1.0, dtype=F64) if w.has_lm_head else torch.tensor(dy, dtype=F64)
    for kind, lo, hi in reversed(plan):
        gout = vjp_chain(lo, hi, gout) + (gout if kind == "res" else 0.0)
    flat = np.zeros(theta1.size)
    for name, off, r, c in lay:
        flat[off:off + r * c] = grads[name].reshape(-1).numpy()
    return gout.numpy(), flat


@pytest.mark.parametrize("key", ["gpt", "bert", "lmhead"])
def test_mismatched_backward_matches_detached_graph(key):
    """Backward with a different parameter version over the WHOLE stage: saved
    activations are the forward's constants, every weight that appears
    (transposed matrices, LayerNorm gains, the tied embedding) comes from the
    new version. A wrong choice of version for any single parameter, or a saved
    activation replaced by a recomputed one, changes some gradient here."""
    w, st, theta, x, aux, dy = _setup(key)
    theta2 = theta + 0.05 * np.random.default_rng(1).standard_normal(theta.size)
    _, saved = st.forward(theta, x, aux)
    dx_a, g_a = st.backward(theta, saved, dy)
    dx_b, g_b = st.backward(theta2, saved, dy)
    dx_ref, g_ref = _two_version_backward_by_local_autograd(w, theta, theta2, x, aux, dy)
    assert np.allclose(dx_b, dx_ref, rtol=1e-9, atol=1e-12)
    for name, off, r, c in st.layout:
        assert np.allclose(g_b[off:off + r * c], g_ref[off:off + r * c], rtol=1e-9, atol=1e-12), name
    # the same construction with one version reproduces the ordinary backward ...
    dx_same, g_same = _two_version_backward_by_local_autograd(w, theta, theta, x, aux, dy)
    assert np.allclose(dx_a, dx_same, rtol=1e-9, atol=1e-12) and np.allclose(g_a, g_same, rtol=1e-9, atol=1e-12)
    # ... and the two versions really give different results
    assert not np.allclose(dx_a, dx_b, rtol=1e-3) and not np.allclose(g_a, g_b, rtol=1e-3)


def test_softmax_rows_and_mask():
    w, st, theta, x, aux, _ = _setup("bert")
    _, (saved, _) = st.forward(theta, x, aux)
    probs = saved[0][1][2]
    for (seq, h), p in probs.items():
        assert np.allclose(p.sum(axis=1), 1.0, atol=1e-14)
        assert np.all(p[:, int(aux[seq]):] == 0.0)
    w, st, theta, x, aux, _ = _setup("gpt")
    _, (saved, _) = st.forward(theta, x, aux)
    for p in saved[0][1][2].values():
        assert np.all(np.triu(p, 1) == 0.0) and np.allclose(p.sum(axis=1), 1.0, atol=1e-14)


def test_causal_independence_of_future():
    w, st, theta, x, aux, _ = _setup("gpt")
    y0, _ = st.forward(theta, x)
    x2 = x.copy()
    pos = 5
    for seq in range(w.microbatch):
        x2[seq * w.seq_len + pos + 1:(seq + 1) * w.seq_len] += 3.0
    y1, _ = st.forward(theta, x2)
    for seq in range(w.microbatch):
        rows = slice(seq * w.seq_len, seq * w.seq_len + pos + 1)
        assert np.array_equal(y0[rows], y1[rows])
    assert not np.allclose(y0, y1)


def test_padding_independence():
    w, st, theta, x, aux, _ = _setup("bert")
    y0, _ = st.forward(theta, x, aux)
    x2 = x.copy()
    for seq in range(w.microbatch):
        x2[seq * w.seq_len + int(aux[seq]):(seq + 1) * w.seq_len] -= 2.0
    y1, _ = st.forward(theta, x2, aux)
    for seq in range(w.microbatch):
        rows = slice(seq * w.seq_len, seq * w.seq_len + int(aux[seq]))
        assert np.allclose(y0[rows], y1[rows], rtol=0, atol=1e-13)


def test_uniform_logits_loss_is_log_vocab():
    w, st, theta, x, aux, _ = _setup("lmhead")
    th = theta.copy()
    for name, off, r, c in st.layout:
        if name == "embed":
            th[off:off + r * c] = 0.0
    loss, saved = st.forward(th, x, aux)
    assert abs(loss - np.log(w.vocab)) < 1e-12
    _, g = st.backward(th, saved)
    for name, off, r, c in st.layout:
        if name == "embed":     # rows sum over vocab to zero: sum_v (p_v - onehot_v) = 0
            assert np.allclose(g[off:off + r * c].reshape(r, c).sum(axis=0), 0.0, atol=1e-14)


def test_table2_parameter_counts(golden_dir):
    facts = json.load(open(os.path.join(golden_dir, "paper_schedule_facts.json")))["table2_parameter_counts"]
    g = facts["gpt"]
    h = g["hidden"]
    per_layer = OS.n_params(OS.param_layout(1, h, 4 * h))
    assert per_layer == 12 * h * h + 13 * h
    # GPT: layers + padded vocabulary embedding + learned positions + final LayerNorm
    assert g["layers"] * per_layer + 50304 * h + g["seq"] * h + 2 * h == g["params"]
    # the stage layout with an LM head reproduces layers + embedding + final LN
    assert OS.n_params(OS.param_layout(g["layers"], h, 4 * h, True, 50304)) + g["seq"] * h == g["params"]
    # BERT: layers + embeddings (vocab 29056, 512 positions, 2 token types) + embedding LN
    #       + pooler + LM-head transform (dense + LN + vocab bias) + 2-way sentence head
    b = facts["bert"]
    bert = (b["layers"] * per_layer + 29056 * h + 512 * h + 2 * h + (h * h + h)
            + (h * h + h) + 2 * h + 29056 + (2 * h + 2) + 2 * h)
    assert bert == b["params"]


# ------------------------------------------------ first stage: input embedding
def _embed_setup(bert=False):
    w = W.TINY["embed"]
    if bert:
        w = w.with_(block_kind=W.configs.BERT_POSTLN_BIDIR)
    st = Stage.from_workload(w)
    theta = W.make_theta(w, st.layout).astype(np.float64)
    tokens = W.make_tokens(w, 0)
    aux = np.concatenate([tokens, np.array([5, 8], dtype=np.int32)]) if bert else tokens
    dy = W.make_dy(w, 0).astype(np.float64) * 1e3
    return w, st, theta, tokens, aux, dy


@pytest.mark.parametrize("bert", [False, True])
def test_embedding_stage_matches_autograd(bert):
    """Token + learned position embedding in front of the blocks, against
    torch.nn.functional.embedding feeding the independent torch model."""
    w, st, theta, tokens, aux, dy = _embed_setup(bert)
    assert [n for n, *_ in st.layout[:2]] == ["tok_embed", "pos_embed"]
    out, saved = st.forward(theta, None, aux)
    dx, g = st.backward(theta, saved, dy)
    V, D, s, b = w.vocab, w.d_model, w.seq_len, w.microbatch
    tt = torch.tensor(theta, dtype=F64, requires_grad=True)
    E, P = tt[: V * D].view(V, D), tt[V * D: V * D + s * D].view(s, D)
    x = TF.embedding(torch.as_tensor(tokens, dtype=torch.long), E) + P.repeat(b, 1)
    body = w.with_(has_embedding=False)
    ref = torch_stage(body, tt[V * D + s * D:], x, aux[len(tokens):] if bert else None)
    assert np.allclose(out, ref.detach().numpy(), rtol=1e-11, atol=1e-12)
    ref.backward(torch.tensor(dy, dtype=F64))
    assert np.allclose(g, tt.grad.numpy(), rtol=1e-9, atol=1e-12)


def test_embedding_gradient_structure():
    """Rows of tokens that do not occur get exactly zero; a token that occurs k
    times gets the sum of k rows of the input gradient; the position gradient
    is the sum over the sequences of the minibatch."""
    w, st, theta, tokens, aux, dy = _embed_setup()
    _, saved = st.forward(theta, None, aux)
    _, g = st.backward(theta, saved, dy)
    V, D, s, b = w.vocab, w.d_model, w.seq_len, w.microbatch
    gE, gP = g[: V * D].reshape(V, D), g[V * D: V * D + s * D].reshape(s, D)
    counts = np.bincount(tokens, minlength=V)
    assert counts.max() >= 2 and counts.min() == 0          # the case has repeats and absentees
    assert np.all(gE[counts == 0] == 0.0)
    # the gradient that reaches the block input, recovered from a body-only stage
    body = Stage.from_workload(w.with_(has_embedding=False))
    x = theta[: V * D].reshape(V, D)[tokens] + np.tile(theta[V * D: V * D + s * D].reshape(s, D), (b, 1))
    _, sv = body.forward(theta[V * D + s * D:], x)
    dx, gb = body.backward(theta[V * D + s * D:], sv, dy)
    assert np.array_equal(g[V * D + s * D:], gb)
    for t in np.flatnonzero(counts):
        assert np.allclose(gE[t], dx[tokens == t].sum(axis=0), rtol=1e-12, atol=1e-14)
    assert np.allclose(gP, dx.reshape(b, s, D).sum(axis=0), rtol=1e-12, atol=1e-14)


def test_embedding_finite_differences():
    w, st, theta, tokens, aux, dy = _embed_setup()
    _, saved = st.forward(theta, None, aux)
    _, g = st.backward(theta, saved, dy)
    scalar = lambda th: float((st.forward(th, None, aux)[0] * dy).sum())
    rng = np.random.default_rng(11)
    n_emb = (w.vocab + w.seq_len) * w.d_model
    for j in rng.choice(n_emb, size=40, replace=False):
        tp, tm = theta.copy(), theta.copy()
        tp[j] += 1e-5
        tm[j] -= 1e-5
        fd = (scalar(tp) - scalar(tm)) / 2e-5
        assert abs(fd - g[j]) <= 1e-6 * max(1.0, abs(fd)) + 1e-9, (j, fd, g[j])
