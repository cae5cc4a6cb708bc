"""Oracle: forward and backward of one pipeline stage (a slice of transformer
blocks, optionally closed by the language-model head and its loss).

TEST INFRASTRUCTURE ONLY (see the package docstring).

The paper trains Megatron-style GPT and BERT models (Section 4.1, Table 2);
it does not print the block equations, so the textbook definitions are written
out here. The per-layer parameter set -- two LayerNorms, a fused QKV
projection, an output projection and a two-matrix GELU MLP, all with biases,
12 h^2 + 13 h numbers per layer -- is the one that reproduces Table 2's
parameter counts exactly (see tests). Block details the paper is silent on:
exact (erf) GELU, LayerNorm with biased variance and eps 1e-5, masked scores
set to -inf before a softmax scaled by 1/sqrt(head_dim), no dropout.

Versioned backward (Section 3.1 defines the mismatch as updates that happen
between a minibatch's forward and backward): every activation that enters a
backward formula is the value saved by that minibatch's forward; every
parameter that enters (the transposed weights, LayerNorm gains, the tied
embedding) is read from the parameter vector handed to backward, which may be
a different version.

All arrays are float64. Token-major activations: row n = sequence * s + pos.
"""
import numpy as np
from scipy.special import erf

GPT_PRELN_CAUSAL = 0
BERT_POSTLN_BIDIR = 1

_LAYER_FIELDS = ("ln1_gamma", "ln1_beta", "w_qkv", "b_qkv", "w_o", "b_o",
                 "ln2_gamma", "ln2_beta", "w_1", "b_1", "w_2", "b_2")


def param_layout(n_layers, d_model, d_ffn, has_lm_head=False, vocab=0, has_embedding=False, seq_len=0):
    """Flat parameter order: on the first stage the token embedding E [V,D] and
    the learned position embedding [s,D]; per layer gamma1, beta1, W_qkv
    [D,3D], b_qkv, W_o [D,D], b_o, gamma2, beta2, W_1 [D,F], b_1, W_2 [F,D],
    b_2; on the last stage then final gamma, beta and the tied embedding E
    [V,D]. Returns a list of (name, offset, rows, cols)."""
    D, Fd = d_model, d_ffn
    shapes = {"ln1_gamma": (1, D), "ln1_beta": (1, D), "w_qkv": (D, 3 * D), "b_qkv": (1, 3 * D),
              "w_o": (D, D), "b_o": (1, D), "ln2_gamma": (1, D), "ln2_beta": (1, D),
              "w_1": (D, Fd), "b_1": (1, Fd), "w_2": (Fd, D), "b_2": (1, D)}
    out, off = [], 0
    if has_embedding:
        for name, (r, c) in (("tok_embed", (vocab, D)), ("pos_embed", (seq_len, D))):
            out.append((name, off, r, c))
            off += r * c
    for l in range(n_layers):
        for f in _LAYER_FIELDS:
            r, c = shapes[f]
            out.append((f"l{l}.{f}", off, r, c))
            off += r * c
    if has_lm_head:
        for name, (r, c) in (("lnf_gamma", (1, D)), ("lnf_beta", (1, D)), ("embed", (vocab, D))):
            out.append((name, off, r, c))
            off += r * c
    return out


def n_params(layout):
    return max(off + r * c for _, off, r, c in layout)


def unpack(theta, layout):
    """Views of the flat vector, keyed by name; vectors are 1-D."""
    out = {}
    for name, off, r, c in layout:
        v = theta[off:off + r * c]
        out[name] = v if r == 1 else v.reshape(r, c)
    return out


# ---------------------------------------------------------------- primitives

def layernorm_fwd(x, gamma, beta, eps):
    mu = x.mean(axis=1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=1, keepdims=True)      # biased
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    return xhat * gamma + beta, (xhat, rstd)


def layernorm_bwd(dy, saved, gamma):
    xhat, rstd = saved
    dgamma = (dy * xhat).sum(axis=0)
    dbeta = dy.sum(axis=0)
    dxhat = dy * gamma
    dx = rstd * (dxhat - dxhat.mean(axis=1, keepdims=True)
                 - xhat * (dxhat * xhat).mean(axis=1, keepdims=True))
    return dx, dgamma, dbeta


def gelu(u):
    return 0.5 * u * (1.0 + erf(u / np.sqrt(2.0)))


def gelu_grad(u):
    return 0.5 * (1.0 + erf(u / np.sqrt(2.0))) + u * np.exp(-0.5 * u * u) / np.sqrt(2.0 * np.pi)


def _mask(kind, s, valid):
    """Boolean [s, s]: True where the key (column) is hidden from the query (row)."""
    q = np.arange(s)[:, None]
    k = np.arange(s)[None, :]
    if kind == GPT_PRELN_CAUSAL:
        return k > q
    return np.broadcast_to(k >= valid, (s, s))


def attention_fwd(qkv, kind, n_heads, seq_len, valid_len):
    """qkv [N, 3D] with column blocks Q | K | V, each split into heads of
    dh contiguous columns. Returns O [N, D] and the saved probabilities."""
    N, D3 = qkv.shape
    D = D3 // 3
    dh = D // n_heads
    b = N // seq_len
    out = np.zeros((N, D))
    probs = {}
    for seq in range(b):
        rows = slice(seq * seq_len, (seq + 1) * seq_len)
        hidden = _mask(kind, seq_len, None if valid_len is None else int(valid_len[seq]))
        for h in range(n_heads):
            q = qkv[rows, h * dh:(h + 1) * dh]
            k = qkv[rows, D + h * dh:D + (h + 1) * dh]
            v = qkv[rows, 2 * D + h * dh:2 * D + (h + 1) * dh]
            sc = (q @ k.T) / np.sqrt(dh)
            sc = np.where(hidden, -np.inf, sc)
            sc = sc - sc.max(axis=1, keepdims=True)
            e = np.exp(sc)
            p = e / e.sum(axis=1, keepdims=True)
            probs[(seq, h)] = p
            out[rows, h * dh:(h + 1) * dh] = p @ v
    return out, probs


def attention_bwd(d_out, qkv, probs, n_heads, seq_len):
    N, D3 = qkv.shape
    D = D3 // 3
    dh = D // n_heads
    b = N // seq_len
    dqkv = np.zeros_like(qkv)
    for seq in range(b):
        rows = slice(seq * seq_len, (seq + 1) * seq_len)
        for h in range(n_heads):
            cq = slice(h * dh, (h + 1) * dh)
            ck = slice(D + h * dh, D + (h + 1) * dh)
            cv = slice(2 * D + h * dh, 2 * D + (h + 1) * dh)
            q, k, v = qkv[rows, cq], qkv[rows, ck], qkv[rows, cv]
            p = probs[(seq, h)]
            do = d_out[rows, cq]
            dv = p.T @ do
            dp = do @ v.T
            ds = p * (dp - (dp * p).sum(axis=1, keepdims=True))
            ds = ds / np.sqrt(dh)
            dqkv[rows, cq] = ds @ k
            dqkv[rows, ck] = ds.T @ q
            dqkv[rows, cv] = dv
    return dqkv


# -------------------------------------------------------------------- blocks

def _mlp_fwd(c, p, l):
    u = c @ p[f"l{l}.w_1"] + p[f"l{l}.b_1"]
    h = gelu(u)
    return h @ p[f"l{l}.w_2"] + p[f"l{l}.b_2"], (c, u, h)


def _mlp_bwd(dout, saved, p, l, g):
    c, u, h = saved
    g[f"l{l}.w_2"] = h.T @ dout
    g[f"l{l}.b_2"] = dout.sum(axis=0)
    dh_ = dout @ p[f"l{l}.w_2"].T
    du = dh_ * gelu_grad(u)
    g[f"l{l}.w_1"] = c.T @ du
    g[f"l{l}.b_1"] = du.sum(axis=0)
    return du @ p[f"l{l}.w_1"].T


def _attn_fwd(a, p, l, kind, H, s, valid):
    qkv = a @ p[f"l{l}.w_qkv"] + p[f"l{l}.b_qkv"]
    o, probs = attention_fwd(qkv, kind, H, s, valid)
    return o @ p[f"l{l}.w_o"] + p[f"l{l}.b_o"], (a, qkv, probs, o)


def _attn_bwd(dout, saved, p, l, H, s, g):
    a, qkv, probs, o = saved
    g[f"l{l}.w_o"] = o.T @ dout
    g[f"l{l}.b_o"] = dout.sum(axis=0)
    do = dout @ p[f"l{l}.w_o"].T
    dqkv = attention_bwd(do, qkv, probs, H, s)
    g[f"l{l}.w_qkv"] = a.T @ dqkv
    g[f"l{l}.b_qkv"] = dqkv.sum(axis=0)
    return dqkv @ p[f"l{l}.w_qkv"].T


def block_fwd(x, p, l, kind, H, s, valid, eps):
    if kind == GPT_PRELN_CAUSAL:
        a, ln1 = layernorm_fwd(x, p[f"l{l}.ln1_gamma"], p[f"l{l}.ln1_beta"], eps)
        att, sa = _attn_fwd(a, p, l, kind, H, s, valid)
        y1 = x + att
        c, ln2 = layernorm_fwd(y1, p[f"l{l}.ln2_gamma"], p[f"l{l}.ln2_beta"], eps)
        mlp, sm = _mlp_fwd(c, p, l)
        return y1 + mlp, (ln1, sa, ln2, sm)
    att, sa = _attn_fwd(x, p, l, kind, H, s, valid)
    y1, ln1 = layernorm_fwd(x + att, p[f"l{l}.ln1_gamma"], p[f"l{l}.ln1_beta"], eps)
    mlp, sm = _mlp_fwd(y1, p, l)
    y, ln2 = layernorm_fwd(y1 + mlp, p[f"l{l}.ln2_gamma"], p[f"l{l}.ln2_beta"], eps)
    return y, (ln1, sa, ln2, sm)


def block_bwd(dy, saved, p, l, kind, H, s, g):
    ln1, sa, ln2, sm = saved
    if kind == GPT_PRELN_CAUSAL:
        dc = _mlp_bwd(dy, sm, p, l, g)
        d2, g[f"l{l}.ln2_gamma"], g[f"l{l}.ln2_beta"] = layernorm_bwd(dc, ln2, p[f"l{l}.ln2_gamma"])
        dy1 = dy + d2
        da = _attn_bwd(dy1, sa, p, l, H, s, g)
        d1, g[f"l{l}.ln1_gamma"], g[f"l{l}.ln1_beta"] = layernorm_bwd(da, ln1, p[f"l{l}.ln1_gamma"])
        return dy1 + d1
    dr2, g[f"l{l}.ln2_gamma"], g[f"l{l}.ln2_beta"] = layernorm_bwd(dy, ln2, p[f"l{l}.ln2_gamma"])
    dy1 = dr2 + _mlp_bwd(dr2, sm, p, l, g)
    dr1, g[f"l{l}.ln1_gamma"], g[f"l{l}.ln1_beta"] = layernorm_bwd(dy1, ln1, p[f"l{l}.ln1_gamma"])
    return dr1 + _attn_bwd(dr1, sa, p, l, H, s, g)


# --------------------------------------------------------------------- stage

class Stage:
    """Shape record plus forward/backward over a flat parameter vector."""

    def __init__(self, block_kind, n_layers, d_model, n_heads, d_ffn, seq_len, microbatch,
                 has_lm_head=False, vocab=0, ln_eps=1e-5, has_embedding=False):
        self.kind, self.L, self.D, self.H, self.Fd = block_kind, n_layers, d_model, n_heads, d_ffn
        self.s, self.b = seq_len, microbatch
        self.has_lm_head, self.V, self.eps = bool(has_lm_head), vocab, ln_eps
        self.has_embedding = bool(has_embedding)
        if self.has_embedding and self.has_lm_head:
            raise ValueError("a stage holds the input embedding or the output head, not both")
        self.layout = param_layout(n_layers, d_model, d_ffn, has_lm_head, vocab, has_embedding, seq_len)
        self.n_params = n_params(self.layout)

    @classmethod
    def from_workload(cls, w):
        return cls(w.block_kind, w.n_layers, w.d_model, w.n_heads, w.d_ffn, w.seq_len,
                   w.microbatch, w.has_lm_head, w.vocab, w.ln_eps, getattr(w, "has_embedding", False))

    def forward(self, theta, x, aux=None):
        """Returns (Y or scalar loss, saved). `aux` is valid_len[b] for the
        bidirectional block, targets[N] on the LM-head stage. On the first
        stage (input embedding) x is ignored and aux holds the token ids [N],
        followed by valid_len[b] for the bidirectional block: the block input
        is the token's embedding row plus the learned embedding of its
        position (the model family's input layer, Section 4.1)."""
        p = unpack(np.asarray(theta, dtype=np.float64), self.layout)
        tokens = None
        if self.has_embedding:
            N = self.s * self.b
            aux = np.asarray(aux)
            tokens = aux[:N].astype(np.int64)
            aux = aux[N:] if self.kind == BERT_POSTLN_BIDIR else None
            h = p["tok_embed"][tokens] + np.tile(p["pos_embed"], (self.b, 1))
        else:
            h = np.asarray(x, dtype=np.float64)
        valid = aux if (self.kind == BERT_POSTLN_BIDIR and not self.has_lm_head) else None
        saved = []
        for l in range(self.L):
            h, sv = block_fwd(h, p, l, self.kind, self.H, self.s, valid, self.eps)
            saved.append(sv)
        if not self.has_lm_head:
            return h, (saved, tokens)
        z, lnf = layernorm_fwd(h, p["lnf_gamma"], p["lnf_beta"], self.eps)
        logits = z @ p["embed"].T
        mx = logits.max(axis=1, keepdims=True)
        lse = mx[:, 0] + np.log(np.exp(logits - mx).sum(axis=1))
        t = np.asarray(aux, dtype=np.int64)
        n = np.arange(logits.shape[0])
        loss = (lse - logits[n, t]).mean()
        sm = np.exp(logits - lse[:, None])
        return loss, (saved, (lnf, z, sm, t))

    def backward(self, theta, saved, dy=None):
        """Returns (dX, flat gradient). On the LM-head stage dy is ignored and
        the seed is d loss = 1."""
        p = unpack(np.asarray(theta, dtype=np.float64), self.layout)
        g = {}
        blocks, head = saved
        if self.has_lm_head:
            lnf, z, sm, t = head
            N = z.shape[0]
            dlogits = sm.copy()
            dlogits[np.arange(N), t] -= 1.0
            dlogits /= N
            g["embed"] = dlogits.T @ z
            dz = dlogits @ p["embed"]
            d, g["lnf_gamma"], g["lnf_beta"] = layernorm_bwd(dz, lnf, p["lnf_gamma"])
        else:
            d = np.asarray(dy, dtype=np.float64)
        for l in reversed(range(self.L)):
            d = block_bwd(d, blocks[l], p, l, self.kind, self.H, self.s, g)
        if self.has_embedding:
            tokens = head
            g["tok_embed"] = np.zeros((self.V, self.D))
            np.add.at(g["tok_embed"], tokens, d)                 # rows of repeated tokens add up
            g["pos_embed"] = d.reshape(self.b, self.s, self.D).sum(axis=0)
        flat = np.zeros(self.n_params)
        for name, off, r, c in self.layout:
            flat[off:off + r * c] = np.asarray(g[name]).reshape(-1)
        return d, flat
