"""Plain numpy definition of one pipeline stage (test infrastructure only).

What is computed.  The paper balances the time t_i^j that stage i of data
parallel group j needs for the forward and the backward pass of its layers
(Section III-A, Eq. 1), over K micro-batches whose gradients are accumulated
before one synchronisation.  The layers themselves are the standard pre-norm
decoder layers of the models it trains (GPT-3, LLaMA; Section V); its third
model, BERT-Large, is read as the same pre-norm block with bidirectional
attention (every position attends to every position of its sequence).  Tensor
parallelism cuts the first matrix of each two-matrix block by columns and the
second by rows (Section II-B); one shard's stage is then a network with
heads/TP heads and FFN/TP hidden units on a residual stream of full width
whose outputs are the partial sums that the tensor-parallel all-reduce would
add up.

Conventions.  Row-major matrices, rows ordered batch-major (row = b*S + s).
Linear layers are y = x @ W + b with W[in, out].  Wqkv columns are
[Q | K | V], each block head-major.  All arithmetic runs in the dtype of the
inputs (float64 for the pins, float32 or float64 for parity).  Nothing here is
blocked, fused or reordered; matrix products use numpy's matmul.
"""
from dataclasses import dataclass
import numpy as np

__all__ = [
    "StageCfg", "layer_norm_fwd", "layer_norm_bwd", "rms_norm_fwd", "rms_norm_bwd",
    "gelu_tanh", "gelu_tanh_grad", "silu", "silu_grad", "rope_tables", "rope_apply",
    "attention_fwd", "attention_bwd", "attention_probs", "layer_fwd", "layer_bwd",
    "stage_fwd", "stage_bwd", "zero_grads_like", "param_names",
    "attn_block_partial", "mlp_block_partial", "shard_layer_params", "stage_loss",
]


@dataclass
class StageCfg:
    arch: str            # "gpt" (LayerNorm, biases, tanh-GeLU), "llama" (RMSNorm, RoPE, SwiGLU, no biases)
                         # or "bert" (the "gpt" block with bidirectional instead of causal attention)
    n_layers: int        # l_i of the layer-partition problem (Section III-C, Eq. 4)
    hidden: int          # h
    n_heads_local: int   # heads / TP
    head_dim: int        # d
    ffn_local: int       # FFN / TP
    seq_len: int         # S
    norm_eps: float = 1e-5
    rope_base: float = 10000.0

    @property
    def h_loc(self):
        return self.n_heads_local * self.head_dim

    @property
    def causal(self):
        return self.arch != "bert"

    @property
    def gpt_block(self):
        return self.arch in ("gpt", "bert")


GPT_PARAMS = ["ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo", "ln2_g", "ln2_b", "w1", "b1", "w2", "b2"]
LLAMA_PARAMS = ["ln1_g", "wqkv", "wo", "ln2_g", "wgu", "wd"]


def param_names(arch):
    return list(GPT_PARAMS if arch in ("gpt", "bert") else LLAMA_PARAMS)


# --------------------------------------------------------------------------
# normalisation
# --------------------------------------------------------------------------
def layer_norm_fwd(x, gamma, beta, eps):
    """a = gamma * (x - mean) / sqrt(var + eps) + beta, biased variance, per row."""
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + x.dtype.type(eps))
    xhat = (x - mu) * rstd
    return gamma * xhat + beta, xhat, rstd


def layer_norm_bwd(da, xhat, rstd, gamma):
    """Returns dx, dgamma, dbeta for a = gamma * xhat + beta."""
    dgamma = (da * xhat).sum(axis=0)
    dbeta = da.sum(axis=0)
    w = da * gamma
    dx = rstd * (w - w.mean(axis=-1, keepdims=True) - xhat * (w * xhat).mean(axis=-1, keepdims=True))
    return dx, dgamma, dbeta


def rms_norm_fwd(x, gamma, eps):
    """a = gamma * x / sqrt(mean(x^2) + eps), per row."""
    r = 1.0 / np.sqrt((x * x).mean(axis=-1, keepdims=True) + x.dtype.type(eps))
    xhat = x * r
    return gamma * xhat, xhat, r


def rms_norm_bwd(da, xhat, r, gamma):
    dgamma = (da * xhat).sum(axis=0)
    w = da * gamma
    dx = r * (w - xhat * (w * xhat).mean(axis=-1, keepdims=True))
    return dx, dgamma


# --------------------------------------------------------------------------
# activations
# --------------------------------------------------------------------------
_KAPPA = 0.7978845608028654  # sqrt(2/pi)


def gelu_tanh(u):
    t = np.tanh(u.dtype.type(_KAPPA) * (u + u.dtype.type(0.044715) * u ** 3))
    return u.dtype.type(0.5) * u * (1 + t)


def gelu_tanh_grad(u):
    k = u.dtype.type(_KAPPA)
    t = np.tanh(k * (u + u.dtype.type(0.044715) * u ** 3))
    return u.dtype.type(0.5) * (1 + t) + u.dtype.type(0.5) * u * (1 - t * t) * k * (1 + u.dtype.type(3 * 0.044715) * u * u)


def _sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


def silu(x):
    return x * _sigmoid(x)


def silu_grad(x):
    s = _sigmoid(x)
    return s * (1 + x * (1 - s))


# --------------------------------------------------------------------------
# rotary position embedding: pairs (i, i + d/2), angle = position * base^(-2i/d)
# --------------------------------------------------------------------------
def rope_tables(seq_len, head_dim, base, dtype):
    i = np.arange(head_dim // 2, dtype=np.float64)
    theta = np.exp(-(2.0 * i / head_dim) * np.log(float(base)))
    ang = np.arange(seq_len, dtype=np.float64)[:, None] * theta[None, :]
    return np.cos(ang).astype(dtype), np.sin(ang).astype(dtype)


def rope_apply(t, cos, sin, sign=1.0):
    """t[..., S, d]; rotates each pair (i, i+d/2) by +angle (sign=1) or -angle (sign=-1)."""
    half = t.shape[-1] // 2
    a, b = t[..., :half], t[..., half:]
    s = sin * t.dtype.type(sign)
    return np.concatenate([a * cos - b * s, b * cos + a * s], axis=-1)


# --------------------------------------------------------------------------
# self-attention, one (batch, head) at a time; causal: query i sees keys k <= i
# --------------------------------------------------------------------------
def attention_probs(q, k, causal=True):
    """softmax(q k^T / sqrt(d)) for one head, over the allowed keys.  q, k: [S, d] -> P[S, S]."""
    S, d = q.shape
    s = (q @ k.T) * q.dtype.type(1.0 / np.sqrt(d))
    if causal:
        allowed = np.tril(np.ones((S, S), dtype=bool))
        s = np.where(allowed, s, -np.inf)
    m = s.max(axis=-1, keepdims=True)
    e = np.exp(s - m)            # masked entries are exp(-inf) = 0 exactly
    return e / e.sum(axis=-1, keepdims=True)


# The (batch, head) pairs are independent.  HEAD_THREADS > 1 hands them to that many threads (same arithmetic per
# head, numpy releases the interpreter lock inside its loops); the full-size parity tests set it, nothing else does.
HEAD_THREADS = 1


def _for_each_head(fn, B, nh):
    pairs = [(b, j) for b in range(B) for j in range(nh)]
    if HEAD_THREADS <= 1:
        for b, j in pairs:
            fn(b, j)
    else:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=HEAD_THREADS) as ex:
            list(ex.map(lambda bj: fn(*bj), pairs))


def attention_fwd(q, k, v, causal=True):
    """q, k, v: [B, nh, S, d] -> o same shape."""
    o = np.empty_like(q)

    def head(b, j):
        o[b, j] = attention_probs(q[b, j], k[b, j], causal) @ v[b, j]

    _for_each_head(head, q.shape[0], q.shape[1])
    return o


def attention_bwd(q, k, v, do, causal=True):
    dq, dk, dv = np.empty_like(q), np.empty_like(k), np.empty_like(v)
    scale = q.dtype.type(1.0 / np.sqrt(q.shape[-1]))

    def head(b, j):
        p = attention_probs(q[b, j], k[b, j], causal)
        dv[b, j] = p.T @ do[b, j]
        dp = do[b, j] @ v[b, j].T
        delta = (p * dp).sum(axis=-1, keepdims=True)
        ds = p * (dp - delta)
        dq[b, j] = (ds @ k[b, j]) * scale
        dk[b, j] = (ds.T @ q[b, j]) * scale

    _for_each_head(head, q.shape[0], q.shape[1])
    return dq, dk, dv


# --------------------------------------------------------------------------
# one decoder layer
# --------------------------------------------------------------------------
def _split_heads(t, B, S, nh, d):
    return t.reshape(B, S, nh, d).transpose(0, 2, 1, 3)


def _merge_heads(t):
    B, nh, S, d = t.shape
    return t.transpose(0, 2, 1, 3).reshape(B * S, nh * d)


def layer_fwd(cfg, p, x):
    """x[T, h] -> (y[T, h], cache).  T = B * S."""
    T = x.shape[0]
    S, nh, d, hl = cfg.seq_len, cfg.n_heads_local, cfg.head_dim, cfg.h_loc
    B = T // S
    c = {"x": x}
    if cfg.gpt_block:
        a, c["xhat1"], c["rstd1"] = layer_norm_fwd(x, p["ln1_g"], p["ln1_b"], cfg.norm_eps)
        qkv = a @ p["wqkv"] + p["bqkv"]
    else:
        a, c["xhat1"], c["rstd1"] = rms_norm_fwd(x, p["ln1_g"], cfg.norm_eps)
        qkv = a @ p["wqkv"]
    c["a"] = a
    q = _split_heads(qkv[:, :hl], B, S, nh, d)
    k = _split_heads(qkv[:, hl:2 * hl], B, S, nh, d)
    v = _split_heads(qkv[:, 2 * hl:], B, S, nh, d)
    if cfg.arch == "llama":
        cos, sin = rope_tables(S, d, cfg.rope_base, x.dtype)
        q, k = rope_apply(q, cos, sin), rope_apply(k, cos, sin)
    c["q"], c["k"], c["v"] = q, k, v
    o = _merge_heads(attention_fwd(q, k, v, cfg.causal))
    c["o"] = o
    if cfg.gpt_block:
        x_mid = x + o @ p["wo"] + p["bo"]
        cc, c["xhat2"], c["rstd2"] = layer_norm_fwd(x_mid, p["ln2_g"], p["ln2_b"], cfg.norm_eps)
        u = cc @ p["w1"] + p["b1"]
        g = gelu_tanh(u)
        y = x_mid + g @ p["w2"] + p["b2"]
        c["u"], c["g"] = u, g
    else:
        x_mid = x + o @ p["wo"]
        cc, c["xhat2"], c["rstd2"] = rms_norm_fwd(x_mid, p["ln2_g"], cfg.norm_eps)
        gu = cc @ p["wgu"]
        F = cfg.ffn_local
        ug, uu = gu[:, :F], gu[:, F:]
        m = silu(ug) * uu
        y = x_mid + m @ p["wd"]
        c["ug"], c["uu"], c["m"] = ug, uu, m
    c["x_mid"], c["c"] = x_mid, cc
    return y, c


def layer_bwd(cfg, p, c, dy, g):
    """Adds this layer's parameter gradients into g (dict of arrays); returns dx."""
    T = dy.shape[0]
    S, nh, d, hl = cfg.seq_len, cfg.n_heads_local, cfg.head_dim, cfg.h_loc
    B = T // S
    if cfg.gpt_block:
        g["w2"] += c["g"].T @ dy
        g["b2"] += dy.sum(axis=0)
        dg = dy @ p["w2"].T
        du = dg * gelu_tanh_grad(c["u"])
        g["w1"] += c["c"].T @ du
        g["b1"] += du.sum(axis=0)
        dc = du @ p["w1"].T
        dx_ln, dgam, dbet = layer_norm_bwd(dc, c["xhat2"], c["rstd2"], p["ln2_g"])
        g["ln2_g"] += dgam
        g["ln2_b"] += dbet
    else:
        g["wd"] += c["m"].T @ dy
        dm = dy @ p["wd"].T
        dug = dm * c["uu"] * silu_grad(c["ug"])
        duu = dm * silu(c["ug"])
        dgu = np.concatenate([dug, duu], axis=1)
        g["wgu"] += c["c"].T @ dgu
        dc = dgu @ p["wgu"].T
        dx_ln, dgam = rms_norm_bwd(dc, c["xhat2"], c["rstd2"], p["ln2_g"])
        g["ln2_g"] += dgam
    dx_mid = dy + dx_ln
    g["wo"] += c["o"].T @ dx_mid
    if cfg.gpt_block:
        g["bo"] += dx_mid.sum(axis=0)
    do = _split_heads(dx_mid @ p["wo"].T, B, S, nh, d)
    dq, dk, dv = attention_bwd(c["q"], c["k"], c["v"], do, cfg.causal)
    if cfg.arch == "llama":
        cos, sin = rope_tables(S, d, cfg.rope_base, dy.dtype)
        dq, dk = rope_apply(dq, cos, sin, -1.0), rope_apply(dk, cos, sin, -1.0)
    dqkv = np.concatenate([_merge_heads(dq), _merge_heads(dk), _merge_heads(dv)], axis=1)
    g["wqkv"] += c["a"].T @ dqkv
    da = dqkv @ p["wqkv"].T
    if cfg.gpt_block:
        g["bqkv"] += dqkv.sum(axis=0)
        dx_ln1, dgam, dbet = layer_norm_bwd(da, c["xhat1"], c["rstd1"], p["ln1_g"])
        g["ln1_b"] += dbet
    else:
        dx_ln1, dgam = rms_norm_bwd(da, c["xhat1"], c["rstd1"], p["ln1_g"])
    g["ln1_g"] += dgam
    return dx_mid + dx_ln1


# --------------------------------------------------------------------------
# the stage: L layers chained; gradients summed over micro-batches (no 1/K)
# --------------------------------------------------------------------------
def zero_grads_like(params):
    return [{k: np.zeros_like(v) for k, v in layer.items()} for layer in params]


def stage_fwd(cfg, params, x):
    """x[T, h] -> (y[T, h], caches, per-layer outputs)."""
    caches, outs = [], []
    for p in params:
        x, c = layer_fwd(cfg, p, x)
        caches.append(c)
        outs.append(x)
    return x, caches, outs


def stage_bwd(cfg, params, caches, dy, grads):
    """dy[T, h] -> dx[T, h]; adds parameter gradients into grads."""
    for p, c, g in zip(reversed(params), reversed(caches), reversed(grads)):
        dy = layer_bwd(cfg, p, c, dy, g)
    return dy


def stage_loss(cfg, params, xs, dys):
    """The scalar whose gradient stage_bwd returns: sum over micro-batches of <dY, Y>."""
    return sum(float((stage_fwd(cfg, params, x)[0].astype(np.float64) * dy).sum()) for x, dy in zip(xs, dys))


# --------------------------------------------------------------------------
# tensor-parallel partial sums (Section II-B: first matrix cut by columns,
# second by rows; rank r owns the r-th contiguous block)
# --------------------------------------------------------------------------
def shard_layer_params(arch, p, tp, r, n_heads, head_dim, ffn):
    """Rank r's shard of one unsharded layer's parameters."""
    hd = n_heads * head_dim
    hl = hd // tp
    Fl = ffn // tp
    cols = np.concatenate([np.arange(b * hd + r * hl, b * hd + (r + 1) * hl) for b in range(3)])
    out = {}
    for k, v in p.items():
        if k == "wqkv":
            out[k] = v[:, cols]
        elif k == "bqkv":
            out[k] = v[cols]
        elif k == "wo":
            out[k] = v[r * hl:(r + 1) * hl, :]
        elif k == "w1":
            out[k] = v[:, r * Fl:(r + 1) * Fl]
        elif k == "b1":
            out[k] = v[r * Fl:(r + 1) * Fl]
        elif k == "wgu":
            out[k] = np.concatenate([v[:, r * Fl:(r + 1) * Fl], v[:, ffn + r * Fl: ffn + (r + 1) * Fl]], axis=1)
        elif k in ("w2", "wd"):
            out[k] = v[r * Fl:(r + 1) * Fl, :]
        else:
            out[k] = v          # norms and post-reduce biases are replicated
    return out


def attn_block_partial(cfg_local, p_shard, x):
    """o_r @ Wo_r for one shard: the addend of the attention block's all-reduce."""
    _, c = layer_fwd(cfg_local, p_shard, x)
    return c["o"] @ p_shard["wo"]


def mlp_block_partial(cfg_local, p_shard, x_mid):
    """g_r @ W2_r (or m_r @ Wd_r) for one shard, from the block's input x_mid."""
    if cfg_local.gpt_block:
        cc, _, _ = layer_norm_fwd(x_mid, p_shard["ln2_g"], p_shard["ln2_b"], cfg_local.norm_eps)
        return gelu_tanh(cc @ p_shard["w1"] + p_shard["b1"]) @ p_shard["w2"]
    cc, _, _ = rms_norm_fwd(x_mid, p_shard["ln2_g"], cfg_local.norm_eps)
    gu = cc @ p_shard["wgu"]
    F = cfg_local.ffn_local
    return (silu(gu[:, :F]) * gu[:, F:]) @ p_shard["wd"]
