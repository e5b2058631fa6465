"""Pins of the CPU oracle against things other than itself (CPU only).

Each test is chosen so that a plausible slip in oracle/stage_ref.py (a dropped
term, a wrong sign or index, a transposed operand) makes it fail.
"""
import os

import numpy as np
import pytest
import torch

from oracle import stage_ref as R
from synth import stage_inputs as SI

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def tiny_cfg(arch, L=2, S=6):
    return R.StageCfg(arch, L, 16, 2, 8, 32, S, 1e-6 if arch == "llama" else 1e-5, 10000.0)


def rand_params(cfg, rng, dtype=np.float64, wstd=0.3):
    h, hl, F = cfg.hidden, cfg.h_loc, cfg.ffn_local
    shapes = {"ln1_g": (h,), "ln1_b": (h,), "wqkv": (h, 3 * hl), "bqkv": (3 * hl,), "wo": (hl, h), "bo": (h,),
              "ln2_g": (h,), "ln2_b": (h,), "w1": (h, F), "b1": (F,), "w2": (F, h), "b2": (h,),
              "wgu": (h, 2 * F), "wd": (F, h)}
    out = []
    for _ in range(cfg.n_layers):
        p = {}
        for n in R.param_names(cfg.arch):
            t = rng.standard_normal(shapes[n]) * wstd
            if n.endswith("_g"):
                t = 1.0 + 0.2 * t
            p[n] = t.astype(dtype)
        out.append(p)
    return out


def run_stage(cfg, params, xs, dys):
    grads = R.zero_grads_like(params)
    ys, dxs = [], []
    for x, dy in zip(xs, dys):
        y, caches, _ = R.stage_fwd(cfg, params, x)
        dxs.append(R.stage_bwd(cfg, params, caches, dy, grads))
        ys.append(y)
    return ys, dxs, grads


# ---------------------------------------------------------------- finite differences
@pytest.mark.parametrize("arch", ["gpt", "llama", "bert"])
def test_backward_matches_central_differences(arch):
    rng = np.random.default_rng(1)
    cfg = tiny_cfg(arch)
    B, K = 2, 2
    params = rand_params(cfg, rng)
    xs = [rng.standard_normal((B * cfg.seq_len, cfg.hidden)) for _ in range(K)]
    dys = [rng.standard_normal((B * cfg.seq_len, cfg.hidden)) for _ in range(K)]
    _, dxs, grads = run_stage(cfg, params, xs, dys)
    eps = 1e-5

    def fd(arr, idx):
        old = arr[idx]
        arr[idx] = old + eps
        lp = R.stage_loss(cfg, params, xs, dys)
        arr[idx] = old - eps
        lm = R.stage_loss(cfg, params, xs, dys)
        arr[idx] = old
        return (lp - lm) / (2 * eps)

    for l in range(cfg.n_layers):
        for name, arr in params[l].items():
            flat = arr.reshape(-1)
            gflat = grads[l][name].reshape(-1)
            for i in rng.choice(flat.size, size=min(6, flat.size), replace=False):
                num = fd(flat, i)
                assert abs(num - gflat[i]) <= 1e-6 * max(1.0, abs(num)), (l, name, i, num, gflat[i])
    for m in range(K):
        flat = xs[m].reshape(-1)
        for i in rng.choice(flat.size, size=8, replace=False):
            num = fd(flat, i)
            assert abs(num - dxs[m].reshape(-1)[i]) <= 1e-6 * max(1.0, abs(num))


def test_activation_derivatives_match_differences():
    u = np.linspace(-6, 6, 241)
    e = 1e-6
    assert np.allclose((R.gelu_tanh(u + e) - R.gelu_tanh(u - e)) / (2 * e), R.gelu_tanh_grad(u), atol=1e-8)
    assert np.allclose((R.silu(u + e) - R.silu(u - e)) / (2 * e), R.silu_grad(u), atol=1e-8)
    # the tanh form stays within 1e-3 of the exact (erf) GeLU, and silu is x*sigmoid(x)
    exact = torch.nn.functional.gelu(torch.from_numpy(u)).numpy()
    assert np.abs(R.gelu_tanh(u) - exact).max() < 1e-3
    assert np.allclose(R.silu(u), torch.nn.functional.silu(torch.from_numpy(u)).numpy(), atol=1e-12)


# ---------------------------------------------------------------- library restatement (autograd)
def torch_layer(arch, p, x, S, nh, d, eps, base):
    F = torch.nn.functional
    T, h = x.shape
    B = T // S
    hl = nh * d
    gpt_block = arch in ("gpt", "bert")
    if gpt_block:
        a = F.layer_norm(x, (h,), p["ln1_g"], p["ln1_b"], eps)
        qkv = torch.addmm(p["bqkv"], a, p["wqkv"])
    else:
        a = x * torch.rsqrt(x.pow(2).mean(-1, keepdim=True) + eps) * p["ln1_g"]
        qkv = a @ p["wqkv"]
    q, k, v = [t.reshape(B, S, nh, d).permute(0, 2, 1, 3) for t in qkv.split(hl, dim=1)]
    if arch == "llama":
        # rotary embedding restated with complex numbers: (a + i b) * exp(i * pos * theta)
        theta = base ** (-torch.arange(0, d, 2, dtype=torch.float64) / d)
        rot = torch.polar(torch.ones(S, d // 2, dtype=torch.float64), torch.outer(torch.arange(S, dtype=torch.float64), theta))

        def rope(t):
            z = torch.complex(t[..., : d // 2], t[..., d // 2:]) * rot
            return torch.cat([z.real, z.imag], dim=-1)
        q, k = rope(q), rope(k)
    o = F.scaled_dot_product_attention(q, k, v, is_causal=(arch != "bert"))
    o = o.permute(0, 2, 1, 3).reshape(T, hl)
    if gpt_block:
        xm = x + o @ p["wo"] + p["bo"]
        c = F.layer_norm(xm, (h,), p["ln2_g"], p["ln2_b"], eps)
        return xm + F.gelu(c @ p["w1"] + p["b1"], approximate="tanh") @ p["w2"] + p["b2"]
    xm = x + o @ p["wo"]
    c = xm * torch.rsqrt(xm.pow(2).mean(-1, keepdim=True) + eps) * p["ln2_g"]
    gate, up = (c @ p["wgu"]).chunk(2, dim=1)
    return xm + (F.silu(gate) * up) @ p["wd"]


@pytest.mark.parametrize("arch", ["gpt", "llama", "bert"])
def test_stage_matches_autograd_restatement(arch):
    rng = np.random.default_rng(2)
    cfg = tiny_cfg(arch, L=3, S=10)
    params = rand_params(cfg, rng)
    B = 2
    x = rng.standard_normal((B * cfg.seq_len, cfg.hidden))
    dy = rng.standard_normal((B * cfg.seq_len, cfg.hidden))
    (y,), (dx,), grads = run_stage(cfg, params, [x], [dy])
    tp = [{k: torch.tensor(v, requires_grad=True) for k, v in p.items()} for p in params]
    tx = torch.tensor(x, requires_grad=True)
    t = tx
    for p in tp:
        t = torch_layer(arch, p, t, cfg.seq_len, cfg.n_heads_local, cfg.head_dim, cfg.norm_eps, cfg.rope_base)
    (t * torch.tensor(dy)).sum().backward()
    assert np.allclose(y, t.detach().numpy(), rtol=1e-9, atol=1e-9)
    assert np.allclose(dx, tx.grad.numpy(), rtol=1e-8, atol=1e-9)
    for l, p in enumerate(tp):
        for k, v in p.items():
            assert np.allclose(grads[l][k], v.grad.numpy(), rtol=1e-8, atol=1e-9), (l, k)


# ---------------------------------------------------------------- softmax / causality
def test_softmax_rows_and_mask():
    rng = np.random.default_rng(3)
    q = rng.standard_normal((33, 8)).astype(np.float32) * 3
    k = rng.standard_normal((33, 8)).astype(np.float32) * 3
    p = R.attention_probs(q, k)
    assert np.abs(p.sum(-1) - 1).max() <= 1e-6
    assert (p >= 0).all()
    assert (p[np.triu_indices(33, 1)] == 0).all()
    assert p[0, 0] == 1.0


def test_bidirectional_probabilities_by_brute_force():
    # every key is allowed: plain loops over a tiny head, and scipy's softmax as a second witness
    from scipy.special import softmax
    rng = np.random.default_rng(31)
    S, d = 7, 4
    q, k = rng.standard_normal((S, d)), rng.standard_normal((S, d))
    p = R.attention_probs(q, k, causal=False)
    for i in range(S):
        w = [np.exp(sum(q[i, c] * k[j, c] for c in range(d)) / np.sqrt(d)) for j in range(S)]
        for j in range(S):
            assert abs(p[i, j] - w[j] / sum(w)) < 1e-14
    assert np.allclose(p, softmax(q @ k.T / 2.0, axis=-1), atol=1e-15)
    assert (p > 0).all()
    # the causal matrix is the same weights renormalised over the allowed prefix
    pc = R.attention_probs(q, k, causal=True)
    low = np.tril(p)
    assert np.allclose(pc, low / low.sum(-1, keepdims=True), atol=1e-14)


def test_bidirectional_stage_sees_the_whole_sequence_and_ignores_its_order():
    rng = np.random.default_rng(32)
    cfg = tiny_cfg("bert", L=2, S=12)
    params = rand_params(cfg, rng)
    B = 2
    x = rng.standard_normal((B, cfg.seq_len, cfg.hidden))
    y = R.stage_fwd(cfg, params, x.reshape(-1, cfg.hidden))[0].reshape(x.shape)
    # no positional signal inside the stage: permuting the tokens of each sequence permutes the outputs
    perm = rng.permutation(cfg.seq_len)
    yp = R.stage_fwd(cfg, params, x[:, perm].reshape(-1, cfg.hidden))[0].reshape(x.shape)
    assert np.allclose(yp, y[:, perm], rtol=1e-11, atol=1e-11)
    # a change at the last position reaches the first one (it would not under the causal mask) ...
    x2 = x.copy()
    x2[:, -1] += rng.standard_normal(cfg.hidden)      # (a constant shift would be removed by the LayerNorm)
    y2 = R.stage_fwd(cfg, params, x2.reshape(-1, cfg.hidden))[0].reshape(x.shape)
    assert np.abs(y2[:, 0] - y[:, 0]).max() > 1e-6
    # ... but never another sequence of the batch
    x3 = x.copy()
    x3[1] += rng.standard_normal(x3[1].shape)
    y3 = R.stage_fwd(cfg, params, x3.reshape(-1, cfg.hidden))[0].reshape(x.shape)
    assert np.array_equal(y3[0], y[0])
    # and the causal stage fails the permutation property (the pin separates the two masks)
    ccfg = tiny_cfg("gpt", L=2, S=12)
    yc = R.stage_fwd(ccfg, params, x.reshape(-1, cfg.hidden))[0].reshape(x.shape)
    ycp = R.stage_fwd(ccfg, params, x[:, perm].reshape(-1, cfg.hidden))[0].reshape(x.shape)
    assert np.abs(ycp - yc[:, perm]).max() > 1e-3


@pytest.mark.parametrize("arch", ["gpt", "llama"])
def test_causality_is_bit_exact(arch):
    rng = np.random.default_rng(4)
    cfg = tiny_cfg(arch, L=2, S=12)
    params = rand_params(cfg, rng, np.float32)
    B, t = 2, 7
    x = rng.standard_normal((B * cfg.seq_len, cfg.hidden)).astype(np.float32)
    x2 = x.copy().reshape(B, cfg.seq_len, -1)
    x2[:, t + 1:] += rng.standard_normal(x2[:, t + 1:].shape).astype(np.float32)
    y1 = R.stage_fwd(cfg, params, x)[0].reshape(B, cfg.seq_len, -1)
    y2 = R.stage_fwd(cfg, params, x2.reshape(x.shape))[0].reshape(B, cfg.seq_len, -1)
    assert np.array_equal(y1[:, : t + 1], y2[:, : t + 1])
    assert not np.array_equal(y1[:, t + 1:], y2[:, t + 1:])


# ---------------------------------------------------------------- accumulation over micro-batches
@pytest.mark.parametrize("arch", ["gpt", "llama", "bert"])
def test_accumulation_equals_concatenated_batch(arch):
    rng = np.random.default_rng(5)
    cfg = tiny_cfg(arch)
    params = rand_params(cfg, rng)
    K, B = 3, 2
    xs = [rng.standard_normal((B * cfg.seq_len, cfg.hidden)) for _ in range(K)]
    dys = [rng.standard_normal((B * cfg.seq_len, cfg.hidden)) for _ in range(K)]
    ys, dxs, g_acc = run_stage(cfg, params, xs, dys)
    (yc,), (dxc,), g_cat = run_stage(cfg, params, [np.concatenate(xs)], [np.concatenate(dys)])
    assert np.allclose(np.concatenate(ys), yc, rtol=1e-12, atol=1e-12)
    assert np.allclose(np.concatenate(dxs), dxc, rtol=1e-12, atol=1e-12)
    for ga, gc in zip(g_acc, g_cat):
        for k in ga:
            assert np.allclose(ga[k], gc[k], rtol=1e-10, atol=1e-11), k


def test_head_threads_change_no_bit():
    rng = np.random.default_rng(61)
    q, k, v, do = (rng.standard_normal((2, 3, 17, 8)) for _ in range(4))
    one = (R.attention_fwd(q, k, v, True),) + R.attention_bwd(q, k, v, do, True)
    R.HEAD_THREADS = 4
    try:
        many = (R.attention_fwd(q, k, v, True),) + R.attention_bwd(q, k, v, do, True)
    finally:
        R.HEAD_THREADS = 1
    assert all(np.array_equal(a, b) for a, b in zip(one, many))


# ---------------------------------------------------------------- tensor-parallel partial sums
@pytest.mark.parametrize("arch", ["gpt", "llama", "bert"])
def test_shard_partials_sum_to_unsharded_block(arch):
    rng = np.random.default_rng(6)
    nh, d, F, h, S, tp = 4, 8, 48, 16, 5, 2
    full = R.StageCfg(arch, 1, h, nh, d, F, S)
    loc = R.StageCfg(arch, 1, h, nh // tp, d, F // tp, S)
    p = rand_params(full, rng)[0]
    x = rng.standard_normal((2 * S, h))
    shards = [R.shard_layer_params(arch, p, tp, r, nh, d, F) for r in range(tp)]
    att = sum(R.attn_block_partial(loc, s, x) for s in shards)
    assert np.allclose(att, R.attn_block_partial(full, p, x), rtol=1e-11, atol=1e-12)
    mlp = sum(R.mlp_block_partial(loc, s, x) for s in shards)
    assert np.allclose(mlp, R.mlp_block_partial(full, p, x), rtol=1e-11, atol=1e-12)
    # the helper against the layer itself (the sum above compares it only with itself): the MLP block's addend is
    # what the layer adds to x_mid, less the bias that is added after the reduce point
    y, cf = R.layer_fwd(full, p, x)
    addend = y - cf["x_mid"] - (p["b2"] if full.gpt_block else 0.0)
    assert np.abs(addend).max() > 1e-3
    assert np.allclose(R.mlp_block_partial(full, p, cf["x_mid"]), addend, rtol=1e-10, atol=1e-12)
    # likewise the attention block's addend: x_mid - x - bo
    assert np.allclose(R.attn_block_partial(full, p, x), cf["x_mid"] - x - (p["bo"] if full.gpt_block else 0.0), rtol=1e-10, atol=1e-12)
    # backward: with the same upstream gradient, each shard's gradient of the row-cut
    # matrix is the matching row block of the unsharded one (gradients are shaped like their shard)
    dy = rng.standard_normal((2 * S, h))
    _, c = R.layer_fwd(full, p, x)
    full_dwo = c["o"].T @ dy
    for r in range(tp):
        _, cs = R.layer_fwd(loc, shards[r], x)
        assert np.allclose(cs["o"].T @ dy, SI.slice_row_parallel(full_dwo, tp, r), rtol=1e-11, atol=1e-12)


def test_shard_slicing_matches_paper_example():
    vals = {}
    for line in open(os.path.join(GOLD, "tp_split_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        vals[k] = np.array(v, dtype=np.float64)
    A = vals["gA"].reshape(2, 2)
    Bm = vals["gB"].reshape(2, 2)
    for r, (ka, kb) in enumerate([("gA1", "gB1"), ("gA2", "gB2")]):
        # the input generator's slicing
        assert np.array_equal(SI.slice_column_parallel(A, 2, r).reshape(-1), vals[ka])
        assert np.array_equal(SI.slice_row_parallel(Bm, 2, r).reshape(-1), vals[kb])
        # the oracle's own slicing (w1 is the column-cut matrix, w2 the row-cut one)
        sh = R.shard_layer_params("gpt", {"w1": A, "w2": Bm}, 2, r, 2, 1, 2)
        assert np.array_equal(sh["w1"].reshape(-1), vals[ka])
        assert np.array_equal(sh["w2"].reshape(-1), vals[kb])


def test_qkv_slicing_takes_each_ranks_heads():
    nh, d, tp = 4, 3, 2
    hd = nh * d
    w = np.arange(2 * 3 * hd).reshape(2, 3 * hd)
    for r in range(tp):
        got = SI.slice_qkv_columns(w, tp, r)
        want_cols = [b * hd + hh * d + i for b in range(3) for hh in range(r * 2, r * 2 + 2) for i in range(d)]
        assert np.array_equal(got, w[:, want_cols])
        assert np.array_equal(R.shard_layer_params("gpt", {"wqkv": w}, tp, r, nh, d, 8)["wqkv"], w[:, want_cols])


# ---------------------------------------------------------------- closed forms / special cases
def test_attention_special_cases():
    rng = np.random.default_rng(7)
    # S = 1: the only allowed key is the query's own position, so o = v
    q, k, v = (rng.standard_normal((2, 3, 1, 8)) for _ in range(3))
    assert np.array_equal(R.attention_fwd(q, k, v), v)
    # equal scores (q = 0): o_i is the running mean of v_0..v_i
    S = 9
    v = rng.standard_normal((1, 1, S, 4))
    o = R.attention_fwd(np.zeros((1, 1, S, 4)), rng.standard_normal((1, 1, S, 4)), v)
    want = np.cumsum(v[0, 0], axis=0) / np.arange(1, S + 1)[:, None]
    assert np.allclose(o[0, 0], want, rtol=1e-13, atol=1e-13)
    # brute-force scalar loops on a tiny case (scale 1/sqrt(d), keys k <= i only)
    S, d = 5, 4
    q, k, v = (rng.standard_normal((1, 1, S, d)) for _ in range(3))
    o = R.attention_fwd(q, k, v)[0, 0]
    for i in range(S):
        sc = [sum(q[0, 0, i, c] * k[0, 0, j, c] for c in range(d)) / np.sqrt(d) for j in range(i + 1)]
        wts = np.exp(np.array(sc) - max(sc))
        wts /= wts.sum()
        ref = sum(wts[j] * v[0, 0, j] for j in range(i + 1))
        assert np.allclose(o[i], ref, rtol=1e-12, atol=1e-13)


def test_norm_closed_forms():
    rng = np.random.default_rng(8)
    x = rng.standard_normal((7, 64)) * 3 + 1.5
    eps = 1e-5
    a, xhat, rstd = R.layer_norm_fwd(x, np.ones(64), np.zeros(64), eps)
    var = x.var(axis=-1)
    assert np.abs(a.mean(-1)).max() < 1e-13
    assert np.allclose(a.var(axis=-1), var / (var + eps), rtol=1e-12)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(x), (64,), eps=eps).numpy()
    assert np.allclose(a, ref, rtol=1e-10, atol=1e-12)
    a, xhat, r = R.rms_norm_fwd(x, np.full(64, 2.0), 1e-6)
    assert np.allclose((a / 2.0) ** 2 @ np.ones(64) / 64, (x * x).mean(-1) / ((x * x).mean(-1) + 1e-6), rtol=1e-12)


def test_rope_properties():
    rng = np.random.default_rng(9)
    S, d = 16, 8
    cos, sin = R.rope_tables(S, d, 10000.0, np.float64)
    q = rng.standard_normal((S, d))
    k = rng.standard_normal((S, d))
    rq = R.rope_apply(q, cos, sin)
    assert np.array_equal(rq[0], q[0])                                    # position 0: identity
    assert np.allclose(rq[:, :4] ** 2 + rq[:, 4:] ** 2, q[:, :4] ** 2 + q[:, 4:] ** 2, rtol=1e-12)   # pair norms kept
    assert np.allclose(R.rope_apply(rq, cos, sin, -1.0), q, rtol=1e-12, atol=1e-13)                   # inverse rotation
    # relative-position property: <rope(q, m), rope(k, n)> depends only on m - n
    q1 = np.tile(q[:1], (S, 1))
    k1 = np.tile(k[:1], (S, 1))
    G = R.rope_apply(q1, cos, sin) @ R.rope_apply(k1, cos, sin).T
    for off in range(-3, 4):
        diag = np.diagonal(G, offset=off)
        assert np.allclose(diag, diag[0], rtol=1e-11, atol=1e-12)
    # angle of pair i at position p is p * base^(-2i/d): check one entry against the definition
    p, i = 5, 2
    ang = p * 10000.0 ** (-2 * i / d)
    assert np.isclose(rq[p, i], q[p, i] * np.cos(ang) - q[p, i + 4] * np.sin(ang), rtol=1e-12)
    assert np.isclose(rq[p, i + 4], q[p, i + 4] * np.cos(ang) + q[p, i] * np.sin(ang), rtol=1e-12)


def test_zero_second_matrix_leaves_residual_plus_bias():
    rng = np.random.default_rng(10)
    cfg = tiny_cfg("gpt", L=1)
    p = rand_params(cfg, rng)[0]
    p["w2"][:] = 0
    x = rng.standard_normal((2 * cfg.seq_len, cfg.hidden))
    y, c = R.layer_fwd(cfg, p, x)
    assert np.array_equal(y, c["x_mid"] + p["b2"])


@pytest.mark.parametrize("arch", ["gpt", "llama"])
def test_float32_instance_tracks_float64(arch):
    rng = np.random.default_rng(11)
    cfg = tiny_cfg(arch, L=2, S=16)
    p64 = rand_params(cfg, rng, wstd=0.1)
    p32 = [{k: v.astype(np.float32) for k, v in p.items()} for p in p64]
    x = rng.standard_normal((2 * cfg.seq_len, cfg.hidden))
    dy = rng.standard_normal((2 * cfg.seq_len, cfg.hidden))
    (y64,), (dx64,), g64 = run_stage(cfg, p64, [x], [dy])
    (y32,), (dx32,), g32 = run_stage(cfg, p32, [x.astype(np.float32)], [dy.astype(np.float32)])
    assert y32.dtype == np.float32 and dx32.dtype == np.float32

    def rel(a, b):
        return np.linalg.norm(a.astype(np.float64) - b) / np.linalg.norm(b)
    assert rel(y32, y64) < 1e-4 and rel(dx32, dx64) < 1e-4
    for a, b in zip(g32, g64):
        for k in a:
            assert a[k].dtype == np.float32
            assert rel(a[k], b[k]) < 1e-4, k


# ---------------------------------------------------------------- input generator
def test_bf16_rounding_is_nearest_even():
    a = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -0.3, 3.1415927, 0.0], dtype=np.float32)
    got = SI.round_bf16(a)
    want = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(got, want)
    rng = np.random.default_rng(0)
    b = rng.standard_normal(4096).astype(np.float32)
    assert np.array_equal(SI.round_bf16(b), torch.from_numpy(b).to(torch.bfloat16).to(torch.float32).numpy())


def test_draws_are_seeded_and_shaped():
    w = SI.WORKLOADS["tiny"]
    p0 = SI.draw_layer_params(w, 0)
    p0b = SI.draw_layer_params(w, 0)
    p1 = SI.draw_layer_params(w, 1)
    assert all(np.array_equal(p0[k], p0b[k]) for k in p0)
    assert not np.array_equal(p0["wqkv"], p1["wqkv"])
    assert p0["wqkv"].shape == (256, 768) and p0["w2"].shape == (1024, 256)
    assert abs(p0["w1"].std() - 0.02) < 1e-3 and (p0["b1"] == 0).all() and (p0["ln1_g"] == 1).all()
    x = SI.draw_activation(w, "x", 0)
    assert x.shape == (256, 256) and abs(x.std() - 1) < 0.02
    assert np.array_equal(SI.round_bf16(x), x)
    w2 = dict(w, tp=2)
    s0 = SI.draw_layer_params(w2, 0, tp_rank=0)
    s1 = SI.draw_layer_params(w2, 0, tp_rank=1)
    assert s0["wqkv"].shape == (256, 384) and s0["wo"].shape == (128, 256) and s0["w1"].shape == (256, 512)
    assert np.array_equal(np.concatenate([s0["w2"], s1["w2"]]), p0["w2"])
    assert np.array_equal(np.concatenate([s0["w1"], s1["w1"]], axis=1), p0["w1"])
