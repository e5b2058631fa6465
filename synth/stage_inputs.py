"""Workload table and seeded tensors for one pipeline stage.

Recipe: activations x ~ N(0,1), upstream gradients dy ~ N(0,1), weight
matrices ~ N(0, 0.02^2), biases 0, norm gains 1, norm offsets 0.  Every tensor
has its own counter-based stream (numpy Philox keyed by seed and a tensor id),
is drawn in float32 and rounded once to bf16 (round to nearest even); both
sides of a parity test receive the same bf16 bits.  For a tensor-parallel
shard the full layer is drawn and rank r's contiguous block is sliced out
(first matrix of a block by columns, second by rows).
"""
import numpy as np

__all__ = ["WORKLOADS", "BASE_SEED", "f32_to_bf16_bits", "bf16_bits_to_f32", "round_bf16",
           "local_dims", "param_spec", "draw_layer_params", "draw_stage_params", "draw_activation",
           "slice_column_parallel", "slice_row_parallel", "slice_qkv_columns"]

BASE_SEED = 20953

# name -> stage description (sizes before tensor-parallel sharding)
WORKLOADS = {
    "tiny":      dict(arch="gpt",   n_layers=2,  hidden=256,  n_heads=4,  head_dim=64,  ffn=1024,  seq=128,  mb=2, n_mb=2,  tp=1, recompute=0),
    "gpt1p3b":   dict(arch="gpt",   n_layers=4,  hidden=2048, n_heads=16, head_dim=128, ffn=8192,  seq=2048, mb=1, n_mb=8,  tp=1, recompute=0),
    "gpt7b_tp2": dict(arch="gpt",   n_layers=4,  hidden=4096, n_heads=32, head_dim=128, ffn=16384, seq=2048, mb=2, n_mb=8,  tp=2, recompute=0),
    "gpt13b":    dict(arch="gpt",   n_layers=10, hidden=5120, n_heads=40, head_dim=128, ffn=20480, seq=2048, mb=1, n_mb=16, tp=1, recompute=0),
    # res32: the stage carries its residual stream in fp32 (8 layers of this block miss the gradient tolerance otherwise)
    "llama7b":   dict(arch="llama", n_layers=8,  hidden=4096, n_heads=32, head_dim=128, ffn=11008, seq=4096, mb=1, n_mb=8,  tp=1, recompute=1, res32=1),
    # bidirectional-attention stages (the BERT-Large shape: 24 layers of h 1024, 16 heads x 64, FFN 4096, S 512; 6 of them here)
    "bert_tiny": dict(arch="bert",  n_layers=2,  hidden=256,  n_heads=4,  head_dim=64,  ffn=1024,  seq=256,  mb=2, n_mb=2,  tp=1, recompute=0),
    "bert_large": dict(arch="bert", n_layers=6,  hidden=1024, n_heads=16, head_dim=64,  ffn=4096,  seq=512,  mb=8, n_mb=8,  tp=1, recompute=0),
}


def f32_to_bf16_bits(a):
    """float32 array -> uint16 array of bf16 bit patterns, round to nearest even."""
    return (_rne_high_half(a) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rne_high_half(a):
    """uint32 view of a float32 array with the low 16 bits rounded away (to nearest, ties to even) and zeroed."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = u >> np.uint32(16)
    r &= np.uint32(1)
    r += np.uint32(0x7FFF)
    r += u
    r &= np.uint32(0xFFFF0000)
    return r


def round_bf16(a):
    return _rne_high_half(a).view(np.float32).reshape(np.shape(a))


def local_dims(w):
    """(local heads, local attention width, local FFN width) of one shard."""
    nh = w["n_heads"] // w["tp"]
    return nh, nh * w["head_dim"], w["ffn"] // w["tp"]


def param_spec(arch, hidden, h_full, ffn_full):
    """[(name, shape, kind)] of the unsharded layer; kind in {'w', 'zero', 'one'}."""
    if arch in ("gpt", "bert"):
        return [("ln1_g", (hidden,), "one"), ("ln1_b", (hidden,), "zero"),
                ("wqkv", (hidden, 3 * h_full), "w"), ("bqkv", (3 * h_full,), "zero"),
                ("wo", (h_full, hidden), "w"), ("bo", (hidden,), "zero"),
                ("ln2_g", (hidden,), "one"), ("ln2_b", (hidden,), "zero"),
                ("w1", (hidden, ffn_full), "w"), ("b1", (ffn_full,), "zero"),
                ("w2", (ffn_full, hidden), "w"), ("b2", (hidden,), "zero")]
    return [("ln1_g", (hidden,), "one"), ("wqkv", (hidden, 3 * h_full), "w"),
            ("wo", (h_full, hidden), "w"), ("ln2_g", (hidden,), "one"),
            ("wgu", (hidden, 2 * ffn_full), "w"), ("wd", (ffn_full, hidden), "w")]


def _gen(seed, tensor_id):
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed), np.uint64(tensor_id)]))


def _normal_bf16(seed, tensor_id, shape, std):
    n = int(np.prod(shape))
    a = _gen(seed, tensor_id).standard_normal(n, dtype=np.float32) * np.float32(std)
    return round_bf16(a).reshape(shape)


# ---- tensor-parallel slicing: index work only ------------------------------
def slice_column_parallel(w, tp, r):
    """Rank r's block of columns (last axis) of a matrix or of a bias vector."""
    n = w.shape[-1] // tp
    return np.ascontiguousarray(w[..., r * n:(r + 1) * n])


def slice_row_parallel(w, tp, r):
    """Rank r's block of rows (first axis)."""
    n = w.shape[0] // tp
    return np.ascontiguousarray(w[r * n:(r + 1) * n])


def slice_qkv_columns(w, tp, r):
    """[Q | K | V] packed along the last axis: rank r's heads of each of the three."""
    third = w.shape[-1] // 3
    return np.concatenate([slice_column_parallel(w[..., b * third:(b + 1) * third], tp, r) for b in range(3)], axis=-1)


def _draw_param(w, layer, idx, name, shape, kind, seed, tp_rank, perturb_vectors):
    tp = w["tp"]
    tid = 1000 * (layer + 1) + idx
    if kind == "w":
        t = _normal_bf16(seed, tid, shape, 0.02)
    elif perturb_vectors:
        t = _normal_bf16(seed, tid, shape, 0.1) + (1.0 if kind == "one" else 0.0)
        t = round_bf16(t.astype(np.float32))
    else:
        t = np.full(shape, 1.0 if kind == "one" else 0.0, dtype=np.float32)
    if tp > 1:
        if name in ("wqkv", "bqkv"):
            t = slice_qkv_columns(t, tp, tp_rank)
        elif name in ("w1", "b1"):
            t = slice_column_parallel(t, tp, tp_rank)
        elif name == "wgu":
            half = t.shape[-1] // 2
            t = np.concatenate([slice_column_parallel(t[:, :half], tp, tp_rank),
                                slice_column_parallel(t[:, half:], tp, tp_rank)], axis=-1)
        elif name in ("wo", "w2", "wd"):
            t = slice_row_parallel(t, tp, tp_rank)
    return np.ascontiguousarray(t, dtype=np.float32)


def draw_layer_params(w, layer, seed=BASE_SEED, tp_rank=0, perturb_vectors=False):
    """Rank tp_rank's shard of layer `layer`: dict name -> float32 array holding bf16 values.

    perturb_vectors=True replaces the 0/1 constants of biases and norm
    parameters by small random values (used by tests that would otherwise not
    see a wrong bias or gain path)."""
    h_full = w["n_heads"] * w["head_dim"]
    return {name: _draw_param(w, layer, idx, name, shape, kind, seed, tp_rank, perturb_vectors)
            for idx, (name, shape, kind) in enumerate(param_spec(w["arch"], w["hidden"], h_full, w["ffn"]))}


def draw_stage_params(w, seed=BASE_SEED, tp_rank=0, perturb_vectors=False, workers=1):
    """draw_layer_params for every layer of the stage; the tensors (each its own stream: same values) are drawn by
    `workers` threads, which is what makes the multi-billion-parameter stages affordable in a test."""
    h_full = w["n_heads"] * w["head_dim"]
    spec = param_spec(w["arch"], w["hidden"], h_full, w["ffn"])
    jobs = [(l, idx) + spec[idx] for l in range(w["n_layers"]) for idx in range(len(spec))]
    jobs.sort(key=lambda j: -int(np.prod(j[3])))     # largest first
    out = [dict.fromkeys(n for n, _, _ in spec) for _ in range(w["n_layers"])]

    def one(job):
        l, idx, name, shape, kind = job
        out[l][name] = _draw_param(w, l, idx, name, shape, kind, seed, tp_rank, perturb_vectors)

    if workers <= 1:
        for j in jobs:
            one(j)
    else:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=workers) as ex:
            list(ex.map(one, jobs))
    return out


def draw_activation(w, what, microbatch, seed=BASE_SEED):
    """what in {'x', 'dy'}: [mb*seq, hidden] float32 array holding bf16 values."""
    tid = 10_000_000 + (0 if what == "x" else 1) * 1_000_000 + microbatch
    return _normal_bf16(seed, tid, (w["mb"] * w["seq"], w["hidden"]), 1.0)
