"""ctypes binding of include/ah_stage.h: argument marshalling only.

Device memory and streams come from PyTorch (ROCm); tensors are passed as raw
device pointers.  The library must have been built (paper_2512_20953_amd/build.py
or __graft_entry__.build()); a missing library is an ImportError-level failure,
there is no fallback path.
"""
import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
AH_ARCH_GPT, AH_ARCH_LLAMA, AH_ARCH_BERT = 0, 1, 2
_ARCH = {"gpt": AH_ARCH_GPT, "llama": AH_ARCH_LLAMA, "bert": AH_ARCH_BERT}
PARAM_INDEX = {"ln1_g": 0, "ln1_b": 1, "wqkv": 2, "bqkv": 3, "wo": 4, "bo": 5,
               "ln2_g": 6, "ln2_b": 7, "w1": 8, "b1": 9, "w2": 10, "b2": 11}
# names the layer's tensors go by elsewhere (LLaMA: fused gate|up and down)
PARAM_ALIASES = {"wgu": "w1", "wd": "w2"}


class AhError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__("ah status %d: %s" % (status, msg))
        self.status = status


class StageConfig(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("arch", C.c_int32), ("n_layers", C.c_int32), ("hidden", C.c_int32),
                ("n_heads", C.c_int32), ("head_dim", C.c_int32), ("ffn_hidden", C.c_int32), ("tp_degree", C.c_int32),
                ("tp_rank", C.c_int32), ("seq_len", C.c_int32), ("microbatch_size", C.c_int32),
                ("n_microbatches", C.c_int32), ("max_in_flight", C.c_int32), ("recompute", C.c_int32),
                ("wgrad_group", C.c_int32), ("norm_eps", C.c_float), ("rope_base", C.c_float), ("residual_fp32", C.c_int32)]

    @classmethod
    def make(cls, arch="gpt", n_layers=1, hidden=256, n_heads=4, head_dim=64, ffn=1024, tp=1, tp_rank=0, seq=128, mb=1,
             n_mb=1, max_in_flight=1, recompute=0, wgrad_group=0, norm_eps=0.0, rope_base=0.0, residual_fp32=0):
        return cls(C.sizeof(cls), _ARCH[arch], n_layers, hidden, n_heads, head_dim,
                   ffn, tp, tp_rank, seq, mb, n_mb, max_in_flight, recompute, wgrad_group, norm_eps, rope_base, residual_fp32)


class _Sizes(C.Structure):
    _fields_ = [("param_elems", C.c_uint64), ("param_bytes", C.c_uint64), ("grad_bytes", C.c_uint64),
                ("activation_bytes_per_slot", C.c_uint64), ("activation_bytes_per_layer_per_slot", C.c_uint64),
                ("workspace_bytes", C.c_uint64)]


class _Buffers(C.Structure):
    _fields_ = [("params", C.c_void_p), ("grads", C.c_void_p), ("activations", C.c_void_p), ("workspace", C.c_void_p)]


class _Profile(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("n_layers", C.c_int32), ("fwd_ms", C.POINTER(C.c_float)),
                ("bwd_ms", C.POINTER(C.c_float)), ("stage_fwd_ms", C.c_float), ("stage_bwd_ms", C.c_float),
                ("iteration_ms", C.c_float), ("peak_activation_bytes", C.c_uint64),
                ("activation_bytes_per_layer_per_slot", C.c_uint64), ("param_bytes", C.c_uint64), ("grad_bytes", C.c_uint64)]


class _TraceEntry(C.Structure):
    _fields_ = [("name", C.c_char * 32), ("launches", C.c_int64), ("total_ms", C.c_double),
                ("flops_per_launch", C.c_double), ("bytes_per_launch", C.c_double)]


def library_path():
    return os.path.join(HERE, "libahstage.so")


def _load():
    path = library_path()
    if not os.path.exists(path):
        raise ImportError("libahstage.so is not built: run `python -m paper_2512_20953_amd.build` "
                          "(or __graft_entry__.build()); there is no fallback implementation")
    # PyTorch ships its own copy of the HIP runtime and must be loaded first: the dynamic linker
    # then resolves this library's runtime dependency to that same copy.  Loaded the other way
    # round the process ends up with two runtimes, and the second one finds no device.
    import torch  # noqa: F401
    L = C.CDLL(path)
    L.ah_last_error.restype = C.c_char_p
    vp, i = C.c_void_p, C.c_int
    L.ah_stage_query_sizes.argtypes = [C.POINTER(StageConfig), C.POINTER(_Sizes)]
    L.ah_stage_create.argtypes = [C.POINTER(StageConfig), C.POINTER(_Buffers), C.POINTER(vp)]
    L.ah_stage_destroy.argtypes = [vp]
    L.ah_stage_param_layout.argtypes = [vp, i, i, C.POINTER(C.c_uint64), C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    L.ah_stage_forward.argtypes = [vp, i, vp, vp, vp]
    L.ah_stage_backward.argtypes = [vp, i, vp, vp, vp]
    L.ah_stage_grads.argtypes = [vp, C.POINTER(vp), C.POINTER(C.c_uint64)]
    L.ah_stage_zero_grads.argtypes = [vp, vp]
    L.ah_stage_flush_grads.argtypes = [vp, vp]
    L.ah_stage_profile.argtypes = [vp, i, i, C.POINTER(_Profile)]
    L.ah_stage_trace_begin.argtypes = [vp]
    L.ah_stage_trace_end.argtypes = [vp, C.POINTER(_TraceEntry), i, C.POINTER(i)]
    dp, ip = C.POINTER(C.c_double), C.POINTER(C.c_int)
    L.ah_cost_layers_time.argtypes = [i, dp, i, dp]
    L.ah_cost_pipeline_time.argtypes = [dp, i, i, dp]
    L.ah_cost_iteration_time.argtypes = [dp, ip, i, i, C.c_double, dp]
    L.ah_cost_idle_fractions.argtypes = [dp, i, i, dp, dp]
    L.ah_cost_partition_layers.argtypes = [i, i, dp, dp, C.c_double, C.c_double, ip, ip, dp]
    L.ah_gemm_nn.argtypes = [vp, vp, vp, vp, i, i, i, vp]
    L.ah_gemm_nt.argtypes = [vp, vp, vp, i, i, i, vp]
    L.ah_gemm_nn_swiglu.argtypes = [vp, vp, vp, vp, i, i, i, vp]
    L.ah_gemm_tn.argtypes = [vp, vp, vp, i, i, i, i, vp]
    L.ah_gemm_tn_segmented.argtypes = [C.POINTER(vp), C.POINTER(vp), i, vp, i, i, i, i, vp]
    L.ah_attention_fwd.argtypes = [vp, vp, vp, i, i, i, i, i, vp]
    L.ah_attention_bwd.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, i, vp]
    L.ah_attention_bwd_static.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, vp]
    L.ah_stage_layer_input.argtypes = [vp, i, i, C.POINTER(vp)]
    return L


lib = _load()


def _check(rc):
    if rc != 0:
        raise AhError(rc, lib.ah_last_error().decode())


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


def _stream(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def query_sizes(cfg):
    s = _Sizes()
    _check(lib.ah_stage_query_sizes(C.byref(cfg), C.byref(s)))
    return {k: int(getattr(s, k)) for k, _ in _Sizes._fields_}


class Stage:
    """A stage over torch-allocated device buffers."""

    def __init__(self, cfg, device="cuda:0"):
        import torch
        self.cfg = cfg
        self.sizes = query_sizes(cfg)
        self.device = torch.device(device)
        self.params = torch.zeros(self.sizes["param_elems"], dtype=torch.bfloat16, device=self.device)
        self.grads = torch.zeros(self.sizes["param_elems"], dtype=torch.float32, device=self.device)
        self.activations = torch.empty(self.sizes["activation_bytes_per_slot"] * cfg.max_in_flight, dtype=torch.uint8,
                                       device=self.device)
        self.workspace = torch.empty(self.sizes["workspace_bytes"], dtype=torch.uint8, device=self.device)
        bufs = _Buffers(self.params.data_ptr(), self.grads.data_ptr(), self.activations.data_ptr(), self.workspace.data_ptr())
        h = C.c_void_p()
        _check(lib.ah_stage_create(C.byref(cfg), C.byref(bufs), C.byref(h)))
        self._h = h

    def close(self):
        if getattr(self, "_h", None) and lib is not None:   # at interpreter shutdown the module globals may be gone already
            lib.ah_stage_destroy(self._h)
            self._h = None

    __del__ = close

    def param_layout(self, layer, name):
        which = PARAM_INDEX[PARAM_ALIASES.get(name, name)]
        off, r, c = C.c_uint64(), C.c_int32(), C.c_int32()
        _check(lib.ah_stage_param_layout(self._h, layer, which, C.byref(off), C.byref(r), C.byref(c)))
        return off.value, r.value, c.value

    def param_view(self, layer, name):
        off, r, c = self.param_layout(layer, name)
        v = self.params[off:off + r * c]
        return v.view(r, c) if r > 1 else v

    def grad_view(self, layer, name):
        off, r, c = self.param_layout(layer, name)
        v = self.grads[off:off + r * c]
        return v.view(r, c) if r > 1 else v

    def layer_input(self, slot, layer):
        """[T, hidden] view (bf16, or fp32 with residual_fp32) of the input the stage keeps for `layer` of the micro-batch in `slot`."""
        import torch
        p = C.c_void_p()
        _check(lib.ah_stage_layer_input(self._h, slot, layer, C.byref(p)))
        T, h = self.cfg.microbatch_size * self.cfg.seq_len, self.cfg.hidden
        dt, nb = (torch.float32, 4) if self.cfg.residual_fp32 else (torch.bfloat16, 2)
        off = p.value - self.activations.data_ptr()
        assert 0 <= off and off + nb * T * h <= self.activations.numel()
        return self.activations[off:off + nb * T * h].view(dt).view(T, h)

    def forward(self, slot, x, y, stream=None):
        _check(lib.ah_stage_forward(self._h, slot, _ptr(x), _ptr(y), _stream(stream)))

    def backward(self, slot, dy, dx, stream=None):
        _check(lib.ah_stage_backward(self._h, slot, _ptr(dy), _ptr(dx), _stream(stream)))

    def zero_grads(self, stream=None):
        _check(lib.ah_stage_zero_grads(self._h, _stream(stream)))

    def flush_grads(self, stream=None):
        _check(lib.ah_stage_flush_grads(self._h, _stream(stream)))

    def grads_ptr(self):
        p, n = C.c_void_p(), C.c_uint64()
        _check(lib.ah_stage_grads(self._h, C.byref(p), C.byref(n)))
        return p.value, n.value

    def trace_begin(self):
        _check(lib.ah_stage_trace_begin(self._h))

    def trace_end(self):
        arr = (_TraceEntry * 32)()
        n = C.c_int()
        _check(lib.ah_stage_trace_end(self._h, arr, 32, C.byref(n)))
        return [{"name": arr[k].name.decode(), "launches": int(arr[k].launches), "total_ms": arr[k].total_ms,
                 "flops_per_launch": arr[k].flops_per_launch, "bytes_per_launch": arr[k].bytes_per_launch}
                for k in range(n.value)]

    def profile(self, warmup=2, iters=5):
        L = self.cfg.n_layers
        f, b = (C.c_float * L)(), (C.c_float * L)()
        p = _Profile(C.sizeof(_Profile), L, f, b)
        _check(lib.ah_stage_profile(self._h, warmup, iters, C.byref(p)))
        return {"fwd_ms": list(f), "bwd_ms": list(b), "stage_fwd_ms": p.stage_fwd_ms, "stage_bwd_ms": p.stage_bwd_ms,
                "iteration_ms": p.iteration_ms, "peak_activation_bytes": int(p.peak_activation_bytes),
                "activation_bytes_per_layer_per_slot": int(p.activation_bytes_per_layer_per_slot),
                "param_bytes": int(p.param_bytes), "grad_bytes": int(p.grad_bytes)}


def gemm_nn(A, B, bias, Cout, stream=None):
    M, K = A.shape
    _check(lib.ah_gemm_nn(_ptr(A), _ptr(B), _ptr(bias), _ptr(Cout), M, B.shape[1], K, _stream(stream)))


def gemm_nn_swiglu(A, B, U, Mout, stream=None):
    M, K = A.shape
    _check(lib.ah_gemm_nn_swiglu(_ptr(A), _ptr(B), _ptr(U), _ptr(Mout), M, B.shape[1] // 2, K, _stream(stream)))


def gemm_nt(A, B, Cout, stream=None):
    M, K = A.shape
    _check(lib.ah_gemm_nt(_ptr(A), _ptr(B), _ptr(Cout), M, B.shape[0], K, _stream(stream)))


def gemm_tn(A, B, Cout, beta, stream=None):
    K, M = A.shape
    _check(lib.ah_gemm_tn(_ptr(A), _ptr(B), _ptr(Cout), M, B.shape[1], K, int(beta), _stream(stream)))


def gemm_tn_segmented(A_list, B_list, Cout, beta, stream=None):
    n = len(A_list)
    seg_k, M = A_list[0].shape
    pa = (C.c_void_p * n)(*[a.data_ptr() for a in A_list])
    pb = (C.c_void_p * n)(*[b.data_ptr() for b in B_list])
    _check(lib.ah_gemm_tn_segmented(pa, pb, n, _ptr(Cout), M, B_list[0].shape[1], seg_k, int(beta), _stream(stream)))


def attention_fwd(qkv, o, lse, B, S, nh, d, causal=True, stream=None):
    _check(lib.ah_attention_fwd(_ptr(qkv), _ptr(o), _ptr(lse), B, S, nh, d, int(bool(causal)), _stream(stream)))


def attention_bwd(qkv, o, lse, d_o, dqkv, delta, B, S, nh, d, causal=True, stream=None):
    _check(lib.ah_attention_bwd(_ptr(qkv), _ptr(o), _ptr(lse), _ptr(d_o), _ptr(dqkv), _ptr(delta), B, S, nh, d, int(bool(causal)), _stream(stream)))


ATTENTION_STATIC_MAX_ROWS = 262144


def attention_bwd_static(qkv, o, lse, d_o, dqkv, B, S, nh, d, causal=True, stream=None):
    _check(lib.ah_attention_bwd_static(_ptr(qkv), _ptr(o), _ptr(lse), _ptr(d_o), _ptr(dqkv), B, S, nh, d, int(bool(causal)), _stream(stream)))


# ---- cost model (include/ah_cost.h): host arrays in, numbers out
def _darr(v):
    return (C.c_double * len(v))(*[float(x) for x in v])


def cost_layers_time(n, t_pow2):
    out = C.c_double()
    _check(lib.ah_cost_layers_time(int(n), _darr(t_pow2), len(t_pow2), C.byref(out)))
    return out.value


def cost_pipeline_time(t_stage, K):
    out = C.c_double()
    _check(lib.ah_cost_pipeline_time(_darr(t_stage), len(t_stage), int(K), C.byref(out)))
    return out.value


def cost_iteration_time(groups, K, t_sync):
    flat = [t for g in groups for t in g]
    stages = (C.c_int * len(groups))(*[len(g) for g in groups])
    out = C.c_double()
    _check(lib.ah_cost_iteration_time(_darr(flat), stages, len(groups), int(K), float(t_sync), C.byref(out)))
    return out.value


def cost_idle_fractions(t_stage, K):
    idle = (C.c_double * len(t_stage))()
    mean = C.c_double()
    _check(lib.ah_cost_idle_fractions(_darr(t_stage), len(t_stage), int(K), idle, C.byref(mean)))
    return list(idle), mean.value


def cost_partition_layers(n_layers, t_layer, mem_bytes, fixed_per_layer, act_per_layer, in_flight):
    P = len(t_layer)
    l = (C.c_int * P)()
    worst = C.c_double()
    _check(lib.ah_cost_partition_layers(P, int(n_layers), _darr(t_layer), _darr(mem_bytes), float(fixed_per_layer),
                                        float(act_per_layer), (C.c_int * P)(*[int(f) for f in in_flight]), l, C.byref(worst)))
    return list(l), worst.value
