"""CPU-side checks of the boundary: the library loads, exports every declared
symbol, validates configurations, and its byte accounting obeys the memory
model's identities (no compute calls here)."""
import ctypes
import os
import re

import pytest

import paper_2512_20953_amd as P
from paper_2512_20953_amd.binding import query_sizes
from synth import stage_inputs as SI

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "ah_stage.h")).read() + open(os.path.join(ROOT, "include", "ah_cost.h")).read()
    names = set(re.findall(r"^(?:int|const char\*)\s+(ah_[a-z_0-9]+)\s*\(", hdr, flags=re.M))
    assert len(names) >= 21 and "ah_cost_partition_layers" in names
    assert {"ah_stage_create", "ah_stage_forward", "ah_stage_backward", "ah_stage_grads", "ah_stage_profile"} <= names
    lib = ctypes.CDLL(P.library_path())
    for n in sorted(names):
        assert hasattr(lib, n), n


def _cfg(name, **kw):
    w = dict(SI.WORKLOADS[name], **kw)
    return P.StageConfig.make(arch=w["arch"], n_layers=w["n_layers"], hidden=w["hidden"], n_heads=w["n_heads"],
                              head_dim=w["head_dim"], ffn=w["ffn"], tp=w["tp"], seq=w["seq"], mb=w["mb"], n_mb=w["n_mb"],
                              max_in_flight=w.get("max_in_flight", 1), recompute=w["recompute"], residual_fp32=w.get("res32", 0))


@pytest.mark.parametrize("name", list(SI.WORKLOADS))
def test_all_workloads_are_supported_and_sized(name):
    w = SI.WORKLOADS[name]
    s = query_sizes(_cfg(name))
    nh, hl, F = SI.local_dims(w)
    h = w["hidden"]
    if w["arch"] != "llama":
        per_layer = 6 * h + h * 3 * hl + 3 * hl + hl * h + h * F + F + F * h
    else:
        per_layer = 2 * h + h * 3 * hl + hl * h + 3 * h * F
    assert s["param_elems"] == per_layer * w["n_layers"]
    assert s["param_bytes"] == 2 * s["param_elems"] and s["grad_bytes"] == 4 * s["param_elems"]
    # memory is additive in the layer count (Section III-D, memory profiling)
    assert s["activation_bytes_per_slot"] == w["n_layers"] * s["activation_bytes_per_layer_per_slot"]
    s1 = query_sizes(_cfg(name, n_layers=1))
    assert s1["activation_bytes_per_layer_per_slot"] == s["activation_bytes_per_layer_per_slot"]
    assert s1["workspace_bytes"] == s["workspace_bytes"]
    T = w["mb"] * w["seq"]
    r = 2 * w.get("res32", 0)   # extra bytes per element of the two residual-stream tensors when they are fp32
    if w["recompute"]:
        assert s["activation_bytes_per_layer_per_slot"] == (2 + r) * T * h
    else:
        saved = 2 * T * (4 * h + 4 * hl + 2 * F) + 2 * r * T * h + 4 * T * nh + 16 * T   # bf16 tensors + lse + two (mean, rstd) pairs
        assert s["activation_bytes_per_layer_per_slot"] == saved
    # the fp32 residual stream costs exactly 2 bytes more per element of the layer input and of x + attention block
    s32 = query_sizes(_cfg(name, res32=1))
    s16 = query_sizes(_cfg(name, res32=0))
    extra = (2 if w["recompute"] else 4) * T * h
    assert s32["activation_bytes_per_layer_per_slot"] - s16["activation_bytes_per_layer_per_slot"] == extra


def test_known_sizes_of_the_benchmark_workload():
    s = query_sizes(_cfg("gpt7b_tp2"))
    assert s["param_elems"] == 4 * 100_702_208
    assert 1.33e9 < s["activation_bytes_per_slot"] < 1.36e9


@pytest.mark.parametrize("kw,status", [
    (dict(head_dim=32), 5), (dict(hidden=200), 5), (dict(seq=100), 5), (dict(ffn=1000), 5),
    (dict(tp=3), 1), (dict(n_layers=0), 1), (dict(mb=0), 1), (dict(max_in_flight=0), 1), (dict(recompute=2), 1),
])
def test_bad_configurations_are_refused(kw, status):
    with pytest.raises(P.AhError) as e:
        query_sizes(_cfg("tiny", **kw))
    assert e.value.status == status
    assert len(str(e.value)) > 10


def test_struct_size_is_checked():
    c = _cfg("tiny")
    c.struct_size = 8
    with pytest.raises(P.AhError) as e:
        query_sizes(c)
    assert e.value.status == 1


def test_create_refuses_missing_or_misaligned_buffers():
    from paper_2512_20953_amd.binding import _Buffers, lib
    c = _cfg("tiny")
    h = ctypes.c_void_p()
    assert lib.ah_stage_create(ctypes.byref(c), ctypes.byref(_Buffers(0, 0, 0, 0)), ctypes.byref(h)) == 1
    assert lib.ah_stage_create(ctypes.byref(c), ctypes.byref(_Buffers(256, 512, 768, 1000)), ctypes.byref(h)) == 1
    assert b"aligned" in lib.ah_last_error()
    # well-formed pointers: the handle is host metadata only, no device access
    assert lib.ah_stage_create(ctypes.byref(c), ctypes.byref(_Buffers(256, 512, 768, 1024)), ctypes.byref(h)) == 0
    off, r, cc = ctypes.c_uint64(), ctypes.c_int32(), ctypes.c_int32()
    assert lib.ah_stage_param_layout(h, 1, P.PARAM_INDEX["w2"], ctypes.byref(off), ctypes.byref(r), ctypes.byref(cc)) == 0
    assert (r.value, cc.value) == (1024, 256)
    assert lib.ah_stage_param_layout(h, 2, 0, ctypes.byref(off), ctypes.byref(r), ctypes.byref(cc)) == 1
    # nothing pending: flushing and restarting the accumulation are host-side no-ops; bad handles and slots are refused
    assert lib.ah_stage_flush_grads(h, None) == 0
    assert lib.ah_stage_zero_grads(h, None) == 0
    assert lib.ah_stage_flush_grads(None, None) == 1
    assert lib.ah_stage_forward(h, 7, 256, 256, None) == 1      # slot out of range
    assert lib.ah_stage_backward(h, 0, 256, 256, None) == 3     # no forward in that slot
    assert lib.ah_stage_destroy(h) == 0


def test_gemm_entry_points_refuse_bad_shapes_without_touching_the_device():
    from paper_2512_20953_amd.binding import lib
    assert lib.ah_gemm_nn(1, 1, None, 1, 100, 128, 128, None) == 5
    assert lib.ah_gemm_nt(None, 1, 1, 128, 128, 128, None) == 1
    assert lib.ah_gemm_tn(1, 1, 1, 128, 128, 128, 2, None) == 1
    C = ctypes
    one = (C.c_void_p * 17)(*([1] * 17))
    assert lib.ah_gemm_tn_segmented(one, one, 17, 1, 128, 128, 128, 0, None) == 5   # too many pieces
    assert lib.ah_gemm_tn_segmented(one, one, 2, 1, 128, 128, 100, 0, None) == 5    # piece length not a multiple of 128
    assert lib.ah_gemm_tn_segmented(one, one, 0, 1, 128, 128, 128, 0, None) == 5
    assert lib.ah_gemm_tn_segmented(None, one, 1, 1, 128, 128, 128, 0, None) == 1
    hole = (C.c_void_p * 2)(1, None)
    assert lib.ah_gemm_tn_segmented(hole, one, 2, 1, 128, 128, 128, 0, None) == 1   # a NULL piece

    assert lib.ah_attention_fwd(1, 1, 1, 1, 100, 1, 128, 1, None) == 5


def test_deferred_weight_gradient_configuration_and_sizes():
    """wgrad_group: range, its two preconditions, and the workspace it adds (G * layers blocks of the four
    output-gradient operands, and per layer the shared partial sums), checked against the byte count written out by hand."""
    base = dict(arch="gpt", n_layers=3, hidden=256, n_heads=4, head_dim=64, ffn=1024, seq=128, mb=2)
    for bad in (dict(wgrad_group=2, max_in_flight=1), dict(wgrad_group=17, max_in_flight=32), dict(wgrad_group=-1),
                dict(wgrad_group=2, max_in_flight=2, recompute=1)):
        with pytest.raises(P.AhError) as e:
            query_sizes(P.StageConfig.make(**base, **bad))
        assert e.value.status == 1, bad
    s0 = query_sizes(P.StageConfig.make(**base, max_in_flight=4))
    s1 = query_sizes(P.StageConfig.make(**base, max_in_flight=4, wgrad_group=1))
    s4 = query_sizes(P.StageConfig.make(**base, max_in_flight=4, wgrad_group=4))
    assert s0 == s1
    T, h, hl, F = 256, 256, 256, 1024
    block = 2 * T * (h + h + F + 3 * hl)
    # plus, per layer, one set of fp32 partial sums for the vector gradients: two norm backward kernels
    # (3 arrays x 64 blocks x h), db1 and dbqkv (T / 64 slabs x their widths)
    vec = 2 * 3 * 64 * h * 4 + (T // 64) * F * 4 + (T // 64) * 3 * hl * 4
    assert s4["workspace_bytes"] - s0["workspace_bytes"] == 4 * 3 * block + 3 * vec
    assert {k: v for k, v in s4.items() if k != "workspace_bytes"} == {k: v for k, v in s0.items() if k != "workspace_bytes"}


def test_layer_input_tap_points_into_the_slot():
    """ah_stage_layer_input is pointer arithmetic over the caller's activation buffer: layer l of slot s sits at
    s * (bytes per slot) + l * (bytes per layer and slot), also when only layer inputs are kept (recompute) and when
    the residual stream is fp32; bad slots and layers are refused."""
    from paper_2512_20953_amd.binding import _Buffers, lib
    for kw in (dict(), dict(recompute=1), dict(res32=1), dict(recompute=1, res32=1)):
        c = _cfg("tiny", n_layers=3, max_in_flight=2, **kw)
        sz = query_sizes(c)
        base = 1 << 20
        h = ctypes.c_void_p()
        assert lib.ah_stage_create(ctypes.byref(c), ctypes.byref(_Buffers(256, 512, base, 1024)), ctypes.byref(h)) == 0
        p = ctypes.c_void_p()
        for slot in (0, 1):
            for layer in (0, 1, 2):
                assert lib.ah_stage_layer_input(h, slot, layer, ctypes.byref(p)) == 0
                assert p.value == base + slot * sz["activation_bytes_per_slot"] + layer * sz["activation_bytes_per_layer_per_slot"]
        assert lib.ah_stage_layer_input(h, 2, 0, ctypes.byref(p)) == 1
        assert lib.ah_stage_layer_input(h, 0, 3, ctypes.byref(p)) == 1
        assert lib.ah_stage_layer_input(h, 0, 0, None) == 1
        assert lib.ah_stage_destroy(h) == 0


def test_residual_fp32_flag_is_validated():
    with pytest.raises(P.AhError) as e:
        query_sizes(_cfg("tiny", res32=2))
    assert e.value.status == 1


def test_new_single_kernel_entry_points_refuse_bad_arguments_without_touching_the_device():
    from paper_2512_20953_amd.binding import lib
    assert lib.ah_gemm_nn_swiglu(1, 1, 1, 1, 128, 100, 128, None) == 5       # F not a multiple of 128
    assert lib.ah_gemm_nn_swiglu(1, 1, 1, 1, 128, 0, 128, None) == 5
    assert lib.ah_gemm_nn_swiglu(1, None, 1, 1, 128, 128, 128, None) == 1
    assert lib.ah_attention_bwd_static(1, 1, 1, 1, None, 1, 128, 1, 64, 1, None) == 1
    assert lib.ah_attention_bwd_static(1, 1, 1, 1, 1, 1, 100, 1, 64, 1, None) == 5
    assert lib.ah_attention_bwd_static(1, 1, 1, 1, 1, 4, 2048, 64, 64, 1, None) == 1     # 524288 rows: beyond the fixed scratch
    assert b"exceeds" in lib.ah_last_error()


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU's stage: any other --gpus exits with a message, before anything touches a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=60)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
