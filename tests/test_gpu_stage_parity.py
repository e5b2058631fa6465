"""HIP stage vs CPU oracle, through the C ABI, on the same seeded inputs.

Tolerances (normalised L2 per tensor): activations 2e-2, gradients 3e-2; index
and mask work (causality, slot bookkeeping, recompute, determinism) bit-exact."""
import numpy as np
import pytest
import torch

import paper_2512_20953_amd as P
from synth import stage_inputs as SI
from tests import gpu_util as U

pytestmark = pytest.mark.gpu


def _inputs(w, n_mb=None, perturb=True):
    params = [SI.draw_layer_params(w, l, perturb_vectors=perturb) for l in range(w["n_layers"])]
    k = w["n_mb"] if n_mb is None else n_mb
    xs = [SI.draw_activation(w, "x", m) for m in range(k)]
    dys = [SI.draw_activation(w, "dy", m) for m in range(k)]
    return params, xs, dys


def _run_case(w, n_mb=None, perturb=True, oracle_dtype=np.float64, **kw):
    gcfg, ocfg = U.make_cfgs(w, **kw)
    params, xs, dys = _inputs(w, n_mb, perturb)
    st = P.Stage(gcfg)
    U.load_params(st, params)
    taps, o_outs, rep = [], [], {}
    ys, dxs = U.run_gpu(st, xs, dys, taps=taps)
    o_ys, o_dxs, o_grads = U.run_oracle(ocfg, params, xs, dys, oracle_dtype, outs=o_outs)
    wa, wg = U.compare_stage(st, params, ys, dxs, o_ys, o_dxs, o_grads, taps=taps, o_outs=o_outs, report=rep)
    print("worst activation err %.3e, worst gradient err %.3e; %s" % (wa, wg, rep))
    return st, ys, dxs


def test_tiny_stage_as_specified():
    """Workload 'tiny' exactly as in the workload table (biases 0, gains 1), all K micro-batches."""
    _run_case(SI.WORKLOADS["tiny"], perturb=False)


def test_tiny_stage_with_nonzero_vectors():
    """Same shapes, biases / gains / offsets perturbed so their paths are visible."""
    _run_case(SI.WORKLOADS["tiny"])


REDUCED = {
    # several tiles in every GEMM dimension, 3 query blocks, head_dim 128, TP shard
    "gpt_d128_tp2": dict(arch="gpt", n_layers=2, hidden=384, n_heads=4, head_dim=128, ffn=1536, seq=384, mb=2, n_mb=3, tp=2, recompute=0),
    "llama_small": dict(arch="llama", n_layers=2, hidden=512, n_heads=4, head_dim=128, ffn=768, seq=256, mb=1, n_mb=2, tp=1, recompute=0),
    "llama_d64": dict(arch="llama", n_layers=1, hidden=256, n_heads=4, head_dim=64, ffn=384, seq=128, mb=2, n_mb=2, tp=1, recompute=0),
    # bidirectional attention: 3 query / key blocks with head_dim 128 on a TP shard; 2 blocks with head_dim 64
    "bert_d128_tp2": dict(arch="bert", n_layers=2, hidden=384, n_heads=4, head_dim=128, ffn=1536, seq=384, mb=2, n_mb=2, tp=2, recompute=0),
    "bert_tiny": SI.WORKLOADS["bert_tiny"],
    # odd multiples of the tile sizes everywhere: 384 rows, hidden 640, 5 heads, FFN 1152 (only 128-wide tiles divide these)
    "gpt_odd": dict(arch="gpt", n_layers=2, hidden=640, n_heads=5, head_dim=128, ffn=1152, seq=128, mb=3, n_mb=2, tp=1, recompute=0),
    # the widest rows the library accepts (hidden 16384) and a width between the row kernels' chunk sizes (12288)
    "gpt_widest": dict(arch="gpt", n_layers=1, hidden=16384, n_heads=2, head_dim=128, ffn=256, seq=128, mb=1, n_mb=2, tp=1, recompute=0),
    "llama_wide": dict(arch="llama", n_layers=1, hidden=12288, n_heads=2, head_dim=64, ffn=128, seq=128, mb=2, n_mb=1, tp=1, recompute=0),
    "llama_odd": dict(arch="llama", n_layers=1, hidden=384, n_heads=6, head_dim=64, ffn=640, seq=384, mb=1, n_mb=3, tp=1, recompute=1),
    # the residual stream carried in fp32 inside the stage: both block types, stored and recomputed activations, three layers
    "gpt_res32": dict(arch="gpt", n_layers=3, hidden=384, n_heads=4, head_dim=128, ffn=1536, seq=256, mb=2, n_mb=2, tp=2, recompute=0, res32=1),
    "llama_res32": dict(arch="llama", n_layers=3, hidden=512, n_heads=4, head_dim=128, ffn=768, seq=256, mb=1, n_mb=2, tp=1, recompute=0, res32=1),
    "llama_res32_recompute": dict(arch="llama", n_layers=2, hidden=384, n_heads=6, head_dim=64, ffn=640, seq=384, mb=1, n_mb=2, tp=1, recompute=1, res32=1),
}


@pytest.mark.parametrize("name", list(REDUCED))
def test_reduced_stages(name):
    _run_case(REDUCED[name])


@pytest.mark.parametrize("name", ["tiny", "llama_small", "llama_res32"])
def test_recompute_is_bit_identical(name):
    w = SI.WORKLOADS[name] if name in SI.WORKLOADS else REDUCED[name]
    outs = []
    for rc in (0, 1):
        st, ys, dxs = _run_case(w, recompute=rc)
        outs.append((ys, dxs, st.grads.clone()))
    for a, b in zip(outs[0][0] + outs[0][1], outs[1][0] + outs[1][1]):
        assert np.array_equal(a, b)
    assert torch.equal(outs[0][2], outs[1][2])


@pytest.mark.parametrize("defer", ["by_size", "all", "all_but_out_projection", "mlp_second_and_out_projection"])
@pytest.mark.parametrize("name,n_mb,group", [("tiny", 4, 2), ("tiny", 5, 3), ("gpt_d128_tp2", 3, 3), ("llama_small", 3, 2),
                                             ("bert_tiny", 2, 16), ("gpt_odd", 3, 2)])
def test_deferred_weight_gradients(name, n_mb, group, defer, monkeypatch):
    """Weight-gradient products taken once per group of micro-batches (full groups, an incomplete last group
    that needs the flush, a group larger than the iteration): against the oracle at the usual gates, and
    against the undeferred run: y and dx bit for bit (their path is the same), the gradients up to fp32
    summation order (a group's sums are formed in the accumulators and in shared partial sums before they
    reach the gradient buffer).  Which matrices wait for the group is the library's choice by output size; at
    these reduced sizes that choice defers none of them (only the vector gradients are grouped), so the other
    variants force it: every matrix deferred (products over pieces of the k axis taken from the slots and the
    pending blocks, everything on the caller's stream), and two mixtures (deferred and per-micro-batch products
    side by side, the second stream in use; the first is what the library picks for the 2048-wide stage)."""
    mask = {"by_size": None, "all": 15, "all_but_out_projection": 11, "mlp_second_and_out_projection": 5}[defer]
    w = dict(SI.WORKLOADS[name] if name in SI.WORKLOADS else REDUCED[name], n_mb=n_mb)
    monkeypatch.delenv("AH_DEFER_MATRICES", raising=False)
    st0, ys0, dxs0 = _run_case(w, n_mb)
    if mask is not None:
        monkeypatch.setenv("AH_DEFER_MATRICES", str(mask))   # read when the stage is created
    st1, ys1, dxs1 = _run_case(w, n_mb, wgrad_group=group)
    assert all(np.array_equal(a, b) for a, b in zip(ys0 + dxs0, ys1 + dxs1))
    for l in range(w["n_layers"]):
        for pname in SI.draw_layer_params(w, l):
            g0, g1 = st0.grad_view(l, pname), st1.grad_view(l, pname)
            assert U.rel_l2(U.to_np(g1), U.to_np(g0)) <= 2e-6, (l, pname)


def test_deferred_weight_gradients_slot_rules():
    w = SI.WORKLOADS["tiny"]
    gcfg, _ = U.make_cfgs(w, max_in_flight=3, wgrad_group=3)
    st = P.Stage(gcfg)
    x = torch.zeros(w["mb"] * w["seq"], w["hidden"], dtype=torch.bfloat16, device="cuda")
    y = torch.empty_like(x)
    st.forward(0, x, y)
    st.backward(0, x, y)
    with pytest.raises(P.AhError) as e:      # slot 0 waits for its group
        st.forward(0, x, y)
    assert e.value.status == 3
    with pytest.raises(P.AhError) as e:      # and has had its backward
        st.backward(0, x, y)
    assert e.value.status == 3
    with pytest.raises(P.AhError) as e:
        st.zero_grads()
    assert e.value.status == 3
    st.flush_grads()
    st.zero_grads()
    st.forward(0, x, y)                      # free again
    st.backward(0, x, y)
    st.forward(1, x, y)
    st.backward(1, x, y)
    st.forward(2, x, y)
    st.backward(2, x, y)                     # closes the group: all three slots free
    for slot in (0, 1, 2):
        st.forward(slot, x, y)
    torch.cuda.synchronize()
    for bad in (dict(wgrad_group=2, max_in_flight=1), dict(wgrad_group=17, max_in_flight=32), dict(wgrad_group=2, max_in_flight=2, recompute=1)):
        cfg = P.StageConfig.make(arch="gpt", n_layers=1, hidden=256, n_heads=4, head_dim=64, ffn=1024, seq=128, mb=2, **bad)
        with pytest.raises(P.AhError) as e:
            P.query_sizes(cfg)
        assert e.value.status == 1


@pytest.mark.parametrize("M,N,seg_k,n_seg,beta", [(128, 128, 128, 1, 0), (384, 256, 128, 3, 1), (256, 640, 384, 2, 1), (512, 384, 256, 5, 0),
                                                  (128, 256, 128, 16, 1)])
def test_gemm_tn_over_pieces_of_the_k_axis(M, N, seg_k, n_seg, beta):
    """C = beta C + sum_i A_i^T B_i with the pieces in separate buffers, element by element against float64."""
    rng = np.random.default_rng(11)
    As = [SI.round_bf16(rng.standard_normal((seg_k, M), dtype=np.float32)) for _ in range(n_seg)]
    Bs = [SI.round_bf16(rng.standard_normal((seg_k, N), dtype=np.float32)) for _ in range(n_seg)]
    C0 = rng.standard_normal((M, N), dtype=np.float32)
    # the pieces live in unrelated allocations, in shuffled order, with guard rows of NaN around each
    order = rng.permutation(n_seg)
    Ad, Bd = [None] * n_seg, [None] * n_seg
    for i in order:
        for src, dst, width in ((As, Ad, M), (Bs, Bd, N)):
            buf = torch.full((seg_k + 16, width), float("nan"), dtype=torch.bfloat16, device="cuda")
            buf[8:8 + seg_k] = U.to_dev(src[i])
            dst[i] = buf[8:8 + seg_k]
    C = torch.from_numpy(C0).cuda()
    P.gemm_tn_segmented(Ad, Bd, C, beta)
    torch.cuda.synchronize()
    ref = beta * C0.astype(np.float64) + sum(a.astype(np.float64).T @ b.astype(np.float64) for a, b in zip(As, Bs))
    got = C.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    assert np.abs(got - ref).max() <= 1e-4 * np.sqrt(seg_k * n_seg) + 1e-5 * np.abs(ref).max()


def test_deterministic_and_slot_independent():
    """Same inputs twice -> same bits; an interleaved 1F1B pattern over 3 slots -> same bits."""
    w = SI.WORKLOADS["tiny"]
    gcfg, _ = U.make_cfgs(w, max_in_flight=3)
    params, xs, dys = _inputs(dict(w, n_mb=4), 4)
    st = P.Stage(gcfg)
    U.load_params(st, params)
    ys1, dxs1 = U.run_gpu(st, xs, dys)
    g1 = st.grads.clone()
    ys2, dxs2 = U.run_gpu(st, xs, dys)
    assert all(np.array_equal(a, b) for a, b in zip(ys1 + dxs1, ys2 + dxs2))
    assert torch.equal(g1, st.grads)
    # warm-up F0 F1 F2, steady B0 F3 B1, drain B2 B3 (slot = micro-batch % 3)
    xd = [U.to_dev(x) for x in xs]
    dyd = [U.to_dev(d) for d in dys]
    y = [torch.empty_like(t) for t in xd]
    dx = [torch.empty_like(t) for t in xd]
    st.zero_grads()
    for m in (0, 1, 2):
        st.forward(m % 3, xd[m], y[m])
    st.backward(0, dyd[0], dx[0])
    st.forward(0, xd[3], y[3])
    st.backward(1, dyd[1], dx[1])
    st.backward(2, dyd[2], dx[2])
    st.backward(0, dyd[3], dx[3])
    torch.cuda.synchronize()
    assert all(np.array_equal(U.to_np(a), b) for a, b in zip(y + dx, ys1 + dxs1))
    assert torch.equal(g1, st.grads)


def test_causality_is_bit_exact_on_gpu():
    w = SI.WORKLOADS["tiny"]
    gcfg, _ = U.make_cfgs(w)
    params, xs, _ = _inputs(w, 1)
    st = P.Stage(gcfg)
    U.load_params(st, params)
    B, S, t = w["mb"], w["seq"], 70
    x = xs[0].reshape(B, S, -1).copy()
    x2 = x.copy()
    x2[:, t + 1:] = SI.round_bf16(x2[:, t + 1:] * 0.5 + 0.25)
    outs = []
    for a in (x, x2):
        xd = U.to_dev(a.reshape(B * S, -1))
        y = torch.empty_like(xd)
        st.forward(0, xd, y)
        dx = torch.empty_like(xd)
        st.backward(0, xd, dx)
        torch.cuda.synchronize()
        outs.append(U.to_np(y).reshape(B, S, -1))
    assert np.array_equal(outs[0][:, : t + 1], outs[1][:, : t + 1])
    assert not np.array_equal(outs[0][:, t + 1:], outs[1][:, t + 1:])


def test_state_errors():
    w = SI.WORKLOADS["tiny"]
    gcfg, _ = U.make_cfgs(w)
    st = P.Stage(gcfg)
    x = torch.zeros(w["mb"] * w["seq"], w["hidden"], dtype=torch.bfloat16, device="cuda")
    y = torch.empty_like(x)
    with pytest.raises(P.AhError) as e:
        st.backward(0, x, y)
    assert e.value.status == 3
    st.forward(0, x, y)
    with pytest.raises(P.AhError) as e:
        st.forward(0, x, y)
    assert e.value.status == 3
    with pytest.raises(P.AhError) as e:
        st.forward(1, x, y)
    assert e.value.status == 1
    st.backward(0, x, y)
    torch.cuda.synchronize()


@pytest.mark.parametrize("name", ["tiny", "llama_res32_recompute"])
def test_profile_reports_layers_and_bytes(name):
    w = dict(SI.WORKLOADS[name] if name in SI.WORKLOADS else REDUCED[name], n_layers=3)
    gcfg, _ = U.make_cfgs(w, max_in_flight=2)
    st = P.Stage(gcfg)
    st.params.normal_(0, 0.02)
    prof = st.profile(warmup=1, iters=3)
    assert len(prof["fwd_ms"]) == 3 and all(t > 0 for t in prof["fwd_ms"] + prof["bwd_ms"])
    assert abs(sum(prof["fwd_ms"]) - prof["stage_fwd_ms"]) <= 0.25 * prof["stage_fwd_ms"] + 0.05
    assert prof["peak_activation_bytes"] == 2 * st.sizes["activation_bytes_per_slot"] + st.sizes["workspace_bytes"]
    assert prof["activation_bytes_per_layer_per_slot"] * 3 == st.sizes["activation_bytes_per_slot"]
    assert prof["param_bytes"] == st.sizes["param_bytes"] and prof["grad_bytes"] == 2 * prof["param_bytes"]
    assert prof["iteration_ms"] > 0


def test_layer_times_add_up_as_the_profiler_assumes():
    """Section III-D: the time of n layers is estimated from the profiles of 1, 2, 4, ... layers;
    memory is the per-layer amount times the layer count (exact)."""
    from paper_2512_20953_amd.profile_study import study
    w = dict(SI.WORKLOADS["gpt1p3b"], n_mb=2)
    prof, rows = study(w, [3], pow2=(1, 2), warmup=2, iters=5)
    r = rows[0]
    print("3 layers: estimated %.2f ms, measured %.2f ms" % (r["estimated_ms"], r["measured_ms"]))
    assert abs(r["rel_err"]) < 0.10
    assert r["activation_bytes_estimated"] == r["activation_bytes_measured"]
    assert abs(sum(prof[3]["fwd_ms"]) - prof[3]["stage_fwd_ms"]) <= 0.1 * prof[3]["stage_fwd_ms"]


def test_bidirectional_stage_is_permutation_equivariant_and_differs_from_causal():
    """Mask work of the bidirectional path: with no positional signal inside the stage, reversing the
    tokens of every sequence reverses the outputs (to rounding: the tiles are summed in another order),
    a late token reaches the first output, and the causal stage on the same inputs gives another result."""
    w = SI.WORKLOADS["bert_tiny"]
    gcfg, _ = U.make_cfgs(w)
    params, xs, dys = _inputs(w, n_mb=1)
    st = P.Stage(gcfg)
    U.load_params(st, params)
    B, S, h = w["mb"], w["seq"], w["hidden"]
    x = xs[0].reshape(B, S, h)

    def fwd(stage, xin):
        xd = U.to_dev(xin.reshape(B * S, h))
        y = torch.empty_like(xd)
        stage.forward(0, xd, y)
        dx = torch.empty_like(xd)
        stage.backward(0, U.to_dev(dys[0]), dx)   # frees the slot
        torch.cuda.synchronize()
        return U.to_np(y).reshape(B, S, h)

    y = fwd(st, x)
    yr = fwd(st, x[:, ::-1])
    assert U.rel_l2(yr, y[:, ::-1]) <= 1e-2
    x2 = x.copy()
    x2[:, -1] = x[:, -1][:, ::-1]
    assert np.abs(fwd(st, x2)[:, 0] - y[:, 0]).max() > 0
    cst = P.Stage(U.make_cfgs(dict(w, arch="gpt"))[0])
    U.load_params(cst, params)
    yc = fwd(cst, x)
    assert np.array_equal(yc[:, 0], fwd(cst, x2)[:, 0])      # causal: position 0 never sees the last token
    # position 0 attends to itself alone under the mask and to all S keys without it (rounding noise is ~3e-3)
    assert U.rel_l2(yc[:, 0], y[:, 0]) > 1e-2


@pytest.mark.parametrize("name", ["tiny", "llama_small"])
def test_second_stream_changes_no_bit(name, monkeypatch):
    """Backward puts weight gradients and reductions on a stream of its own; with that switched off (everything on
    the caller's stream) the outputs and every gradient must be bit-identical, also with recompute."""
    w = SI.WORKLOADS[name] if name in SI.WORKLOADS else REDUCED[name]
    outs = []
    for off in (False, True):
        if off:
            monkeypatch.setenv("AH_NO_SIDE_STREAM", "1")
        else:
            monkeypatch.delenv("AH_NO_SIDE_STREAM", raising=False)
        for rc in (0, 1):
            gcfg, _ = U.make_cfgs(w, recompute=rc)
            params, xs, dys = _inputs(w)
            st = P.Stage(gcfg)
            U.load_params(st, params)
            ys, dxs = U.run_gpu(st, xs, dys)
            ys2, dxs2 = U.run_gpu(st, xs, dys)          # a second iteration on the same stage (streams already exist)
            outs.append((ys + dxs + ys2 + dxs2, st.grads.clone()))
    for arrs, g in outs[1:]:
        for a, b in zip(arrs, outs[0][0]):
            assert np.array_equal(a, b)
        assert torch.equal(g, outs[0][1])


@pytest.mark.parametrize("name,group", [("gpt_d128_tp2", 0), ("gpt_d128_tp2", 2), ("llama_res32", 0)])
def test_forward_beside_backward_changes_no_bit(name, group):
    """Micro-batches are independent until their gradients meet (Section III-A): without recompute the forward of
    micro-batch m + 1 may run on a second stream beside the backward of micro-batch m.  Outputs, input gradients and
    the accumulated gradients must equal those of the serial order F0 B0 F1 B1 ... bit for bit.  Two slots; with
    wgrad_group 2 a slot is free again only after the backward that closes its group, so that forward follows it."""
    w = REDUCED[name]
    K = 5
    gcfg, _ = U.make_cfgs(w, max_in_flight=2, recompute=0, wgrad_group=group)
    params, xs, dys = _inputs(w, n_mb=K)
    st = P.Stage(gcfg)
    U.load_params(st, params)
    ys, dxs = U.run_gpu(st, xs, dys)
    g_serial = st.grads.clone()

    G, slots = max(group, 1), 2
    main, ahead_stream = torch.cuda.current_stream(), torch.cuda.Stream()
    xd, dyd = [U.to_dev(x) for x in xs], [U.to_dev(d) for d in dys]
    yd, dxd = [torch.empty_like(x) for x in xd], [torch.empty_like(x) for x in xd]
    fdone = [torch.cuda.Event() for _ in range(K)]
    bdone = [torch.cuda.Event() for _ in range(K)]

    def frees_slot_of(j):
        return j if G == 1 else min((j // G) * G + G - 1, K - 1)

    def forward(j):
        if j - slots >= 0:
            ahead_stream.wait_event(bdone[frees_slot_of(j - slots)])
        st.forward(j % slots, xd[j], yd[j], ahead_stream)
        fdone[j].record(ahead_stream)

    for rep in range(2):
        torch.cuda.synchronize()
        st.grads.fill_(float("nan"))      # the first backward after zero_grads overwrites
        st.zero_grads()
        ahead_stream.wait_stream(main)
        forward(0)
        for m in range(K):
            early = m + 1 < K and (m + 1 - slots < 0 or frees_slot_of(m + 1 - slots) < m)
            if early:
                forward(m + 1)
            main.wait_event(fdone[m])
            st.backward(m % slots, dyd[m], dxd[m], main)
            bdone[m].record(main)
            if m + 1 < K and not early:
                forward(m + 1)
        st.flush_grads()
        torch.cuda.synchronize()
        for m in range(K):
            assert np.array_equal(U.to_np(yd[m]), ys[m]), (rep, m)
            assert np.array_equal(U.to_np(dxd[m]), dxs[m]), (rep, m)
        assert torch.equal(st.grads, g_serial), rep


@pytest.mark.parametrize("group", [
    0,
    pytest.param(2, marks=pytest.mark.skip(
        reason="host-side segmentation fault inside the graph launch (torch.cuda.CUDAGraph.replay) in two runs of the whole suite, "
               "after passing alone and in earlier suite runs; the library's own code does not run during a replay and no cause "
               "has been established, so this case stays off the GPU; the library now refuses to be captured in this mode "
               "(test_capture_with_deferred_gradients_is_refused)")),
])
def test_a_step_replays_from_a_hip_graph(group):
    """The library enqueues kernels and stream-ordering events only (no memset, no allocation, no host
    synchronisation), so a whole step can be captured into a HIP graph by the caller.  Replays, with eager steps
    and synchronisations between them, give the eager result bit for bit.  The case runs in a process of its own
    (tests/graph_replay_case.py)."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, "-m", "tests.graph_replay_case", str(group)], cwd=root, capture_output=True, text=True, timeout=110)
    assert r.returncode == 0, (r.returncode, r.stdout[-2000:], r.stderr[-2000:])
    assert "graph replay ok" in r.stdout


def test_capture_with_deferred_gradients_is_refused():
    """With wgrad_group > 1 a backward on a capturing stream returns AH_EUNSUPPORTED before it enqueues anything; the
    capture itself stays valid and ends normally (one fill kernel, never launched)."""
    w = SI.WORKLOADS["tiny"]
    gcfg, _ = U.make_cfgs(w, max_in_flight=2, wgrad_group=2)
    st = P.Stage(gcfg)
    x = torch.zeros(w["mb"] * w["seq"], w["hidden"], dtype=torch.bfloat16, device="cuda")
    y = torch.empty_like(x)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        st.forward(0, x, y, s)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            y.zero_()
            with pytest.raises(P.AhError) as e:
                st.backward(0, x, y, s)
            assert e.value.status == 5
            with pytest.raises(P.AhError) as e:
                st.flush_grads(s)
            assert e.value.status == 5
        del g
        st.backward(0, x, y, s)      # outside a capture the same call works
        st.flush_grads(s)
        torch.cuda.synchronize()


@pytest.mark.parametrize("arch", ["gpt", "llama"])
def test_shard_outputs_sum_to_the_unsharded_block_on_gpu(arch):
    """Section II-B on the device: with the first matrix of a block cut by columns and the second by rows, the
    two shards' outputs are the addends of the unsharded block's output.  A one-layer stage exposes one block at
    a time: with the second MLP matrix zero y = x + o Wo + bo (the attention block), with the out-projection zero
    y = x + g W2 + b2 (the MLP block).  Both tensor-parallel ranks run through the C ABI on their own shard; their
    addends are summed and compared with the unsharded stage's addend and with the oracle's partial sums."""
    from oracle import stage_ref as R
    tp = 2
    w = dict(arch=arch, n_layers=1, hidden=384, n_heads=4, head_dim=128, ffn=1536, seq=256, mb=2, n_mb=1, tp=tp, recompute=0)
    w_full = dict(w, tp=1)
    x = SI.draw_activation(w, "x", 0)
    second, out_proj = ("w2", "wo") if arch == "gpt" else ("wd", "wo")
    post_bias = {"w2": "b2", "wd": None, "wo": "bo"}

    def run(wl, params):
        gcfg, _ = U.make_cfgs(wl)
        st = P.Stage(gcfg)
        U.load_params(st, [params])
        xd = U.to_dev(x)
        y = torch.empty_like(xd)
        st.forward(0, xd, y)
        dx = torch.empty_like(xd)
        st.backward(0, xd, dx)       # frees the slot
        torch.cuda.synchronize()
        return U.to_np(y)

    for zeroed, block in ((second, "attention"), (out_proj, "mlp")):
        def prep(p):
            p = dict(p)
            p[zeroed] = np.zeros_like(p[zeroed])
            for b in ("b2", "bo"):
                if b in p and post_bias[zeroed] == b:
                    p[b] = np.zeros_like(p[b])
            return p
        kept_bias = "bo" if block == "attention" else "b2"
        full = prep(SI.draw_layer_params(w_full, 0, perturb_vectors=True))
        bias = full[kept_bias].astype(np.float64) if kept_bias in full else 0.0
        addend_full = run(w_full, full) - x - bias
        shards = [prep(SI.draw_layer_params(w, 0, tp_rank=r, perturb_vectors=True)) for r in range(tp)]
        addends = [run(w, s) - x - bias for s in shards]
        # y is rounded to bf16 at |x + addend| ~ 1, so each recovered addend carries ~2^-9 absolute error
        noise = 2.0 ** -9 * np.sqrt(np.mean((x + addend_full) ** 2)) / np.sqrt(np.mean(addend_full ** 2))
        assert U.rel_l2(sum(addends), addend_full) <= 4 * noise + 1e-2, block
        # and each shard's addend against the oracle's partial sum for that shard
        nh, hl, Fl = SI.local_dims(w)
        ocfg = R.StageCfg(arch, 1, w["hidden"], nh, w["head_dim"], Fl, w["seq"], 1e-6 if arch == "llama" else 1e-5)
        for r, s in enumerate(shards):
            s64 = {k: v.astype(np.float64) for k, v in s.items()}
            ref = R.attn_block_partial(ocfg, s64, x.astype(np.float64)) if block == "attention" else R.mlp_block_partial(ocfg, s64, x.astype(np.float64))
            assert U.rel_l2(addends[r], ref) <= 4 * noise + 1e-2, (block, r)
        assert U.rel_l2(addends[0], addend_full) > 0.3    # one shard alone is not the block
