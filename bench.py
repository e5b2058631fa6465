#!/usr/bin/env python3
"""Throughput of one pipeline stage on one MI355X.

A step is one training iteration of the stage: K micro-batches, each a forward
and a backward pass through all layers, gradients accumulated in fp32 (restarted
at micro-batch 0).  Workload: the 7B-class TP=2 shard (4 layers, hidden 4096,
16 local heads x 128, local FFN 8192, seq 2048, micro-batch 2, K = 8), synthetic
seeded data already resident in HBM.  Prints one JSON line.

The weight-gradient products are deferred by default (--wgrad-group, default K): each layer's four products run
once per step over the K micro-batches' tokens instead of once per micro-batch, all inside the timed step;
--wgrad-group 1 gives the per-micro-batch accumulation.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0


def model_flops_per_iter(w):
    """2 flop per MAC, causal attention at its real half cost (bidirectional: all S keys), backward = 2 x forward,
    recompute not counted."""
    tp = w["tp"]
    h, hl, F = w["hidden"], w["n_heads"] // tp * w["head_dim"], w["ffn"] // tp
    S = w["seq"]
    mlp = (6 if w["arch"] == "llama" else 4) * h * F
    keys = S if w["arch"] == "bert" else (S + 1) / 2
    per_token_layer = 2 * h * 3 * hl + 2 * hl * h + mlp + 4 * hl * keys
    return 3.0 * per_token_layer * w["n_layers"] * w["mb"] * S * w["n_mb"]


def cpu_baseline(w, name):
    """The oracle as it stands, float32, on a bounded sample: one layer, two micro-batches, forward + backward."""
    import numpy as np
    from oracle import stage_ref as R
    from synth import stage_inputs as SI
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count()])
    except Exception:
        cores = os.cpu_count()
    # one layer, two of the workload's micro-batches: about 10-30 s of numpy on the box's share of host cores
    ws = dict(w, n_layers=1)
    reps = 2
    nh, hl, Fl = SI.local_dims(ws)
    cfg = R.StageCfg(ws["arch"], 1, ws["hidden"], nh, ws["head_dim"], Fl, ws["seq"], 1e-6 if ws["arch"] == "llama" else 1e-5)
    rng = np.random.default_rng(0)
    params = [{n: (np.ones(s, np.float32) if k == "one" else np.zeros(s, np.float32) if k == "zero"
                   else (rng.standard_normal(s, dtype=np.float32) * np.float32(0.02)))
               for n, s, k in SI.param_spec(ws["arch"], ws["hidden"], hl, Fl)}]
    T = ws["mb"] * ws["seq"]
    xs = [rng.standard_normal((T, ws["hidden"]), dtype=np.float32) for _ in range(reps)]
    dys = [rng.standard_normal((T, ws["hidden"]), dtype=np.float32) for _ in range(reps)]
    grads = R.zero_grads_like(params)
    t0 = time.perf_counter()
    for x, dy in zip(xs, dys):
        y, caches, _ = R.stage_fwd(cfg, params, x)
        R.stage_bwd(cfg, params, caches, dy, grads)
    dt = time.perf_counter() - t0
    tokens = T * reps
    return {"value": tokens / (dt * w["n_layers"]), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": "workload %s: 1 of %d layers, %d micro-batches of %d x %d tokens, forward+backward with fp32 gradient accumulation "
                      "in float32 numpy, %.1f s; tokens/s = %d / (%d layers x that time)"
                      % (name, w["n_layers"], reps, ws["mb"], ws["seq"], dt, tokens, w["n_layers"])}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="gpt7b_tp2")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--trace-steps", type=int, default=2)
    ap.add_argument("--no-ungrouped", action="store_true", help="skip the comparison run with wgrad_group 1")
    ap.add_argument("--overlap", type=int, default=0,
                    help="1: forward of micro-batch m+1 is enqueued on a second stream beside backward of micro-batch m (they are "
                         "independent; the stage is then created with at least two activation slots)")
    ap.add_argument("--no-side-stream", action="store_true",
                    help="keep all of backward on one stream, as the per-site trace does: kernel durations in a profile are then "
                         "those of kernels that own the chip (the timed figure is ~1 %% lower)")
    ap.add_argument("--wgrad-group", type=int, default=0,
                    help="micro-batches per weight-gradient product (ah_stage_config_t.wgrad_group); 0 = all K of a step "
                         "(1 with activation recomputation, which cannot defer)")
    args = ap.parse_args()
    if args.no_side_stream:
        os.environ["AH_NO_SIDE_STREAM"] = "1"
    if args.gpus != 1:
        print("bench.py measures one GPU's stage; this build has no multi-GPU path (--gpus %d refused)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2512_20953_amd as P
    from synth import stage_inputs as SI

    w = SI.WORKLOADS[args.workload]
    torch.manual_seed(SI.BASE_SEED)
    dev = torch.device("cuda:0")
    G = args.wgrad_group if args.wgrad_group > 0 else (1 if w["recompute"] else min(w["n_mb"], 16))
    # forward of micro-batch m + 1 beside backward of micro-batch m: both need a slot, and with recomputation both would use
    # the stage's one per-layer workspace, so that mode stays serial
    overlap = bool(args.overlap) and w["n_mb"] >= 2 and not w["recompute"]
    slots = max(G, 2) if overlap else G
    cfg = P.StageConfig.make(arch=w["arch"], n_layers=w["n_layers"], hidden=w["hidden"], n_heads=w["n_heads"],
                             head_dim=w["head_dim"], ffn=w["ffn"], tp=w["tp"], seq=w["seq"], mb=w["mb"], n_mb=w["n_mb"],
                             max_in_flight=slots, recompute=w["recompute"], wgrad_group=G, residual_fp32=w.get("res32", 0))
    st = P.Stage(cfg, device=dev)
    # synthetic weights of the stated distribution, generated on the device: N(0, 0.02), gains 1, biases 0
    st.params.normal_(0.0, 0.02)
    for l in range(w["n_layers"]):
        for name in (["ln1_g", "ln2_g"]):
            st.param_view(l, name).fill_(1.0)
        if w["arch"] != "llama":
            for name in ("ln1_b", "ln2_b", "bqkv", "bo", "b1", "b2"):
                st.param_view(l, name).zero_()
    T, K = w["mb"] * w["seq"], w["n_mb"]
    xs = [torch.randn(T, w["hidden"], device=dev).to(torch.bfloat16) for _ in range(K)]
    dys = [torch.randn(T, w["hidden"], device=dev).to(torch.bfloat16) for _ in range(K)]
    y, dx = torch.empty_like(xs[0]), torch.empty_like(xs[0])
    stream = torch.cuda.current_stream()

    if overlap:
        fstream = torch.cuda.Stream()
        fdone = [torch.cuda.Event() for _ in range(K)]
        bdone = [torch.cuda.Event() for _ in range(K)]
        ys2 = [torch.empty_like(xs[0]) for _ in range(2)]
        step_end = torch.cuda.Event()

    def step():
        st.zero_grads(stream)
        if not overlap:
            for m in range(K):
                st.forward(m % slots, xs[m], y, stream)
                st.backward(m % slots, dys[m], dx, stream)
        else:
            # the forward passes run ahead on their own stream: F(m+1) beside B(m); B(m) waits for F(m).  A slot is free
            # again once its previous micro-batch has had its backward (wgrad_group 1) or that micro-batch's group has been
            # taken (the backward that closes the group): F waits for that backward, and is enqueued after it if need be.
            step_end.record(stream)
            fstream.wait_event(step_end)          # the slots were freed by the previous step's work on `stream`

            def frees_slot_of(j):                 # the backward after which micro-batch j's slot is free again
                return j if G == 1 else min((j // G) * G + G - 1, K - 1)

            def forward(j):
                if j - slots >= 0:
                    fstream.wait_event(bdone[frees_slot_of(j - slots)])
                st.forward(j % slots, xs[j], ys2[j % 2], fstream)
                fdone[j].record(fstream)

            forward(0)
            for m in range(K):
                ahead = m + 1 < K and (m + 1 - slots < 0 or frees_slot_of(m + 1 - slots) < m)
                if ahead:
                    forward(m + 1)
                stream.wait_event(fdone[m])
                st.backward(m % slots, dys[m], dx, stream)
                bdone[m].record(stream)
                if m + 1 < K and not ahead:
                    forward(m + 1)
        st.flush_grads(stream)   # an incomplete last group (K not a multiple of G); otherwise nothing is pending

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(args.steps):
        step()
    e1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = e0.elapsed_time(e1) / args.steps
    assert torch.isfinite(st.grads).all() and torch.isfinite(dx.float()).all()
    tokens = T * K
    flops = model_flops_per_iter(w)
    tflops = flops / (ms_per_step * 1e-3) / 1e12

    # per-call-site durations, measured with HIP event pairs on the launch stream over the same steps
    st.trace_begin()
    for _ in range(max(1, args.trace_steps)):
        step()
    sites = st.trace_end()
    for s in sites:
        avg = s["total_ms"] / s["launches"]
        s["avg_us"] = avg * 1e3
        if s["flops_per_launch"] > 0:
            s["tflops"] = s["flops_per_launch"] / (avg * 1e-3) / 1e12
        elif s["bytes_per_launch"] > 0:
            s["gbs"] = s["bytes_per_launch"] / (avg * 1e-3) / 1e9
    # The dominant kernel: call sites that launch the same kernel instantiation on the same shape are one
    # entry (the weight-gradient GEMMs of the two MLP matrices are: same tile, layout, epilogue and flops).
    groups = {}
    for s in sites:
        if s["flops_per_launch"] <= 0:
            continue
        key = (s["name"].split(".")[0], s["flops_per_launch"]) if s["name"].startswith("gemm_tn.") else (s["name"], 0)
        g = groups.setdefault(key, {"names": [], "total_ms": 0.0, "launches": 0, "flops_per_launch": s["flops_per_launch"]})
        g["names"].append(s["name"])
        g["total_ms"] += s["total_ms"]
        g["launches"] += s["launches"]
    dom = max(groups.values(), key=lambda g: g["total_ms"])
    avg_ms = dom["total_ms"] / dom["launches"]
    achieved = dom["flops_per_launch"] / (avg_ms * 1e-3) / 1e12
    # HBM-side traffic of that kernel comes from hardware counters, which a plain run cannot read: it is taken from the
    # committed rocprofv3 counter summary, and only if that summary was made with this very GEMM source and launch
    # shape (it records the hash of csrc/gemm.hip); otherwise null.
    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic_%s.md" % args.workload)
    is_mlp_wgrad = any(n.startswith("gemm_tn.fc") for n in dom["names"])
    if os.path.exists(tpath) and is_mlp_wgrad:
        import hashlib
        sha = hashlib.sha256(open(os.path.join(ROOT, "paper_2512_20953_amd", "csrc", "gemm.hip"), "rb").read()).hexdigest()[:16]
        meta = dict(l.split(":", 1) for l in open(tpath) if l.startswith(("traffic_bytes_per_launch:", "wgrad_group:", "gemm_hip_sha256:")))
        if int(meta.get("wgrad_group", -1)) == G and meta.get("gemm_hip_sha256", "").strip() == sha:
            traffic = float(meta["traffic_bytes_per_launch"])
            traffic_source = "profiles/hbm_traffic_%s.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, csrc/gemm.hip %s)" % (args.workload, sha)
    # algorithmic bytes of one launch of the dominant kernel: each bf16 operand once, the fp32 result written once
    algorithmic_bytes = None
    if is_mlp_wgrad:
        Tk, h_, F_ = T * G, w["hidden"], (2 if w["arch"] == "llama" else 1) * (w["ffn"] // w["tp"])
        algorithmic_bytes = 2.0 * Tk * (h_ + F_) + 4.0 * h_ * F_ * (1 if G == K else 2)
    roofline = {"bound": "mfma", "scope": "dominant kernel (largest total time in the step)", "kernel": "+".join(dom["names"]),
                "achieved": achieved, "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS, "traffic": traffic, "traffic_source": traffic_source,
                "algorithmic_bytes": algorithmic_bytes, "avg_launch_us": avg_ms * 1e3,
                "launches": dom["launches"], "flops_per_launch": dom["flops_per_launch"],
                "whole_step_frac": tflops / PEAK_BF16_TFLOPS}

    # the same step with per-micro-batch accumulation (wgrad_group 1: one activation slot instead of G), for comparison
    ungrouped = None
    if G > 1 and not args.no_ungrouped:
        act_g = st.sizes["activation_bytes_per_slot"] * G + st.sizes["workspace_bytes"]
        st.close()
        del st
        torch.cuda.empty_cache()
        cfg1 = P.StageConfig.make(arch=w["arch"], n_layers=w["n_layers"], hidden=w["hidden"], n_heads=w["n_heads"],
                                  head_dim=w["head_dim"], ffn=w["ffn"], tp=w["tp"], seq=w["seq"], mb=w["mb"], n_mb=w["n_mb"],
                                  max_in_flight=1, recompute=w["recompute"], wgrad_group=1, residual_fp32=w.get("res32", 0))
        st1 = P.Stage(cfg1, device=dev)
        st1.params.normal_(0.0, 0.02)
        for l in range(w["n_layers"]):
            for name in ("ln1_g", "ln2_g"):
                st1.param_view(l, name).fill_(1.0)

        def step1():
            st1.zero_grads(stream)
            for m in range(K):
                st1.forward(0, xs[m], y, stream)
                st1.backward(0, dys[m], dx, stream)

        n1 = max(2, min(args.steps, 5))
        for _ in range(2):
            step1()
        torch.cuda.synchronize()
        e0.record(stream)
        for _ in range(n1):
            step1()
        e1.record(stream)
        torch.cuda.synchronize()
        ms1 = e0.elapsed_time(e1) / n1
        ungrouped = {"wgrad_group": 1, "ms_per_step": ms1, "steps": n1, "tokens_per_s": tokens / (ms1 * 1e-3),
                     "pct_of_bf16_mfma_peak": 100.0 * flops / (ms1 * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                     "activation_and_workspace_bytes": st1.sizes["activation_bytes_per_slot"] + st1.sizes["workspace_bytes"],
                     "activation_and_workspace_bytes_of_the_timed_configuration": act_g}

    out = {"metric": "stage fwd+bwd tokens/s and TFLOP/s (% bf16 MFMA peak) at 1 MI355X",
           "value": tokens / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
           "data": "synthetic", "model_tflops": tflops, "pct_of_bf16_mfma_peak": 100.0 * tflops / PEAK_BF16_TFLOPS,
           "wall_ms_per_step": wall * 1e3 / args.steps,
           "config": {"workload": args.workload, "arch": w["arch"], "layers": w["n_layers"], "hidden": w["hidden"],
                      "local_heads": w["n_heads"] // w["tp"], "head_dim": w["head_dim"], "local_ffn": w["ffn"] // w["tp"],
                      "seq_len": w["seq"], "microbatch": w["mb"], "microbatches": K, "tokens_per_step": tokens,
                      "tp_degree": w["tp"], "recompute": w["recompute"], "residual_fp32": w.get("res32", 0), "wgrad_group": G, "forward_beside_backward": int(overlap), "parallelism": "1 GPU (one TP shard of one stage)"},
           "roofline": roofline, "per_microbatch_accumulation": ungrouped,
           "sites": [{k: (round(v, 3) if isinstance(v, float) else v) for k, v in s.items()} for s in sites]}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, args.workload)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
