"""Profiling by binary decomposition, as the paper's planner does it (Section III-D, Eq. 5):
profile a stage at 1, 2, 4, 8 layers, estimate other layer counts as sums of those blocks, and
compare with a direct measurement; same for the additive memory model.

Usage (on an MI355X):  python -m paper_2512_20953_amd.profile_study --workload gpt13b --layers 3 5 6 7 10
Prints a Markdown table."""
import argparse
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def profile_layers(w, n_layers, warmup=2, iters=5, max_in_flight=1):
    """Runs ah_stage_profile for workload dict `w` with n_layers layers; returns its report."""
    import paper_2512_20953_amd as P
    cfg = P.StageConfig.make(arch=w["arch"], n_layers=n_layers, hidden=w["hidden"], n_heads=w["n_heads"],
                             head_dim=w["head_dim"], ffn=w["ffn"], tp=w["tp"], seq=w["seq"], mb=w["mb"], n_mb=w["n_mb"],
                             max_in_flight=max_in_flight, recompute=w["recompute"], residual_fp32=w.get("res32", 0))
    st = P.Stage(cfg)
    st.params.normal_(0.0, 0.02)
    rep = st.profile(warmup=warmup, iters=iters)
    rep["sizes"] = st.sizes
    st.close()
    return rep


def study(w, targets, pow2=(1, 2, 4, 8), warmup=2, iters=5):
    import paper_2512_20953_amd as P
    prof = {n: profile_layers(w, n, warmup, iters) for n in sorted(set(pow2) | set(targets))}
    t_pow2 = [prof[n]["iteration_ms"] for n in pow2]
    per_layer_bytes = prof[1]["activation_bytes_per_layer_per_slot"]
    rows = []
    for n in targets:
        est = P.cost_layers_time(n, t_pow2)
        meas = prof[n]["iteration_ms"]
        mem_est = n * per_layer_bytes
        mem_meas = prof[n]["sizes"]["activation_bytes_per_slot"]
        rows.append({"layers": n, "estimated_ms": est, "measured_ms": meas, "rel_err": (est - meas) / meas,
                     "activation_bytes_estimated": mem_est, "activation_bytes_measured": mem_meas})
    return prof, rows


def main():
    from synth import stage_inputs as SI
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="gpt13b")
    ap.add_argument("--layers", type=int, nargs="+", default=[3, 5, 6, 7, 10])
    ap.add_argument("--iters", type=int, default=5)
    args = ap.parse_args()
    w = SI.WORKLOADS[args.workload]
    prof, rows = study(w, args.layers, iters=args.iters)
    print("| layers | profiled iteration ms | per-layer fwd ms (median of layers) | per-layer bwd ms |")
    print("|---|---|---|---|")
    for n in sorted(prof):
        f, b = sorted(prof[n]["fwd_ms"]), sorted(prof[n]["bwd_ms"])
        print("| %d | %.2f | %.3f | %.3f |" % (n, prof[n]["iteration_ms"], f[len(f) // 2], b[len(b) // 2]))
    print()
    print("| layers | Eq. 5 estimate ms | measured ms | relative error | activation bytes: n x one layer | measured |")
    print("|---|---|---|---|---|---|")
    for r in rows:
        print("| %d | %.2f | %.2f | %+.2f %% | %d | %d |" % (r["layers"], r["estimated_ms"], r["measured_ms"], 100 * r["rel_err"],
                                                             r["activation_bytes_estimated"], r["activation_bytes_measured"]))


if __name__ == "__main__":
    main()
