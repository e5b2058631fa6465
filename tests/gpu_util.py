"""Helpers shared by the GPU parity tests: move seeded inputs to the device, run
the HIP stage through the C ABI, run the numpy oracle, compare."""
import numpy as np
import torch

import paper_2512_20953_amd as P
from oracle import stage_ref as R
from synth import stage_inputs as SI


def to_dev(a):
    """float32 array holding bf16 values -> bf16 device tensor (exact)."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16).cuda()


def to_np(t, dtype=np.float64):
    return t.detach().float().cpu().numpy().astype(dtype)


def rel_l2(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(got - ref) / den) if den > 0 else float(np.linalg.norm(got))


def make_cfgs(w, max_in_flight=1, recompute=None, wgrad_group=0):
    nh, hl, Fl = SI.local_dims(w)
    gcfg = P.StageConfig.make(arch=w["arch"], n_layers=w["n_layers"], hidden=w["hidden"], n_heads=w["n_heads"],
                              head_dim=w["head_dim"], ffn=w["ffn"], tp=w["tp"], seq=w["seq"], mb=w["mb"], n_mb=w["n_mb"],
                              max_in_flight=max(max_in_flight, wgrad_group), recompute=w["recompute"] if recompute is None else recompute,
                              wgrad_group=wgrad_group)
    ocfg = R.StageCfg(w["arch"], w["n_layers"], w["hidden"], nh, w["head_dim"], Fl, w["seq"],
                      1e-6 if w["arch"] == "llama" else 1e-5, 10000.0)
    return gcfg, ocfg


def load_params(stage, params):
    """params: list (per layer) of dict name -> float32 array holding bf16 values."""
    for l, p in enumerate(params):
        for name, arr in p.items():
            stage.param_view(l, name).copy_(to_dev(arr).view(stage.param_view(l, name).shape))


def run_gpu(stage, xs, dys):
    """F0 B0 F1 B1 ... ; returns ys, dxs (numpy float64) and leaves grads in the stage.  Undeferred everything
    runs on slot 0; with deferred weight gradients a micro-batch keeps its slot until its group is taken, so the
    slots rotate, the input buffers are overwritten after each call (the library must have kept what it still
    needs) and an incomplete last group is flushed."""
    stage.zero_grads()
    group = max(int(stage.cfg.wgrad_group), 1)
    ys, dxs = [], []
    for m, (x, dy) in enumerate(zip(xs, dys)):
        xd, dyd = to_dev(x), to_dev(dy)
        y, dx = torch.empty_like(xd), torch.empty_like(xd)
        slot = m % stage.cfg.max_in_flight if group > 1 else 0
        stage.forward(slot, xd, y)
        stage.backward(slot, dyd, dx)
        xd.zero_()
        dyd.zero_()
        torch.cuda.synchronize()
        ys.append(to_np(y))
        dxs.append(to_np(dx))
    stage.flush_grads()
    torch.cuda.synchronize()
    return ys, dxs


def run_oracle(ocfg, params, xs, dys, dtype=np.float64):
    ps = [{k: v.astype(dtype) for k, v in p.items()} for p in params]
    grads = R.zero_grads_like(ps)
    ys, dxs = [], []
    for x, dy in zip(xs, dys):
        y, caches, _ = R.stage_fwd(ocfg, ps, x.astype(dtype))
        dxs.append(R.stage_bwd(ocfg, ps, caches, dy.astype(dtype), grads))
        ys.append(y)
    return ys, dxs, grads


def compare_stage(stage, params, ys, dxs, o_ys, o_dxs, o_grads, act_tol=2e-2, grad_tol=3e-2):
    """Normalised-L2 gates: activations (y, dx) 2e-2, every gradient tensor 3e-2."""
    worst_a, worst_g = 0.0, 0.0
    for m, (y, dx, oy, odx) in enumerate(zip(ys, dxs, o_ys, o_dxs)):
        ea, eb = rel_l2(y, oy), rel_l2(dx, odx)
        worst_a = max(worst_a, ea, eb)
        assert ea <= act_tol, "y of micro-batch %d: %g" % (m, ea)
        assert eb <= act_tol, "dx of micro-batch %d: %g" % (m, eb)
    for l, g in enumerate(o_grads):
        for name, ref in g.items():
            got = to_np(stage.grad_view(l, name)).reshape(ref.shape)
            if np.linalg.norm(ref) == 0:
                assert np.abs(got).max() == 0
                continue
            e = rel_l2(got, ref)
            worst_g = max(worst_g, e)
            assert e <= grad_tol, "grad %s of layer %d: %g" % (name, l, e)
    return worst_a, worst_g
