"""Helpers shared by the GPU parity tests: move seeded inputs to the device, run
the HIP stage through the C ABI, run the numpy oracle, compare.

The comparison arithmetic (norms of differences) runs in float64; for the large
tensors it runs on the device with PyTorch, which is test plumbing here: it
touches neither side's results before they are compared."""
import numpy as np
import torch

import paper_2512_20953_amd as P
from oracle import stage_ref as R
from synth import stage_inputs as SI

# Gates.  Tensor level (normalised L2): activations 2e-2, parameter gradients 3e-2 (the stated tolerances).  Finer
# views, so that one wrong row or tile (error ~1 on its own, invisible in the norm of a large tensor) fails:
#  * every row of y, dx and the layer outputs against its own norm, at twice the tensor's bound.  A row is a sum of
#    thousands of independently rounded terms like the whole, so its error is of the tensor's order, but not evenly
#    spread: the rows of the first positions of a sequence carry two to three times the average.  Attention backward
#    takes delta_i = do_i . o_i from the bf16 output, an absolute error in every dp_ik - delta_i of row i that weighs
#    most where the softmax is peaked (few keys).  Measured at full size: worst row 1.3e-2 .. 2.0e-2 beside
#    0.8e-2 .. 1.0e-2 for the tensor.
#  * every 128 x 128 tile of a matrix gradient against its own norm, at TILE_TOL = 0.15.  The worst tiles are always
#    key (and query) columns of the fused QKV gradient: the key gradients of a sequence sum to exactly zero over its
#    tokens (sum_k ds_ik = 0 for every query), so the part of the layer input common to the tokens contributes rounding
#    noise to a^T dk but no signal, and a tile there has several times the tensor's relative error (1.8e-2 .. 6.5e-2
#    measured beside 0.7e-2 .. 1.0e-2 for the tensor) whatever the kernel does in bf16.
#  * the largest element error relative to the largest reference element, at twice the tensor's bound: element errors
#    are near-Gaussian with standard deviation e * rms(ref) (e the tensor's normalised L2 error), the reference
#    elements near-Gaussian with standard deviation rms(ref), and the maxima of N such variables scale by the same
#    sqrt(2 ln N), so the ratio would be about e if the errors were evenly spread; the maximum is taken by the rows
#    that carry two to three times the average (measured: 1.0e-2 .. 2.1e-2).
ACT_TOL, GRAD_TOL = 2e-2, 3e-2
TILE = 128
TILE_TOL = 0.15
FLOOR = 0.05


def to_dev(a):
    """float32 array holding bf16 values -> bf16 device tensor (exact: the conversion drops 16 zero bits)."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda().to(torch.bfloat16)


def to_np(t, dtype=np.float64):
    return t.detach().float().cpu().numpy().astype(dtype)


def rel_l2(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(got - ref) / den) if den > 0 else float(np.linalg.norm(got))


def _dev64(a):
    if isinstance(a, torch.Tensor):
        return a.detach().cuda().double()
    a = np.asarray(a)
    if a.dtype == np.float64:
        return torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda().double()


def error_views(got, ref, tile=None):
    """Errors of `got` against `ref` (arrays or tensors of one shape), float64 on the device.
    Returns dict: l2 (normalised L2 of the tensor), maxabs (max |got - ref| / max |ref|), rows (worst normalised L2
    of a row, 2-D inputs), tiles (worst normalised L2 of a tile x tile block, if `tile` divides both extents)."""
    g, r = _dev64(got), _dev64(ref)
    g = g.reshape(r.shape)
    d = g - r
    out = {}
    den = r.norm().item()
    out["l2"] = d.norm().item() / den if den > 0 else d.norm().item()
    mx = r.abs().max().item()
    out["maxabs"] = d.abs().max().item() / mx if mx > 0 else d.abs().max().item()
    if r.dim() == 2:
        # A row (tile) is measured against its own norm, but not against less than FLOOR of the root-mean-square
        # row (tile) norm of the tensor: a reference row that is zero or nearly so (the first query's dq under the
        # causal mask is exactly 0) has no relative error of its own.
        rn = r.norm(dim=1)
        q = d.norm(dim=1) / rn.clamp_min(FLOOR * (rn ** 2).mean().sqrt().item() + 1e-300)
        out["rows"] = q.max().item()
        out["rows_argmax"] = int(q.argmax().item())
        if tile and r.shape[0] % tile == 0 and r.shape[1] % tile == 0:
            sh = (r.shape[0] // tile, tile, r.shape[1] // tile, tile)
            dn = (d.view(sh) ** 2).sum(dim=(1, 3)).sqrt()
            tn = (r.view(sh) ** 2).sum(dim=(1, 3)).sqrt()
            q = dn / tn.clamp_min(FLOOR * (tn ** 2).mean().sqrt().item() + 1e-300)
            out["tiles"] = q.max().item()
            out["tiles_argmax"] = tuple(int(v) for v in np.unravel_index(int(q.argmax().item()), q.shape))
    return out


def make_cfgs(w, max_in_flight=1, recompute=None, wgrad_group=0, res32=None):
    nh, hl, Fl = SI.local_dims(w)
    gcfg = P.StageConfig.make(arch=w["arch"], n_layers=w["n_layers"], hidden=w["hidden"], n_heads=w["n_heads"],
                              head_dim=w["head_dim"], ffn=w["ffn"], tp=w["tp"], seq=w["seq"], mb=w["mb"], n_mb=w["n_mb"],
                              max_in_flight=max(max_in_flight, wgrad_group), recompute=w["recompute"] if recompute is None else recompute,
                              wgrad_group=wgrad_group, residual_fp32=w.get("res32", 0) if res32 is None else res32)
    ocfg = R.StageCfg(w["arch"], w["n_layers"], w["hidden"], nh, w["head_dim"], Fl, w["seq"],
                      1e-6 if w["arch"] == "llama" else 1e-5, 10000.0)
    return gcfg, ocfg


def load_params(stage, params):
    """params: list (per layer) of dict name -> float32 array holding bf16 values."""
    for l, p in enumerate(params):
        for name, arr in p.items():
            stage.param_view(l, name).copy_(to_dev(arr).view(stage.param_view(l, name).shape))


def run_gpu(stage, xs, dys, taps=None):
    """F0 B0 F1 B1 ... ; returns ys, dxs (numpy float64) and leaves grads in the stage.  Undeferred everything
    runs on slot 0; with deferred weight gradients a micro-batch keeps its slot until its group is taken, so the
    slots rotate, the input buffers are overwritten after each call (the library must have kept what it still
    needs) and an incomplete last group is flushed.  taps: a list that receives, per micro-batch, the outputs of
    layers 0 .. L-2 as the stage keeps them (bf16 device tensors: the inputs of layers 1 .. L-1)."""
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
        if taps is not None:
            taps.append([stage.layer_input(slot, l).clone() for l in range(1, stage.cfg.n_layers)])
        ys.append(to_np(y))
        dxs.append(to_np(dx))
    stage.flush_grads()
    torch.cuda.synchronize()
    return ys, dxs


def run_oracle(ocfg, params, xs, dys, dtype=np.float64, outs=None, progress=None):
    """outs: a list that receives every micro-batch's per-layer outputs; progress: called with a line of text after
    each pass (the full-size cases take minutes and report as they go)."""
    ps = [{k: v.astype(dtype, copy=False) for k, v in p.items()} for p in params]
    grads = R.zero_grads_like(ps)
    ys, dxs = [], []
    for m, (x, dy) in enumerate(zip(xs, dys)):
        y, caches, layer_ys = R.stage_fwd(ocfg, ps, x.astype(dtype, copy=False))
        if progress:
            progress("oracle forward of micro-batch %d done" % m)
        dxs.append(R.stage_bwd(ocfg, ps, caches, dy.astype(dtype, copy=False), grads))
        if progress:
            progress("oracle backward of micro-batch %d done" % m)
        ys.append(y)
        if outs is not None:
            outs.append(layer_ys)
    return ys, dxs, grads


def compare_stage(stage, params, ys, dxs, o_ys, o_dxs, o_grads, act_tol=ACT_TOL, grad_tol=GRAD_TOL, taps=None, o_outs=None,
                  report=None):
    """Gates, per compared tensor: normalised L2 (activations act_tol, gradients grad_tol); twice that bound on
    max |gpu - ref| / max |ref| and on every row of y and dx; TILE_TOL on every 128 x 128 tile of every matrix
    gradient (see the head of this file).  With taps / o_outs (run_gpu, run_oracle) each layer's output is gated
    like y.  Every view is evaluated before the first failure is raised, so that `report` (a dict, filled with the
    worst of every view) is complete.  Returns the worst tensor-level activation and gradient errors."""
    worst = {"act_l2": 0.0, "act_rows": 0.0, "act_maxabs": 0.0, "grad_l2": 0.0, "grad_tiles": 0.0, "grad_maxabs": 0.0, "layer_l2": []}
    bad = []

    def check(ok, msg):
        if not ok:
            bad.append(msg)

    def gate_act(what, got, ref):
        e = error_views(got, ref)
        worst.setdefault("act_l2_by_tensor", {})[what] = e["l2"]
        worst["act_l2"] = max(worst["act_l2"], e["l2"])
        if e["rows"] > worst["act_rows"]:
            worst["act_rows"], worst["act_rows_where"] = e["rows"], "%s, row %d" % (what, e["rows_argmax"])
        worst["act_maxabs"] = max(worst["act_maxabs"], e["maxabs"])
        check(e["l2"] <= act_tol, "%s: normalised L2 %g" % (what, e["l2"]))
        check(e["rows"] <= 2 * act_tol, "%s: row %d has normalised L2 %g" % (what, e["rows_argmax"], e["rows"]))
        check(e["maxabs"] <= 2 * act_tol, "%s: max abs error / max abs reference %g" % (what, e["maxabs"]))
        return e

    for m, (y, dx, oy, odx) in enumerate(zip(ys, dxs, o_ys, o_dxs)):
        gate_act("y of micro-batch %d" % m, y, oy)
        gate_act("dx of micro-batch %d" % m, dx, odx)
    if taps is not None and o_outs is not None:
        L = len(o_outs[0])
        per_layer = [0.0] * L
        for m, (tp, oo) in enumerate(zip(taps, o_outs)):
            assert len(tp) == L - 1
            for l in range(L - 1):
                per_layer[l] = max(per_layer[l], gate_act("output of layer %d, micro-batch %d" % (l, m), tp[l], oo[l])["l2"])
            per_layer[L - 1] = max(per_layer[L - 1], error_views(ys[m], oo[L - 1])["l2"])
        worst["layer_l2"] = per_layer
    for l, g in enumerate(o_grads):
        for name, ref in g.items():
            got = stage.grad_view(l, name)
            if not np.any(ref):
                check(float(got.abs().max()) == 0, "grad %s of layer %d: reference is zero, result is not" % (name, l))
                continue
            e = error_views(got, ref.reshape(tuple(got.shape)), tile=TILE if ref.ndim == 2 else None)
            worst["grad_l2"] = max(worst["grad_l2"], e["l2"])
            worst["grad_maxabs"] = max(worst["grad_maxabs"], e["maxabs"])
            worst.setdefault("grad_l2_by_tensor", {})["%d.%s" % (l, name)] = e["l2"]
            check(e["l2"] <= grad_tol, "grad %s of layer %d: normalised L2 %g" % (name, l, e["l2"]))
            check(e["maxabs"] <= 2 * grad_tol, "grad %s of layer %d: max abs error / max abs reference %g" % (name, l, e["maxabs"]))
            if "tiles" in e:
                if e["tiles"] > worst["grad_tiles"]:
                    worst["grad_tiles"], worst["grad_tiles_where"] = e["tiles"], "%s of layer %d, tile %s" % (name, l, e["tiles_argmax"])
                check(e["tiles"] <= TILE_TOL, "grad %s of layer %d: tile %s has normalised L2 %g" % (name, l, e["tiles_argmax"], e["tiles"]))
    if report is not None:
        report.update(worst)
    assert not bad, "%d gates failed, first: %s" % (len(bad), "; ".join(bad[:40]))
    return worst["act_l2"], worst["grad_l2"]
