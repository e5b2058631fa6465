"""One training step of a tiny stage captured into a HIP graph and replayed against eager steps (run as a child
process by tests/test_gpu_stage_parity.py, so that a fault inside the graph launch cannot take the test session down).
Usage: python -m tests.graph_replay_case <wgrad_group>"""
import sys

import torch

import paper_2512_20953_amd as P
from synth import stage_inputs as SI
from tests import gpu_util as U


def main(group):
    w = dict(SI.WORKLOADS["tiny"], n_mb=4)
    gcfg, _ = U.make_cfgs(w, max_in_flight=2, wgrad_group=group)
    params = [SI.draw_layer_params(w, l, perturb_vectors=True) for l in range(w["n_layers"])]
    xs = [SI.draw_activation(w, "x", m) for m in range(4)]
    dys = [SI.draw_activation(w, "dy", m) for m in range(4)]
    st = P.Stage(gcfg)
    U.load_params(st, params)
    xd, dyd = [U.to_dev(x) for x in xs], [U.to_dev(d) for d in dys]
    y, dx = [torch.empty_like(t) for t in xd], [torch.empty_like(t) for t in xd]
    s = torch.cuda.Stream()

    def step():
        st.zero_grads(s)
        for m in range(4):
            st.forward(m % 2, xd[m], y[m], s)
            st.backward(m % 2, dyd[m], dx[m], s)
        st.flush_grads(s)

    with torch.cuda.stream(s):
        step()                      # also creates the library's own stream and events, outside the capture
        torch.cuda.synchronize()
        want = (st.grads.clone(), [t.clone() for t in y + dx])
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            step()
        for rep in range(3):
            st.grads.fill_(float("nan"))
            for t in y + dx:
                t.zero_()
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(st.grads, want[0]), rep
            assert all(torch.equal(a, b) for a, b in zip(y + dx, want[1])), rep
            step()                  # eager work between replays
            torch.cuda.synchronize()
            assert torch.equal(st.grads, want[0]), rep
    # the graph goes before the stage whose stream it was captured on
    del g
    torch.cuda.synchronize()
    st.close()
    print("graph replay ok, wgrad_group", group, flush=True)


if __name__ == "__main__":
    main(int(sys.argv[1]))
