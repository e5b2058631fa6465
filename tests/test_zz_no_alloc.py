"""The entry point that allocates nothing (ah_attention_bwd_static: the scratch of attention backward lives in the
library's device image) against ah_attention_bwd with a caller-supplied scratch buffer, through the C ABI: same
kernels, so the outputs must agree bit for bit; two calls in a row, the second on a smaller input (the array keeps the
first call's contents); sizes beyond the fixed maximum are refused before anything is launched."""
import numpy as np
import pytest
import torch

import paper_2512_20953_amd as P
from synth import stage_inputs as SI
from tests import gpu_util as U

pytestmark = pytest.mark.gpu


def _case(B, S, nh, d, causal, seed):
    rng = np.random.default_rng(seed)
    T, hl = B * S, nh * d
    qkv = U.to_dev(SI.round_bf16(rng.standard_normal((T, 3 * hl), dtype=np.float32)))
    d_o = U.to_dev(SI.round_bf16(rng.standard_normal((T, hl), dtype=np.float32)))
    o = torch.empty(T, hl, dtype=torch.bfloat16, device="cuda")
    lse = torch.empty(B * nh * S, dtype=torch.float32, device="cuda")
    P.attention_fwd(qkv, o, lse, B, S, nh, d, causal)
    want = torch.full((T, 3 * hl), float("nan"), dtype=torch.bfloat16, device="cuda")
    delta = torch.empty(B * nh * S, dtype=torch.float32, device="cuda")
    P.attention_bwd(qkv, o, lse, d_o, want, delta, B, S, nh, d, causal)
    torch.cuda.synchronize()
    return qkv, o, lse, d_o, want


def test_static_scratch_entry_point_matches_the_one_with_a_caller_buffer():
    big = (2, 512, 4, 128, True)
    small = (1, 256, 2, 64, False)
    cases = [(_case(*big, seed=21), big), (_case(*small, seed=22), small)]
    free_before = torch.cuda.mem_get_info()[0]
    for (qkv, o, lse, d_o, want), (B, S, nh, d, causal) in cases:      # two calls in a row, the second smaller
        got = torch.full_like(want, float("nan"))
        P.attention_bwd_static(qkv, o, lse, d_o, got, B, S, nh, d, causal)
        torch.cuda.synchronize()
        assert torch.isfinite(got.float()).all()
        assert torch.equal(got.view(torch.int16), want.view(torch.int16)), (B, S, nh, d, causal)
    # and once more on the first input: what the smaller call left in the array does not leak into a larger one
    (qkv, o, lse, d_o, want), (B, S, nh, d, causal) = cases[0]
    got = torch.full_like(want, float("nan"))
    P.attention_bwd_static(qkv, o, lse, d_o, got, B, S, nh, d, causal)
    torch.cuda.synchronize()
    assert torch.equal(got.view(torch.int16), want.view(torch.int16))
    del got
    assert torch.cuda.mem_get_info()[0] >= free_before - (64 << 20)    # nothing of the order of the inputs was allocated behind the call


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    B, S, nh, d = 2, 2048, 128, 64          # 524288 rows of scratch: twice the fixed array
    assert B * S * nh > P.ATTENTION_STATIC_MAX_ROWS
    t = torch.zeros(8, dtype=torch.bfloat16, device="cuda")    # never touched: the call must fail before any launch
    f = torch.zeros(8, dtype=torch.float32, device="cuda")
    with pytest.raises(P.AhError) as e:
        P.attention_bwd_static(t, t, f, t, t, B, S, nh, d, True)
    assert e.value.status == 1 and "exceeds" in str(e.value)
    torch.cuda.synchronize()
