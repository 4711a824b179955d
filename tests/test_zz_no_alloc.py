"""The allocation-free split forward call (ap_sparse_attn_fwd_split_static) against the ordinary
split call: same kernels, so the results must agree bit for bit; two calls in a row share the
library's one scratch array, the second with a smaller input."""
import numpy as np
import pytest
import torch

import oracle
from paper_2012_02030_amd import binding as ap
from paper_2012_02030_amd import synth

from gpu_util import TOL, to_device

pytestmark = pytest.mark.gpu


def _case(seed, B, H, Lq, Lk, D, density, causal, splits, use_sched):
    rng = np.random.default_rng([synth.SEED, 777, seed])
    Q, K, V = (rng.standard_normal(s, dtype=np.float32) for s in ((B, H, Lq, D), (B, H, Lk, D), (B, H, Lk, D)))
    mask = synth.random_mask(H, Lq, Lk, density, seed=seed)
    dq, rq = to_device(Q, "bf16")
    dk, rk = to_device(K, "bf16")
    dv, rv = to_device(V, "bf16")
    lay = ap.ap_build_layout(torch.from_numpy(mask).cuda(), 64, 64)
    sched = ap.ap_build_schedule(lay, causal=causal) if use_sched else None
    want_O, want_lse = ap.ap_sparse_attn_fwd_split(dq, dk, dv, lay, splits, causal=causal, sched=sched)
    ref = oracle.masked_attention(rq, rk, rv, mask, causal=causal)
    out = torch.full_like(dq, float("nan"))
    lse = torch.full((B, H, Lq), float("nan"), dtype=torch.float32, device="cuda")
    return (dq, dk, dv, lay, splits, out, lse, causal, sched), (want_O, want_lse), ref


def _check(got, want, ref, what):
    O, lse = got
    assert torch.equal(O, want[0]), what + ": O differs from the workspace call"
    assert torch.equal(lse, want[1]), what + ": lse differs from the workspace call"
    err = float(np.abs(O.double().cpu().numpy() - ref[0]).max())
    assert err <= TOL["bf16"], (what, err)
    fin = np.isfinite(ref[1])
    assert float(np.abs(lse.double().cpu().numpy()[fin] - ref[1][fin]).max()) <= TOL["bf16"]


def test_static_split_call_matches_the_workspace_call_twice_in_a_row():
    big = _case(1, 2, 4, 100, 2048, 128, 0.3, True, 8, True)
    small = _case(2, 1, 2, 64, 700, 64, 0.2, False, 3, False)
    torch.cuda.synchronize()
    for name, (args, want, ref) in (("first call", big), ("second, smaller call", small)):
        print("static split:", name, flush=True)
        dq, dk, dv, lay, splits, out, lse, causal, sched = args
        got = ap.ap_sparse_attn_fwd_split_static(dq, dk, dv, lay, splits, out, lse, causal=causal, sched=sched)
        torch.cuda.synchronize()
        _check(got, want, ref, name)


def test_static_split_call_rejects_what_does_not_fit():
    q = torch.zeros((4, 16, 64, 128), dtype=torch.bfloat16, device="cuda")
    k = torch.zeros((4, 16, 128, 128), dtype=torch.bfloat16, device="cuda")
    lay = ap.ap_build_layout(torch.ones((16, 64, 128), dtype=torch.uint8, device="cuda"), 64, 64)
    with pytest.raises(ap.ApError) as e:
        ap.ap_sparse_attn_fwd_split_static(q, k, k, lay, 16, torch.empty_like(q))
    assert e.value.status == ap.AP_ERR_CAPACITY
