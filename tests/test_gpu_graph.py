"""The library's calls under HIP graph capture: a captured forward call (and a captured backward
call) is replayed several times, with new inputs written into the same buffers, eager work of the
program and synchronisations between the replays, and every replay is compared bit for bit with the
eager call on the same inputs.  (The calls launch kernels only: no allocation and no memset is
recorded when the caller passes outputs and workspaces.)"""
import numpy as np
import pytest
import torch

from paper_2012_02030_amd import binding as ap
from paper_2012_02030_amd import synth

pytestmark = pytest.mark.gpu


def fresh(shape, seed, dtype):
    rng = np.random.default_rng([synth.SEED, 4242, seed])
    return torch.from_numpy(rng.standard_normal(shape, dtype=np.float32)).to(dtype).cuda()


@pytest.mark.parametrize("dtype,D,causal", [(torch.bfloat16, 64, True), (torch.bfloat16, 128, False),
                                            (torch.float32, 32, True)])
def test_forward_graph_replays_match_eager(dtype, D, causal):
    B, H, Lq, Lk = 2, 3, 200, 264
    mask = synth.random_mask(H, Lq, Lk, 0.2, seed=D)
    lay = ap.ap_build_layout(torch.from_numpy(mask).cuda(), 64, 64)
    sched = ap.ap_build_schedule(lay, causal=causal) if dtype == torch.bfloat16 else None
    q, k, v = fresh((B, H, Lq, D), 1, dtype), fresh((B, H, Lk, D), 2, dtype), fresh((B, H, Lk, D), 3, dtype)
    out = torch.empty_like(q)
    lse = torch.empty((B, H, Lq), dtype=torch.float32, device="cuda")

    def call():
        ap.ap_sparse_attn_fwd(q, k, v, lay, causal=causal, out=out, lse=lse, sched=sched)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call()                                               # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        call()
    for rep in range(4):
        print("graph replay", dtype, D, rep, flush=True)
        q.copy_(fresh(tuple(q.shape), 10 + rep, dtype))      # new inputs in the captured buffers
        v.copy_(fresh(tuple(v.shape), 20 + rep, dtype))
        out.zero_()
        lse.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got_o, got_l = out.clone(), lse.clone()
        O_e, lse_e = ap.ap_sparse_attn_fwd(q, k, v, lay, causal=causal, sched=sched)   # eager, own outputs
        torch.cuda.synchronize()
        assert torch.equal(got_o, O_e), "replay %d differs from the eager call" % rep
        assert torch.equal(got_l, lse_e)


def test_backward_graph_replays_match_eager():
    B, H, Lq, Lk, D = 1, 2, 192, 192, 64
    mask = synth.random_mask(H, Lq, Lk, 0.3, seed=9)
    lay = ap.ap_build_layout(torch.from_numpy(mask).cuda(), 64, 64)
    lay_t = ap.ap_build_layout_transpose(lay)
    sched = ap.ap_build_schedule(lay, causal=True)
    csched = ap.ap_build_col_schedule(lay, lay_t, causal=True)
    bf = torch.bfloat16
    q, k, v = fresh((B, H, Lq, D), 1, bf), fresh((B, H, Lk, D), 2, bf), fresh((B, H, Lk, D), 3, bf)
    do = fresh((B, H, Lq, D), 4, bf)
    O, lse = ap.ap_sparse_attn_fwd(q, k, v, lay, causal=True, sched=sched)
    torch.cuda.synchronize()

    def eager():
        return ap.ap_sparse_attn_bwd(q, k, v, O, do, lse, lay, lay_t, causal=True, sched=sched, col_sched=csched)

    ref = [t.clone() for t in eager()]
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        eager()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        outs = eager()                                       # outputs and workspace come from the graph's pool
    for rep in range(3):
        print("backward graph replay", rep, flush=True)
        for t in outs:
            t.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for got, want in zip(outs, ref):
            assert torch.equal(got, want), "replay %d differs from the eager call" % rep
        _ = (q.float() @ k.float().transpose(-1, -2)).sum().item()   # eager work between replays
