"""GPU parity of the backward pass of masked attention with the 1.5-entmax normaliser (Section 6)
against the fp64 oracle.

Tolerance: as for the softmax backward pass (P, dS and the results are rounded to bf16; the bar is
max-abs error <= 2e-2 * max(1, max|oracle gradient|), per tensor and per row).  The forward
pass's tau leaves |sum p - 1| <= 1e-4 (tests/test_gpu_entmax.py), and the backward pass forms
p = u^2 from it without renormalising: far below that bar.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2012_02030_amd import binding as ap
from paper_2012_02030_amd import synth

from gpu_util import assert_grad_close, to_device
from test_gpu_bwd import BWD_CASES, rand_inputs

pytestmark = pytest.mark.gpu


def run_entmax_bwd(Q, K, V, dO, mask_np, causal, scale=0.0, min_cols=0, min_rows=0):
    dq, rq = to_device(Q, "bf16")
    dk, rk = to_device(K, "bf16")
    dv, rv = to_device(V, "bf16")
    dg, rg = to_device(dO, "bf16")
    lay = ap.ap_build_layout(torch.from_numpy(mask_np).cuda(), 64, 64)
    lt = ap.ap_build_layout_transpose(lay)
    rs = ap.ap_build_schedule(lay, causal=causal, min_cols=min_cols)
    cs = ap.ap_build_col_schedule(lay, lt, causal=causal, min_rows=min_rows)
    _, tau = ap.ap_sparse_attn_entmax15_fwd(dq, dk, dv, lay, causal=causal, softmax_scale=scale, sched=rs)
    print("entmax bwd", Q.shape, K.shape, "causal" if causal else "full", flush=True)
    got3 = ap.ap_sparse_attn_entmax15_bwd(dq, dk, dv, dg, tau, lay, lt, rs, cs, causal=causal, softmax_scale=scale)
    torch.cuda.synchronize()
    ref = oracle.masked_entmax15_attention_backward(rq, rk, rv, mask_np, rg, causal=causal, scale=scale)
    for name, got, want in zip(("dQ", "dK", "dV"), got3, ref):
        assert_grad_close(name, got.double().cpu().numpy(), want)


@pytest.mark.parametrize("case", BWD_CASES, ids=lambda c: "B%d_H%d_%dx%d_D%d_%s_%g" % (c[:5] + ("causal" if c[5] else "full", c[6])))
def test_entmax_backward_matches_oracle(case):
    B, H, Lq, Lk, D, causal, density = case
    Q, K, V, dO = rand_inputs(Lq + Lk + D + 1, B, H, Lq, Lk, D)
    mask = synth.random_mask(H, Lq, Lk, density, seed=D + Lq + 1)
    run_entmax_bwd(Q, K, V, dO, mask, causal)


@pytest.mark.parametrize("mins", [(1, 1), (65, 65)])
def test_entmax_backward_any_packing_and_sharp_scores(mins):
    """All entries consecutive / all gathered; scores scaled up so that supports are small."""
    Q, K, V, dO = rand_inputs(23, 2, 2, 200, 260, 64)
    mask = synth.random_mask(2, 200, 260, 0.1, seed=78)
    mask[:, 50:120, 64:128] = 1
    run_entmax_bwd(2.0 * Q, 2.0 * K, V, dO, mask, True, scale=0.3, min_cols=mins[0], min_rows=mins[1])


def test_entmax_backward_on_the_structured_mask():
    cfg = synth.CONFIGS["C3"]
    mask = np.stack([synth.head_mask(cfg, h) for h in range(2)]).astype(np.uint8)
    Q, K, V, dO = rand_inputs(8, 1, 2, cfg.Lq, cfg.Lk, cfg.D)
    run_entmax_bwd(Q, K, V, dO, mask, cfg.causal)


def test_entmax_backward_full_size_c5_one_slice_against_oracle():
    """The benchmark's shape and launch configuration (B4 H16 L4096 D128 causal, C5's mask)."""
    cfg = synth.CONFIGS["C5"]
    mask = synth.make_mask(cfg)
    Q, K, V = synth.make_qkv(cfg)
    dO = np.random.default_rng([synth.SEED, 4244]).standard_normal(Q.shape, dtype=np.float32)
    dq, dk, dv, dg = (torch.from_numpy(x).to(torch.bfloat16).cuda() for x in (Q, K, V, dO))
    lay = ap.ap_build_layout(torch.from_numpy(mask).cuda(), 64, 64)
    lt = ap.ap_build_layout_transpose(lay)
    rs = ap.ap_build_schedule(lay, causal=True)
    cs = ap.ap_build_col_schedule(lay, lt, causal=True)
    _, tau = ap.ap_sparse_attn_entmax15_fwd(dq, dk, dv, lay, causal=True, sched=rs)
    gQ, gK, gV = ap.ap_sparse_attn_entmax15_bwd(dq, dk, dv, dg, tau, lay, lt, rs, cs, causal=True)
    torch.cuda.synchronize()
    for t in (gQ, gK, gV):
        assert bool(torch.isfinite(t).all())
    b, h = 2, 5
    sl = lambda t: t[b:b + 1, h:h + 1].double().cpu().numpy()
    ref = oracle.masked_entmax15_attention_backward(sl(dq), sl(dk), sl(dv), mask[h:h + 1], sl(dg), causal=True)
    for name, got, want in zip(("dQ", "dK", "dV"), (gQ, gK, gV), ref):
        print("C5 entmax bwd", name, assert_grad_close(name, sl(got), want, "[%d,%d]" % (b, h)), flush=True)
