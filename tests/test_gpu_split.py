"""GPU parity of the split forward call (few queries against many keys, Section 4.1's
Transformer-XL setting: a short segment attends to a long memory, causal limit bottom-right)
against the fp64 oracle, and agreement with the ordinary call."""
import numpy as np
import pytest
import torch

import oracle
from paper_2012_02030_amd import binding as ap
from paper_2012_02030_amd import synth

from gpu_util import TOL, to_device

pytestmark = pytest.mark.gpu


def run_split(B, H, Lq, Lk, D, causal, density, splits, use_sched, seed):
    rng = np.random.default_rng([synth.SEED, 31337, seed])
    Q = rng.standard_normal((B, H, Lq, D), dtype=np.float32)
    K = rng.standard_normal((B, H, Lk, D), dtype=np.float32)
    V = rng.standard_normal((B, H, Lk, D), dtype=np.float32)
    mask = synth.random_mask(H, Lq, Lk, density, seed=seed)
    dq, rq = to_device(Q, "bf16")
    dk, rk = to_device(K, "bf16")
    dv, rv = to_device(V, "bf16")
    lay = ap.ap_build_layout(torch.from_numpy(mask).cuda(), 64, 64)
    sched = ap.ap_build_schedule(lay, causal=causal) if use_sched else None
    O, lse = ap.ap_sparse_attn_fwd_split(dq, dk, dv, lay, splits, causal=causal, sched=sched)
    O1, lse1 = ap.ap_sparse_attn_fwd(dq, dk, dv, lay, causal=causal, sched=sched)
    torch.cuda.synchronize()
    O_ref, lse_ref = oracle.masked_attention(rq, rk, rv, mask, causal=causal)
    Oh, lh = O.double().cpu().numpy(), lse.double().cpu().numpy()
    assert np.isfinite(Oh).all()
    assert np.abs(Oh - O_ref).max() <= TOL["bf16"]
    empty = np.isneginf(lse_ref)
    assert np.array_equal(np.isneginf(lh), empty)
    if (~empty).any():
        assert np.abs(lh[~empty] - lse_ref[~empty]).max() <= TOL["bf16"]
    # against the ordinary call: same inputs, other summation order and one more rounding
    assert float((O.float() - O1.float()).abs().max()) <= TOL["bf16"]


SPLIT_CASES = [
    # B, H, Lq, Lk, D, causal, density, splits, schedule
    (2, 3, 1, 2000, 64, True, 0.3, 8, False),
    (2, 3, 1, 2000, 64, True, 0.1, 8, True),
    (1, 2, 16, 4096, 128, True, 0.1, 16, True),
    (1, 2, 64, 1000, 128, False, 0.5, 5, False),
    (1, 2, 100, 3000, 32, True, 0.05, 7, True),       # two block rows, ragged
    (1, 1, 8, 300, 64, True, 0.02, 64, False),        # more splits than tiles: empty chunks
    (1, 1, 8, 640, 64, False, 1.0, 1, False),         # splits = 1
    # more than 128 and more than 192 entries in one workgroup's walk: the window of entry starts
    # that a wavefront keeps in registers moves on once and twice
    (1, 1, 40, 9000, 128, False, 0.5, 1, True),
    (1, 1, 40, 9000, 64, True, 0.5, 1, False),
    (1, 1, 8, 13000, 128, False, 0.5, 1, True),
    (1, 1, 8, 13000, 32, True, 0.5, 2, False),
]


@pytest.mark.parametrize("case", SPLIT_CASES, ids=lambda c: "B%d_H%d_%dx%d_D%d_s%d" % (c[:5] + (c[7],)))
def test_split_forward_matches_oracle(case):
    B, H, Lq, Lk, D, causal, density, splits, use_sched = case
    run_split(B, H, Lq, Lk, D, causal, density, splits, use_sched, seed=Lk + splits)


def test_split_forward_rows_without_kept_keys():
    B, H, Lq, Lk, D = 1, 1, 4, 512, 64
    rng = np.random.default_rng(5)
    Q, K, V = (rng.standard_normal(s, dtype=np.float32) for s in ((B, H, Lq, D), (B, H, Lk, D), (B, H, Lk, D)))
    mask = synth.random_mask(H, Lq, Lk, 0.2, seed=9)
    mask[0, 2, :] = 0
    dq, rq = to_device(Q, "bf16")
    dk, rk = to_device(K, "bf16")
    dv, rv = to_device(V, "bf16")
    lay = ap.ap_build_layout(torch.from_numpy(mask).cuda(), 64, 64)
    O, lse = ap.ap_sparse_attn_fwd_split(dq, dk, dv, lay, 4)
    torch.cuda.synchronize()
    assert float(O[0, 0, 2].float().abs().max()) == 0.0 and bool(torch.isneginf(lse[0, 0, 2]))
    O_ref, _ = oracle.masked_attention(rq, rk, rv, mask)
    assert np.abs(O.double().cpu().numpy() - O_ref).max() <= TOL["bf16"]
