"""One layout for every sequence length (Section 6: lengths vary across a data set while a layer's
masks are fixed): ap_sparse_attn_fwd_cropped under the top-left corner of a stored mask, against
the fp64 oracle evaluated on that corner of the mask.  The layout and the visit schedule are built
once, for the full stored size."""
import numpy as np
import pytest
import torch

import oracle
from paper_2012_02030_amd import binding as ap
from paper_2012_02030_amd import synth

from gpu_util import TOL, to_device

pytestmark = pytest.mark.gpu


def stored_mask(H, Lq, Lk, seed, causal):
    """Band next to the (bottom-right aligned) diagonal, a sink column and isolated connections."""
    rng = np.random.default_rng([synth.SEED, 606, seed])
    i = np.arange(Lq)[:, None] + (Lk - Lq)
    j = np.arange(Lk)[None, :]
    m = (np.abs(i - j) < 24) | (j == 0) | (rng.random((H, Lq, Lk)) < 0.02)
    return np.broadcast_to(m, (H, Lq, Lk)).astype(np.uint8).copy()


def run_crop(mask, Lq, Lk, D, causal, bm, use_sched, seed, B=2):
    H = mask.shape[0]
    rng = np.random.default_rng([synth.SEED, 607, seed])
    Q, K, V = (rng.standard_normal(s, dtype=np.float32) for s in ((B, H, Lq, D), (B, H, Lk, D), (B, H, Lk, D)))
    dq, rq = to_device(Q, "bf16")
    dk, rk = to_device(K, "bf16")
    dv, rv = to_device(V, "bf16")
    lay = ap.ap_build_layout(torch.from_numpy(mask).cuda(), bm, 64)       # once, full stored size
    sched = ap.ap_build_schedule(lay, causal=causal) if use_sched else None
    print("crop", mask.shape, "->", (Lq, Lk), "D", D, "causal", causal, "bm", bm, "sched", use_sched, flush=True)
    O, lse = ap.ap_sparse_attn_fwd(dq, dk, dv, lay, causal=causal, sched=sched, crop=True)
    torch.cuda.synchronize()
    corner = np.ascontiguousarray(mask[:, :Lq, :Lk])
    O_ref, lse_ref = oracle.masked_attention(rq, rk, rv, corner, causal=causal)
    Oh, lh = O.double().cpu().numpy(), lse.double().cpu().numpy()
    assert np.isfinite(Oh).all()
    err = float(np.abs(Oh - O_ref).max())
    assert err <= TOL["bf16"], "max |O - oracle| = %.3e" % err
    empty = np.isneginf(lse_ref)
    assert np.array_equal(np.isneginf(lh), empty)
    if (~empty).any():
        assert float(np.abs(lh[~empty] - lse_ref[~empty]).max()) <= TOL["bf16"]


@pytest.mark.parametrize("use_sched", [False, True])
@pytest.mark.parametrize("bm", [64, 128])
def test_causal_self_attention_cropped_to_shorter_lengths(bm, use_sched):
    mask = stored_mask(2, 300, 300, 1, True)
    for L, D in ((300, 64), (257, 128), (200, 64), (64, 128), (63, 32), (1, 64)):
        run_crop(mask, L, L, D, True, bm, use_sched, seed=L)


@pytest.mark.parametrize("use_sched", [False, True])
def test_cross_attention_cropped_in_both_directions(use_sched):
    mask = stored_mask(3, 200, 330, 2, False)
    mask[:, :, 100:] |= synth.random_mask(3, 200, 230, 0.3, seed=9)      # dense region beyond some crops
    for (Lq, Lk), D in (((200, 330), 64), ((130, 330), 128), ((200, 100), 64), ((70, 65), 128), ((200, 129), 32)):
        run_crop(mask, Lq, Lk, D, False, 64, use_sched, seed=Lq + Lk)


def test_causal_memory_layout_cropped_without_a_schedule():
    """Few queries against a longer memory, bottom-right aligned; the call's own offset applies."""
    mask = stored_mask(2, 100, 300, 3, True)
    for Lq, Lk in ((100, 300), (50, 120), (100, 100), (10, 299)):
        run_crop(mask, Lq, Lk, 64, True, 64, False, seed=Lq * Lk)


def test_gathered_keys_beyond_the_cropped_length_are_hidden():
    """Isolated connections only: every entry is gathered, and most gathered keys lie beyond Lk."""
    mask = synth.random_mask(2, 128, 2000, 0.01, seed=4)
    mask[:, :, 0] = 1
    for Lk in (2000, 700, 65, 3):
        run_crop(mask, 128, Lk, 64, False, 64, True, seed=Lk)


def test_cropped_call_rejects_what_it_cannot_do():
    mask = stored_mask(1, 128, 256, 5, True)
    lay = ap.ap_build_layout(torch.from_numpy(mask).cuda(), 64, 64)
    sched = ap.ap_build_schedule(lay, causal=True)
    q = torch.zeros((1, 1, 64, 64), dtype=torch.bfloat16, device="cuda")
    k = torch.zeros((1, 1, 100, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(ap.ApError) as e:                                  # offset 36 against the schedule's 128
        ap.ap_sparse_attn_fwd(q, k, k.clone(), lay, causal=True, sched=sched, crop=True)
    assert e.value.status == ap.AP_ERR_INVALID_ARG
    with pytest.raises(ValueError):                                       # not asked for
        ap.ap_sparse_attn_fwd(q, k, k.clone(), lay, causal=True)
    k2 = torch.zeros((1, 1, 300, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(ValueError):                                       # larger than the layout
        ap.ap_sparse_attn_fwd(q, k2, k2.clone(), lay, causal=True, crop=True)
    qf, kf = q.float(), k.float()
    with pytest.raises(ap.ApError) as e:
        ap.ap_sparse_attn_fwd(qf, kf, kf.clone(), lay, causal=True, crop=True)
    assert e.value.status == ap.AP_ERR_UNSUPPORTED
