"""GPU parity of masked attention with the 1.5-entmax normaliser (Section 6) against the fp64
oracle: O within the forward tolerance (bf16 inputs and output, P rounded to bf16 before the
second product), tau within 1e-3, and the residual |sum p - 1| at the returned tau within the
bound the header states (1e-4: Newton's iteration stops a row at a residual <= 1e-5, or one
quadratically converging step after a residual <= 1e-2; scores are formed in fp32)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2012_02030_amd import binding as ap
from paper_2012_02030_amd import synth

from gpu_util import TOL, to_device

pytestmark = pytest.mark.gpu


def run_entmax(Q, K, V, mask, causal, scale=0.0):
    """Both walks (layout tiles, visit schedule) against the oracle."""
    dq, rq = to_device(Q, "bf16")
    dk, rk = to_device(K, "bf16")
    dv, rv = to_device(V, "bf16")
    lay = ap.ap_build_layout(torch.from_numpy(mask).cuda(), 64, 64)
    sched = ap.ap_build_schedule(lay, causal=causal)
    O_ref, tau_ref = oracle.masked_entmax15_attention(rq, rk, rv, mask, causal=causal, scale=scale)
    err = 0.0
    for sc in (None, sched):
        O, tau = ap.ap_sparse_attn_entmax15_fwd(dq, dk, dv, lay, causal=causal, softmax_scale=scale, sched=sc)
        torch.cuda.synchronize()
        err = max(err, check_entmax(O, tau, O_ref, tau_ref))
    return err


def check_entmax(O, tau, O_ref, tau_ref):
    Oh, th = O.double().cpu().numpy(), tau.double().cpu().numpy()
    assert np.isfinite(Oh).all()
    err = float(np.abs(Oh - O_ref).max())
    assert err <= TOL["bf16"], "max |O - oracle| = %.3e" % err
    empty = np.isinf(tau_ref)
    assert np.array_equal(np.isinf(th), empty)
    if (~empty).any():
        terr = float(np.abs(th[~empty] - tau_ref[~empty]).max())
        assert terr <= 1e-3, "max |tau - oracle| = %.3e" % terr
    return err


def rand_qkv(seed, B, H, Lq, Lk, D, gain=1.0):
    rng = np.random.default_rng([synth.SEED, 1515, seed])
    return (gain * rng.standard_normal((B, H, Lq, D), dtype=np.float32),
            rng.standard_normal((B, H, Lk, D), dtype=np.float32),
            rng.standard_normal((B, H, Lk, D), dtype=np.float32))


ENTMAX_CASES = [
    # B, H, Lq, Lk, D, causal, density, query gain (sharper scores -> smaller supports)
    (2, 2, 128, 128, 64, False, 0.5, 1.0),
    (1, 2, 200, 200, 64, True, 0.3, 3.0),
    (1, 2, 100, 157, 32, False, 0.3, 1.0),
    (1, 2, 100, 300, 128, True, 0.2, 0.2),      # nearly equal scores: large supports
    (1, 1, 192, 192, 128, False, 1.0, 1.0),     # nothing pruned
    (1, 2, 64, 64, 64, True, 0.05, 1.0),        # empty rows
    (1, 1, 1, 1, 32, False, 1.0, 1.0),
]


@pytest.mark.parametrize("case", ENTMAX_CASES, ids=lambda c: "B%d_H%d_%dx%d_D%d_%s_g%g" % (c[:5] + ("causal" if c[5] else "full", c[7])))
def test_entmax_forward_matches_oracle(case):
    B, H, Lq, Lk, D, causal, density, gain = case
    Q, K, V = rand_qkv(Lq + Lk + D, B, H, Lq, Lk, D, gain)
    mask = synth.random_mask(H, Lq, Lk, density, seed=Lq + D)
    run_entmax(Q, K, V, mask, causal)


@pytest.mark.parametrize("case", ENTMAX_CASES[:5], ids=lambda c: "%dx%d_D%d_g%g" % (c[2], c[3], c[4], c[7]))
def test_entmax_returned_tau_leaves_the_documented_residual(case):
    """sum_j [x_ij - tau_i]_+^2 recomputed in fp64 from the returned tau (scores from the same
    bf16-rounded inputs) is within 1e-4 of 1 for every query with a visible kept key, for both
    walks."""
    B, H, Lq, Lk, D, causal, density, gain = case
    Q, K, V = rand_qkv(Lq + Lk + D, B, H, Lq, Lk, D, gain)
    mask = synth.random_mask(H, Lq, Lk, density, seed=Lq + D)
    dq, rq = to_device(Q, "bf16")
    dk, rk = to_device(K, "bf16")
    dv, _ = to_device(V, "bf16")
    lay = ap.ap_build_layout(torch.from_numpy(mask).cuda(), 64, 64)
    sched = ap.ap_build_schedule(lay, causal=causal)
    keep = mask != 0
    if causal:
        keep = keep & (np.arange(Lk)[None, :] <= np.arange(Lq)[:, None] + (Lk - Lq))[None]
    x = np.einsum("bhid,bhjd->bhij", rq, rk) / (2.0 * np.sqrt(D))
    for sc in (None, sched):
        _, tau = ap.ap_sparse_attn_entmax15_fwd(dq, dk, dv, lay, causal=causal, sched=sc)
        torch.cuda.synchronize()
        th = tau.double().cpu().numpy()
        u = np.where(keep[None], np.maximum(x - th[..., None], 0.0), 0.0)
        total = (u * u).sum(-1)
        rows = keep.any(-1)[None].repeat(B, 0)
        resid = float(np.abs(total[rows] - 1.0).max())
        assert resid <= 1e-4, "max |sum p - 1| = %.3e" % resid


def test_entmax_zero_queries_give_the_mean_of_kept_values():
    Q, K, V = rand_qkv(3, 1, 2, 96, 96, 64)
    mask = synth.random_mask(2, 96, 96, 0.4, seed=8)
    run_entmax(0.0 * Q, K, V, mask, False)


def test_entmax_on_a_structured_mask_and_explicit_scale():
    cfg = synth.CONFIGS["C3"]
    mask = np.stack([synth.head_mask(cfg, h) for h in range(2)]).astype(np.uint8)
    Q, K, V = rand_qkv(5, 1, 2, cfg.Lq, cfg.Lk, cfg.D, 2.0)
    run_entmax(Q, K, V, mask, True, scale=0.2)


def test_entmax_full_size_c5_two_slices_against_oracle():
    """The benchmark's shape (B4 H16 L4096 D128 causal, C5's mask): two (example, head) slices
    element by element, and the rows of every slice are finite."""
    cfg = synth.CONFIGS["C5"]
    mask = synth.make_mask(cfg)
    Q, K, V = synth.make_qkv(cfg)
    dq, dk, dv = (torch.from_numpy(x).to(torch.bfloat16).cuda() for x in (Q, K, V))
    lay = ap.ap_build_layout(torch.from_numpy(mask).cuda(), 64, 64)
    sched = ap.ap_build_schedule(lay, causal=True)
    O, tau = ap.ap_sparse_attn_entmax15_fwd(dq, dk, dv, lay, causal=True, sched=sched)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(O).all()) and bool(torch.isfinite(tau).all())
    for b, h in ((0, 1), (3, 14)):
        sl = lambda t: t[b:b + 1, h:h + 1].double().cpu().numpy()
        rows = slice(0, cfg.Lq, 7)                               # every 7th query keeps the oracle quick
        O_ref, tau_ref = oracle.masked_entmax15_attention(sl(dq)[:, :, rows], sl(dk), sl(dv),
                                                          _rows_mask(mask[h:h + 1], rows, cfg), causal=False)
        assert np.abs(sl(O)[:, :, rows] - O_ref).max() <= TOL["bf16"]
        assert np.abs(sl(tau)[:, :, rows] - tau_ref).max() <= 1e-3


def _rows_mask(mask_h, rows, cfg):
    """Mask rows of the sampled queries with the causal limit folded in (the oracle is then called
    without its causal flag, which would align a query subset differently)."""
    i = np.arange(cfg.Lq)[rows][:, None]
    j = np.arange(cfg.Lk)[None, :]
    return (mask_h[:, rows, :] != 0) & (j <= i + (cfg.Lk - cfg.Lq))[None]


def test_entmax_block_row_with_more_than_64_schedule_entries():
    """Dense 64 x 5000 mask: 79 consecutive entries in the one block row, more than the kernel
    keeps gather keys for, so it walks the layout's tiles."""
    Q, K, V = rand_qkv(11, 1, 1, 64, 5000, 64)
    mask = np.ones((1, 64, 5000), np.uint8)
    run_entmax(Q, K, V, mask, False)


def test_entmax_block_row_with_more_than_16_gathered_entries():
    """Sparse 64 x 3000 mask (2 % kept, about 45 distinct columns per tile): every tile of the one
    block row is packed, into more gathered entries than the kernel keeps keys for in LDS, so it
    walks the layout's tiles; a 64 x 900 mask of the same kind stays within the limit."""
    for Lk, seed in ((3000, 12), (900, 13)):
        print("entmax gathered", Lk, flush=True)
        Q, K, V = rand_qkv(seed, 1, 1, 64, Lk, 64, gain=2.0)
        mask = synth.random_mask(1, 64, Lk, 0.02, seed=seed)
        lay = ap.ap_build_layout(torch.from_numpy(mask).cuda(), 64, 64)
        sched = ap.ap_build_schedule(lay, causal=False)
        torch.cuda.synchronize()
        n_gathered = int((sched.start[: int(sched.cnt[0].item())] < 0).sum().item())
        assert (n_gathered > 16) == (Lk == 3000), n_gathered
        run_entmax(Q, K, V, mask, False)
