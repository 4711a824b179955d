"""GPU parity of mask construction (Section 3.2, Eq. (1) and Eq. (2)) against the fp64 oracle.

Mean maps: max-abs error at most MAP_TOL per unit of weight * B.  Both sides start from the same
bf16 inputs; the kernel forms the scores in fp32 on the matrix cores (relative error of a score
about 2^-23 * sqrt(D), absolute about 5e-5 for |s| ~ 40), takes exp2 and log2 with the
hardware approximations (about 2^-22 relative) and sums B probabilities <= 1 in fp32, so a
probability is off by at most about 1e-4 of itself.
Threshold and mask: bit-exact on the same float32 input; so is the layout built straight from the
map and the threshold (ap_build_layout_from_map) against the layout oracle on the oracle's mask.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2012_02030_amd import binding as ap
from paper_2012_02030_amd import synth

from gpu_util import assert_layout_equal, to_device

pytestmark = pytest.mark.gpu
MAP_TOL = 1e-4


def run_maps(Q, K, causal, scale=0.0, weight=None, abar=None):
    dq, rq = to_device(Q, "bf16")
    dk, rk = to_device(K, "bf16")
    B = Q.shape[0]
    weight = 1.0 / B if weight is None else weight
    out = ap.ap_accumulate_attention_maps(dq, dk, abar=abar, causal=causal, softmax_scale=scale,
                                          weight=weight)
    torch.cuda.synchronize()
    return out, rq, rk


MAP_CASES = [
    # B, H, Lq, Lk, D, causal
    (3, 2, 200, 200, 64, False),
    (3, 2, 200, 200, 64, True),
    (2, 3, 100, 300, 32, False),
    (2, 3, 100, 300, 32, True),
    (2, 1, 192, 192, 128, True),
    (2, 2, 70, 157, 64, False),        # Lk not a multiple of 4: element-wise update path
    (2, 2, 70, 157, 64, True),
    (1, 1, 1, 1, 32, True),
    (5, 1, 64, 64, 128, False),
]


@pytest.mark.parametrize("case", MAP_CASES, ids=lambda c: "B%d_H%d_%dx%d_D%d_%s" % (c[:5] + ("causal" if c[5] else "full",)))
def test_mean_map_matches_oracle(case):
    B, H, Lq, Lk, D, causal = case
    Q, K = synth.make_qk_positional(B, H, Lq, Lk, D, seed=Lq + Lk + D)
    abar, rq, rk = run_maps(Q, K, causal)
    ref = oracle.mean_attention_map(rq, rk, causal=causal)
    got = abar.double().cpu().numpy()
    assert np.isfinite(got).all()
    err = np.abs(got - ref).max()
    assert err <= MAP_TOL, "max |abar - oracle| = %.3e" % err


@pytest.mark.parametrize("case", MAP_CASES[:7], ids=lambda c: "B%d_H%d_%dx%d_D%d_%s" % (c[:5] + ("causal" if c[5] else "full",)))
def test_mean_map_with_the_forward_calls_lse(case):
    """ap_accumulate_attention_maps_lse: the row statistics come from the unpruned attention call
    (all-ones mask) on the same inputs instead of a pass of their own; same oracle, same bar."""
    B, H, Lq, Lk, D, causal = case
    Q, K = synth.make_qk_positional(B, H, Lq, Lk, D, seed=Lq + Lk + D)
    dq, rq = to_device(Q, "bf16")
    dk, rk = to_device(K, "bf16")
    ones = torch.ones((H, Lq, Lk), dtype=torch.uint8, device="cuda")
    lay = ap.ap_build_layout(ones, 64, 64)
    _, lse = ap.ap_sparse_attn_fwd(dq, dk, dk, lay, causal=causal)       # V plays no role in lse
    abar = ap.ap_accumulate_attention_maps(dq, dk, causal=causal, weight=1.0 / B, lse=lse)
    torch.cuda.synchronize()
    ref = oracle.mean_attention_map(rq, rk, causal=causal)
    got = abar.double().cpu().numpy()
    assert np.isfinite(got).all()
    err = np.abs(got - ref).max()
    assert err <= MAP_TOL, "max |abar - oracle| = %.3e" % err


def test_hidden_entries_are_not_touched():
    B, H, Lq, Lk, D = 2, 2, 130, 200, 64
    Q, K = synth.make_qk_positional(B, H, Lq, Lk, D, seed=5)
    abar0 = torch.full((H, Lq, Lk), -7.0, dtype=torch.float32, device="cuda")
    abar, rq, rk = run_maps(Q, K, True, abar=abar0)
    got = abar.double().cpu().numpy()
    vis = np.arange(Lk)[None, :] <= np.arange(Lq)[:, None] + (Lk - Lq)
    assert np.all(got[:, ~vis] == -7.0)
    ref = oracle.mean_attention_map(rq, rk, causal=True)
    assert np.abs(got[:, vis] - (ref[:, vis] - 7.0)).max() <= MAP_TOL


def test_streaming_over_batches_gives_eq1_mean():
    """Two calls with weight 1/n, n = all examples of both batches (Eq. (1))."""
    H, Lq, Lk, D = 2, 150, 150, 64
    Q1, K1 = synth.make_qk_positional(3, H, Lq, Lk, D, seed=11)
    Q2, K2 = synth.make_qk_positional(2, H, Lq, Lk, D, seed=12)
    abar, rq1, rk1 = run_maps(Q1, K1, False, weight=1.0 / 5)
    abar, rq2, rk2 = run_maps(Q2, K2, False, weight=1.0 / 5, abar=abar)
    ref = oracle.mean_attention_map(np.concatenate([rq1, rq2]), np.concatenate([rk1, rk2]))
    assert np.abs(abar.double().cpu().numpy() - ref).max() <= MAP_TOL


def test_explicit_scale_and_strided_inputs():
    B, H, Lq, Lk, D = 2, 2, 96, 96, 64
    Q, K = synth.make_qk_positional(B, H, Lq, Lk, D, seed=21)
    # [B, L, H, D] storage viewed as [B, H, L, D]
    dq = torch.from_numpy(Q).to(torch.bfloat16).cuda().permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    dk = torch.from_numpy(K).to(torch.bfloat16).cuda().permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    abar = ap.ap_accumulate_attention_maps(dq, dk, softmax_scale=0.05, weight=0.5)
    torch.cuda.synchronize()
    ref = oracle.mean_attention_map(dq.double().cpu().numpy(), dk.double().cpu().numpy(), scale=0.05)
    assert np.abs(abar.double().cpu().numpy() - ref).max() <= MAP_TOL


# --- threshold and mask: bit-exact ------------------------------------------------------------------

def abar_from_oracle(H, Lq, Lk, causal, seed):
    Q, K = synth.make_qk_positional(2, H, Lq, Lk, 32, seed=seed)
    return oracle.mean_attention_map(Q, K, causal=causal).astype(np.float32)


def check_prune(abar_np, p, causal, layout_block_ms=(64, 128)):
    d = torch.from_numpy(abar_np).cuda()
    mask, tau = ap.ap_prune_mask(d, p, causal=causal)
    torch.cuda.synchronize()
    ref_mask, ref_tau = oracle.prune_mask(abar_np, p, causal=causal)
    got_tau = tau.cpu().numpy()[0]
    assert got_tau == ref_tau or (np.isinf(got_tau) and np.isinf(ref_tau)), (got_tau, ref_tau)
    assert np.array_equal(mask.cpu().numpy(), ref_mask)
    # the same without the byte mask: threshold only, then the layout straight from the map; it must
    # be the layout of the oracle's mask (Eq. (2)'s strict comparison, ties kept, hidden entries never)
    none, tau2 = ap.ap_prune_mask(d, p, causal=causal, threshold_only=True)
    assert none is None
    for bm in layout_block_ms:
        lay = ap.ap_build_layout_from_map(d, tau2, causal=causal, block_m=bm)
        torch.cuda.synchronize()
        assert torch.equal(tau2, tau)
        assert_layout_equal(lay, ref_mask)


@pytest.mark.parametrize("p", [0.0, 0.1, 0.5, 0.9, 0.999, 1.0])
@pytest.mark.parametrize("shape", [(2, 64, 64, False), (3, 100, 157, True), (2, 300, 300, True),
                                   (4, 33, 1000, False), (1, 1, 1, False)])
def test_prune_mask_bit_exact_on_mean_maps(shape, p):
    H, Lq, Lk, causal = shape
    check_prune(abar_from_oracle(H, Lq, Lk, causal, seed=Lq + Lk), p, causal)


@pytest.mark.parametrize("p", [0.0, 0.25, 0.5, 0.75, 0.97])
@pytest.mark.parametrize("causal", [False, True])
def test_prune_mask_with_ties_zeros_and_tiny_values(p, causal):
    rng = np.random.default_rng(31)
    H, Lq, Lk = 3, 90, 120
    a = rng.integers(0, 12, size=(H, Lq, Lk)).astype(np.float32) / 16.0      # 12 distinct values: heavy ties
    a[rng.random(a.shape) < 0.05] = np.float32(1e-41)                          # denormals
    a[rng.random(a.shape) < 0.05] = np.float32(-0.0)                           # counts as zero
    a[rng.random(a.shape) < 0.02] = np.float32(3e38)
    check_prune(a, p, causal)


def test_prune_mask_values_that_differ_in_the_last_bits():
    rng = np.random.default_rng(37)
    base = np.float32(0.125)
    steps = rng.integers(0, 3000, size=(2, 128, 128))
    a = (base.view(np.uint32) + steps.astype(np.uint32)).view(np.float32).reshape(2, 128, 128)
    for p in (0.3, 0.9):
        check_prune(a, p, False)


@pytest.mark.parametrize("spread", [3000, 3, 1])
def test_prune_mask_more_ties_than_the_candidate_buffer_holds(spread):
    """Over two million entries inside one 1 %-wide value interval: the selection has to fix
    more digits with further sweeps (spread 3000), down to the last bit (spread 3), or finds
    every entry equal (spread 1)."""
    rng = np.random.default_rng(43)
    shape = (2, 1024, 1024)
    steps = rng.integers(0, spread, size=shape).astype(np.uint32)
    a = (np.float32(0.5).view(np.uint32) + steps).view(np.float32).reshape(shape)
    a[0, :7, :5] = 0.0                                                    # a few entries elsewhere
    a[1, 5, 100:140] = 0.75
    for p, causal in ((0.5, False), (0.9, True), (0.0, False)):
        check_prune(a, p, causal)


def test_mask_feeds_layout_and_attention_end_to_end():
    """Q, K -> mean map -> mask -> layout on the GPU; entries whose oracle mean is not within
    the map tolerance of the oracle's threshold must agree with the oracle's mask."""
    B, H, L, D, p = 4, 3, 256, 64, 0.9
    Q, K = synth.make_qk_positional(B, H, L, L, D, seed=41, strength=1.5)
    abar, rq, rk = run_maps(Q, K, True)
    mask, tau = ap.ap_prune_mask(abar, p, causal=True)
    lay = ap.ap_build_layout(mask, 64, 64)
    torch.cuda.synchronize()
    ref_abar = oracle.mean_attention_map(rq, rk, causal=True)
    ref_mask, ref_tau = oracle.prune_mask(ref_abar, p, causal=True)
    assert abs(float(tau.item()) - ref_tau) <= MAP_TOL
    clear = np.abs(ref_abar - ref_tau) > 2 * MAP_TOL
    got = mask.cpu().numpy()
    assert np.array_equal(got[clear], ref_mask[clear])
    vis = np.tril(np.ones((L, L), bool))
    n = int(vis.sum()) * H
    assert abs(int(got.sum()) - (n - int(np.floor(p * n)))) <= 4            # exact up to ties at tau
    from gpu_util import assert_layout_equal
    assert_layout_equal(lay, got)


# --- the benchmark's shape and launch configuration ---------------------------------------------------

def test_full_size_mean_map_rows_sampled_against_oracle():
    """C5's shape (B4 H16 L4096 D128 causal): rows sum to 1, hidden entries stay untouched, and
    windows of rows of three heads match the oracle element by element."""
    cfg = synth.CONFIGS["C5"]
    Q, K = synth.make_qk_positional(cfg.B, cfg.H, cfg.Lq, cfg.Lk, cfg.D, seed=cfg.index)
    abar, rq, rk = run_maps(Q, K, True)
    rs = abar.sum(-1)
    assert float((rs - 1.0).abs().max()) <= MAP_TOL
    assert float(abar.min()) >= 0.0
    upper = torch.triu(torch.ones(cfg.Lq, cfg.Lk, dtype=torch.bool, device="cuda"), diagonal=1)
    assert float(abar[:, upper].abs().max()) == 0.0                       # never written
    for h, r0, r1 in ((0, 0, 8), (7, 2040, 2056), (15, 4088, 4096), (3, 1000, 1003)):
        ref = oracle.attention_maps(rq[:, h:h + 1, r0:r1], rk[:, h:h + 1, :r1], causal=True).mean(0)[0]
        got = abar[h, r0:r1, :r1].double().cpu().numpy()
        assert np.abs(got - ref).max() <= MAP_TOL


def test_full_size_threshold_and_mask_bit_exact():
    """H16 x 4096 x 4096 causal map (the benchmark's shape), prune 90 %: tau and every mask byte
    equal the oracle's on the same float32 input."""
    a = synth.make_mean_map(16, 4096, 4096, seed=5)
    check_prune(a, 0.9, True, layout_block_ms=(64,))
