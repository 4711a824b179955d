"""The visit schedule (a derived re-packing of the layout): structural validity of what
ap_build_schedule emits, and parity of ap_sparse_attn_fwd when it walks a schedule.

Several schedules are valid for one mask, so the structural test checks what must hold for
any of them: every visible kept (query, key) pair appears in exactly one entry slot, no other
pair appears, slots of a gathered entry name real keys or the empty marker, and a block row
has no more entries than stored tiles."""
import numpy as np
import pytest
import torch

import oracle
from paper_2012_02030_amd import binding as ap
from paper_2012_02030_amd import synth

from gpu_util import TOL, assert_c5_matches_oracle, c5_reference, to_device

pytestmark = pytest.mark.gpu


def expand_schedule(lay, sched, causal):
    """Rebuild the visible mask [H, Lq, Lk] from a schedule; asserts that no pair repeats."""
    torch.cuda.synchronize()
    H, Lq, Lk, BM = lay.H, lay.Lq, lay.Lk, lay.block_m
    nqb = -(-Lq // BM)
    rp = lay.row_ptr.cpu().numpy()
    cnt = sched.cnt.cpu().numpy()
    start = sched.start.cpu().numpy()
    cols = sched.cols.cpu().numpy()
    words = sched.bitmaps.cpu().numpy().view(np.uint64)
    out = np.zeros((H, Lq, Lk), np.uint8)
    bit = (np.uint64(1) << np.arange(64, dtype=np.uint64))
    for r in range(H * nqb):
        h, qb = divmod(r, nqb)
        assert 0 <= cnt[r] <= rp[r + 1] - rp[r]
        for e in range(rp[r], rp[r] + cnt[r]):
            if start[e] >= 0:
                keys = start[e] + np.arange(64)
            else:
                assert start[e] == -1
                keys = cols[e]
                real = keys[keys < Lk]
                assert len(set(real.tolist())) == len(real), "a gathered entry lists a key twice"
                assert np.all((keys >= 0) & (keys <= Lk))
            for rr in range(BM):
                w = words[e, rr]
                if w == 0:
                    continue
                i = qb * BM + rr
                assert i < Lq
                js = keys[(w & bit) != 0]
                assert np.all(js < Lk), "bit set on an empty slot or beyond the last key"
                assert not out[h, i, js].any(), "pair scheduled twice"
                out[h, i, js] = 1
    return out


def visible(mask, causal):
    m = (mask != 0)
    if causal:
        H, Lq, Lk = mask.shape
        m = m & (np.arange(Lk)[None, :] <= np.arange(Lq)[:, None] + (Lk - Lq))[None]
    return m.astype(np.uint8)


@pytest.mark.parametrize("min_cols", [0, 1, 17, 65])
@pytest.mark.parametrize("bm", [64, 128])
def test_schedule_covers_exactly_the_visible_mask(bm, min_cols):
    cases = [
        (synth.make_mask(synth.CONFIGS["C3"])[:3], True),
        (synth.random_mask(2, 200, 330, 0.01, 1), False),
        (synth.random_mask(2, 130, 260, 0.2, 2), True),
        (np.ones((1, 100, 100), np.uint8), True),
        (np.zeros((2, 70, 70), np.uint8), False),
    ]
    for mask, causal in cases:
        print("schedule", bm, min_cols, mask.shape, causal, flush=True)
        lay = ap.ap_build_layout(torch.from_numpy(mask).cuda(), bm, 64)
        sched = ap.ap_build_schedule(lay, causal=causal, min_cols=min_cols)
        got = expand_schedule(lay, sched, causal)
        assert np.array_equal(got, visible(mask, causal))


def test_schedule_packs_isolated_connections():
    # band + isolated connections: the schedule needs clearly fewer entries than stored tiles
    cfg = synth.CONFIGS["C3"]
    mask = synth.make_mask(cfg)
    lay = ap.ap_build_layout(torch.from_numpy(mask).cuda(), 64, 64)
    sched = ap.ap_build_schedule(lay, causal=True)
    torch.cuda.synchronize()
    tiles = int(lay.nnz.item())
    entries = int(sched.cnt.sum().item())
    assert entries < 0.8 * tiles, (entries, tiles)
    # min_cols = 1 keeps every visible tile as it is
    same = ap.ap_build_schedule(lay, causal=True, min_cols=1)
    torch.cuda.synchronize()
    assert int(same.cnt.sum().item()) == tiles
    assert bool((same.start[:tiles] >= 0).all())


def run_sched(Q, K, V, mask, causal, bm, min_cols, dtype="bf16"):
    dq, rq = to_device(Q, dtype)
    dk, rk = to_device(K, dtype)
    dv, rv = to_device(V, dtype)
    lay = ap.ap_build_layout(torch.from_numpy(mask).cuda(), bm, 64)
    sched = ap.ap_build_schedule(lay, causal=causal, min_cols=min_cols)
    O, lse = ap.ap_sparse_attn_fwd(dq, dk, dv, lay, causal=causal, sched=sched)
    torch.cuda.synchronize()
    O_ref, lse_ref = oracle.masked_attention(rq, rk, rv, mask, causal=causal)
    O_h = O.to(torch.float64).cpu().numpy()
    lse_h = lse.to(torch.float64).cpu().numpy()
    assert np.all(np.isfinite(O_h))
    err = np.abs(O_h - O_ref).max()
    assert err <= TOL[dtype], "max |O - oracle| = %.3e" % err
    empty = np.isneginf(lse_ref)
    assert np.array_equal(np.isneginf(lse_h), empty)
    if (~empty).any():
        assert np.abs(lse_h[~empty] - lse_ref[~empty]).max() <= TOL[dtype]
    return O, lse, lay, (dq, dk, dv)


@pytest.mark.parametrize("name", ["C2", "C3", "C4"])
@pytest.mark.parametrize("bm", [64, 128])
def test_configs_with_schedule(name, bm):
    cfg = synth.CONFIGS[name]
    print("attn sched", name, bm, flush=True)
    Q, K, V = synth.make_qkv(cfg)
    mask = synth.make_mask(cfg)
    for min_cols in (0, 65):
        run_sched(Q, K, V, mask, cfg.causal, bm, min_cols)


@pytest.mark.parametrize("D", [32, 64, 128])
def test_adversarial_masks_with_schedule(D):
    rng = np.random.default_rng(D)
    H, Lq, Lk = 2, 150, 333
    Q = rng.standard_normal((2, H, Lq, D), dtype=np.float32)
    K = rng.standard_normal((2, H, Lk, D), dtype=np.float32)
    V = rng.standard_normal((2, H, Lk, D), dtype=np.float32)
    column = np.zeros((H, Lq, Lk), np.uint8)
    column[:, :, 0] = 1
    column[:, :, 200] = 1
    holes = synth.random_mask(H, Lq, Lk, 0.05, 3)
    holes[:, ::2] = 0
    masks = {"bern01": synth.random_mask(H, Lq, Lk, 0.01, 1), "bern30": synth.random_mask(H, Lq, Lk, 0.3, 2),
             "column": column, "empty_rows": holes, "ones": np.ones((H, Lq, Lk), np.uint8),
             "none": np.zeros((H, Lq, Lk), np.uint8)}
    for mname, mask in masks.items():
        for causal in (False, True):
            for bm in (64, 128):
                for min_cols in (0, 65):
                    print("attn sched", D, mname, causal, bm, min_cols, flush=True)
                    run_sched(Q, K, V, mask, causal, bm, min_cols)


def test_unpacked_schedule_is_bitwise_the_layout_walk():
    cfg = synth.CONFIGS["C3"]
    Q, K, V = synth.make_qkv(cfg)
    mask = synth.make_mask(cfg)
    O, lse, lay, (dq, dk, dv) = run_sched(Q[:2], K[:2], V[:2], mask, True, 64, 1)
    O2, lse2 = ap.ap_sparse_attn_fwd(dq, dk, dv, lay, causal=True)
    torch.cuda.synchronize()
    assert torch.equal(O, O2) and torch.equal(lse, lse2)


def test_schedule_causal_flag_must_match():
    lay = ap.ap_build_layout(torch.ones((1, 64, 64), dtype=torch.uint8, device="cuda"), 64, 64)
    sched = ap.ap_build_schedule(lay, causal=True)
    q = torch.zeros((1, 1, 64, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(ValueError):
        ap.ap_sparse_attn_fwd(q, q.clone(), q.clone(), lay, causal=False, sched=sched)


def test_long_context_with_schedule_every_slice():
    """C5 with the visit schedule (the benchmark's launch configuration, and 128-query block
    rows): every output element of all 64 (batch, head) slices against the oracle."""
    cfg, mask, dq, dk, dv, O_ref, lse_ref = c5_reference()
    print("attn sched C5 full size", flush=True)
    dmask = torch.from_numpy(mask).cuda()
    for bm in (64, 128):
        lay = ap.ap_build_layout(dmask, bm, 64)
        sched = ap.ap_build_schedule(lay, causal=True)
        O, lse = ap.ap_sparse_attn_fwd(dq, dk, dv, lay, causal=True, sched=sched)
        torch.cuda.synchronize()
        assert torch.isfinite(O).all() and torch.isfinite(lse).all()
        print("  block_m", bm, "worst (O, lse) error over 64 slices:",
              assert_c5_matches_oracle(O, lse, O_ref, lse_ref, "sched block_m %d" % bm), flush=True)
        O1, _ = ap.ap_sparse_attn_fwd(dq, dk, torch.ones_like(dv), lay, causal=True, sched=sched)
        torch.cuda.synchronize()
        assert (O1.float() - 1.0).abs().max().item() <= 4e-3
