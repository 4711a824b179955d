"""GPU tests of the backward pass over visit schedules: the column schedule against its definition
(expanded on the host and compared with the mask itself), and the gradients against the fp64
oracle, to the same bar as the unscheduled backward pass (per row and per tensor, derived in
test_gpu_bwd.py; gpu_util.assert_grad_close).
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


def visible_mask(mask, causal):
    H, Lq, Lk = mask.shape
    m = mask.astype(bool)
    if causal:
        m = m & (np.arange(Lk)[None, None, :] <= (np.arange(Lq)[:, None] + (Lk - Lq))[None])
    return m


def check_col_schedule(mask, causal, min_rows):
    """Every (query, 64-key word) the schedule lists for a block column is exactly the nonzero
    word of the visible mask, each once; the entry kinds follow the min_rows rule."""
    H, Lq, Lk = mask.shape
    lay = ap.ap_build_layout(torch.from_numpy(mask).cuda(), 64, 64)
    lt = ap.ap_build_layout_transpose(lay)
    cs = ap.ap_build_col_schedule(lay, lt, causal=causal, min_rows=min_rows)
    torch.cuda.synchronize()
    eff = 48 if min_rows == 0 else min_rows
    col_ptr = lt.col_ptr.cpu().numpy()
    cnt, start = cs.cnt.cpu().numpy(), cs.start.cpu().numpy()
    cols, words = cs.cols.cpu().numpy(), cs.bitmaps.cpu().numpy().view(np.uint64)
    vis = visible_mask(mask, causal)
    nKB = -(-Lk // 64)
    # behind the counts: every head's visiting order (columns with >= twice the mean count first)
    order = cnt[H * nKB:2 * H * nKB].reshape(H, nKB)
    n_heavy = cnt[2 * H * nKB:]
    cnt = cnt[:H * nKB]
    for h in range(H):
        ch = cnt[h * nKB:(h + 1) * nKB]
        heavy = (ch * nKB >= 2 * ch.sum()) & (ch > 1)
        assert n_heavy[h] == heavy.sum()
        assert np.array_equal(order[h], np.concatenate([np.nonzero(heavy)[0], np.nonzero(~heavy)[0]]))
    pad = np.zeros((H, Lq, nKB * 64), bool)
    pad[:, :, :Lk] = vis
    want_words = np.zeros((H, Lq, nKB), np.uint64)
    for bit in range(64):
        want_words |= pad[:, :, bit::64].astype(np.uint64) << np.uint64(bit)
    for c in range(H * nKB):
        h, kb = divmod(c, nKB)
        c0 = col_ptr[c]
        assert 0 <= cnt[c] <= col_ptr[c + 1] - c0
        seen = {}
        consecutive_done = False
        last_gathered = -1
        for e in range(c0, c0 + cnt[c]):
            if start[e] >= 0:
                assert not consecutive_done, "runs of consecutive queries come first"
                assert start[e] % 64 == 0
                rows = start[e] + np.arange(64)
                nz = 0
                for slot, q in enumerate(rows):
                    w = int(words[e, slot])
                    if q >= Lq:
                        assert w == 0
                        continue
                    if w:
                        assert q not in seen
                        seen[int(q)] = w
                        nz += 1
                assert nz >= eff
            else:
                consecutive_done = True
                for slot in range(64):
                    q, w = int(cols[e, slot]), int(words[e, slot])
                    if q >= Lq:
                        assert q == Lq and w == 0
                        continue
                    assert w != 0 and q not in seen and q > last_gathered
                    seen[q] = w
                    last_gathered = q
        want = {int(q): int(want_words[h, q, kb]) for q in np.nonzero(want_words[h, :, kb])[0]}
        assert seen == want, "block column %d of head %d" % (kb, h)
        # rows left to gathered entries come from tiles with fewer than min_rows visible rows
        for e in range(c0, c0 + cnt[c]):
            if start[e] < 0:
                for q in cols[e][cols[e] < Lq]:
                    qb = q // 64
                    assert np.count_nonzero(want_words[h, qb * 64:(qb + 1) * 64, kb]) < eff


@pytest.mark.parametrize("min_rows", [0, 1, 17, 65])
@pytest.mark.parametrize("shape", [(2, 64, 64, 0.5, False), (3, 200, 330, 0.02, True), (1, 1000, 70, 0.01, False),
                                   (2, 130, 130, 0.0, False), (2, 300, 300, 0.004, True)])
def test_col_schedule_matches_definition(shape, min_rows):
    H, Lq, Lk, density, causal = shape
    mask = synth.random_mask(H, Lq, Lk, density, seed=Lq + 1)
    check_col_schedule(mask, causal, min_rows)


def test_col_schedule_on_the_structured_mask():
    cfg = synth.CONFIGS["C3"]
    mask = np.stack([synth.head_mask(cfg, h) for h in range(2)]).astype(np.uint8)
    check_col_schedule(mask, cfg.causal, 0)


def run_bwd_sched(Q, K, V, dO, mask_np, causal, scale=0.0, min_cols=0, min_rows=0, which=("both",)):
    dq, rq = to_device(Q, "bf16")
    dk, rk = to_device(K, "bf16")
    dv, rv = to_device(V, "bf16")
    dg, rg = to_device(dO, "bf16")
    lay = ap.ap_build_layout(torch.from_numpy(mask_np).cuda(), 64, 64)
    lt = ap.ap_build_layout_transpose(lay)
    rs = ap.ap_build_schedule(lay, causal=causal, min_cols=min_cols)
    cs = ap.ap_build_col_schedule(lay, lt, causal=causal, min_rows=min_rows)
    O, lse = ap.ap_sparse_attn_fwd(dq, dk, dv, lay, causal=causal, softmax_scale=scale, sched=rs)
    ref = oracle.masked_attention_backward(rq, rk, rv, mask_np, rg, causal=causal, scale=scale)
    for w in which:
        kw = {"both": dict(sched=rs, col_sched=cs), "row": dict(sched=rs), "col": dict(col_sched=cs)}[w]
        print("bwd_sched", Q.shape, K.shape, "causal" if causal else "full", w, flush=True)
        got3 = ap.ap_sparse_attn_bwd(dq, dk, dv, O, dg, lse, lay, lt, causal=causal, softmax_scale=scale, **kw)
        torch.cuda.synchronize()
        for name, got, want in zip(("dQ", "dK", "dV"), got3, ref):
            assert_grad_close(name, got.double().cpu().numpy(), want, " (%s)" % (w,))


@pytest.mark.parametrize("case", BWD_CASES, ids=lambda c: "B%d_H%d_%dx%d_D%d_%s_%g" % (c[:5] + ("causal" if c[5] else "full", c[6])))
def test_scheduled_backward_matches_oracle(case):
    B, H, Lq, Lk, D, causal, density = case
    Q, K, V, dO = rand_inputs(Lq + Lk + D, B, H, Lq, Lk, D)
    mask = synth.random_mask(H, Lq, Lk, density, seed=D + Lq)
    run_bwd_sched(Q, K, V, dO, mask, causal, which=("both", "row", "col"))


@pytest.mark.parametrize("mins", [(1, 1), (65, 65), (20, 9)])
def test_scheduled_backward_any_packing(mins):
    """Everything consecutive, everything gathered, and a mixture: the result must not depend on it."""
    Q, K, V, dO = rand_inputs(21, 2, 2, 260, 330, 64)
    mask = synth.random_mask(2, 260, 330, 0.06, seed=77)
    mask[:, 100:180, 64:128] = 1                     # a few dense tiles among sparse ones
    run_bwd_sched(Q, K, V, dO, mask, True, min_cols=mins[0], min_rows=mins[1])


@pytest.mark.parametrize("B,H", [(2, 4), (8, 2), (1, 8)])
def test_scheduled_backward_heavy_columns_first(B, H):
    """B * H divisible by 8: the dK/dV workgroups take the heavy block columns of all their pairs
    first.  One or two key blocks that every query attends to are such columns."""
    Lq = Lk = 448
    Q, K, V, dO = rand_inputs(33 + B, B, H, Lq, Lk, 64)
    mask = synth.random_mask(H, Lq, Lk, 0.01, seed=5)
    mask[:, :, 0:64] = 1
    mask[1::2, :, 128:192] = 1
    run_bwd_sched(Q, K, V, dO, mask, True)
    run_bwd_sched(Q, K, V, dO, mask, False)


def test_scheduled_backward_on_the_structured_masks():
    for name, heads, batch in (("C3", 2, 1), ("C2", 3, 2)):
        cfg = synth.CONFIGS[name]
        mask = np.stack([synth.head_mask(cfg, h) for h in range(heads)]).astype(np.uint8)
        Q, K, V, dO = rand_inputs(7, batch, heads, cfg.Lq, cfg.Lk, cfg.D)
        run_bwd_sched(Q, K, V, dO, mask, cfg.causal)


def test_scheduled_backward_full_size_c5_two_slices_against_oracle():
    """The benchmark's shape and launch configuration (B4 H16 L4096 D128 causal, C5's mask)."""
    cfg = synth.CONFIGS["C5"]
    mask = synth.make_mask(cfg)
    Q, K, V = synth.make_qkv(cfg)
    dO = np.random.default_rng([synth.SEED, 4243]).standard_normal(Q.shape, dtype=np.float32)
    dq, dk, dv, dg = (torch.from_numpy(x).to(torch.bfloat16).cuda() for x in (Q, K, V, dO))
    lay = ap.ap_build_layout(torch.from_numpy(mask).cuda(), 64, 64)
    lt = ap.ap_build_layout_transpose(lay)
    rs = ap.ap_build_schedule(lay, causal=True)
    cs = ap.ap_build_col_schedule(lay, lt, causal=True)
    O, lse = ap.ap_sparse_attn_fwd(dq, dk, dv, lay, causal=True, sched=rs)
    gQ, gK, gV = ap.ap_sparse_attn_bwd(dq, dk, dv, O, dg, lse, lay, lt, causal=True, sched=rs, col_sched=cs)
    torch.cuda.synchronize()
    for t in (gQ, gK, gV):
        assert bool(torch.isfinite(t).all())
    for b, h in ((0, 0), (3, 11)):
        sl = lambda t: t[b:b + 1, h:h + 1].double().cpu().numpy()
        ref = oracle.masked_attention_backward(sl(dq), sl(dk), sl(dv), mask[h:h + 1], sl(dg), causal=True)
        for name, got, want in zip(("dQ", "dK", "dV"), (gQ, gK, gV), ref):
            print("C5 bwd sched", name, (b, h), assert_grad_close(name, sl(got), want, "[%d,%d]" % (b, h)), flush=True)


def nan_padded(t, extra=64):
    """The same values as t [B, H, L, D], stored with `extra` rows of NaN behind every head's last row."""
    B, H, L, D = t.shape
    store = torch.full((B, H, L + extra, D), float("nan"), dtype=t.dtype, device=t.device)
    store[:, :, :L] = t
    return store[:, :, :L]


@pytest.mark.parametrize("use_sched", [False, True])
def test_rows_behind_the_last_row_are_never_used(use_sched):
    """Ragged last tiles: whatever is stored behind row L - 1 of Q, K, V, O, dO must not reach a gradient."""
    B, H, Lq, Lk, D = 2, 2, 130, 150, 128
    Q, K, V, dO = rand_inputs(41, B, H, Lq, Lk, D)
    mask = synth.random_mask(H, Lq, Lk, 0.4, seed=42)
    mask[:, :, Lk - 1] = 1
    mask[:, Lq - 1, :] = 1
    dq, rq = to_device(Q, "bf16")
    dk, rk = to_device(K, "bf16")
    dv, rv = to_device(V, "bf16")
    dg, rg = to_device(dO, "bf16")
    lay = ap.ap_build_layout(torch.from_numpy(mask).cuda(), 64, 64)
    lt = ap.ap_build_layout_transpose(lay)
    kw = {}
    if use_sched:
        kw = dict(sched=ap.ap_build_schedule(lay, causal=False), col_sched=ap.ap_build_col_schedule(lay, lt, causal=False))
    pq, pk, pv, pg = nan_padded(dq), nan_padded(dk), nan_padded(dv), nan_padded(dg)
    O, lse = ap.ap_sparse_attn_fwd(pq, pk, pv, lay)
    pO = nan_padded(O)
    got3 = ap.ap_sparse_attn_bwd(pq, pk, pv, pO, pg, lse, lay, lt, **kw)
    torch.cuda.synchronize()
    ref = oracle.masked_attention_backward(rq, rk, rv, mask, rg)
    for name, got, want in zip(("dQ", "dK", "dV"), got3, ref):
        g = got.double().cpu().numpy()
        assert np.isfinite(g).all(), name + " picked up padding"
        assert_grad_close(name, g, want)
