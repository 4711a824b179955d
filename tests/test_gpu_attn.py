"""ap_sparse_attn_fwd on the GPU against the fp64 oracle, element by element.

Tolerances (max-abs on O and on lse): 2e-2 for bf16 inputs with fp32 accumulation, 1e-5 for fp32.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2012_02030_amd import binding as ap
from paper_2012_02030_amd import synth

from gpu_util import assert_c5_matches_oracle, c5_reference, TOL, run_and_compare, to_device

pytestmark = pytest.mark.gpu


def qkv(seed, B, H, Lq, Lk, D):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((B, H, Lq, D), dtype=np.float32),
            rng.standard_normal((B, H, Lk, D), dtype=np.float32),
            rng.standard_normal((B, H, Lk, D), dtype=np.float32))


# ---- the benchmark configurations at full size (C5 below, sampled) -----------------------------

@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4"])
def test_config_full_size(name):
    cfg = synth.CONFIGS[name]
    print("attn", name, flush=True)
    Q, K, V = synth.make_qkv(cfg)
    mask = synth.make_mask(cfg)
    run_and_compare(Q, K, V, mask, cfg.dtype, cfg.causal)


@pytest.mark.parametrize("name", ["C2", "C3", "C4"])
def test_config_wide_block_rows(name):
    cfg = synth.CONFIGS[name]
    print("attn bm128", name, flush=True)
    Q, K, V = synth.make_qkv(cfg)
    mask = synth.make_mask(cfg)
    run_and_compare(Q, K, V, mask, cfg.dtype, cfg.causal, block_m=128)


@pytest.mark.parametrize("name", ["C2", "C3"])
def test_config_dense_mask_run(name):
    # the p = 0 case the benchmark uses as its dense-mask baseline
    cfg = synth.CONFIGS[name]
    print("attn dense", name, flush=True)
    Q, K, V = synth.make_qkv(cfg)
    run_and_compare(Q[:4], K[:4], V[:4], synth.dense_mask(cfg), cfg.dtype, cfg.causal)


# ---- adversarial masks ---------------------------------------------------------------------------

CASES = [
    # name, H, Lq, Lk, D, causal
    ("square", 2, 192, 192, 64, False),
    ("square_causal", 2, 192, 192, 64, True),
    ("ragged", 3, 100, 150, 64, False),
    ("ragged_causal_lk_gt_lq", 2, 70, 201, 128, True),
    ("d32", 2, 130, 130, 32, True),
    ("d128", 1, 257, 300, 128, False),
    ("one_row", 1, 1, 77, 64, False),
]


def adversarial_masks(H, Lq, Lk, seed):
    rng = np.random.default_rng(seed)
    ones = np.ones((H, Lq, Lk), np.uint8)
    diag = np.zeros((H, Lq, Lk), np.uint8)
    ii = np.arange(Lq)
    diag[:, ii, np.minimum(ii + (Lk - Lq if Lk >= Lq else 0), Lk - 1)] = 1
    single = np.zeros((H, Lq, Lk), np.uint8)
    for h in range(H):
        single[h, ii, rng.integers(0, Lk, Lq)] = 1
    holes = synth.random_mask(H, Lq, Lk, 0.3, seed)
    holes[:, ::3] = 0                                   # every third query has no key at all
    column = np.zeros((H, Lq, Lk), np.uint8)
    column[:, :, Lk // 2] = 1
    column[:, :, 0] = 1
    return {
        "ones": ones, "diag": diag, "single": single, "empty_rows": holes, "column": column,
        "bern01": synth.random_mask(H, Lq, Lk, 0.01, seed + 1),
        "bern10": synth.random_mask(H, Lq, Lk, 0.10, seed + 2),
        "bern50": synth.random_mask(H, Lq, Lk, 0.50, seed + 3),
        "none": np.zeros((H, Lq, Lk), np.uint8),
    }


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_adversarial_masks(case, dtype):
    name, H, Lq, Lk, D, causal = case
    Q, K, V = qkv(sum(map(ord, name)), 2, H, Lq, Lk, D)
    for mname, mask in adversarial_masks(H, Lq, Lk, seed=len(name)).items():
        print("attn", name, dtype, mname, flush=True)
        run_and_compare(Q, K, V, mask, dtype, causal)
        if dtype == "bf16":
            run_and_compare(Q, K, V, mask, dtype, causal, block_m=128)


def test_single_kept_entry_returns_value_row_bitwise():
    H, Lq, Lk, D = 2, 128, 128, 64
    Q, K, V = qkv(3, 2, H, Lq, Lk, D)
    rng = np.random.default_rng(4)
    cols = rng.integers(0, Lk, (H, Lq))
    mask = np.zeros((H, Lq, Lk), np.uint8)
    for h in range(H):
        mask[h, np.arange(Lq), cols[h]] = 1
    for dtype in ("bf16", "f32"):
        dq, _ = to_device(Q, dtype)
        dk, _ = to_device(K, dtype)
        dv, _ = to_device(V, dtype)
        lay = ap.ap_build_layout(torch.from_numpy(mask).cuda(), 64, 64)
        O, _ = ap.ap_sparse_attn_fwd(dq, dk, dv, lay)
        torch.cuda.synchronize()
        for h in range(H):
            expect = dv[:, h, torch.from_numpy(cols[h]).cuda()]
            assert torch.equal(O[:, h], expect)


def test_constant_values_pass_through():
    H, Lq, Lk, D = 2, 200, 200, 64
    Q, K, _ = qkv(5, 1, H, Lq, Lk, D)
    V = np.ones((1, H, Lk, D), np.float32)
    mask = synth.random_mask(H, Lq, Lk, 0.2, 6)
    mask[:, np.arange(Lq), np.arange(Lq)] = 1
    run_and_compare(Q, K, V, mask, "bf16", False, tol=4e-3)    # one bf16 ulp at 1.0
    run_and_compare(Q, K, V, mask, "f32", False, tol=1e-6)


def test_explicit_scale_and_large_scores():
    H, Lq, Lk, D = 1, 128, 128, 64
    Q, K, V = qkv(7, 1, H, Lq, Lk, D)
    mask = synth.random_mask(H, Lq, Lk, 0.3, 8)
    mask[:, np.arange(Lq), np.arange(Lq)] = 1
    for dtype in ("bf16", "f32"):
        run_and_compare(Q, K, V, mask, dtype, False, scale=0.05)
        # scores up to about +-100: the softmax is nearly one-hot and exp must not overflow
        run_and_compare(Q * 2, K * 2, V, mask, dtype, True, scale=1.0,
                        tol=TOL[dtype] if dtype == "bf16" else 1e-4)


def test_strided_inputs():
    # [B, L, H, D] storage viewed as [B, H, L, D], and a head-dim padded to a wider row pitch
    B, H, L, D = 2, 3, 160, 64
    Q, K, V = qkv(9, B, H, L, L, D)
    mask = synth.random_mask(H, L, L, 0.15, 10)
    mask[:, np.arange(L), np.arange(L)] = 1
    lay = ap.ap_build_layout(torch.from_numpy(mask).cuda(), 64, 64)
    for dtype in ("bf16", "f32"):
        dq, rq = to_device(Q, dtype)
        dk, rk = to_device(K, dtype)
        dv, rv = to_device(V, dtype)
        sq = dq.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)            # BLHD storage
        pk = torch.zeros((B, H, L, D + 16), dtype=dk.dtype, device="cuda")
        pk[..., :D] = dk
        sk = pk[..., :D]                                                        # padded row pitch
        out_store = torch.empty((B, L, H, D), dtype=dq.dtype, device="cuda").permute(0, 2, 1, 3)
        assert not sq.is_contiguous() and not sk.is_contiguous()
        O, lse = ap.ap_sparse_attn_fwd(sq, sk, dv, lay, causal=True, out=out_store)
        torch.cuda.synchronize()
        O_ref, lse_ref = oracle.masked_attention(rq, rk, rv, mask, causal=True)
        assert np.abs(O.to(torch.float64).cpu().numpy() - O_ref).max() <= TOL[dtype]
        assert np.abs(lse.to(torch.float64).cpu().numpy() - lse_ref).max() <= TOL[dtype]


def nan_padded(t, extra=64):
    """The same values as t [B, H, L, D], stored with `extra` rows of NaN behind every head's last row."""
    B, H, L, D = t.shape
    store = torch.full((B, H, L + extra, D), float("nan"), dtype=t.dtype, device=t.device)
    store[:, :, :L] = t
    return store[:, :, :L]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_rows_behind_the_last_key_are_never_used(dtype):
    # a ragged last key tile must not pick up what is stored behind row Lk - 1 of a head
    H, Lq, Lk, D = 2, 130, 150, 128
    Q, K, V = qkv(31, 2, H, Lq, Lk, D)
    mask = synth.random_mask(H, Lq, Lk, 0.4, 32)
    mask[:, :, Lk - 1] = 1
    dq, rq = to_device(Q, dtype)
    dk, rk = to_device(K, dtype)
    dv, rv = to_device(V, dtype)
    lay = ap.ap_build_layout(torch.from_numpy(mask).cuda(), 64, 64)
    O_ref, lse_ref = oracle.masked_attention(rq, rk, rv, mask, causal=False)
    for sched in (None, ap.ap_build_schedule(lay, causal=False)) if dtype == "bf16" else (None,):
        O, lse = ap.ap_sparse_attn_fwd(dq, nan_padded(dk), nan_padded(dv), lay, sched=sched)
        torch.cuda.synchronize()
        O_h = O.to(torch.float64).cpu().numpy()
        assert np.all(np.isfinite(O_h))
        assert np.abs(O_h - O_ref).max() <= TOL[dtype]
        assert np.abs(lse.to(torch.float64).cpu().numpy() - lse_ref).max() <= TOL[dtype]


def test_output_is_bitwise_reproducible():
    cfg = synth.CONFIGS["C3"]
    Q, K, V = synth.make_qkv(cfg)
    mask = synth.make_mask(cfg)
    dq, dk, dv = (to_device(x[:2], "bf16")[0] for x in (Q, K, V))
    lay = ap.ap_build_layout(torch.from_numpy(mask).cuda(), 64, 64)
    O1, l1 = ap.ap_sparse_attn_fwd(dq, dk, dv, lay, causal=True)
    O2, l2 = ap.ap_sparse_attn_fwd(dq, dk, dv, lay, causal=True)
    torch.cuda.synchronize()
    assert torch.equal(O1, O2) and torch.equal(l1, l2)


def test_causal_with_fewer_keys_than_queries_is_rejected():
    H, Lq, Lk, D = 1, 128, 64, 64
    Q, K, V = qkv(11, 1, H, Lq, Lk, D)
    dq, dk, dv = (to_device(x, "bf16")[0] for x in (Q, K, V))
    lay = ap.ap_build_layout(torch.ones((H, Lq, Lk), dtype=torch.uint8, device="cuda"), 64, 64)
    with pytest.raises(ap.ApError) as e:
        ap.ap_sparse_attn_fwd(dq, dk, dv, lay, causal=True)
    assert e.value.status == ap.AP_ERR_INVALID_ARG


# ---- the long-context configuration at full size --------------------------------------------------

def test_long_context_full_size_every_slice():
    """C5 in the launch configuration the benchmark times (and with 128-query block rows): every
    output element of all 64 (batch, head) slices against the oracle, and V = 1 as a property
    check."""
    cfg, mask, dq, dk, dv, O_ref, lse_ref = c5_reference()
    print("attn C5 full size", flush=True)
    dmask = torch.from_numpy(mask).cuda()
    for bm in (64, 128):
        lay = ap.ap_build_layout(dmask, bm, 64)
        O, lse = ap.ap_sparse_attn_fwd(dq, dk, dv, lay, causal=True)
        torch.cuda.synchronize()
        assert torch.isfinite(O).all() and torch.isfinite(lse).all()
        print("  block_m", bm, "worst (O, lse) error over 64 slices:",
              assert_c5_matches_oracle(O, lse, O_ref, lse_ref, "block_m %d" % bm), flush=True)
        ones = torch.ones_like(dv)
        O1, _ = ap.ap_sparse_attn_fwd(dq, dk, ones, lay, causal=True)
        torch.cuda.synchronize()
        assert (O1.float() - 1.0).abs().max().item() <= 4e-3
