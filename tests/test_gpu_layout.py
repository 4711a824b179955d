"""ap_build_layout on the GPU against the layout oracle: bit-exact."""
import numpy as np
import pytest
import torch

import oracle
from paper_2012_02030_amd import binding as ap
from paper_2012_02030_amd import synth

from gpu_util import assert_layout_equal, layout_to_host

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4"])
@pytest.mark.parametrize("bm,bn", [(64, 64), (128, 64), (16, 16), (32, 128)])
def test_paper_shaped_masks(name, bm, bn):
    print("layout", name, bm, bn, flush=True)
    mask = synth.make_mask(synth.CONFIGS[name])
    lay = ap.ap_build_layout(torch.from_numpy(mask).cuda(), bm, bn)
    assert_layout_equal(lay, mask)


@pytest.mark.parametrize("H,Lq,Lk,bm,bn,density", [
    (3, 70, 130, 64, 64, 0.02),      # ragged, Lk not a multiple of 16 -> byte path
    (2, 100, 160, 64, 64, 0.001),    # almost empty, Lk multiple of 16 -> vector path with clipped last tile
    (1, 1, 1, 64, 64, 1.0),
    (2, 257, 513, 32, 32, 0.01),
    (1, 300, 4200, 16, 128, 0.003),  # more than 64 block columns: several ballot rounds per row
    (2, 129, 8200, 64, 64, 0.0005),
    (4, 64, 64, 128, 128, 0.5),
    (2, 96, 96, 64, 64, 0.0),        # empty mask
])
def test_random_masks(H, Lq, Lk, bm, bn, density):
    print("layout random", H, Lq, Lk, bm, bn, density, flush=True)
    mask = synth.random_mask(H, Lq, Lk, density, seed=Lq + Lk)
    lay = ap.ap_build_layout(torch.from_numpy(mask).cuda(), bm, bn)
    assert_layout_equal(lay, mask)


def test_any_nonzero_byte_is_kept():
    rng = np.random.default_rng(5)
    mask = (rng.random((2, 128, 128)) < 0.05).astype(np.uint8) * rng.integers(1, 256, (2, 128, 128)).astype(np.uint8)
    lay = ap.ap_build_layout(torch.from_numpy(mask).cuda(), 64, 64)
    assert_layout_equal(lay, mask)


def test_count_only_and_truncation():
    mask = synth.random_mask(2, 256, 256, 0.01, seed=3)
    dmask = torch.from_numpy(mask).cuda()
    rp_o, ci_o, bm_o = oracle.build_layout(mask, 64, 64)
    cnt = ap.ap_build_layout(dmask, 64, 64, count_only=True)
    torch.cuda.synchronize()
    assert int(cnt.nnz.item()) == len(ci_o)
    assert np.array_equal(cnt.row_ptr.cpu().numpy(), rp_o)
    # exact-size second call
    lay = ap.ap_build_layout(dmask, 64, 64, cap=len(ci_o))
    assert_layout_equal(lay, mask)
    # too small: the true count is still reported, the first cap tiles are written, nothing else
    cap = len(ci_o) // 2
    lay = ap.ap_build_layout(dmask, 64, 64, cap=cap)
    nnz, rp, ci, bm = layout_to_host(lay)
    assert nnz == len(ci_o) and len(ci) == cap
    assert np.array_equal(ci, ci_o[:cap]) and np.array_equal(bm, bm_o[:cap])


def test_layout_is_deterministic():
    mask = synth.random_mask(3, 512, 512, 0.01, seed=8)
    dmask = torch.from_numpy(mask).cuda()
    a = layout_to_host(ap.ap_build_layout(dmask, 64, 64))
    b = layout_to_host(ap.ap_build_layout(dmask, 64, 64))
    assert a[0] == b[0] and all(np.array_equal(x, y) for x, y in zip(a[1:], b[1:]))


def test_full_size_long_context_mask():
    cfg = synth.CONFIGS["C5"]
    print("layout C5 full size", flush=True)
    mask = synth.make_mask(cfg)
    lay = ap.ap_build_layout(torch.from_numpy(mask).cuda(), 64, 64)
    assert_layout_equal(lay, mask)


@pytest.mark.parametrize("stored,crop,bm,bn", [
    ((3, 300, 512), (300, 512), 64, 64),     # the whole mask
    ((3, 300, 512), (130, 256), 64, 64),     # vector path: pitch and cropped width multiples of 16
    ((3, 300, 512), (257, 201), 64, 64),     # byte path: the cropped width ends inside a 16-byte group
    ((2, 200, 333), (64, 70), 64, 64),       # pitch not a multiple of 16
    ((2, 200, 333), (1, 1), 64, 64),
    ((2, 260, 260), (129, 129), 128, 64),
    ((2, 100, 160), (33, 48), 16, 16),
])
def test_cropped_layout_is_the_layout_of_the_corner(stored, crop, bm, bn):
    """One stored mask serves every shorter sequence through its top-left corner; kept entries
    right of and below the corner must not leak in."""
    H, LqS, LkS = stored
    mask = synth.random_mask(H, LqS, LkS, 0.05, seed=LqS + LkS + crop[0])
    mask[:, :, LkS - 1] = 1
    mask[:, LqS - 1, :] = 1
    lay = ap.ap_build_layout(torch.from_numpy(mask).cuda(), bm, bn, crop=crop)
    assert (lay.Lq, lay.Lk) == crop
    assert_layout_equal(lay, np.ascontiguousarray(mask[:, :crop[0], :crop[1]]))


def test_attention_under_a_cropped_mask():
    from gpu_util import to_device, TOL
    H, LqS, LkS, D = 2, 256, 320, 64
    Lq, Lk = 150, 201
    mask = synth.random_mask(H, LqS, LkS, 0.2, seed=9)
    rng = np.random.default_rng(10)
    Q, K, V = (rng.standard_normal(s, dtype=np.float32) for s in ((2, H, Lq, D), (2, H, Lk, D), (2, H, Lk, D)))
    lay = ap.ap_build_layout(torch.from_numpy(mask).cuda(), 64, 64, crop=(Lq, Lk))
    sched = ap.ap_build_schedule(lay, causal=False)
    dq, rq = to_device(Q, "bf16")
    dk, rk = to_device(K, "bf16")
    dv, rv = to_device(V, "bf16")
    O, lse = ap.ap_sparse_attn_fwd(dq, dk, dv, lay, sched=sched)
    torch.cuda.synchronize()
    O_ref, lse_ref = oracle.masked_attention(rq, rk, rv, mask[:, :Lq, :Lk])
    assert np.abs(O.double().cpu().numpy() - O_ref).max() <= TOL["bf16"]
    ok = ~np.isneginf(lse_ref)
    assert np.abs(lse.double().cpu().numpy()[ok] - lse_ref[ok]).max() <= TOL["bf16"]
