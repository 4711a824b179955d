"""Pins for the layout oracle: a hand-written fixture, the round trip back to the element
mask, structural invariants, and an independent numpy formulation."""
import json
import os

import numpy as np
import pytest

import oracle
from paper_2012_02030_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def expand(row_ptr, col_idx, bitmaps, H, Lq, Lk, bm, bn):
    """Rebuild the element mask from a layout, bit by bit."""
    nqb = -(-Lq // bm)
    out = np.zeros((H, Lq, Lk), np.uint8)
    for r in range(H * nqb):
        h, qb = divmod(r, nqb)
        for t in range(row_ptr[r], row_ptr[r + 1]):
            kb = col_idx[t]
            for rr in range(bm):
                for c in range(bn):
                    if (int(bitmaps[t, rr, c // 64]) >> (c % 64)) & 1:
                        i, j = qb * bm + rr, kb * bn + c
                        assert i < Lq and j < Lk, "bit set outside the mask"
                        out[h, i, j] = 1
    return out


def numpy_tiles(mask, bm, bn):
    """Non-empty tiles via pad + reshape + any (a different route to the same answer)."""
    H, Lq, Lk = mask.shape
    nqb, nkb = -(-Lq // bm), -(-Lk // bn)
    pad = np.zeros((H, nqb * bm, nkb * bn), bool)
    pad[:, :Lq, :Lk] = mask != 0
    present = pad.reshape(H, nqb, bm, nkb, bn).any(axis=(2, 4)).reshape(H * nqb, nkb)
    counts = present.sum(axis=1)
    row_ptr = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    col_idx = np.nonzero(present)[1].astype(np.int32)
    return row_ptr, col_idx, pad


def test_hand_written_fixture():
    with open(os.path.join(GOLDEN, "layout_4x6_bm2_bn4.json")) as f:
        g = json.load(f)
    mask = np.array(g["mask"], np.uint8)[None]
    rp, ci, bmaps = oracle.build_layout(mask, g["block_m"], g["block_n"])
    assert rp.tolist() == g["row_ptr"]
    assert ci.tolist() == g["col_idx"]
    assert bmaps[:, :, 0].tolist() == g["bitmaps"]


@pytest.mark.parametrize("H,Lq,Lk,bm,bn,density", [
    (2, 16, 16, 4, 4, 0.2), (3, 37, 53, 8, 16, 0.05), (1, 70, 130, 16, 64, 0.02),
    (2, 65, 200, 32, 128, 0.01), (1, 5, 3, 64, 64, 0.5), (2, 64, 64, 64, 64, 0.0)])
def test_round_trip_and_invariants(H, Lq, Lk, bm, bn, density):
    mask = synth.random_mask(H, Lq, Lk, density, seed=Lq * 1000 + Lk)
    rp, ci, bmaps = oracle.build_layout(mask, bm, bn)
    nqb = -(-Lq // bm)
    assert rp[0] == 0 and len(rp) == H * nqb + 1 and np.all(np.diff(rp) >= 0)
    assert rp[-1] == len(ci) == len(bmaps)
    for r in range(H * nqb):
        cols = ci[rp[r]:rp[r + 1]]
        assert np.all(np.diff(cols) > 0), "columns must ascend strictly inside a block row"
    # no stored tile is empty, and the bits are exactly the kept entries
    pop = np.array([sum(bin(int(w)).count("1") for w in t.ravel()) for t in bmaps], dtype=np.int64)
    assert np.all(pop > 0) if len(pop) else True
    assert pop.sum() == int((mask != 0).sum())
    assert np.array_equal(expand(rp, ci, bmaps, H, Lq, Lk, bm, bn), (mask != 0).astype(np.uint8))
    # independent numpy route
    rp2, ci2, _ = numpy_tiles(mask, bm, bn)
    assert np.array_equal(rp, rp2) and np.array_equal(ci, ci2)


def test_any_nonzero_byte_counts_as_kept():
    mask = np.zeros((1, 4, 4), np.uint8)
    mask[0, 1, 2] = 255
    mask[0, 3, 0] = 2
    rp, ci, bmaps = oracle.build_layout(mask, 2, 2)
    assert rp.tolist() == [0, 1, 2] and ci.tolist() == [1, 0]
    assert bmaps[:, :, 0].tolist() == [[0, 1], [0, 1]]


def test_generators_reproduce_the_workload_structure():
    # structure of the synthetic masks: kept counts are exact, tile occupancy as designed
    c1 = synth.CONFIGS["C1"]
    m = synth.head_mask(c1, 0)
    assert m.sum() >= 208 and np.all(np.diag(m)) and not np.any(np.triu(m, 1))
    c2 = synth.CONFIGS["C2"]
    m = synth.head_mask(c2, 0)
    assert 8192 <= m.sum() <= 8192 + 128 and np.all(np.diag(m))
    assert m[:, 0].mean() > 0.9 and m[:, 127].mean() > 0.9          # separator columns survive
    c3 = synth.CONFIGS["C3"]
    m = synth.head_mask(c3, 0)
    assert 13133 <= m.sum() <= 13133 + 512 and not np.any(np.triu(m, 1))
    st = synth.tile_stats(m, 64, 64, True)
    assert st["nonempty_tiles"] == st["valid_tiles"] == 36              # spikes touch every tile
    st16 = synth.tile_stats(m, 16, 16, True)
    assert 0.90 < st16["nonempty_tiles"] / st16["valid_tiles"] < 0.99
    assert np.all(m[:, 0])                                              # sink column kept
    c4 = synth.CONFIGS["C4"]
    m = synth.head_mask(c4, 0)
    assert 8192 <= m.sum() <= 8192 + 128 and np.all(m.sum(axis=1) >= 1)
    # the same seed gives the same mask, different heads differ
    assert np.array_equal(synth.head_mask(c3, 1), synth.head_mask(c3, 1))
    assert not np.array_equal(synth.head_mask(c3, 0), synth.head_mask(c3, 1))
    # tensors: seeded, standard normal
    q, k = synth.make_qkv(c1, "QK")
    assert q.shape == (1, 2, 64, 32) and q.dtype == np.float32 and not np.array_equal(q, k)
    assert np.array_equal(q, synth.make_qkv(c1, "Q")[0])
