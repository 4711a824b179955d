"""Helpers shared by the GPU parity tests (data movement only)."""
import numpy as np
import torch

import oracle
from paper_2012_02030_amd import binding as ap

TOL = {"bf16": 2e-2, "f32": 1e-5}      # max-abs error allowed against the fp64 oracle
TORCH_DTYPE = {"bf16": torch.bfloat16, "f32": torch.float32}


def to_device(x_f32: np.ndarray, dtype: str):
    """float32 numpy -> (device tensor in dtype, float64 numpy of the values after rounding)."""
    t = torch.from_numpy(x_f32).to(TORCH_DTYPE[dtype])
    return t.cuda(), t.to(torch.float64).numpy()


def layout_to_host(lay: ap.Layout):
    torch.cuda.synchronize()
    nnz = int(lay.nnz.item())
    rp = lay.row_ptr.cpu().numpy()
    n = min(nnz, lay.col_idx.shape[0])
    ci = lay.col_idx[:n].cpu().numpy()
    bm = lay.bitmaps[:n].cpu().numpy().view(np.uint64)
    return nnz, rp, ci, bm


def assert_layout_equal(lay: ap.Layout, mask_np: np.ndarray):
    rp_o, ci_o, bm_o = oracle.build_layout(mask_np, lay.block_m, lay.block_n)
    nnz, rp, ci, bm = layout_to_host(lay)
    assert nnz == len(ci_o), (nnz, len(ci_o))
    assert np.array_equal(rp, rp_o)
    assert np.array_equal(ci, ci_o)
    assert np.array_equal(bm, bm_o)


def run_and_compare(Q, K, V, mask_np, dtype, causal, block_m=64, scale=0.0, tol=None,
                    check_lse=True):
    """Run the GPU path on float32 numpy inputs and compare every output with the oracle."""
    tol = TOL[dtype] if tol is None else tol
    dq, rq = to_device(Q, dtype)
    dk, rk = to_device(K, dtype)
    dv, rv = to_device(V, dtype)
    dmask = torch.from_numpy(mask_np).cuda()
    lay = ap.ap_build_layout(dmask, block_m, 64)
    O, lse = ap.ap_sparse_attn_fwd(dq, dk, dv, lay, causal=causal, softmax_scale=scale)
    torch.cuda.synchronize()
    O_ref, lse_ref = oracle.masked_attention(rq, rk, rv, mask_np, causal=causal, scale=scale)
    O_h = O.to(torch.float64).cpu().numpy()
    lse_h = lse.to(torch.float64).cpu().numpy()
    assert np.all(np.isfinite(O_h)), "non-finite output"
    err = np.abs(O_h - O_ref).max()
    assert err <= tol, "max |O - oracle| = %.3e > %.1e" % (err, tol)
    if check_lse:
        empty = np.isneginf(lse_ref)
        assert np.array_equal(np.isneginf(lse_h), empty), "empty rows differ"
        if (~empty).any():
            lerr = np.abs(lse_h[~empty] - lse_ref[~empty]).max()
            assert lerr <= tol, "max |lse - oracle| = %.3e > %.1e" % (lerr, tol)
    return err
