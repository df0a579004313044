"""GPU vs CPU oracle for the other sparsity structures of the paper: whole-block pruning (the comparison of
Sec. 4.4 / Table 4) and the row-segment division (Eq. 2; Alg. 1 as printed) on the matrix as it is stored,
alone and together with the column division.  Sums, factors and masks are compared bit for bit."""
import numpy as np
import pytest
import torch

import bsp_workloads as wl
import paper_2009_08065_amd as bsp
from oracle import bsp_oracle as orc
from test_gpu_parity import CODE, assert_y_close, bits_equal, dev, host, run_layer

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("B,N,Ct", [(48, 768, 16), (7, 96, 3), (5, 64, 64), (3, 40, 1), (64, 4096, 32)])
def test_tile_sums_and_mask_expansion_bit_exact(B, N, Ct):
    s = (wl.normal(B + N + Ct, (B, N), 0.02, "f32") ** 2).astype(np.float32)
    ts = bsp.bsp_tile_sumsq(dev(s), Ct)
    ts_ref = orc.tile_sumsq(s, Ct)
    assert bits_equal(host(ts), ts_ref)
    tk_ref, _ = orc.mask_rank(ts_ref, ts_ref.size // 5, orc.SCOPE_MATRIX)
    tk, _ = bsp.bsp_prune_mask(ts, n_keep=ts_ref.size // 5, scope=bsp.SCOPE_MATRIX)
    assert np.array_equal(host(tk), tk_ref)
    assert np.array_equal(host(bsp.bsp_expand_tile_mask(tk, Ct)), orc.expand_tile_mask(tk_ref, Ct))


@pytest.mark.parametrize("Ct", [8, 32])
def test_whole_block_pruning_end_to_end(Ct):
    """Norms -> tile sums -> percentile over the tiles (5x) -> column mask -> storage -> layer, against the oracle's chain."""
    R, M, N, T = 16, 512, 1024, 200
    d = wl.layer(300 + Ct, T, M, N, "bf16")
    s, _, _ = bsp.bsp_group_norms(dev(d["W"], "bf16"), R)
    ts = bsp.bsp_tile_sumsq(s, Ct)
    n_keep = ts.numel() // 5
    tk, _ = bsp.bsp_prune_mask(ts, n_keep=n_keep, scope=bsp.SCOPE_MATRIX)
    keep = bsp.bsp_expand_tile_mask(tk, Ct)
    k_ref = orc.expand_tile_mask(orc.mask_rank(orc.tile_sumsq(orc.sumsq(d["W"], R), Ct), n_keep, orc.SCOPE_MATRIX)[0], Ct)
    assert np.array_equal(host(keep), k_ref)
    assert abs(bsp.bsp_compression_rate(M, N, R, int(k_ref.sum())) - 5.0) < 0.05
    run_layer(d["X"], d["W"], d["bias"], R, k_ref, 32, "bf16")   # storage bit for bit, both layer entry points


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("M,N,Cs", [(96, 1024, 16), (33, 777, 3), (20, 640, 64), (5, 64, 1), (7, 36, 12)])
def test_rowseg_norms_bit_exact(dtype, M, N, Cs):
    W = wl.normal(M * 7 + N + Cs, (M, N), 0.02, dtype)
    W[0, :Cs] = 0.0                                      # an all-zero group
    for mode in (orc.ALPHA_SQNORM, orc.ALPHA_NORM):
        s, nrm, alpha = bsp.bsp_rowseg_norms(dev(W, dtype), Cs, eps=1e-6, mode=mode)
        s_ref = orc.rowseg_sumsq(W, Cs)
        n_ref, a_ref = orc.norm_alpha(s_ref, 1e-6, mode)
        assert bits_equal(host(s), s_ref) and bits_equal(host(nrm), n_ref) and bits_equal(host(alpha), a_ref)


def test_row_segment_variant_on_the_stored_matrix_and_both_divisions_together():
    """Alg. 1 as printed (column blocks, a group is a row of a block) on W as it is stored, then both divisions on one
    matrix (Sec. 3.1): the matrix is masked by the column groups of its row-blocks and by the row segments of its
    column blocks, stored by its kept column groups, and the layer must give the dense product of the doubly masked W."""
    R, Cs, M, N, T = 16, 16, 256, 512, 150
    d = wl.layer(411, T, M, N, "bf16")
    W = d["W"]
    Wd = dev(W, "bf16")
    # row segments: sums, a matrix-scope percentile (keep half), masked weights
    s_seg, _, _ = bsp.bsp_rowseg_norms(Wd, Cs)
    s_seg_ref = orc.rowseg_sumsq(W, Cs)
    assert bits_equal(host(s_seg), s_seg_ref)
    k_seg, _ = bsp.bsp_prune_mask(s_seg, n_keep=s_seg_ref.size // 2, scope=bsp.SCOPE_MATRIX)
    k_seg_ref, _ = orc.mask_rank(s_seg_ref, s_seg_ref.size // 2, orc.SCOPE_MATRIX)
    assert np.array_equal(host(k_seg), k_seg_ref)
    # the same decision as the column-group route takes on the transposed matrix (the first round's way to this variant)
    kT_ref, _ = orc.mask_rank(orc.sumsq(np.ascontiguousarray(W.T), Cs), s_seg_ref.size // 2, orc.SCOPE_MATRIX)
    assert np.array_equal(k_seg_ref, kT_ref.T)
    W1 = Wd.clone()
    bsp.bsp_mask_weights_rowseg(W1, Cs, k_seg)
    W1_ref = np.ascontiguousarray(orc.mask_weights(np.ascontiguousarray(W.T), Cs, np.ascontiguousarray(k_seg_ref.T)).T)
    assert bits_equal(host(W1), W1_ref)
    # column groups of the row-blocks on top (a third of the groups of what is left)
    s_col, _, _ = bsp.bsp_group_norms(W1, R)
    s_col_ref = orc.sumsq(W1_ref, R)
    assert bits_equal(host(s_col), s_col_ref)
    k_col_ref, _ = orc.mask_rank(s_col_ref, s_col_ref.size // 3, orc.SCOPE_MATRIX)
    Y, p = run_layer(d["X"], W1_ref, d["bias"], R, k_col_ref, 32, "bf16")
    both = W.astype(np.float64) * np.repeat(k_seg_ref, Cs, axis=1) * np.repeat(k_col_ref, R, axis=0)
    want = d["X"].astype(np.float64) @ both.T + d["bias"]
    assert_y_close(Y, orc.round_to(want, orc.BF16), "bf16")
    assert (both != 0).sum() < 0.2 * both.size          # two thirds of a half: about a sixth of the weights survive
