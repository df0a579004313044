"""The whole path replayed from a HIP graph gives, on every replay, the bits of the eager run."""
import numpy as np
import pytest
import torch

import bsp_workloads as wl
import paper_2009_08065_amd as bsp

pytestmark = pytest.mark.gpu


def test_graph_replays_match_eager():
    T, M, N, R = 200, 512, 1024, 16
    d = wl.layer(31, T, M, N, "bf16")
    W = torch.from_numpy(d["W"]).bfloat16().cuda()
    bias = torch.from_numpy(d["bias"]).bfloat16().cuda()
    Xs = [torch.from_numpy(wl.normal(100 + i, (T, N), 1.0, "bf16")).bfloat16().cuda() for i in range(3)]
    n_keep = (M // R) * N // 5
    B = M // R
    cap = n_keep + B * 31
    dev = "cuda"
    X = Xs[0].clone()
    sumsq = torch.empty((B, N), dtype=torch.float32, device=dev)
    alpha = torch.empty_like(sumsq)
    grad = torch.empty_like(W)
    keep = torch.empty((B, N), dtype=torch.uint8, device=dev)
    ws = torch.empty(bsp.lib().bsp_prune_mask_workspace_bytes(B, N, bsp.SCOPE_MATRIX), dtype=torch.uint8, device=dev)
    cnt = torch.empty(B, dtype=torch.int32, device=dev)
    ptr = torch.empty(B + 1, dtype=torch.int32, device=dev)
    col = torch.empty(cap, dtype=torch.int32, device=dev)
    vals = torch.empty(R * cap, dtype=torch.bfloat16, device=dev)
    plan = torch.empty(bsp.lib().bsp_linear_plan_bytes(M, R, cap), dtype=torch.uint8, device=dev)
    Y = torch.empty((T, M), dtype=torch.bfloat16, device=dev)
    Z = torch.empty((T, N), dtype=torch.bfloat16, device=dev)     # the input gradient of the layer for dY = Y
    Yf = torch.empty((T, M), dtype=torch.bfloat16, device=dev)    # the layer with GELU in its epilogue
    D = torch.empty(R * cap, dtype=torch.bfloat16, device=dev)    # the weight gradient for dY = Y
    dws = torch.empty(bsp.lib().bsp_linear_dvals_workspace_bytes(M, N, R, cap), dtype=torch.uint8, device=dev)
    p = bsp.Packed(M, N, R, 32, cnt, ptr, col, vals, cap)

    def path():
        bsp.bsp_group_norms(W, R, sumsq=sumsq, alpha=alpha, want=())
        bsp.bsp_penalty_grad(W, R, alpha, 1e-4, grad=grad)
        bsp.bsp_prune_mask(sumsq, n_keep=n_keep, scope=bsp.SCOPE_MATRIX, keep=keep, ws=ws)
        bsp.bsp_pack_count(keep, 32, blk_cnt=cnt, blk_ptr=ptr)
        st = bsp.lib().bsp_pack(W.data_ptr(), bsp.BF16, M, N, R, keep.data_ptr(), 32, cnt.data_ptr(), ptr.data_ptr(),
                                cap, col.data_ptr(), vals.data_ptr(), bsp.BF16,
                                torch.cuda.current_stream().cuda_stream)
        assert st == 0
        bsp.bsp_linear_plan(p, plan=plan)
        bsp.bsp_linear_planned(X, p, plan, bias, Y=Y)
        bsp.bsp_linear_transposed(Y, p, None, Z=Z)
        bsp.bsp_linear_planned_fused(X, p, plan, bias, act=bsp.ACT_GELU, Y=Yf)
        # (D is as long as the storage's capacity; the call writes the R * blk_ptr[B] elements that are in use)
        st = bsp.lib().bsp_linear_dvals(X.data_ptr(), Y.data_ptr(), bsp.BF16, T, M, N, R, 32, cnt.data_ptr(),
                                        ptr.data_ptr(), col.data_ptr(), cap, D.data_ptr(), bsp.BF16, dws.data_ptr(),
                                        dws.numel(), bsp.DVALS_BUILD, torch.cuda.current_stream().cuda_stream)
        assert st == 0

    want = []
    for Xi in Xs:                       # eager reference (also the warm-up before capture)
        X.copy_(Xi)
        path()
        torch.cuda.synchronize()
        want.append((Y.clone(), keep.clone(), grad.clone(), Z.clone(), Yf.clone(), D[:R * int(ptr[-1])].clone()))
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        path()
    for rep in range(2):
        for Xi, (y_ref, k_ref, g_ref, z_ref, yf_ref, d_ref) in zip(Xs, want):
            X.copy_(Xi)
            Y.zero_(); keep.zero_(); grad.zero_(); col.zero_(); plan.zero_(); Z.zero_()   # eager work between replays
            Yf.zero_(); D.zero_(); dws.zero_()
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(Y, y_ref) and torch.equal(keep, k_ref) and torch.equal(grad, g_ref)
            assert torch.equal(Z, z_ref) and torch.equal(Yf, yf_ref) and torch.equal(D[:d_ref.numel()], d_ref)


def test_graph_replays_of_the_mask_with_its_storage_sizes():
    """bsp_prune_mask_count elects its last workgroup through a counter that the call's first launch clears: replays of
    a captured call (the workspace trashed in between) give the mask and the sizes of the separate calls."""
    B, N, k_align = 192, 1024, 32
    dev = "cuda"
    ws = torch.empty(bsp.lib().bsp_prune_mask_workspace_bytes(B, N, bsp.SCOPE_MATRIX), dtype=torch.uint8, device=dev)
    sumsq = torch.empty((B, N), dtype=torch.float32, device=dev)
    keep = torch.empty((B, N), dtype=torch.uint8, device=dev)
    cnt = torch.empty(B, dtype=torch.int32, device=dev)
    ptr = torch.empty(B + 1, dtype=torch.int32, device=dev)
    n_keep = B * N // 5
    inputs = [torch.from_numpy(wl.normal(500 + i, (B, N), 1.0) ** 2).float().cuda() for i in range(3)]
    want = []
    for s in inputs:
        k, _ = bsp.bsp_prune_mask(s, n_keep=n_keep, scope=bsp.SCOPE_MATRIX)
        c, p = bsp.bsp_pack_count(k, k_align)
        want.append((k.clone(), c.clone(), p.clone()))
    sumsq.copy_(inputs[0])
    bsp.bsp_prune_mask_count(sumsq, n_keep=n_keep, scope=bsp.SCOPE_MATRIX, k_align=k_align, keep=keep, ws=ws,
                             blk_cnt=cnt, blk_ptr=ptr)               # warm-up before capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        bsp.bsp_prune_mask_count(sumsq, n_keep=n_keep, scope=bsp.SCOPE_MATRIX, k_align=k_align, keep=keep, ws=ws,
                                 blk_cnt=cnt, blk_ptr=ptr)
    for rep in range(3):
        for s, (k_ref, c_ref, p_ref) in zip(inputs, want):
            sumsq.copy_(s)
            keep.zero_(); cnt.zero_(); ptr.zero_(); ws.random_(0, 256)   # eager work between replays
            g.replay()
            g.replay()                                                   # twice in a row on one stream
            torch.cuda.synchronize()
            assert torch.equal(keep, k_ref) and torch.equal(cnt, c_ref) and torch.equal(ptr, p_ref)
