"""The entry point that allocates nothing (bsp_prune_mask_static), called through the raw C ABI: its mask and
threshold must equal, bit for bit, those of bsp_prune_mask on the same input (same kernels, the scratch taken from
the library's device array instead of a workspace), on two calls in a row, the second on a smaller input, so that
whatever the first call left in the shared array is there when the second runs.  Both are also held against the
CPU oracle's percentile."""
import ctypes as C

import numpy as np
import pytest
import torch

import bsp_workloads as wl
import paper_2009_08065_amd as bsp
from oracle import bsp_oracle as orc

pytestmark = pytest.mark.gpu


def _static(L, s, n_keep, scope, t=0.0):
    B, N = s.shape
    keep = torch.full((B, N), 7, dtype=torch.uint8, device="cuda")
    t_used = torch.full((B if scope == bsp.SCOPE_BLOCK else 1,), 123.0, dtype=torch.float32, device="cuda")
    st = L.bsp_prune_mask_static(C.c_void_p(s.data_ptr()), B, N, C.c_float(t), n_keep, scope,
                                 C.c_void_p(keep.data_ptr()), C.c_void_p(t_used.data_ptr()),
                                 C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert st == 0, L.bsp_status_string(st)
    return keep, t_used


def _workspace(L, s, n_keep, scope, t=0.0):
    B, N = s.shape
    keep = torch.full((B, N), 9, dtype=torch.uint8, device="cuda")
    t_used = torch.full((B if scope == bsp.SCOPE_BLOCK else 1,), 321.0, dtype=torch.float32, device="cuda")
    need = L.bsp_prune_mask_workspace_bytes(B, N, scope)
    ws = torch.empty(max(need, 4), dtype=torch.uint8, device="cuda")
    st = L.bsp_prune_mask(C.c_void_p(s.data_ptr()), B, N, C.c_float(t), n_keep, scope, C.c_void_p(keep.data_ptr()),
                          C.c_void_p(t_used.data_ptr()), C.c_void_p(ws.data_ptr()), need,
                          C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert st == 0, L.bsp_status_string(st)
    return keep, t_used


def test_prune_mask_static_equals_workspace_form_twice_second_smaller():
    L = bsp.lib()
    # first: 4.2 M groups (all 256 histogram slots in use); second: 3 x 1000 groups (one slot), ties included
    for seed, (B, N), frac in ((1, (4096, 1024), 5), (2, (3, 1000), 3)):
        s_np = (wl.normal(seed, (B, N), 0.02, "f32") ** 2).astype(np.float32)
        s_np[0, : N // 2] = s_np[0, 0]                                   # ties at and around the cut
        s = torch.from_numpy(s_np).cuda()
        n_keep = B * N // frac
        k_st, t_st = _static(L, s, n_keep, bsp.SCOPE_MATRIX)
        k_ws, t_ws = _workspace(L, s, n_keep, bsp.SCOPE_MATRIX)
        torch.cuda.synchronize()
        assert torch.equal(k_st, k_ws)
        assert torch.equal(t_st.view(torch.int32), t_ws.view(torch.int32))
        k_ref, t_ref = orc.mask_rank(s_np, n_keep, orc.SCOPE_MATRIX)
        assert np.array_equal(k_st.cpu().numpy(), k_ref)
        assert np.array_equal(t_st.cpu().numpy().view(np.uint32), np.asarray(t_ref, dtype=np.float32).view(np.uint32))


def test_prune_mask_static_other_forms_and_limits():
    L = bsp.lib()
    s_np = (wl.normal(3, (7, 300), 0.02, "f32") ** 2).astype(np.float32)
    s = torch.from_numpy(s_np).cuda()
    for scope, n_keep, t in ((bsp.SCOPE_BLOCK, 100, 0.0), (bsp.SCOPE_MATRIX, -1, 0.02), (bsp.SCOPE_MATRIX, 7 * 300, 0.0)):
        k_st, _ = _static(L, s, n_keep, scope, t)
        k_ws, _ = _workspace(L, s, n_keep, scope, t)
        torch.cuda.synchronize()
        assert torch.equal(k_st, k_ws)
    one = C.c_void_p(16)
    assert L.bsp_prune_mask_static(one, 1 << 20, 1 << 20, C.c_float(0.0), 5, 1, one, None, None) == 2   # too large: shape
    assert L.bsp_prune_mask_static(None, 2, 8, C.c_float(0.0), 5, 1, one, None, None) == 1
