"""The C-ABI library loads, exports every symbol the header declares, and rejects bad
arguments on the host before anything is launched (so these run without a GPU)."""
import ctypes as C
import os
import re

import paper_2009_08065_amd as bsp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "bsp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bsp_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    L = bsp.lib()
    names = declared_symbols()
    assert {"bsp_group_norms", "bsp_penalty_grad", "bsp_prune_mask", "bsp_pack_count", "bsp_pack", "bsp_linear",
            "bsp_packed_validate", "bsp_compression_rate", "bsp_status_string"} <= set(names)
    for n in names:
        assert hasattr(L, n), n


def test_status_strings_and_rate():
    L = bsp.lib()
    assert L.bsp_status_string(0) == b"ok"
    assert all(L.bsp_status_string(i) for i in range(8))
    assert bsp.bsp_compression_rate(768, 768, 16, 48 * 384) == 2.0
    assert abs(bsp.bsp_compression_rate(100, 100, 10, 700) - 1 / 0.7) < 1e-12   # Sec. 4.4: 30 % sparsity
    assert bsp.bsp_compression_rate(8, 8, 4, 0) == float("inf")


def test_host_side_argument_checks():
    L = bsp.lib()
    one = C.c_void_p(16)   # never dereferenced: every call below fails validation first
    OK, NULL, SHAPE, DTYPE, CAP = 0, 1, 2, 3, 4
    assert L.bsp_group_norms(None, 0, 16, 8, 16, 1e-6, 0, one, one, one, None) == NULL
    assert L.bsp_group_norms(one, 0, 17, 8, 16, 1e-6, 0, one, one, one, None) == SHAPE      # M % R
    assert L.bsp_group_norms(one, 0, 16, 8, 0, 1e-6, 0, one, one, one, None) == SHAPE       # R < 1
    assert L.bsp_group_norms(one, 0, 130, 8, 65, 1e-6, 0, one, one, one, None) == SHAPE     # R > 64
    assert L.bsp_group_norms(one, 7, 16, 8, 16, 1e-6, 0, one, one, one, None) == DTYPE
    assert L.bsp_group_norms(one, 0, 16, 8, 16, 1e-6, 5, one, one, one, None) == DTYPE
    assert L.bsp_group_norms(one, 0, 16, 8, 16, 1e-6, 0, None, None, None, None) == OK      # nothing to do
    assert L.bsp_penalty_grad(one, 0, 16, 8, 16, None, 0.1, 0, 0, one, None, None, 0, None) == NULL
    assert L.bsp_penalty_grad(one, 0, 16, 8, 16, one, 0.1, 0, 0, one, one, one, 0, None) == CAP
    assert L.bsp_prune_mask(None, 1, 8, 0.0, -1, 0, one, None, None, 0, None) == NULL
    assert L.bsp_prune_mask(one, 0, 8, 0.0, -1, 0, one, None, None, 0, None) == SHAPE
    assert L.bsp_prune_mask(one, 1 << 20, 1 << 20, 0.0, -1, 0, one, None, None, 0, None) == SHAPE
    assert L.bsp_prune_mask(one, 2, 8, 0.0, 3, 1, one, None, one, 4, None) == CAP
    assert L.bsp_prune_mask(one, 2, 8, 0.0, 3, 9, one, None, one, 1 << 20, None) == DTYPE
    assert L.bsp_prune_mask_static(one, 1 << 20, 1 << 20, 0.0, 5, 1, one, None, None) == SHAPE   # beyond its scratch
    assert L.bsp_prune_mask_count(one, 2, 8, 0.0, 3, 1, one, None, 32, None, one, one, 1 << 20, None) == NULL
    assert L.bsp_prune_mask_count(one, 2, 8, 0.0, 3, 1, one, None, 5, one, one, one, 1 << 20, None) == SHAPE
    assert L.bsp_prune_mask_count(one, 2, 8, 0.0, 3, 1, one, None, 32, one, one, one, 4, None) == CAP
    assert L.bsp_prune_mask_count(one, 2, 8, 0.0, 3, 1, one, None, 32, one, one, None, 0, None) == NULL
    assert L.bsp_prune_mask_static(one, 0, 8, 0.0, -1, 0, one, None, None) == SHAPE
    assert L.bsp_pack_count(one, 2, 8, 3, one, one, None) == SHAPE                           # k_align
    assert L.bsp_pack_count(None, 2, 8, 16, one, one, None) == NULL
    assert L.bsp_pack(one, 0, 16, 8, 16, one, 16, one, one, -1, one, one, 0, None) == CAP
    assert L.bsp_pack(one, 0, 16, 8, 16, one, 16, one, one, 0, None, None, 0, None) == OK    # empty storage
    assert L.bsp_pack(one, 0, 16, 8, 16, one, 16, one, one, 5, None, one, 0, None) == NULL
    assert L.bsp_pack(one, 0, 16, 8, 16, one, 16, one, one, 5, one, one, 9, None) == DTYPE
    assert L.bsp_linear(None, 1, 4, 16, 8, 16, 32, one, one, one, one, None, one, None) == NULL
    assert L.bsp_linear(one, 1, 4, 24, 8, 16, 32, one, one, one, one, None, one, None) == SHAPE
    assert L.bsp_linear(one, 1, 0, 16, 8, 16, 32, one, one, one, one, None, one, None) == OK  # no tokens
    assert L.bsp_linear(C.c_void_p(8), 1, 4, 16, 8, 16, 32, one, one, one, one, None, one, None) == SHAPE  # alignment
    assert L.bsp_linear(one, 5, 4, 16, 8, 16, 32, one, one, one, one, None, one, None) == DTYPE
    assert L.bsp_linear_transposed(None, 1, 4, 16, 8, 16, 32, one, one, one, one, None, one, None) == NULL
    assert L.bsp_linear_transposed(one, 1, 4, 24, 8, 16, 32, one, one, one, one, None, one, None) == SHAPE
    assert L.bsp_linear_transposed(one, 1, 4, 16, 70000, 16, 32, one, one, one, one, None, one, None) == SHAPE
    assert L.bsp_linear_transposed(one, 1, 0, 16, 8, 16, 32, one, one, one, one, None, one, None) == OK  # no tokens
    assert L.bsp_linear_transposed(one, 7, 4, 16, 8, 16, 32, one, one, one, one, None, one, None) == DTYPE
    assert L.bsp_linear_transposed_dense(None, 1, 4, 16, 8, one, None, one, None) == NULL
    assert L.bsp_linear_transposed_dense(one, 9, 4, 16, 8, one, None, one, None) == DTYPE
    assert L.bsp_linear_transposed_dense(one, 1, 4, 0, 8, one, None, one, None) == SHAPE
    assert L.bsp_linear_transposed_dense(one, 1, 0, 16, 8, one, None, one, None) == OK       # no tokens
    # (X, dY, xdt, T, M, N, R, k_align, blk_cnt, blk_ptr, col_idx, capacity_cols, D, gdt, ws, ws_bytes, stream)
    assert L.bsp_linear_dvals(one, one, 1, 4, 16, 8, 16, 32, None, one, one, 32, one, 1, None, 0, 0, None) == NULL
    assert L.bsp_linear_dvals(one, one, 1, 4, 24, 8, 16, 32, one, one, one, 32, one, 1, None, 0, 0, None) == SHAPE  # M % R
    assert L.bsp_linear_dvals(one, one, 1, 4, 16, 8, 16, 5, one, one, one, 32, one, 1, None, 0, 0, None) == SHAPE   # k_align
    assert L.bsp_linear_dvals(one, one, 7, 4, 16, 8, 16, 32, one, one, one, 32, one, 1, None, 0, 0, None) == DTYPE
    assert L.bsp_linear_dvals(one, one, 1, 4, 16, 8, 16, 32, one, one, one, 32, one, 9, None, 0, 0, None) == DTYPE
    assert L.bsp_linear_dvals(one, one, 1, 4, 16, 8, 16, 32, one, one, None, 0, None, 1, None, 0, 0, None) == OK    # nothing kept
    assert L.bsp_linear_dvals(one, one, 1, 4, 16, 8, 16, 32, one, one, one, 32, None, 1, None, 0, 0, None) == NULL  # no D
    ws = C.c_void_p(4096)
    assert L.bsp_linear_dvals(C.c_void_p(64), C.c_void_p(64), 1, 4, 16, 8, 16, 32, one, one, one, 32, one, 1, ws, 16, 0, None) == CAP
    assert L.bsp_linear_dvals(one, one, 1, 4, 16, 8, 16, 32, one, one, one, 32, one, 1, None, 0, 5, None) == SHAPE  # ws_state
    assert L.bsp_linear_dvals_workspace_bytes(3072, 1024, 16, 45000) > 256 * 12 * 4096 * 4      # 256 units of partial sums
    assert L.bsp_linear_dvals_workspace_bytes(3072, 1024, 5, 45000) == 0                         # M % R
    assert L.bsp_packed_validate(16, 8, 16, 16, None, one, one, 0, one, None) == NULL
    assert L.bsp_penalty_grad_workspace_bytes(32, 300, 16) == 2 * 2 * 8
    assert L.bsp_prune_mask_workspace_bytes(4, 100, 1) >= 2 * (2048 + 64) * 4   # two histogram slots at least
    assert L.bsp_prune_mask_workspace_bytes(256, 4096, 1) > L.bsp_prune_mask_workspace_bytes(4, 100, 1)
    assert L.bsp_prune_mask_workspace_bytes(4, 100, 0) == 0
