"""ctypes binding of include/bsp.h.  Same names as the C entry points; argument marshalling
only.  Tensors must live on the GPU, be contiguous and have the dtype the C call expects; the
kernels are enqueued on torch's current stream.  There is no CPU fallback: if libbsp.so cannot
be loaded the import of `lib()` raises."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

F32, BF16, F16 = 0, 1, 2
ALPHA_SQNORM, ALPHA_NORM = 0, 1
SCOPE_BLOCK, SCOPE_MATRIX = 0, 1

_DT = {torch.float32: F32, torch.bfloat16: BF16, torch.float16: F16}
_TORCH = {F32: torch.float32, BF16: torch.bfloat16, F16: torch.float16}

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class BspError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().bsp_status_string(status).decode()
        if status == 6:
            msg += f" [hipError {lib().bsp_last_hip_error()}]"
        super().__init__(f"{where}: {msg} (status {status})")


def library_path() -> str:
    return os.path.join(_HERE, "libbsp.so")


def lib():
    """Load libbsp.so (building it in-tree with hipcc first if it is not there)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    from . import build as _build
    if not os.path.exists(path):
        _build.build(force=True)
    elif _build.stale():
        # a built library is loaded as it is (GPU runs must not compile); say so when a source is newer
        import warnings
        warnings.warn("libbsp.so is older than its sources: run `python -m paper_2009_08065_amd.build`")
    L = C.CDLL(path)
    i64, i32, f32, vp, sz = C.c_int64, C.c_int32, C.c_float, C.c_void_p, C.c_size_t
    L.bsp_group_norms.argtypes = [vp, C.c_int, i64, i64, i32, f32, C.c_int, vp, vp, vp, vp]
    L.bsp_penalty_grad.argtypes = [vp, C.c_int, i64, i64, i32, vp, f32, C.c_int, C.c_int, vp, vp, vp, sz, vp]
    L.bsp_penalty_grad_workspace_bytes.argtypes = [i64, i64, i32]
    L.bsp_penalty_grad_workspace_bytes.restype = sz
    L.bsp_prune_mask.argtypes = [vp, i64, i64, f32, i64, C.c_int, vp, vp, vp, sz, vp]
    L.bsp_prune_mask_static.argtypes = [vp, i64, i64, f32, i64, C.c_int, vp, vp, vp]
    L.bsp_prune_mask_count.argtypes = [vp, i64, i64, f32, i64, C.c_int, vp, vp, i32, vp, vp, vp, sz, vp]
    L.bsp_prune_mask_workspace_bytes.argtypes = [i64, i64, C.c_int]
    L.bsp_prune_mask_workspace_bytes.restype = sz
    L.bsp_mask_weights.argtypes = [vp, C.c_int, i64, i64, i32, vp, vp]
    L.bsp_tile_sumsq.argtypes = [vp, i64, i64, i32, vp, vp]
    L.bsp_expand_tile_mask.argtypes = [vp, i64, i64, i32, vp, vp]
    L.bsp_rowseg_norms.argtypes = [vp, C.c_int, i64, i64, i32, f32, C.c_int, vp, vp, vp, vp]
    L.bsp_mask_weights_rowseg.argtypes = [vp, C.c_int, i64, i64, i32, vp, vp]
    L.bsp_adam_step.argtypes = [vp, vp, C.c_int, vp, vp, i64, i64, i32, vp, f32, C.c_int, vp, f32, f32, f32, f32, i64, vp]
    L.bsp_group_norms_grad.argtypes = [vp, C.c_int, i64, i64, i32, f32, C.c_int, f32, C.c_int, vp, vp, vp, vp, vp]
    L.bsp_pack_count.argtypes = [vp, i64, i64, i32, vp, vp, vp]
    L.bsp_pack.argtypes = [vp, C.c_int, i64, i64, i32, vp, i32, vp, vp, i64, vp, vp, C.c_int, vp]
    L.bsp_packed_validate.argtypes = [i64, i64, i32, i32, vp, vp, vp, i64, vp, vp]
    L.bsp_linear.argtypes = [vp, C.c_int, i64, i64, i64, i32, i32, vp, vp, vp, vp, vp, vp, vp]
    L.bsp_linear_transposed.argtypes = [vp, C.c_int, i64, i64, i64, i32, i32, vp, vp, vp, vp, vp, vp, vp]
    L.bsp_linear_transposed_dense.argtypes = [vp, C.c_int, i64, i64, i64, vp, vp, vp, vp]
    L.bsp_linear_dvals_workspace_bytes.argtypes = [i64, i64, i32, i64]
    L.bsp_linear_dvals_workspace_bytes.restype = sz
    L.bsp_linear_dvals.argtypes = [vp, vp, C.c_int, i64, i64, i64, i32, i32, vp, vp, vp, i64, vp, C.c_int, vp, sz, C.c_int, vp]
    L.bsp_linear_plan_supported.argtypes = [C.c_int, i64, i32]
    L.bsp_linear_plan_supported.restype = C.c_int
    L.bsp_linear_plan_bytes.argtypes = [i64, i32, i64]
    L.bsp_linear_plan_bytes.restype = sz
    L.bsp_linear_plan.argtypes = [C.c_int, i64, i64, i32, i32, vp, vp, vp, vp, i64, vp, sz, vp]
    L.bsp_linear_planned.argtypes = [vp, C.c_int, i64, i64, i64, i32, i32, vp, i64, vp, vp, vp]
    L.bsp_linear_planned_fused.argtypes = [vp, C.c_int, i64, i64, i64, i32, i32, vp, i64, vp, C.c_int, vp, vp, vp]
    L.bsp_compression_rate.argtypes = [i64, i64, i32, i64]
    L.bsp_compression_rate.restype = C.c_double
    L.bsp_status_string.argtypes = [C.c_int]
    L.bsp_status_string.restype = C.c_char_p
    L.bsp_last_hip_error.restype = C.c_int
    L.bsp_version.restype = C.c_char_p
    for name in ("bsp_group_norms", "bsp_penalty_grad", "bsp_prune_mask", "bsp_pack_count", "bsp_pack",
                 "bsp_packed_validate", "bsp_linear", "bsp_linear_transposed", "bsp_linear_transposed_dense", "bsp_linear_dvals", "bsp_linear_plan", "bsp_linear_planned", "bsp_linear_planned_fused",
                 "bsp_mask_weights",
                 "bsp_group_norms_grad", "bsp_adam_step", "bsp_prune_mask_count"):
        getattr(L, name).restype = C.c_int
    _LIB = L
    return L


def _ptr(t: Optional[torch.Tensor], dtype=None):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensor must be a contiguous GPU tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected dtype {dtype}, got {t.dtype}")
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(st: int, where: str):
    if st != 0:
        raise BspError(st, where)


def bsp_group_norms(W, R, eps=1e-6, mode=ALPHA_SQNORM, sumsq=None, norm=None, alpha=None, want=("sumsq", "norm", "alpha")):
    """Returns (sumsq, norm, alpha) [B, N] fp32; entries not in `want` (and not passed) are None."""
    M, N = W.shape
    B = M // max(R, 1)
    mk = lambda: torch.empty((B, N), dtype=torch.float32, device=W.device)
    if sumsq is None and "sumsq" in want:
        sumsq = mk()
    if norm is None and "norm" in want:
        norm = mk()
    if alpha is None and "alpha" in want:
        alpha = mk()
    st = lib().bsp_group_norms(_ptr(W), _DT[W.dtype], M, N, R, eps, mode, _ptr(sumsq, torch.float32),
                               _ptr(norm, torch.float32), _ptr(alpha, torch.float32), _stream())
    _check(st, "bsp_group_norms")
    return sumsq, norm, alpha


def bsp_group_norms_grad(W, R, lam, eps=1e-6, mode=ALPHA_SQNORM, sumsq=None, norm=None, alpha=None, grad=None,
                         accumulate=False, want=("sumsq", "alpha")):
    """bsp_group_norms and bsp_penalty_grad in one pass over W.  Returns (sumsq, norm, alpha, grad)."""
    M, N = W.shape
    B = M // max(R, 1)
    mk = lambda: torch.empty((B, N), dtype=torch.float32, device=W.device)
    if sumsq is None and "sumsq" in want:
        sumsq = mk()
    if norm is None and "norm" in want:
        norm = mk()
    if alpha is None and "alpha" in want:
        alpha = mk()
    if grad is None:
        grad = torch.empty_like(W)
        accumulate = False
    if grad.dtype != W.dtype or grad.shape != W.shape:
        raise ValueError("grad must have the shape and dtype of W")
    st = lib().bsp_group_norms_grad(_ptr(W), _DT[W.dtype], M, N, R, eps, mode, lam, int(bool(accumulate)),
                                    _ptr(sumsq, torch.float32), _ptr(norm, torch.float32), _ptr(alpha, torch.float32),
                                    _ptr(grad), _stream())
    _check(st, "bsp_group_norms_grad")
    return sumsq, norm, alpha, grad


def bsp_adam_step(W, G, m, v, R, lr, beta1=0.9, beta2=0.999, eps=1e-8, t=1, alpha=None, lam=0.0, mode=ALPHA_SQNORM,
                  keep=None):
    """One Adam update of Alg. 2 in place on fp32 W, m, v: optional regulariser gradient (alpha, lam, mode) added
    to G, optional W = W * Mask (keep)."""
    M, N = W.shape
    for x in (W, m, v):
        if x.dtype != torch.float32 or x.shape != W.shape or not x.is_contiguous():
            raise ValueError("W, m, v must be contiguous fp32 tensors of one shape")
    if G.shape != W.shape or not G.is_contiguous():
        raise ValueError("G must be contiguous and have the shape of W")
    st = lib().bsp_adam_step(_ptr(W), _ptr(G), _DT[G.dtype], _ptr(m), _ptr(v), M, N, R, _ptr(alpha, torch.float32), lam,
                             mode, _ptr(keep, torch.uint8), lr, beta1, beta2, eps, t, _stream())
    _check(st, "bsp_adam_step")
    return W, m, v


def bsp_penalty_grad(W, R, alpha, lam, mode=ALPHA_SQNORM, grad=None, accumulate=False, want_penalty=False, ws=None):
    """Returns (grad, penalty) with penalty a 1-element fp64 GPU tensor or None."""
    M, N = W.shape
    if grad is None:
        grad = torch.empty_like(W)
        accumulate = False
    if grad.dtype != W.dtype or grad.shape != W.shape:
        raise ValueError("grad must have the shape and dtype of W")
    penalty = None
    ws_bytes = 0
    if want_penalty:
        penalty = torch.empty(1, dtype=torch.float64, device=W.device)
        need = lib().bsp_penalty_grad_workspace_bytes(M, N, R)
        if ws is None:
            ws = torch.empty(max(need, 8), dtype=torch.uint8, device=W.device)
        ws_bytes = ws.numel() * ws.element_size()
    st = lib().bsp_penalty_grad(_ptr(W), _DT[W.dtype], M, N, R, _ptr(alpha, torch.float32), lam, mode,
                                int(bool(accumulate)), _ptr(grad), _ptr(penalty), _ptr(ws), ws_bytes, _stream())
    _check(st, "bsp_penalty_grad")
    return grad, penalty


def bsp_prune_mask(sumsq, t=0.0, n_keep=-1, scope=SCOPE_BLOCK, keep=None, t_used=None, ws=None, want_t_used=False):
    """Returns (keep uint8 [B, N], t_used or None)."""
    B, N = sumsq.shape
    if keep is None:
        keep = torch.empty((B, N), dtype=torch.uint8, device=sumsq.device)
    if t_used is None and want_t_used and n_keep >= 0:
        t_used = torch.empty(B if scope == SCOPE_BLOCK else 1, dtype=torch.float32, device=sumsq.device)
    ws_bytes = 0
    if n_keep >= 0:
        need = lib().bsp_prune_mask_workspace_bytes(B, N, scope)
        if ws is None and need:
            ws = torch.empty(need, dtype=torch.uint8, device=sumsq.device)
        ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    st = lib().bsp_prune_mask(_ptr(sumsq, torch.float32), B, N, t, n_keep, scope, _ptr(keep, torch.uint8),
                              _ptr(t_used, torch.float32), _ptr(ws), ws_bytes, _stream())
    _check(st, "bsp_prune_mask")
    return keep, t_used


def bsp_prune_mask_static(sumsq, keep, t=0.0, n_keep=-1, scope=SCOPE_BLOCK, t_used=None):
    """bsp_prune_mask for callers that cannot allocate: the outputs are the caller's, the scratch is the library's
    own device array.  Calls on one GPU must not overlap."""
    B, N = sumsq.shape
    st = lib().bsp_prune_mask_static(_ptr(sumsq, torch.float32), B, N, t, n_keep, scope, _ptr(keep, torch.uint8),
                                     _ptr(t_used, torch.float32), _stream())
    _check(st, "bsp_prune_mask_static")
    return keep, t_used


def bsp_mask_weights(W, R, keep):
    """In place: zero every pruned group of W (Alg. 1; the W = W * Mask step of Alg. 2).  Returns W."""
    M, N = W.shape
    st = lib().bsp_mask_weights(_ptr(W), _DT[W.dtype], M, N, R, _ptr(keep, torch.uint8), _stream())
    _check(st, "bsp_mask_weights")
    return W


def bsp_tile_sumsq(sumsq, Ct, out=None):
    """Sums of squares of the R x Ct tiles from the column-group sums [B, N] (whole-block pruning)."""
    B, N = sumsq.shape
    if out is None:
        out = torch.empty((B, N // Ct), dtype=torch.float32, device=sumsq.device)
    _check(lib().bsp_tile_sumsq(_ptr(sumsq, torch.float32), B, N, Ct, _ptr(out, torch.float32), _stream()), "bsp_tile_sumsq")
    return out


def bsp_expand_tile_mask(tile_keep, Ct, out=None):
    B, NT = tile_keep.shape
    if out is None:
        out = torch.empty((B, NT * Ct), dtype=torch.uint8, device=tile_keep.device)
    _check(lib().bsp_expand_tile_mask(_ptr(tile_keep, torch.uint8), B, NT * Ct, Ct, _ptr(out, torch.uint8), _stream()),
           "bsp_expand_tile_mask")
    return out


def bsp_rowseg_norms(W, Cs, eps=1e-6, mode=ALPHA_SQNORM):
    """Returns (sumsq, norm, alpha), each [M, N / Cs] fp32: the groups are row segments of Cs columns."""
    M, N = W.shape
    outs = [torch.empty((M, N // Cs), dtype=torch.float32, device=W.device) for _ in range(3)]
    _check(lib().bsp_rowseg_norms(_ptr(W), _DT[W.dtype], M, N, Cs, eps, mode, _ptr(outs[0]), _ptr(outs[1]), _ptr(outs[2]),
                                  _stream()), "bsp_rowseg_norms")
    return tuple(outs)


def bsp_mask_weights_rowseg(W, Cs, keep_seg):
    """In place: zero every pruned row segment of W.  Returns W."""
    M, N = W.shape
    _check(lib().bsp_mask_weights_rowseg(_ptr(W), _DT[W.dtype], M, N, Cs, _ptr(keep_seg, torch.uint8), _stream()),
           "bsp_mask_weights_rowseg")
    return W


def bsp_pack_count(keep, k_align=32, blk_cnt=None, blk_ptr=None):
    B, N = keep.shape
    if blk_cnt is None:
        blk_cnt = torch.empty(B, dtype=torch.int32, device=keep.device)
    if blk_ptr is None:
        blk_ptr = torch.empty(B + 1, dtype=torch.int32, device=keep.device)
    st = lib().bsp_pack_count(_ptr(keep, torch.uint8), B, N, k_align, _ptr(blk_cnt, torch.int32),
                              _ptr(blk_ptr, torch.int32), _stream())
    _check(st, "bsp_pack_count")
    return blk_cnt, blk_ptr


def bsp_prune_mask_count(sumsq, t=0.0, n_keep=-1, scope=SCOPE_BLOCK, k_align=32, keep=None, t_used=None, ws=None,
                         blk_cnt=None, blk_ptr=None):
    """bsp_prune_mask and bsp_pack_count in one call.  Returns (keep, t_used, blk_cnt, blk_ptr)."""
    B, N = sumsq.shape
    dev = sumsq.device
    if keep is None:
        keep = torch.empty((B, N), dtype=torch.uint8, device=dev)
    if blk_cnt is None:
        blk_cnt = torch.empty(B, dtype=torch.int32, device=dev)
    if blk_ptr is None:
        blk_ptr = torch.empty(B + 1, dtype=torch.int32, device=dev)
    ws_bytes = 0
    if n_keep >= 0:
        need = lib().bsp_prune_mask_workspace_bytes(B, N, scope)
        if ws is None and need:
            ws = torch.empty(need, dtype=torch.uint8, device=dev)
        ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    st = lib().bsp_prune_mask_count(_ptr(sumsq, torch.float32), B, N, t, n_keep, scope, _ptr(keep, torch.uint8),
                                    _ptr(t_used, torch.float32), k_align, _ptr(blk_cnt, torch.int32),
                                    _ptr(blk_ptr, torch.int32), _ptr(ws), ws_bytes, _stream())
    _check(st, "bsp_prune_mask_count")
    return keep, t_used, blk_cnt, blk_ptr


@dataclass
class Packed:
    """The compact storage of one pruned weight (device tensors, canonical layout of bsp.h)."""
    M: int
    N: int
    R: int
    k_align: int
    blk_cnt: torch.Tensor
    blk_ptr: torch.Tensor
    col_idx: torch.Tensor
    vals: torch.Tensor
    total_cols: int


def bsp_pack(W, R, keep, k_align=32, vdt=None, blk_cnt=None, blk_ptr=None, total_cols=None):
    """Two-phase pack.  Reads blk_ptr[B] back to the host once to size the buffers (unless
    total_cols is given)."""
    M, N = W.shape
    if blk_cnt is None or blk_ptr is None:
        blk_cnt, blk_ptr = bsp_pack_count(keep, k_align)
    if total_cols is None:
        total_cols = int(blk_ptr[-1].item())
    vdtype = W.dtype if vdt is None else _TORCH[vdt]
    col_idx = torch.empty(max(total_cols, 1), dtype=torch.int32, device=W.device)
    vals = torch.empty(max(R * total_cols, 1), dtype=vdtype, device=W.device)
    st = lib().bsp_pack(_ptr(W), _DT[W.dtype], M, N, R, _ptr(keep, torch.uint8), k_align, _ptr(blk_cnt, torch.int32),
                        _ptr(blk_ptr, torch.int32), total_cols, _ptr(col_idx), _ptr(vals), _DT[vdtype], _stream())
    _check(st, "bsp_pack")
    return Packed(M, N, R, k_align, blk_cnt, blk_ptr, col_idx[:total_cols], vals[:R * total_cols], total_cols)


def bsp_packed_validate(p: Packed) -> bool:
    flag = torch.zeros(1, dtype=torch.int32, device=p.blk_ptr.device)
    st = lib().bsp_packed_validate(p.M, p.N, p.R, p.k_align, _ptr(p.blk_cnt), _ptr(p.blk_ptr),
                                   _ptr(p.col_idx) if p.total_cols else None, p.total_cols, _ptr(flag), _stream())
    if st == 5:
        return False
    _check(st, "bsp_packed_validate")
    return True


def bsp_linear(X, p: Packed, bias=None, Y=None):
    T, N = X.shape
    if N != p.N:
        raise ValueError("X has the wrong number of columns")
    if p.vals.dtype != X.dtype or (bias is not None and bias.dtype != X.dtype):
        raise ValueError("X, vals and bias must share one dtype")
    if Y is None:
        Y = torch.empty((T, p.M), dtype=X.dtype, device=X.device)
    has = p.total_cols > 0
    st = lib().bsp_linear(_ptr(X), _DT[X.dtype], T, p.M, N, p.R, p.k_align, _ptr(p.blk_cnt), _ptr(p.blk_ptr),
                          _ptr(p.col_idx) if has else None, _ptr(p.vals) if has else None, _ptr(bias), _ptr(Y),
                          _stream())
    _check(st, "bsp_linear")
    return Y


def bsp_linear_transposed(U, p: Packed, bias=None, Z=None):
    T, M = U.shape
    if M != p.M:
        raise ValueError("U has the wrong number of columns")
    if p.vals.dtype != U.dtype or (bias is not None and bias.dtype != U.dtype):
        raise ValueError("U, vals and bias must share one dtype")
    if Z is None:
        Z = torch.empty((T, p.N), dtype=U.dtype, device=U.device)
    has = p.total_cols > 0
    st = lib().bsp_linear_transposed(_ptr(U), _DT[U.dtype], T, M, p.N, p.R, p.k_align, _ptr(p.blk_cnt),
                                     _ptr(p.blk_ptr), _ptr(p.col_idx) if has else None,
                                     _ptr(p.vals) if has else None, _ptr(bias), _ptr(Z), _stream())
    _check(st, "bsp_linear_transposed")
    return Z


def bsp_linear_transposed_dense(U, Wm, bias=None, Z=None):
    """Z = U Wm (+ bias) with Wm the masked dense matrix [M, N]: the transposed product as a dense library product."""
    T, M = U.shape
    if Wm.shape[0] != M or Wm.dtype != U.dtype or (bias is not None and bias.dtype != U.dtype):
        raise ValueError("U [T, M], Wm [M, N] and bias must fit and share one dtype")
    N = Wm.shape[1]
    if Z is None:
        Z = torch.empty((T, N), dtype=U.dtype, device=U.device)
    st = lib().bsp_linear_transposed_dense(_ptr(U), _DT[U.dtype], T, M, N, _ptr(Wm), _ptr(bias), _ptr(Z), _stream())
    _check(st, "bsp_linear_transposed_dense")
    return Z


DVALS_BUILD, DVALS_REUSE = 0, 1


def bsp_linear_dvals(X, dY, p: Packed, out_dtype=None, D=None, ws=None, ws_state=DVALS_BUILD):
    """Gradient with respect to the kept weights, in the layout of p.vals: a tensor of R * p.total_cols elements.
    ws_state=DVALS_REUSE: ws is the workspace of an earlier call on the same storage (its work list is reused)."""
    T, N = X.shape
    if N != p.N or dY.shape != (T, p.M):
        raise ValueError("X must be [T, N] and dY [T, M]")
    if dY.dtype != X.dtype:
        raise ValueError("X and dY must share one dtype")
    out_dtype = out_dtype or X.dtype
    if D is None:
        D = torch.empty(p.R * p.total_cols, dtype=out_dtype, device=X.device)
    need = lib().bsp_linear_dvals_workspace_bytes(p.M, p.N, p.R, p.total_cols)
    if ws is None:
        ws = torch.empty(max(need, 256), dtype=torch.uint8, device=X.device)
    has = p.total_cols > 0
    st = lib().bsp_linear_dvals(_ptr(X), _ptr(dY), _DT[X.dtype], T, p.M, p.N, p.R, p.k_align, _ptr(p.blk_cnt),
                                _ptr(p.blk_ptr), _ptr(p.col_idx) if has else None, p.total_cols,
                                _ptr(D) if has else None, _DT[D.dtype], _ptr(ws), ws.numel(), ws_state, _stream())
    _check(st, "bsp_linear_dvals")
    return D


def bsp_linear_plan_supported(dtype, N, k_align) -> bool:
    return bool(lib().bsp_linear_plan_supported(_DT[dtype], N, k_align))


def bsp_linear_plan(p: Packed, plan=None):
    """Build the derived operand buffer of a compact storage.  Returns a uint8 GPU tensor."""
    need = lib().bsp_linear_plan_bytes(p.M, p.R, p.total_cols)
    if plan is None:
        plan = torch.empty(max(need, 16), dtype=torch.uint8, device=p.blk_ptr.device)
    has = p.total_cols > 0
    st = lib().bsp_linear_plan(_DT[p.vals.dtype], p.M, p.N, p.R, p.k_align, _ptr(p.blk_cnt), _ptr(p.blk_ptr),
                               _ptr(p.col_idx) if has else None, _ptr(p.vals) if has else None, p.total_cols,
                               _ptr(plan), plan.numel(), _stream())
    _check(st, "bsp_linear_plan")
    return plan


def bsp_linear_planned(X, p: Packed, plan, bias=None, Y=None):
    T, N = X.shape
    if N != p.N:
        raise ValueError("X has the wrong number of columns")
    if bias is not None and bias.dtype != X.dtype:
        raise ValueError("X and bias must share one dtype")
    if Y is None:
        Y = torch.empty((T, p.M), dtype=X.dtype, device=X.device)
    st = lib().bsp_linear_planned(_ptr(X), _DT[X.dtype], T, p.M, N, p.R, p.k_align, _ptr(plan),
                                  p.total_cols, _ptr(bias), _ptr(Y), _stream())
    _check(st, "bsp_linear_planned")
    return Y


ACT_NONE, ACT_GELU = 0, 1


def bsp_linear_planned_fused(X, p: Packed, plan, bias=None, act=ACT_NONE, residual=None, Y=None):
    """Y = round(act(X Wp^T + bias) + residual) in the layer kernel (raises BspError where that layer is not fused)."""
    T, N = X.shape
    if N != p.N:
        raise ValueError("X has the wrong number of columns")
    if bias is not None and bias.dtype != X.dtype:
        raise ValueError("X and bias must share one dtype")
    if residual is not None and (residual.dtype != X.dtype or tuple(residual.shape) != (T, p.M)
                                 or not residual.is_contiguous()):
        raise ValueError("residual must be a contiguous [T, M] tensor of the dtype of X")
    if Y is None:
        Y = torch.empty((T, p.M), dtype=X.dtype, device=X.device)
    st = lib().bsp_linear_planned_fused(_ptr(X), _DT[X.dtype], T, p.M, N, p.R, p.k_align, _ptr(plan),
                                        p.total_cols, _ptr(bias), act, _ptr(residual), _ptr(Y), _stream())
    _check(st, "bsp_linear_planned_fused")
    return Y


def bsp_compression_rate(M, N, R, kept_cols_total) -> float:
    return lib().bsp_compression_rate(M, N, R, kept_cols_total)
