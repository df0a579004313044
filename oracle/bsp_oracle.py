"""ctypes front end of the C oracle (oracle/bsp_oracle.c).  Test infrastructure only.

Every function takes and returns numpy arrays on the host.  Low-precision tensors travel as
float32 arrays whose values are exactly representable in the low-precision type; dtype codes
F32 / BF16 / F16 say what a result is rounded to.  Citations of the paper are in the C file.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

F32, BF16, F16 = 0, 1, 2
ALPHA_SQNORM, ALPHA_NORM = 0, 1
SCOPE_BLOCK, SCOPE_MATRIX = 0, 1

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = C.CDLL(path)
        _lib.orc_round.restype = C.c_double
        _lib.orc_round.argtypes = [C.c_double, C.c_int]
        _lib.orc_compression_rate.restype = C.c_double
        _lib.orc_compression_rate.argtypes = [C.c_int64, C.c_int64, C.c_int32, C.c_int64]
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def round_to(v, dtype):
    """Round python floats / arrays (as doubles) to dtype, RNE; returns float64 array."""
    v = np.asarray(v, dtype=np.float64)
    out = np.empty_like(v)
    L = lib()
    flat_in, flat_out = v.ravel(), out.ravel()
    for i in range(flat_in.size):
        flat_out[i] = L.orc_round(float(flat_in[i]), dtype)
    return out


def sumsq(W, R):
    W = _f32(W)
    M, N = W.shape
    assert M % R == 0
    s = np.empty((M // R, N), dtype=np.float32)
    lib().orc_sumsq(_p(W), C.c_int64(M), C.c_int64(N), C.c_int32(R), _p(s))
    return s


def sumsq_exact(W, R):
    W = _f32(W)
    M, N = W.shape
    assert M % R == 0
    s = np.empty((M // R, N), dtype=np.float64)
    lib().orc_sumsq_exact(_p(W), C.c_int64(M), C.c_int64(N), C.c_int32(R), _p(s))
    return s


def norm_alpha(s, eps, mode):
    s = _f32(s)
    norm = np.empty_like(s)
    alpha = np.empty_like(s)
    lib().orc_norm_alpha(_p(s), C.c_int64(s.size), C.c_float(eps), C.c_int32(mode), _p(norm), _p(alpha))
    return norm, alpha


def penalty_grad(W, R, alpha, lam, mode, gdt=F32, G0=None):
    """Returns (G, penalty).  G0 given => accumulate into a copy of it."""
    W = _f32(W)
    M, N = W.shape
    alpha = _f32(alpha)
    assert alpha.shape == (M // R, N)
    G = np.zeros_like(W) if G0 is None else _f32(G0).copy()
    pen = C.c_double(0.0)
    lib().orc_penalty_grad(_p(W), C.c_int64(M), C.c_int64(N), C.c_int32(R), _p(alpha), C.c_float(lam),
                           C.c_int32(mode), C.c_int32(0 if G0 is None else 1), C.c_int32(gdt), _p(G),
                           C.byref(pen))
    return G, pen.value


def mask_threshold(s, t):
    s = _f32(s)
    keep = np.empty(s.shape, dtype=np.uint8)
    lib().orc_mask_threshold(_p(s), C.c_int64(s.size), C.c_float(t), _p(keep))
    return keep


def mask_rank(s, n_keep, scope):
    s = _f32(s)
    B, N = s.shape
    keep = np.empty((B, N), dtype=np.uint8)
    t_used = np.empty(B if scope == SCOPE_BLOCK else 1, dtype=np.float32)
    lib().orc_mask_rank(_p(s), C.c_int64(B), C.c_int64(N), C.c_int64(n_keep), C.c_int32(scope), _p(keep),
                        _p(t_used))
    return keep, t_used


def pack_count(keep, k_align):
    keep = np.ascontiguousarray(keep, dtype=np.uint8)
    B, N = keep.shape
    cnt = np.empty(B, dtype=np.int32)
    ptr = np.empty(B + 1, dtype=np.int32)
    lib().orc_pack_count(_p(keep), C.c_int64(B), C.c_int64(N), C.c_int32(k_align), _p(cnt), _p(ptr))
    return cnt, ptr


def pack(W, R, keep, k_align, vdt=F32):
    """Returns dict(blk_cnt, blk_ptr, col_idx, vals) in the canonical compact layout."""
    W = _f32(W)
    M, N = W.shape
    keep = np.ascontiguousarray(keep, dtype=np.uint8)
    assert keep.shape == (M // R, N)
    cnt, ptr = pack_count(keep, k_align)
    total = int(ptr[-1])
    col_idx = np.empty(total, dtype=np.int32)
    vals = np.empty(R * total, dtype=np.float32)
    lib().orc_pack(_p(W), C.c_int64(M), C.c_int64(N), C.c_int32(R), _p(keep), C.c_int32(k_align), _p(cnt),
                   _p(ptr), C.c_int32(vdt), _p(col_idx), _p(vals))
    return dict(blk_cnt=cnt, blk_ptr=ptr, col_idx=col_idx, vals=vals, R=R, M=M, N=N, k_align=k_align)


def linear_dense(X, W, keep, bias, R, ydt=F32):
    """Brute force: dense product with pruned entries zeroed.  Returns (Y rounded, Y double)."""
    X, W = _f32(X), _f32(W)
    T, N = X.shape
    M = W.shape[0]
    keep = np.ascontiguousarray(keep, dtype=np.uint8)
    bias = None if bias is None else _f32(bias)
    Y = np.empty((T, M), dtype=np.float32)
    Yd = np.empty((T, M), dtype=np.float64)
    lib().orc_linear_dense(_p(X), _p(W), _p(keep), _p(bias), C.c_int64(T), C.c_int64(M), C.c_int64(N),
                           C.c_int32(R), C.c_int32(ydt), _p(Y), _p(Yd))
    return Y, Yd


def linear_packed(X, packed, bias, ydt=F32, t0=0, t1=None, n_threads=1):
    """The layer through the compact storage, rows t0..t1-1 of X.  Returns (Y, Yd) of full
    shape [T, M]; rows outside [t0, t1) are left as NaN."""
    X = _f32(X)
    T, N = X.shape
    M, R = packed["M"], packed["R"]
    assert N == packed["N"]
    t1 = T if t1 is None else t1
    bias = None if bias is None else _f32(bias)
    Y = np.full((T, M), np.nan, dtype=np.float32)
    Yd = np.full((T, M), np.nan, dtype=np.float64)
    lib().orc_linear_packed(_p(X), C.c_int64(t0), C.c_int64(t1), C.c_int64(M), C.c_int64(N), C.c_int32(R),
                            _p(packed["blk_cnt"]), _p(packed["blk_ptr"]), _p(packed["col_idx"]),
                            _p(packed["vals"]), _p(bias), C.c_int32(ydt), _p(Y), _p(Yd), C.c_int32(n_threads))
    return Y, Yd


def linear_t_dense(U, W, keep, bias, R, zdt=F32):
    """Brute force transposed product: U times the matrix with pruned entries zeroed.  Returns (Z rounded, Z double)."""
    U, W = _f32(U), _f32(W)
    T, M = U.shape
    N = W.shape[1]
    assert W.shape[0] == M
    keep = np.ascontiguousarray(keep, dtype=np.uint8)
    bias = None if bias is None else _f32(bias)
    Z = np.empty((T, N), dtype=np.float32)
    Zd = np.empty((T, N), dtype=np.float64)
    lib().orc_linear_t_dense(_p(U), _p(W), _p(keep), _p(bias), C.c_int64(T), C.c_int64(M), C.c_int64(N),
                             C.c_int32(R), C.c_int32(zdt), _p(Z), _p(Zd))
    return Z, Zd


def linear_t_packed(U, packed, bias, zdt=F32, t0=0, t1=None, n_threads=1):
    """The transposed product through the compact storage, rows t0..t1-1 of U.  Returns (Z, Zd) of full
    shape [T, N]; rows outside [t0, t1) are left as NaN."""
    U = _f32(U)
    T, M = U.shape
    N, R = packed["N"], packed["R"]
    assert M == packed["M"]
    t1 = T if t1 is None else t1
    bias = None if bias is None else _f32(bias)
    Z = np.full((T, N), np.nan, dtype=np.float32)
    Zd = np.full((T, N), np.nan, dtype=np.float64)
    lib().orc_linear_t_packed(_p(U), C.c_int64(t0), C.c_int64(t1), C.c_int64(M), C.c_int64(N), C.c_int32(R),
                              _p(packed["blk_cnt"]), _p(packed["blk_ptr"]), _p(packed["col_idx"]),
                              _p(packed["vals"]), _p(bias), C.c_int32(zdt), _p(Z), _p(Zd), C.c_int32(n_threads))
    return Z, Zd


def mask_weights(W, R, keep):
    """Returns a copy of W with every pruned group set to +0 (Alg. 1; the W = W * Mask step of Alg. 2)."""
    W = _f32(W).copy()
    M, N = W.shape
    keep = np.ascontiguousarray(keep, dtype=np.uint8)
    assert keep.shape == (M // R, N)
    lib().orc_mask_weights(_p(W), C.c_int64(M), C.c_int64(N), C.c_int32(R), _p(keep))
    return W


def adam_step(W, G, m, v, R, lr, beta1=0.9, beta2=0.999, eps=1e-8, t=1, alpha=None, lam=0.0, mode=ALPHA_SQNORM,
              keep=None):
    """One Adam update of Alg. 2 (fp32): optional regulariser gradient (Eq. 3, factors alpha fixed) added to G,
    moments, weight update, optional W = W * Mask.  Returns new copies (W, m, v)."""
    W, m, v = _f32(W).copy(), _f32(m).copy(), _f32(v).copy()
    G = _f32(G)
    M, N = W.shape
    assert G.shape == W.shape and m.shape == W.shape and v.shape == W.shape
    if alpha is not None:
        alpha = _f32(alpha)
        assert alpha.shape == (M // R, N)
    if keep is not None:
        keep = np.ascontiguousarray(keep, dtype=np.uint8)
        assert keep.shape == (M // R, N)
    lib().orc_adam_step(_p(W), _p(G), _p(m), _p(v), C.c_int64(M), C.c_int64(N), C.c_int32(R),
                        _p(alpha) if alpha is not None else None, C.c_float(lam), C.c_int32(mode),
                        _p(keep) if keep is not None else None, C.c_float(lr), C.c_float(beta1), C.c_float(beta2),
                        C.c_float(eps), C.c_int64(t))
    return W, m, v


def compression_rate(M, N, R, kept_cols_total):
    return lib().orc_compression_rate(M, N, R, kept_cols_total)


ACT_NONE, ACT_GELU = 0, 1


def epilogue(Yd, act=ACT_NONE, residual=None, ydt=F32):
    """Element-wise tail of a layer on its unrounded sums: optional exact (erf) GELU, optional residual addition,
    one rounding.  Returns (Y rounded, Y double)."""
    Yd = np.ascontiguousarray(Yd, dtype=np.float64)
    res = None if residual is None else _f32(residual)
    assert res is None or res.shape == Yd.shape
    Y = np.empty(Yd.shape, dtype=np.float32)
    Ye = np.empty(Yd.shape, dtype=np.float64)
    lib().orc_epilogue(_p(Yd), _p(res), C.c_int64(Yd.size), C.c_int32(act), C.c_int32(ydt), _p(Y), _p(Ye))
    return Y, Ye


def linear_packed_fused(X, packed, bias, act=ACT_NONE, residual=None, ydt=F32, n_threads=1):
    """The layer followed by its epilogue: (Y rounded, Y double)."""
    _, Yd = linear_packed(X, packed, bias, ydt=ydt, n_threads=n_threads)
    return epilogue(Yd, act, residual, ydt)


def linear_dvals(X, dY, packed, gdt=F32, n_threads=1):
    """Gradient with respect to the kept weights, in the layout of the value panels: (D rounded, D double)."""
    X, dY = _f32(X), _f32(dY)
    T, N = X.shape
    M, R = packed["M"], packed["R"]
    assert dY.shape == (T, M) and N == packed["N"]
    n = R * int(packed["blk_ptr"][-1])
    D = np.empty(n, dtype=np.float32)
    Dd = np.empty(n, dtype=np.float64)
    lib().orc_linear_dvals(_p(X), _p(dY), C.c_int64(T), C.c_int64(M), C.c_int64(N), C.c_int32(R),
                           _p(packed["blk_cnt"]), _p(packed["blk_ptr"]), _p(packed["col_idx"]), C.c_int32(gdt),
                           _p(D), _p(Dd), C.c_int32(n_threads))
    return D, Dd


def tile_sumsq(s, Ct):
    """Sums of squares of the R x Ct tiles from the column-group sums s [B, N] (fp32, columns ascending)."""
    s = _f32(s)
    B, N = s.shape
    assert N % Ct == 0
    ts = np.empty((B, N // Ct), dtype=np.float32)
    lib().orc_tile_sumsq(_p(s), C.c_int64(B), C.c_int64(N), C.c_int32(Ct), _p(ts))
    return ts


def expand_tile_mask(tkeep, Ct):
    tkeep = np.ascontiguousarray(tkeep, dtype=np.uint8)
    B, NT = tkeep.shape
    keep = np.empty((B, NT * Ct), dtype=np.uint8)
    lib().orc_expand_tile_mask(_p(tkeep), C.c_int64(B), C.c_int64(NT * Ct), C.c_int32(Ct), _p(keep))
    return keep


def rowseg_sumsq(W, Cs):
    """Sums of squares of the row segments of Cs columns (the other division of Alg. 1), fp32 canonical chain."""
    W = _f32(W)
    M, N = W.shape
    assert N % Cs == 0
    s = np.empty((M, N // Cs), dtype=np.float32)
    lib().orc_rowseg_sumsq(_p(W), C.c_int64(M), C.c_int64(N), C.c_int32(Cs), _p(s))
    return s
