"""GPU vs CPU oracle, element by element, through the C ABI (paper_2009_08065_amd.bsp).

Bars: bit-exact for sums of squares, norms, reweighting factors, gradients, masks and the
compact storage; for Y, |y - y_oracle| <= tol * (|y_oracle| + rms(y_oracle)) with tol = 2e-2
for bf16 / fp16 and 1e-5 for fp32."""
import numpy as np
import pytest
import torch

import bsp_workloads as wl
import paper_2009_08065_amd as bsp
from oracle import bsp_oracle as orc

pytestmark = pytest.mark.gpu

TDT = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}
CODE = {"f32": orc.F32, "bf16": orc.BF16, "f16": orc.F16}
TOL = {"f32": 1e-5, "bf16": 2e-2, "f16": 2e-2}


def dev(a, dtype="f32"):
    """numpy float32 (values representable in dtype) -> GPU tensor of that dtype."""
    if a is None:
        return None
    return torch.from_numpy(np.ascontiguousarray(a)).to(TDT[dtype]).cuda()


def host(t):
    return t.detach().float().cpu().numpy() if t.is_floating_point() else t.detach().cpu().numpy()


def bits_equal(gpu_f32, ref_f32):
    a = np.ascontiguousarray(gpu_f32, dtype=np.float32).view(np.uint32)
    b = np.ascontiguousarray(ref_f32, dtype=np.float32).view(np.uint32)
    return np.array_equal(a, b)


# What the arithmetic allows, far inside the stated tolerance: both sides round one fp32 / fp64 sum to the output
# type, so they differ by at most one unit in the last place of that type where the sums straddle a rounding
# boundary (2^-7 relative for bf16, 2^-10 for fp16), plus the fp32 accumulation error of the kernel, which is of
# the order sqrt(k) 2^-24 of the rms of the outputs (k <= 4096 terms): 1e-3 rms leaves two decimal orders of room.
ULP = {"bf16": 2.0 ** -7, "f16": 2.0 ** -10}


def assert_y_close(y_gpu, y_ref, dtype, rows=None):
    y_ref = y_ref.astype(np.float64)
    y_gpu = y_gpu.astype(np.float64)
    if rows is not None:
        y_ref, y_gpu = y_ref[rows], y_gpu[rows]
    rms = np.sqrt(np.mean(y_ref ** 2))
    err = np.abs(y_gpu - y_ref)
    bound = TOL[dtype] * (np.abs(y_ref) + rms)          # the stated tolerance: max relative error, rms as the floor
    if dtype in ULP:
        bound = np.minimum(bound, ULP[dtype] * np.abs(y_ref) + 1e-3 * rms)
    if not np.all(err <= bound):     # (an all-zero reference has bound 0 and must be matched exactly)
        with np.errstate(divide="ignore", invalid="ignore"):
            worst = np.nanmax(np.where(err > bound, err / bound, 0.0))
        raise AssertionError(f"worst err/bound = {worst:.3f}")


def pack_equal(p_gpu, p_ref):
    assert np.array_equal(host(p_gpu.blk_cnt), p_ref["blk_cnt"])
    assert np.array_equal(host(p_gpu.blk_ptr), p_ref["blk_ptr"])
    assert p_gpu.total_cols == int(p_ref["blk_ptr"][-1])
    assert np.array_equal(host(p_gpu.col_idx), p_ref["col_idx"])
    assert bits_equal(host(p_gpu.vals), p_ref["vals"])


# ------------------------------------------------------------------------------ norms
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("R,M,N", [(16, 96, 1024), (8, 64, 777), (32, 64, 520), (1, 5, 64), (3, 27, 130), (64, 128, 72)])
def test_group_norms_bit_exact(dtype, R, M, N):
    W = wl.normal(R * 100 + N, (M, N), 0.02, dtype)
    W[0:R, 3] = 0.0                                    # an all-zero group
    for mode in (orc.ALPHA_SQNORM, orc.ALPHA_NORM):
        s, nrm, alpha = bsp.bsp_group_norms(dev(W, dtype), R, eps=1e-6, mode=mode)
        s_ref = orc.sumsq(W, R)
        n_ref, a_ref = orc.norm_alpha(s_ref, 1e-6, mode)
        assert bits_equal(host(s), s_ref)
        assert bits_equal(host(nrm), n_ref)
        assert bits_equal(host(alpha), a_ref)


def test_group_norms_wide_value_range_and_partial_outputs():
    rng = np.random.default_rng(5)
    W = (rng.standard_normal((64, 256)) * np.exp(rng.uniform(-20, 20, (64, 256)))).astype(np.float32)
    s_ref = orc.sumsq(W, 16)
    s, nrm, alpha = bsp.bsp_group_norms(dev(W), 16, want=("sumsq",))
    assert nrm is None and alpha is None and bits_equal(host(s), s_ref)
    _, nrm, _ = bsp.bsp_group_norms(dev(W), 16, want=("norm",))
    assert bits_equal(host(nrm), orc.norm_alpha(s_ref, 1e-6, 0)[0])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("R,M,N", [(16, 64, 512), (8, 32, 264), (32, 64, 100), (5, 20, 77)])
@pytest.mark.parametrize("mode", [orc.ALPHA_SQNORM, orc.ALPHA_NORM])
def test_penalty_grad(dtype, R, M, N, mode):
    W = wl.normal(R + N, (M, N), 0.02, dtype)
    W[0:R, 1] = 0.0
    lam = 1e-4
    _, alpha = orc.norm_alpha(orc.sumsq(W, R), 1e-6, mode)
    G_ref, pen_ref = orc.penalty_grad(W, R, alpha, lam, mode, gdt=CODE[dtype])
    Wd, ad = dev(W, dtype), dev(alpha)
    G, pen = bsp.bsp_penalty_grad(Wd, R, ad, lam, mode=mode, want_penalty=True)
    assert bits_equal(host(G), G_ref)
    assert abs(pen.item() - pen_ref) <= 1e-11 * abs(pen_ref)
    G2, pen2 = bsp.bsp_penalty_grad(Wd, R, ad, lam, mode=mode, want_penalty=True)
    assert pen2.item() == pen.item()                   # fixed summation order
    G3, _ = bsp.bsp_penalty_grad(Wd, R, ad, lam, mode=mode)
    assert bits_equal(host(G3), G_ref)
    G0 = wl.normal(99, (M, N), 0.01, dtype)
    Gacc_ref, _ = orc.penalty_grad(W, R, alpha, lam, mode, gdt=CODE[dtype], G0=G0)
    Gacc, _ = bsp.bsp_penalty_grad(Wd, R, ad, lam, mode=mode, grad=dev(G0, dtype), accumulate=True)
    assert bits_equal(host(Gacc), Gacc_ref)


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("R,M,N", [(16, 64, 512), (8, 32, 264), (32, 64, 1024), (5, 20, 77), (64, 128, 520)])
@pytest.mark.parametrize("mode", [orc.ALPHA_SQNORM, orc.ALPHA_NORM])
def test_group_norms_grad_one_pass(dtype, R, M, N, mode):
    """The fused refresh + gradient is the chain sumsq -> factors -> Eq. 3 gradient, bit for bit."""
    W = wl.normal(7 * R + N, (M, N), 0.02, dtype)
    W[0:R, 1] = 0.0
    lam = 1e-4
    s_ref = orc.sumsq(W, R)
    n_ref, a_ref = orc.norm_alpha(s_ref, 1e-6, mode)
    G_ref, _ = orc.penalty_grad(W, R, a_ref, lam, mode, gdt=CODE[dtype])
    Wd = dev(W, dtype)
    s, nrm, alpha, G = bsp.bsp_group_norms_grad(Wd, R, lam, eps=1e-6, mode=mode, want=("sumsq", "norm", "alpha"))
    assert bits_equal(host(s), s_ref) and bits_equal(host(nrm), n_ref) and bits_equal(host(alpha), a_ref)
    assert bits_equal(host(G), G_ref)
    s2, nrm2, alpha2, G2 = bsp.bsp_group_norms_grad(Wd, R, lam, eps=1e-6, mode=mode, want=())
    assert s2 is None and nrm2 is None and alpha2 is None and bits_equal(host(G2), G_ref)
    G0 = wl.normal(98, (M, N), 0.01, dtype)
    Gacc_ref, _ = orc.penalty_grad(W, R, a_ref, lam, mode, gdt=CODE[dtype], G0=G0)
    _, _, _, Gacc = bsp.bsp_group_norms_grad(Wd, R, lam, eps=1e-6, mode=mode, grad=dev(G0, dtype), accumulate=True)
    assert bits_equal(host(Gacc), Gacc_ref)
    # the two separate calls give the same bits
    _, _, alpha_d = bsp.bsp_group_norms(Wd, R, eps=1e-6, mode=mode)
    G_sep, _ = bsp.bsp_penalty_grad(Wd, R, alpha_d, lam, mode=mode)
    assert torch.equal(G_sep.view(torch.uint8), G.view(torch.uint8))


@pytest.mark.parametrize("gdt", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("R,M,N", [(16, 64, 512), (8, 32, 264), (5, 20, 77), (64, 128, 1028)])
def test_adam_step_bit_exact(gdt, R, M, N):
    """The Adam update of Alg. 2 (plain, on the mixed loss, and followed by W = W * Mask): fp32, one rounding per
    operation on both sides, so W, m and v agree bit for bit over several steps with the state carried by each side."""
    B = M // R
    W0 = wl.normal(11 * R + N, (M, N), 0.05)
    W0[0:R, 1] = 0.0
    rng = np.random.default_rng(R * 1000 + N)
    keep = (rng.random((B, N)) < 0.3).astype(np.uint8)
    hp = dict(lr=3e-5, beta1=0.9, beta2=0.999, eps=1e-8)
    lam = 1e-3
    for mode, use_alpha, use_keep in ((orc.ALPHA_SQNORM, False, False), (orc.ALPHA_SQNORM, True, False),
                                      (orc.ALPHA_NORM, True, False), (orc.ALPHA_SQNORM, False, True),
                                      (orc.ALPHA_NORM, True, True)):
        W, m, v = W0.copy(), np.zeros_like(W0), np.zeros_like(W0)
        Wd, md, vd = dev(W), dev(m), dev(v)
        _, alpha = orc.norm_alpha(orc.sumsq(W0, R), 1e-6, mode)
        ad = dev(alpha) if use_alpha else None
        kd = torch.from_numpy(keep).cuda() if use_keep else None
        for t in (1, 2, 3, 1000):
            G = wl.normal(100 + t, (M, N), 1e-3, gdt)
            W, m, v = orc.adam_step(W, G, m, v, R, t=t, alpha=alpha if use_alpha else None, lam=lam, mode=mode,
                                    keep=keep if use_keep else None, **hp)
            bsp.bsp_adam_step(Wd, dev(G, gdt), md, vd, R, t=t, alpha=ad, lam=lam, mode=mode, keep=kd, **hp)
            assert bits_equal(host(Wd), W), (mode, use_alpha, use_keep, t)
            assert bits_equal(host(md), m) and bits_equal(host(vd), v)
        if use_keep:
            assert not host(Wd)[~np.repeat(keep, R, axis=0).astype(bool)].any()


def test_adam_step_argument_checks():
    W = torch.zeros(32, 64, device="cuda")
    L = bsp.lib()
    args = lambda **k: dict(dict(W=W.data_ptr(), G=W.data_ptr(), gdt=bsp.F32, m=W.data_ptr(), v=W.data_ptr(), M=32, N=64,
                                 R=16, t=1), **k)

    def call(a):
        return L.bsp_adam_step(a["W"], a["G"], a["gdt"], a["m"], a["v"], a["M"], a["N"], a["R"], None, 0.0, 0, None,
                               1e-5, 0.9, 0.999, 1e-8, a["t"], None)
    assert call(args(W=None)) != 0 and call(args(G=None)) != 0 and call(args(m=None)) != 0 and call(args(v=None)) != 0
    assert call(args(gdt=7)) != 0 and call(args(R=5)) != 0 and call(args(R=0)) != 0 and call(args(t=0)) != 0
    torch.cuda.synchronize()
    assert not W.any()


# ------------------------------------------------------------------------------ masks
def test_mask_threshold_bit_exact_with_ties():
    W = wl.normal(3, (64, 333), 0.02)
    s = orc.sumsq(W, 16)
    t = np.float32(np.sqrt(np.median(s)))
    s[1, 5] = np.float32(float(t) * float(t))           # as close to the tie as fp32 allows
    for tt in (-1.0, 0.0, float(t), 0.05, 10.0):
        keep, _ = bsp.bsp_prune_mask(dev(s), t=tt)
        assert np.array_equal(host(keep), orc.mask_threshold(s, tt))
    sq = np.array([[0.25, 0.2500001, 0.2499999, 0.0]], np.float32)   # Alg. 1: norm == t is pruned
    assert host(bsp.bsp_prune_mask(dev(sq), t=0.5)[0]).tolist() == [[0, 1, 0, 0]]


@pytest.mark.parametrize("scope", [orc.SCOPE_BLOCK, orc.SCOPE_MATRIX])
@pytest.mark.parametrize("B,N", [(48, 768), (7, 1000), (3, 65), (1, 1), (64, 4096)])
def test_mask_rank_bit_exact(scope, B, N):
    W = wl.normal(B + N, (B * 16, N), 0.02)
    s = orc.sumsq(W, 16)
    if N > 8:
        s[0, 1] = s[0, 2] = s[0, 3]                    # ties
        s[B - 1, :] = s[B - 1, 0]                      # a constant row
    if B > 2:
        s[1, 0] = 0.0
    n = N if scope == orc.SCOPE_BLOCK else B * N
    sd = dev(s)
    for n_keep in sorted({0, 1, n // 5, n // 3, n // 2, n - 1, n, n + 5}):
        keep, t_used = bsp.bsp_prune_mask(sd, n_keep=n_keep, scope=scope, want_t_used=True)
        k_ref, t_ref = orc.mask_rank(s, n_keep, scope)
        assert np.array_equal(host(keep), k_ref), n_keep
        assert bits_equal(host(t_used), t_ref), n_keep


@pytest.mark.parametrize("scope", [orc.SCOPE_BLOCK, orc.SCOPE_MATRIX])
@pytest.mark.parametrize("B,N,k_align", [(48, 768, 32), (7, 1000, 8), (3, 65, 1), (1, 1, 32), (64, 4096, 32),
                                         (256, 1024, 32), (1500, 258, 16), (33, 2047, 64)])
def test_mask_and_storage_sizes_in_one_call(scope, B, N, k_align):
    # the mask of bsp_prune_mask and the counts of bsp_pack_count from one call: the oracle's mask, its counts
    W = wl.normal(B * 3 + N, (B * 4, N), 0.02)
    s = orc.sumsq(W, 4)
    if N > 8:
        s[0, 1] = s[0, 2] = s[0, 3]
    n = N if scope == orc.SCOPE_BLOCK else B * N
    sd = dev(s)
    ws = torch.empty(max(bsp.lib().bsp_prune_mask_workspace_bytes(B, N, scope), 16), dtype=torch.uint8, device="cuda")
    for n_keep in sorted({0, n // 5, n // 2, n - 1, n}):
        ws.random_(0, 256)                              # nothing in the workspace has to be cleared by the caller
        t_used = torch.empty(B if scope == orc.SCOPE_BLOCK else 1, dtype=torch.float32, device="cuda")
        keep, t_used, cnt, ptr = bsp.bsp_prune_mask_count(sd, n_keep=n_keep, scope=scope, k_align=k_align,
                                                          t_used=t_used, ws=ws)
        k_ref, t_ref = orc.mask_rank(s, n_keep, scope)
        cnt_ref, ptr_ref = orc.pack_count(k_ref, k_align)
        assert np.array_equal(host(keep), k_ref), n_keep
        assert bits_equal(host(t_used), t_ref), n_keep
        assert np.array_equal(host(cnt), cnt_ref) and np.array_equal(host(ptr), ptr_ref), n_keep
    # the threshold form
    keep, _, cnt, ptr = bsp.bsp_prune_mask_count(sd, t=0.04, k_align=k_align)
    k_ref = orc.mask_threshold(s, 0.04)
    cnt_ref, ptr_ref = orc.pack_count(k_ref, k_align)
    assert np.array_equal(host(keep), k_ref) and np.array_equal(host(cnt), cnt_ref) and np.array_equal(host(ptr), ptr_ref)


def test_mask_rank_wide_range_and_negative_values():
    rng = np.random.default_rng(11)
    s = (rng.standard_normal((16, 500)) * np.exp(rng.uniform(-30, 30, (16, 500)))).astype(np.float32)
    for scope in (orc.SCOPE_BLOCK, orc.SCOPE_MATRIX):
        n = 500 if scope == orc.SCOPE_BLOCK else 8000
        for n_keep in (n // 7, n // 2, n - 3):
            keep, t_used = bsp.bsp_prune_mask(dev(s), n_keep=n_keep, scope=scope, want_t_used=True)
            k_ref, t_ref = orc.mask_rank(s, n_keep, scope)
            assert np.array_equal(host(keep), k_ref) and bits_equal(host(t_used), t_ref)


# ------------------------------------------------------------------------------ packing
@pytest.mark.parametrize("k_align", [1, 8, 16, 32, 64])
@pytest.mark.parametrize("R,N,wdt,vdt", [(16, 768, "f32", "f32"), (8, 300, "f32", "bf16"), (32, 1030, "bf16", "bf16"),
                                         (3, 75, "f16", "f16"), (1, 40, "f32", "f16"), (64, 129, "bf16", "f32")])
def test_pack_bit_exact(R, N, wdt, vdt, k_align):
    M = 6 * R
    W = wl.normal(R + N, (M, N), 0.02, wdt)
    keep = wl.bernoulli_keep_mask(R * 7 + k_align, M // R, N, 0.3)
    keep[1, :] = 0
    keep[2, :] = 1
    keep[3, :] = 0
    keep[3, N - 1] = 1
    p = bsp.bsp_pack(dev(W, wdt), R, torch.from_numpy(keep).cuda(), k_align,
                     vdt=CODE[vdt])
    pack_equal(p, orc.pack(W, R, keep, k_align, CODE[vdt]))
    assert bsp.bsp_packed_validate(p)
    if p.total_cols:
        bad = bsp.Packed(p.M, p.N, p.R, p.k_align, p.blk_cnt, p.blk_ptr, p.col_idx.clone(), p.vals, p.total_cols)
        bad.col_idx[0] = N
        assert not bsp.bsp_packed_validate(bad)


@pytest.mark.parametrize("B,N", [(1024, 32), (1025, 31), (43, 749), (1, 1), (1024, 33), (37, 14000), (2, 16384)])
@pytest.mark.parametrize("k_align", [1, 32])
def test_pack_count_one_launch_and_two(B, N, k_align):
    # small masks are counted and scanned by one workgroup, larger ones by a count launch and a scan launch
    keep = wl.bernoulli_keep_mask(B * 7 + N, B, N, 0.3)
    keep[B // 2, :] = 0
    keep[keep != 0] = np.random.default_rng(B + N).integers(1, 256, size=int(np.count_nonzero(keep)), dtype=np.uint8)
    cnt_ref, ptr_ref = orc.pack_count(keep, k_align)
    cnt, ptr = bsp.bsp_pack_count(torch.from_numpy(keep).cuda(), k_align)
    assert np.array_equal(host(cnt), cnt_ref) and np.array_equal(host(ptr), ptr_ref)


def test_pack_all_empty_and_capacity_guard():
    W = wl.normal(1, (32, 64), 0.02)
    keep0 = torch.zeros((2, 64), dtype=torch.uint8, device="cuda")
    p = bsp.bsp_pack(dev(W), 16, keep0, 32)
    assert p.total_cols == 0 and host(p.blk_ptr).tolist() == [0, 0, 0] and bsp.bsp_packed_validate(p)
    Y = bsp.bsp_linear(dev(wl.normal(2, (5, 64), 1.0)), p, dev(wl.normal(3, (32,), 0.02)))
    assert bits_equal(host(Y), np.broadcast_to(wl.normal(3, (32,), 0.02), (5, 32)))
    # capacity smaller than needed: blocks beyond it stay unwritten, nothing out of bounds
    keep = torch.from_numpy(wl.random_keep_mask(4, 2, 64, 20)).cuda()
    cnt, ptr = bsp.bsp_pack_count(keep, 32)
    assert host(ptr).tolist() == [0, 32, 64]
    col = torch.full((64,), -7, dtype=torch.int32, device="cuda")
    vals = torch.full((16 * 64,), 5.0, device="cuda")
    st = bsp.lib().bsp_pack(dev(W).data_ptr(), 0, 32, 64, 16, keep.data_ptr(), 32, cnt.data_ptr(), ptr.data_ptr(), 32,
                            col.data_ptr(), vals.data_ptr(), 0, None)
    torch.cuda.synchronize()
    assert st == 0 and (host(col)[32:] == -7).all() and (host(col)[:20] >= 0).all() and (host(vals)[16 * 32:] == 5).all()


# ------------------------------------------------------------------------------ masked weights
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("R,M,N", [(16, 96, 1024), (8, 64, 777), (3, 27, 130), (64, 128, 73), (1, 5, 1)])
def test_mask_weights_bit_exact(dtype, R, M, N):
    W = wl.normal(R * 10 + N, (M, N), 0.02, dtype)
    W[0, 0] = -0.0
    keep = wl.bernoulli_keep_mask(R + M + N, M // R, N, 0.3)
    keep[0, :] = 0
    if M // R > 1:
        keep[1, :] = 1
    Wd = dev(W, dtype)
    out = bsp.bsp_mask_weights(Wd, R, torch.from_numpy(keep).cuda())
    assert out.data_ptr() == Wd.data_ptr()
    assert bits_equal(host(Wd), orc.mask_weights(W, R, keep))
    # a view that starts on an odd element: the two-element stores must not be used
    holder = dev(np.concatenate([np.zeros(1, np.float32), W.reshape(-1)]), dtype)
    Wo = holder[1:].view(M, N)
    bsp.bsp_mask_weights(Wo, R, torch.from_numpy(keep).cuda())
    assert bits_equal(host(Wo), orc.mask_weights(W, R, keep)) and float(holder[0]) == 0.0


# ------------------------------------------------------------------------------ the layer
def run_layer(X, W, bias, R, keep, k_align, dtype, T_rows=None):
    code = CODE[dtype]
    p_ref = orc.pack(W, R, keep, k_align, code)
    Xd, bd = dev(X, dtype), dev(bias, dtype)
    p = bsp.bsp_pack(dev(W, dtype), R, torch.from_numpy(np.ascontiguousarray(keep)).cuda(), k_align)
    pack_equal(p, p_ref)
    check = lambda y: _check_y(y, X, p_ref, bias, code, dtype, T_rows)
    Y = host(bsp.bsp_linear(Xd, p, bd))
    if k_align % 32 == 0 and bsp.bsp_linear_plan_supported(TDT[dtype], X.shape[1], k_align):
        # the planned path computes the same sums from a re-ordered copy of the storage
        Yp = host(bsp.bsp_linear_planned(Xd, p, bsp.bsp_linear_plan(p), bd))
        check(Yp)
    check(Y)
    return Y, p


def _check_y(Y, X, p_ref, bias, code, dtype, T_rows):
    if T_rows is None:
        Y_ref, _ = orc.linear_packed(X, p_ref, bias, ydt=code, n_threads=16)
        assert_y_close(Y, Y_ref, dtype)
    else:
        for (t0, t1) in T_rows:
            Y_ref, _ = orc.linear_packed(X, p_ref, bias, ydt=code, t0=t0, t1=t1, n_threads=16)
            assert_y_close(Y, Y_ref, dtype, rows=slice(t0, t1))


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("k_align", [1, 16, 32])
@pytest.mark.parametrize("R,T,M,N,p_keep", [(16, 100, 64, 200, 0.5), (8, 70, 40, 333, 0.2), (32, 130, 96, 256, 0.33),
                                            (1, 9, 7, 50, 0.5), (3, 65, 12, 100, 0.7), (64, 17, 128, 96, 0.4)])
def test_linear_small_shapes(dtype, k_align, R, T, M, N, p_keep):
    d = wl.layer(R * 1000 + T, T, M, N, dtype)
    keep = wl.bernoulli_keep_mask(T + N, M // R, N, p_keep)
    keep[0, :] = 0                                      # a row-block with nothing kept: bias only
    if M // R > 1:
        keep[1, :] = 1                                  # a dense row-block
    run_layer(d["X"], d["W"], d["bias"], R, keep, k_align, dtype)
    run_layer(d["X"], d["W"], None, R, keep, k_align, dtype)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("R,T,M,N,p_keep", [(16, 150, 272, 2304, 0.2), (16, 64, 48, 1032, 0.5), (32, 70, 160, 4096, 0.1),
                                            (64, 33, 192, 3000, 0.3), (8, 129, 136, 1280, 0.25)])
def test_linear_wide_layers_in_column_chunks(dtype, R, T, M, N, p_keep):
    # more than 1024 input columns: the planned path walks X in chunks of 1024 columns (the last one
    # ragged) and carries several row-blocks per wavefront across the chunks
    d = wl.layer(R * 7 + N, T, M, N, dtype)
    B = M // R
    keep = wl.bernoulli_keep_mask(T + N + 1, B, N, p_keep)
    keep[0, :] = 0                                      # nothing kept
    keep[1, :] = 1                                      # dense
    keep[2, :1024] = 0                                  # first chunk empty
    if B > 3:
        keep[3, 1024:] = 0                              # only the first chunk
    if B > 4:
        keep[4, :] = 0
        keep[4, 1023:1025] = 1                          # one column on each side of a chunk border
    run_layer(d["X"], d["W"], d["bias"], R, keep, 32, dtype)
    run_layer(d["X"], d["W"], None, R, keep, 64, dtype)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("R,T,M,N", [(16, 100, 80, 200), (16, 4100, 2128, 512), (32, 200, 224, 1024), (64, 130, 320, 640),
                                     (8, 130, 88, 512), (8, 300, 1048, 1024)])
def test_linear_planned_output_paths(dtype, R, T, M, N):
    # layers of up to 1024 columns on the planned path: an odd number of row-blocks (the last one leaves
    # alone), several strips and groups, one and two fragments per staged row, ragged token tiles
    d = wl.layer(R + T + M, T, M, N, dtype)
    keep = wl.bernoulli_keep_mask(R + T + M + 1, M // R, N, 0.25)
    keep[1, :] = 0
    keep[M // R - 1, :] = 0                              # the lone last block with nothing kept
    rows = None if T < 1000 else [(0, 70), (2040, 2060), (4090, 4100)]
    run_layer(d["X"], d["W"], d["bias"], R, keep, 32, dtype, T_rows=rows)
    keep[M // R - 1, ::3] = 1
    run_layer(d["X"], d["W"], None, R, keep, 32, dtype, T_rows=rows)


@pytest.mark.parametrize("T,M,N", [(130, 96, 512), (70, 160, 1024), (100, 64, 2048), (65, 208, 3000), (64, 32, 777)])
def test_linear_planned_pairs_of_8_row_blocks(T, M, N):
    # 8-row blocks in a layer of even block count: a block of the plan is the union of two stored blocks' columns.
    # Pairs with the same columns, with disjoint columns, with one or both blocks empty, a full block beside a
    # sparse one; one chunk and several
    R, B = 8, M // 8
    d = wl.layer(T + M + N, T, M, N, "bf16")
    keep = wl.bernoulli_keep_mask(T + M + N + 1, B, N, 0.22)
    keep[1, :] = keep[0, :]                              # the same columns
    keep[2, :] = 0
    keep[2, ::5] = 1
    keep[3, :] = 0
    keep[3, 1::5] = 1                                    # disjoint
    if B >= 8:
        keep[4, :] = 0                                   # first of the pair empty
        keep[6, :] = 0
        keep[7, :] = 0                                   # both empty
    if B >= 12:
        keep[9, :] = 0                                   # second of the pair empty
        keep[10, :] = 1                                  # everything kept beside a sparse block
        keep[11, :] = 0
        keep[11, N - 1] = 1
    run_layer(d["X"], d["W"], d["bias"], R, keep, 32, "bf16")
    run_layer(d["X"], d["W"], None, R, keep, 64, "bf16")


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("R,T,M,N", [(32, 130, 96, 512), (32, 4100, 2144, 1024), (64, 70, 320, 2048), (48, 65, 240, 3000),
                                     (64, 100, 64, 777), (32, 64, 1056, 4096)])
def test_linear_planned_slabs_of_tall_row_blocks(dtype, R, T, M, N):
    # 32-, 48- and 64-row blocks: a block of the plan is a 16-row slab of a stored block.  An empty block, a full
    # block, an odd number of stored blocks, one chunk and several, ragged token tiles
    d = wl.layer(R + T + M + N, T, M, N, dtype)
    keep = wl.bernoulli_keep_mask(R + T + M + N + 1, M // R, N, 0.22)
    keep[0, :] = 0
    if M // R > 2:
        keep[2, :] = 1
    rows = None if T < 1000 else [(0, 70), (2040, 2060), (4090, 4100)]
    run_layer(d["X"], d["W"], d["bias"], R, keep, 32, dtype, T_rows=rows)
    run_layer(d["X"], d["W"], None, R, keep, 64, dtype, T_rows=rows)


@pytest.mark.parametrize("R", [16, 8])
def test_linear_planned_bias_at_odd_address(R):
    # a bias that starts on a 2-byte boundary cannot be read in 4-byte words: the element-wise output path
    T, M, N = 90, 96, 256
    d = wl.layer(5150, T, M, N, "bf16")
    keep = wl.bernoulli_keep_mask(5151, M // R, N, 0.3)
    p_ref = orc.pack(d["W"], R, keep, 32, CODE["bf16"])
    p = bsp.bsp_pack(dev(d["W"], "bf16"), R, torch.from_numpy(keep).cuda(), 32)
    holder = torch.zeros(M + 1, dtype=torch.bfloat16, device="cuda")
    holder[1:] = dev(d["bias"], "bf16")
    bias_odd = holder[1:]
    assert bias_odd.data_ptr() % 4 == 2
    Xd = dev(d["X"], "bf16")
    Y_ref, _ = orc.linear_packed(d["X"], p_ref, d["bias"], ydt=CODE["bf16"], n_threads=16)
    assert_y_close(host(bsp.bsp_linear_planned(Xd, p, bsp.bsp_linear_plan(p), bias_odd)), Y_ref, "bf16")
    assert_y_close(host(bsp.bsp_linear(Xd, p, bias_odd)), Y_ref, "bf16")
    # an output that does not start on a 16-byte boundary is refused (and left untouched)
    ybuf = torch.full((T * M + 1,), 7.0, dtype=torch.bfloat16, device="cuda")
    Y_odd = ybuf[1:].view(T, M)
    assert Y_odd.data_ptr() % 16 == 2
    with pytest.raises(bsp.BspError):
        bsp.bsp_linear_planned(Xd, p, bsp.bsp_linear_plan(p), bias_odd, Y=Y_odd)
    torch.cuda.synchronize()
    assert torch.all(ybuf == 7.0)


def test_linear_wide_layer_many_tokens_ragged_strips():
    # enough token tiles that every wavefront carries 4 row-blocks across the chunks; 133 row-blocks
    # leave the last strip with one group and that group with 5 of its 8 row-blocks
    R, T, M, N = 16, 4100, 2128, 2304
    d = wl.layer(991, T, M, N, "bf16")
    keep = wl.bernoulli_keep_mask(992, M // R, N, 0.2)
    keep[5, :] = 0
    keep[130, 1024:2048] = 0
    run_layer(d["X"], d["W"], d["bias"], R, keep, 32, "bf16", T_rows=[(0, 70), (2040, 2060), (4090, 4100)])


def test_linear_seeded_random_shapes():
    """Eighty seeded draws over block sizes, widths (one tile and column chunks), ragged token counts, densities,
    alignments, dtypes, empty row-blocks, no bias: both layer entry points against the oracle."""
    rng = np.random.default_rng(20250)
    for it in range(80):
        R = int(rng.choice([16, 16, 16, 32, 32, 64, 8, 4, 24]))
        B = int(rng.integers(1, 70))
        M = R * B
        N = int(rng.choice([32, 64, 200, 256, 520, 768, 1000, 1024, 1032, 2048, 3000, 4096]))
        T = int(rng.integers(1, 330))
        dt = str(rng.choice(["bf16", "f16"]))
        p_keep = float(rng.choice([0.05, 0.2, 0.5, 0.9]))
        k_align = int(rng.choice([32, 64]))
        d = wl.layer(1000 + it, T, M, N, dt)
        keep = wl.bernoulli_keep_mask(5000 + it, B, N, p_keep)
        if it % 7 == 0:
            keep[int(rng.integers(0, B))] = 0          # an empty row-block
        if it % 11 == 0:
            keep[:] = 0                                 # nothing kept: the bias alone
        use_bias = it % 3 != 0
        p_ref = orc.pack(d["W"], R, keep, k_align, CODE[dt])
        p = bsp.bsp_pack(dev(d["W"], dt), R, torch.from_numpy(keep).cuda(), k_align)
        bias = dev(d["bias"], dt) if use_bias else None
        Y_ref, _ = orc.linear_packed(d["X"], p_ref, d["bias"] if use_bias else None, ydt=CODE[dt], n_threads=16)
        Xd = dev(d["X"], dt)
        case = dict(it=it, R=R, B=B, N=N, T=T, dt=dt, p=p_keep, k_align=k_align, bias=use_bias)
        try:
            assert_y_close(host(bsp.bsp_linear_planned(Xd, p, bsp.bsp_linear_plan(p), bias)), Y_ref, dt)
            assert_y_close(host(bsp.bsp_linear(Xd, p, bias)), Y_ref, dt)
        except AssertionError as e:
            raise AssertionError(f"{case}: {e}")


# ------------------------------------------------------------------------------ the layer with its epilogue
FUSED_CASES = [
    # (dtype, R, T, M, N, act, residual): the kernel for narrow layers (activation only) ...
    ("bf16", 16, 200, 1536, 768, True, False), ("f16", 16, 77, 512 + 16, 1000, True, False),
    ("bf16", 8, 130, 1280, 512, True, False),
    # ... and the kernel that streams X (wide layers; layers of few row-blocks): activation, residual, both
    ("bf16", 16, 150, 256, 2048, False, True), ("bf16", 16, 333, 1024, 1024, False, True),
    ("f16", 16, 100, 96, 4096, True, True), ("bf16", 8, 65, 336, 3000, True, True),
    ("bf16", 16, 64, 1024, 768, True, False),
    # row-blocks of 32, 48 and 64 rows run as their 16-row slabs
    ("bf16", 32, 130, 1280, 512, True, False), ("f16", 64, 70, 320, 2048, True, True),
    ("bf16", 48, 65, 480, 1024, False, True), ("bf16", 32, 100, 2144, 3000, True, True),
]


@pytest.mark.parametrize("dtype,R,T,M,N,act,with_res", FUSED_CASES)
def test_linear_fused_epilogue(dtype, R, T, M, N, act, with_res):
    """Exact GELU and residual inside the layer kernel against the oracle's layer followed by its epilogue (one
    rounding); also with an empty row-block and without a bias."""
    d = wl.layer(7000 + T + N, T, M, N, dtype)
    keep = wl.bernoulli_keep_mask(7100 + M, M // R, N, 0.25)
    keep[1, :] = 0
    res = wl.layer(7200 + T, T, 16, M, dtype)["X"] if with_res else None   # a [T, M] tensor of N(0, 1) values
    p_ref = orc.pack(d["W"], R, keep, 32, CODE[dtype])
    p = bsp.bsp_pack(dev(d["W"], dtype), R, torch.from_numpy(keep).cuda(), 32)
    plan = bsp.bsp_linear_plan(p)
    code = orc.ACT_GELU if act else orc.ACT_NONE
    for bias in (d["bias"], None):
        Y_ref, _ = orc.linear_packed_fused(d["X"], p_ref, bias, act=code, residual=res, ydt=CODE[dtype], n_threads=16)
        Y = bsp.bsp_linear_planned_fused(dev(d["X"], dtype), p, plan, dev(bias, dtype),
                                         act=bsp.ACT_GELU if act else bsp.ACT_NONE, residual=dev(res, dtype))
        assert_y_close(host(Y), Y_ref, dtype)


def test_linear_fused_epilogue_refuses_what_is_not_fused():
    """Row-blocks of other heights, and a residual for a layer whose kernel stores block by block: an error and
    nothing written."""
    for (R, M, N, act, with_res) in [(24, 240, 512, bsp.ACT_GELU, False), (16, 2048, 1024, bsp.ACT_NONE, True),
                                     (16, 256, 512, 7, False)]:
        d = wl.layer(7300 + R, 64, M, N, "bf16")
        keep = wl.bernoulli_keep_mask(7301, M // R, N, 0.3)
        p = bsp.bsp_pack(dev(d["W"], "bf16"), R, torch.from_numpy(keep).cuda(), 32)
        plan = bsp.bsp_linear_plan(p)
        Y = torch.full((64, M), 3.0, dtype=torch.bfloat16, device="cuda")
        res = torch.zeros((64, M), dtype=torch.bfloat16, device="cuda") if with_res else None
        with pytest.raises(bsp.BspError):
            bsp.bsp_linear_planned_fused(dev(d["X"], "bf16"), p, plan, None, act=act, residual=res, Y=Y)
        assert float(Y.float().min()) == 3.0 and float(Y.float().max()) == 3.0


# ------------------------------------------------------------------------------ the transposed product
def run_transposed(U, W, bias, R, keep, k_align, dtype, T_rows=None):
    code = CODE[dtype]
    p_ref = orc.pack(W, R, keep, k_align, code)
    p = bsp.bsp_pack(dev(W, dtype), R, torch.from_numpy(np.ascontiguousarray(keep)).cuda(), k_align)
    pack_equal(p, p_ref)
    Z = host(bsp.bsp_linear_transposed(dev(U, dtype), p, dev(bias, dtype)))
    assert Z.shape == (U.shape[0], W.shape[1])
    for (t0, t1) in (T_rows or [(0, U.shape[0])]):
        Z_ref, _ = orc.linear_t_packed(U, p_ref, bias, zdt=code, t0=t0, t1=t1, n_threads=16)
        assert_y_close(Z, Z_ref, dtype, rows=slice(t0, t1))
    return Z, p_ref


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("k_align", [1, 8, 32])
@pytest.mark.parametrize("R,T,M,N,p_keep", [(16, 100, 64, 200, 0.5), (8, 70, 40, 333, 0.2), (32, 130, 96, 256, 0.33),
                                            (1, 9, 7, 50, 0.5), (3, 65, 12, 100, 0.7), (64, 17, 128, 96, 0.4),
                                            (4, 33, 36, 515, 0.6), (24, 64, 48, 1024, 0.25), (48, 40, 96, 300, 0.5),
                                            (40, 50, 80, 260, 0.4), (64, 200, 192, 520, 0.9)])
def test_linear_transposed_small_shapes(dtype, k_align, R, T, M, N, p_keep):
    d = wl.layer(R * 1000 + T + 7, T, M, N, dtype)
    U = wl.normal(R * 77 + T, (T, M), 1.0, dtype)
    zb = wl.normal(R * 78 + T, (N,), 0.5, dtype)
    keep = wl.bernoulli_keep_mask(T + N + 1, M // R, N, p_keep)
    keep[0, :] = 0                                      # a row-block with nothing kept
    if M // R > 1:
        keep[1, :] = 1                                  # a dense row-block
    keep[:, N // 2] = 0                                 # a column no row-block keeps: the bias alone
    Z, _ = run_transposed(U, d["W"], zb, R, keep, k_align, dtype)
    assert bits_equal(Z[:, N // 2], np.broadcast_to(zb[N // 2], (T,)))
    Z, _ = run_transposed(U, d["W"], None, R, keep, k_align, dtype)
    assert np.all(Z[:, N // 2] == 0)


def test_linear_transposed_seeded_random_shapes():
    """Sixty seeded draws over block sizes, widths (one column range and several, ragged last range), ragged token
    counts, densities, alignments, dtypes, empty row-blocks, nothing kept, no bias."""
    rng = np.random.default_rng(31337)
    for it in range(60):
        R = int(rng.choice([16, 16, 16, 32, 32, 64, 8, 4, 24, 12]))
        B = int(rng.integers(1, 70))
        M = R * B
        N = int(rng.choice([32, 64, 200, 256, 257, 520, 768, 1000, 1024, 1032, 2048, 3000, 4096]))
        T = int(rng.integers(1, 330))
        dt = str(rng.choice(["bf16", "f16"]))
        p_keep = float(rng.choice([0.05, 0.2, 0.5, 0.9]))
        k_align = int(rng.choice([8, 16, 32, 64]))
        W = wl.normal(2000 + it, (M, N), 0.02, dt)
        U = wl.normal(3000 + it, (T, M), 1.0, dt)
        zb = wl.normal(4000 + it, (N,), 0.5, dt) if it % 3 != 0 else None
        keep = wl.bernoulli_keep_mask(6000 + it, B, N, p_keep)
        if it % 7 == 0:
            keep[int(rng.integers(0, B))] = 0
        if it % 11 == 0:
            keep[:] = 0
        case = dict(it=it, R=R, B=B, N=N, T=T, dt=dt, p=p_keep, k_align=k_align, bias=zb is not None)
        try:
            run_transposed(U, W, zb, R, keep, k_align, dt)
        except AssertionError as e:
            raise AssertionError(f"{case}: {e}")


def test_linear_transposed_more_row_blocks_than_one_table_pass():
    R, B, N, T = 4, 2100, 300, 70
    W = wl.normal(91, (R * B, N), 0.02, "bf16")
    U = wl.normal(92, (T, R * B), 1.0, "bf16")
    run_transposed(U, W, None, R, wl.bernoulli_keep_mask(93, B, N, 0.3), 8, "bf16")


def test_linear_transposed_passes_without_any_kept_column():
    """300 row-blocks are walked in three passes of the range table; here the whole first pass and, in one column
    range, every pass keeps nothing."""
    R, B, N, T = 8, 300, 600, 90
    W = wl.normal(94, (R * B, N), 0.02, "f16")
    U = wl.normal(95, (T, R * B), 1.0, "f16")
    keep = wl.bernoulli_keep_mask(96, B, N, 0.4)
    keep[:128] = 0
    keep[:, 256:512] = 0
    run_transposed(U, W, wl.normal(97, (N,), 0.5, "f16"), R, keep, 16, "f16")


def test_linear_transposed_is_the_adjoint_of_the_layer_and_skips_pads():
    T, M, N, R = 200, 256, 1024, 16
    d = wl.layer(314, T, M, N, "bf16")
    U = wl.normal(315, (T, M), 1.0, "bf16")
    keep = wl.bernoulli_keep_mask(316, M // R, N, 0.3)
    p = bsp.bsp_pack(dev(d["W"], "bf16"), R, torch.from_numpy(keep).cuda(), 32)
    Y = bsp.bsp_linear(dev(d["X"], "bf16"), p, None).double().cpu().numpy()
    Z = bsp.bsp_linear_transposed(dev(U, "bf16"), p, None).double().cpu().numpy()
    lhs, rhs = float((Y * U).sum()), float((d["X"] * Z).sum())
    scale = float(np.abs(Y * U).sum())
    assert abs(lhs - rhs) <= 2e-3 * scale               # both sides carry one bf16 rounding per output
    # an infinite input meets the pad slots (zero values) of its row-block: they must not be multiplied in
    Ui = U.copy()
    Ui[3, 5] = np.inf
    Zi = host(bsp.bsp_linear_transposed(dev(Ui, "bf16"), p, None))
    p_ref = orc.pack(d["W"], R, keep, 32, orc.BF16)
    Zi_ref, _ = orc.linear_t_packed(Ui, p_ref, None, zdt=orc.BF16)
    assert np.array_equal(np.isnan(Zi), np.isnan(Zi_ref)) and np.array_equal(np.isinf(Zi), np.isinf(Zi_ref))
    fin = np.isfinite(Zi_ref)
    assert fin[3].sum() > 0 and (~fin[3]).sum() > 0
    assert_y_close(np.where(fin, Zi, 0.0), np.where(fin, Zi_ref, 0.0), "bf16")


@pytest.mark.parametrize("C", [16, 32])
def test_row_segment_variant_end_to_end_on_transposed_storage(C):
    """The other division of Alg. 1: V [out, in] is cut into column blocks of C columns and a group is one row's
    segment inside a column block.  Stored transposed (V^T is [in, out], its row-blocks are V's column blocks),
    the same entry points compute its norms, percentile mask and compact storage, and the transposed product is
    its layer Y = X Vp^T + bias.  Checked against definitions written directly on V."""
    T, out_f, in_f = 150, 384, 512
    V = wl.normal(811 + C, (out_f, in_f), 0.05, "bf16")
    X = wl.normal(812 + C, (T, in_f), 1.0, "bf16")
    bias = wl.normal(813 + C, (out_f,), 0.5, "bf16")
    Vt = np.ascontiguousarray(V.T)
    # norms of the row segments, straight from V
    seg = (V.astype(np.float64).reshape(out_f, in_f // C, C) ** 2).sum(axis=2)          # [out, in / C]
    s, _, _ = bsp.bsp_group_norms(dev(Vt, "bf16"), C)                                   # [in / C, out]
    assert np.allclose(host(s).T, seg, rtol=1e-6, atol=0)
    assert bits_equal(host(s), orc.sumsq(Vt, C))
    # keep the n_keep largest segments of the whole matrix
    n_keep = seg.size // 3
    keep, _ = bsp.bsp_prune_mask(s, n_keep=n_keep, scope=bsp.SCOPE_MATRIX)
    keep_h = host(keep)
    assert keep_h.sum() == n_keep
    thr = np.sort(host(s).ravel())[::-1][n_keep - 1]
    assert np.array_equal(keep_h, (host(s) >= thr).astype(np.uint8))                    # no ties in this draw
    p = bsp.bsp_pack(dev(Vt, "bf16"), C, keep, 32)
    Y = host(bsp.bsp_linear_transposed(dev(X, "bf16"), p, dev(bias, "bf16")))
    Vp = V.astype(np.float64) * np.repeat(keep_h.T, C, axis=1)                          # pruned segments zeroed
    want = X.astype(np.float64) @ Vp.T + bias
    assert_y_close(Y, orc.round_to(want, orc.BF16), "bf16")
    # and the input gradient of that layer is the forward entry point on the same storage
    G = wl.normal(814 + C, (T, out_f), 1.0, "bf16")
    dX = host(bsp.bsp_linear(dev(G, "bf16"), p, None))
    assert_y_close(dX, G.astype(np.float64) @ Vp, "bf16")


@pytest.mark.parametrize("R", [8, 16, 32])
def test_config4_bert_large_layer_set_transposed(R):
    """The input gradient of every BERT-large matrix at the benchmark's token count, on sampled token rows."""
    for i, d in enumerate(wl.config4(R=R)):
        W = d["W"]
        s_ref = orc.sumsq(W, R)
        k_ref, _ = orc.mask_rank(s_ref, d["n_keep"], orc.SCOPE_MATRIX)
        T, M = d["X"].shape[0], W.shape[0]
        U = wl.normal(7000 + 10 * R + i, (T, M), 1.0, "bf16")
        run_transposed(U, W, None, R, k_ref, 32, "bf16",
                       T_rows=None if R == 16 else [(0, 40), (5000, 5030), (T - 12, T)])   # R = 16: every token row


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("R,T,M,N,p_keep", [(16, 200, 256, 1024, 0.2), (8, 70, 40, 333, 0.5), (32, 130, 96, 256, 0.33)])
def test_linear_transposed_dense_on_the_masked_matrix(dtype, R, T, M, N, p_keep):
    """The same product as a dense one on W after Alg. 1 (bsp_mask_weights), against the oracle's transposed product
    on the compact storage of the same mask."""
    d = wl.layer(R * 1000 + T + 13, T, M, N, dtype)
    U = wl.normal(R * 81 + T, (T, M), 1.0, dtype)
    zb = wl.normal(R * 82 + T, (N,), 0.5, dtype)
    keep = wl.bernoulli_keep_mask(T + N + 5, M // R, N, p_keep)
    Wm = dev(d["W"], dtype)
    bsp.bsp_mask_weights(Wm, R, torch.from_numpy(keep).cuda())
    p_ref = orc.pack(d["W"], R, keep, 32, CODE[dtype])
    for bias in (zb, None):
        Z = host(bsp.bsp_linear_transposed_dense(dev(U, dtype), Wm, dev(bias, dtype)))
        Z_ref, _ = orc.linear_t_packed(U, p_ref, bias, zdt=CODE[dtype], n_threads=16)
        assert_y_close(Z, Z_ref, dtype)


# ------------------------------------------------------------------------------ the weight gradient
def run_dvals(X, dY, W, R, keep, k_align, dtype, gdt=None):
    """bsp_linear_dvals against the oracle on the same storage: kept positions to the layer's tolerance (one rounding
    of an fp32 / fp64 sum to gdt), pad slots exactly +0."""
    gdt = gdt or dtype
    p_ref = orc.pack(W, R, keep, k_align, CODE[dtype])
    p = bsp.bsp_pack(dev(W, dtype), R, torch.from_numpy(np.ascontiguousarray(keep)).cuda(), k_align)
    pack_equal(p, p_ref)
    D = bsp.bsp_linear_dvals(dev(X, dtype), dev(dY, dtype), p, out_dtype=TDT[gdt])
    D_ref, _ = orc.linear_dvals(X, dY, p_ref, gdt=CODE[gdt], n_threads=16)
    D = host(D)
    assert D.shape == D_ref.shape == (R * int(p_ref["blk_ptr"][-1]),)
    if D.size:
        assert_y_close(D, D_ref, gdt)
    ptr, cnt = p_ref["blk_ptr"], p_ref["blk_cnt"]
    for b in range(len(cnt)):                            # pad slots: +0, whatever X and dY hold
        kp = int(ptr[b + 1] - ptr[b])
        panel = D[R * int(ptr[b]):R * int(ptr[b + 1])].reshape(R, kp)
        assert bits_equal(panel[:, int(cnt[b]):], np.zeros((R, kp - int(cnt[b])), np.float32))
    return D, p


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("R,T,M,N,p_keep,k_align", [
    (16, 100, 64, 200, 0.5, 32), (16, 257, 320, 1024, 0.2, 32), (8, 70, 40, 332, 0.2, 8), (32, 130, 96, 256, 0.33, 16),
    (64, 33, 128, 96, 0.4, 64), (16, 64, 48, 2048, 0.25, 32), (24, 90, 48, 1000, 0.3, 1), (16, 31, 512, 1100, 0.05, 32),
    (4, 33, 36, 516, 0.6, 8), (3, 65, 12, 100, 0.7, 1), (16, 300, 32, 4096, 0.9, 32), (40, 50, 80, 260, 0.4, 8)])
def test_linear_dvals_small_shapes(dtype, R, T, M, N, p_keep, k_align):
    """Block heights with one to four 16-row slabs and half a slab, widths of one to four column ranges with a ragged
    last range, ragged token tiles, an empty and a dense row-block (several items), both kernels (fp32 inputs and
    the odd block heights take the plain one)."""
    d = wl.layer(R * 1000 + T + 11, T, M, N, dtype)
    dY = wl.normal(R * 79 + T, (T, M), 1.0, dtype)
    keep = wl.bernoulli_keep_mask(T + N + 3, M // R, N, p_keep)
    keep[0, :] = 0
    if M // R > 1:
        keep[1, :] = 1
    run_dvals(d["X"], dY, d["W"], R, keep, k_align, dtype)
    if dtype != "f32":
        run_dvals(d["X"], dY, d["W"], R, keep, k_align, dtype, gdt="f32")   # the sums themselves, unrounded


def test_linear_dvals_seeded_random_shapes():
    rng = np.random.default_rng(4242)
    for it in range(40):
        R = int(rng.choice([16, 16, 16, 32, 8, 64, 48, 24]))
        B = int(rng.integers(1, 60))
        M = R * B
        N = int(rng.choice([32, 64, 200, 256, 520, 768, 1000, 1024, 1028, 2048, 3000, 4096]))
        T = int(rng.integers(1, 700))
        dt = str(rng.choice(["bf16", "f16"]))
        p_keep = float(rng.choice([0.02, 0.2, 0.5, 0.95]))
        k_align = int(rng.choice([1, 8, 16, 32, 64]))
        W = wl.normal(12000 + it, (M, N), 0.02, dt)
        X = wl.normal(13000 + it, (T, N), 1.0, dt)
        dY = wl.normal(14000 + it, (T, M), 1.0, dt)
        keep = wl.bernoulli_keep_mask(16000 + it, B, N, p_keep)
        if it % 7 == 0:
            keep[int(rng.integers(0, B))] = 0
        if it % 11 == 0:
            keep[:] = 0
        case = dict(it=it, R=R, B=B, N=N, T=T, dt=dt, p=p_keep, k_align=k_align)
        try:
            run_dvals(X, dY, W, R, keep, k_align, dt, gdt="f32" if it % 3 == 0 else None)
        except AssertionError as e:
            raise AssertionError(f"{case}: {e}")


def test_linear_dvals_same_bits_twice_and_is_the_gradient_of_the_layer():
    T, M, N, R = 1000, 256, 1024, 16
    d = wl.layer(414, T, M, N, "bf16")
    dY = wl.normal(415, (T, M), 1.0, "bf16")
    keep = wl.bernoulli_keep_mask(416, M // R, N, 0.3)
    D, p = run_dvals(d["X"], dY, d["W"], R, keep, 32, "bf16", gdt="f32")
    D2 = host(bsp.bsp_linear_dvals(dev(d["X"], "bf16"), dev(dY, "bf16"), p, out_dtype=torch.float32))
    assert bits_equal(D, D2)
    # the work list of a workspace serves later calls on the same storage, whatever the tokens
    ws = torch.empty(bsp.lib().bsp_linear_dvals_workspace_bytes(M, N, R, p.total_cols), dtype=torch.uint8, device="cuda")
    D3 = host(bsp.bsp_linear_dvals(dev(d["X"], "bf16"), dev(dY, "bf16"), p, out_dtype=torch.float32, ws=ws))
    D4 = host(bsp.bsp_linear_dvals(dev(d["X"], "bf16"), dev(dY, "bf16"), p, out_dtype=torch.float32, ws=ws,
                                   ws_state=bsp.DVALS_REUSE))
    assert bits_equal(D, D3) and bits_equal(D, D4)
    Xs, dYs = d["X"][:333], dY[:333]
    D5 = host(bsp.bsp_linear_dvals(dev(Xs, "bf16"), dev(dYs, "bf16"), p, out_dtype=torch.bfloat16, ws=ws,
                                   ws_state=bsp.DVALS_REUSE))
    p_ref = orc.pack(d["W"], R, keep, 32, orc.BF16)
    assert_y_close(D5, orc.linear_dvals(Xs, dYs, p_ref, gdt=orc.BF16, n_threads=16)[0], "bf16")
    # <dY, layer(X; V)> = <V, D> for the panel values V of the storage (pads are zero on both sides)
    Y = bsp.bsp_linear(dev(d["X"], "bf16"), p, None).double().cpu().numpy()
    lhs = float((Y * dY).sum())
    V = p.vals.double().cpu().numpy()
    rhs = float((V * D.astype(np.float64)).sum())
    assert abs(lhs - rhs) <= 2e-3 * float(np.abs(Y * dY).sum())      # Y carries one bf16 rounding per output


def test_config4_bert_large_layer_set_dvals():
    """The weight gradient of every BERT-large matrix at the benchmark's size (8192 tokens, 5x), every kept position."""
    for i, d in enumerate(wl.config4(R=16)):
        W = d["W"]
        k_ref, _ = orc.mask_rank(orc.sumsq(W, 16), d["n_keep"], orc.SCOPE_MATRIX)
        dY = wl.normal(7100 + i, (d["X"].shape[0], W.shape[0]), 1.0, "bf16")
        run_dvals(d["X"], dY, W, 16, k_ref, 32, "bf16")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_linear_keep_all_is_dense_gemm_keep_none_is_bias(dtype):
    d = wl.layer(77, 96, 64, 160, dtype)
    ones = np.ones((4, 160), np.uint8)
    Y, _ = run_layer(d["X"], d["W"], d["bias"], 16, ones, 32, dtype)
    want = d["X"].astype(np.float64) @ d["W"].astype(np.float64).T + d["bias"]
    assert_y_close(Y, want, dtype)
    Y0, _ = run_layer(d["X"], d["W"], d["bias"], 16, np.zeros((4, 160), np.uint8), 32, dtype)
    assert bits_equal(Y0, np.broadcast_to(d["bias"], (96, 64)))


def test_config1_fp32_attention_projection():
    c = wl.config1()
    run_layer(c["X"], c["W"], c["bias"], c["R"], c["keep"], 32, "f32")


def test_config2_bf16_ffn_up_full_chain():
    c = wl.config2()
    W, R = c["W"], c["R"]
    Wd = dev(W, "bf16")
    s, _, _ = bsp.bsp_group_norms(Wd, R)
    s_ref = orc.sumsq(W, R)
    assert bits_equal(host(s), s_ref)
    keep, _ = bsp.bsp_prune_mask(s, n_keep=c["n_keep"], scope=bsp.SCOPE_BLOCK)
    k_ref, _ = orc.mask_rank(s_ref, c["n_keep"], orc.SCOPE_BLOCK)
    assert np.array_equal(host(keep), k_ref)
    assert (k_ref.sum(axis=1) == 256).all()
    run_layer(c["X"], W, c["bias"], R, k_ref, 32, "bf16", T_rows=[(0, 64), (1000, 1100), (4090, 4096)])


def chain_matrix(d, k_align=32, rows=((0, 48), (5000, 5040), (8180, 8192))):
    """rows=None: every token row is compared (the oracle needs about a second per matrix on 16 threads)."""
    W, R = d["W"], d["R"]
    Wd = dev(W, "bf16")
    s, _, _ = bsp.bsp_group_norms(Wd, R)
    s_ref = orc.sumsq(W, R)
    assert bits_equal(host(s), s_ref)
    keep, t_used = bsp.bsp_prune_mask(s, n_keep=d["n_keep"], scope=bsp.SCOPE_MATRIX, want_t_used=True)
    k_ref, t_ref = orc.mask_rank(s_ref, d["n_keep"], orc.SCOPE_MATRIX)
    assert np.array_equal(host(keep), k_ref) and bits_equal(host(t_used), t_ref)
    T = d["X"].shape[0]
    if rows is not None:
        rows = [(min(a, T - 1), min(b, T)) for a, b in rows]
    run_layer(d["X"], W, d["bias"], R, k_ref, k_align, "bf16", T_rows=rows)


def test_config3_bert_base_layer_set():
    for d in wl.config3():
        chain_matrix(d)


@pytest.mark.parametrize("R", [8, 16, 32])
def test_config4_bert_large_layer_set(R):
    """The benchmark's set at its full size, in the launch configuration the benchmark times.  R = 16 (the benchmark's
    block size): all 8192 token rows of all four matrices, element by element; R = 8, 32: sampled token rows."""
    for d in wl.config4(R=R):
        chain_matrix(d, rows=None if R == 16 else ((0, 48), (5000, 5040), (8180, 8192)))


def test_config5_full_weight_set_sampled():
    # 24-layer BERT-large weight set, fp32, 302 M parameters: norms, factors, gradient, one global 5x percentile
    # over all 18.9 M groups, pack.  Full size on the GPU; the oracle checks sampled row-blocks element by
    # element and the global threshold by its own sort.
    c = wl.config5()
    R, eps, lam = c["R"], c["eps"], c["lam"]
    Wh = c["W"]
    Wd = torch.from_numpy(Wh).cuda()
    runs = []                                            # matrices of one width, adjacent in the buffer, stacked
    for off, m, n in c["desc"]:
        if runs and runs[-1][2] == n and runs[-1][0] + runs[-1][1] * n == off:
            runs[-1] = (runs[-1][0], runs[-1][1] + m, n)
        else:
            runs.append((off, m, n))
    assert len(runs) == 2 and sum(r * n for _, r, n in runs) == Wh.size == 301989888
    groups = Wh.size // R
    sumsq = torch.empty(groups, dtype=torch.float32, device="cuda")
    alpha = torch.empty(groups, dtype=torch.float32, device="cuda")
    grad = torch.empty_like(Wd)
    keep = torch.empty(groups, dtype=torch.uint8, device="cuda")
    rng = np.random.default_rng(5)
    views = []
    for off, rows, n in runs:
        g0, ng = off // R, rows // R * n
        v = dict(off=off, rows=rows, n=n, g0=g0, W=Wd[off:off + rows * n].view(rows, n),
                 G=grad[off:off + rows * n].view(rows, n), s=sumsq[g0:g0 + ng].view(rows // R, n),
                 a=alpha[g0:g0 + ng].view(rows // R, n), k=keep[g0:g0 + ng].view(rows // R, n))
        bsp.bsp_group_norms(v["W"], R, eps=eps, mode=bsp.ALPHA_SQNORM, sumsq=v["s"], alpha=v["a"], want=())
        bsp.bsp_penalty_grad(v["W"], R, v["a"], lam, mode=bsp.ALPHA_SQNORM, grad=v["G"])
        v["blocks"] = sorted(set([0, rows // R - 1] + rng.integers(0, rows // R, 6).tolist()))
        views.append(v)
    n_keep = groups // 5
    _, t_used = bsp.bsp_prune_mask(sumsq.view(groups // 1024, 1024), n_keep=n_keep, scope=bsp.SCOPE_MATRIX,
                                   keep=keep.view(groups // 1024, 1024), want_t_used=True)
    s_host = host(sumsq)
    # sampled row-blocks: sums, factors, gradient
    for v in views:
        Wm = Wh[v["off"]:v["off"] + v["rows"] * v["n"]].reshape(v["rows"], v["n"])
        for b in v["blocks"]:
            Wb = Wm[b * R:(b + 1) * R]
            s_ref = orc.sumsq(Wb, R)
            _, a_ref = orc.norm_alpha(s_ref, eps, orc.ALPHA_SQNORM)
            g_ref, _ = orc.penalty_grad(Wb, R, a_ref, lam, orc.ALPHA_SQNORM)
            assert bits_equal(host(v["s"][b:b + 1]), s_ref) and bits_equal(host(v["a"][b:b + 1]), a_ref)
            assert bits_equal(host(v["G"][b * R:(b + 1) * R]), g_ref)
    # the global threshold and mask
    k_ref, t_ref = orc.mask_rank(s_host.reshape(1, -1), n_keep, orc.SCOPE_MATRIX)
    assert bits_equal(host(t_used), t_ref)
    k_host = host(keep)
    assert np.array_equal(k_host, k_ref.reshape(-1))
    assert 0 <= n_keep - int(k_host.sum()) < 64           # fewer than n_keep only by ties at the cut
    # pack (bf16 panels): counts everywhere, sampled row-blocks element by element
    for v in views:
        p = bsp.bsp_pack(v["W"], R, v["k"], 32, vdt=bsp.BF16)
        assert bsp.bsp_packed_validate(p)
        kv = k_host[v["g0"]:v["g0"] + v["rows"] // R * v["n"]].reshape(v["rows"] // R, v["n"])
        cnt_ref, ptr_ref = orc.pack_count(kv, 32)
        assert np.array_equal(host(p.blk_cnt), cnt_ref) and np.array_equal(host(p.blk_ptr), ptr_ref)
        Wm = Wh[v["off"]:v["off"] + v["rows"] * v["n"]].reshape(v["rows"], v["n"])
        col, ptr = host(p.col_idx), ptr_ref
        for b in v["blocks"]:
            ref = orc.pack(Wm[b * R:(b + 1) * R], R, kv[b:b + 1], 32, orc.BF16)
            lo, hi = int(ptr[b]), int(ptr[b + 1])
            assert np.array_equal(col[lo:hi], ref["col_idx"])
            assert bits_equal(host(p.vals[R * lo:R * hi]), ref["vals"])


def test_skewed_weights_ragged_blocks():
    R, M, N, T = 16, 512, 1024, 300
    W = wl.skewed_weight(21, M, N, R, "bf16", sigma=1.5)
    X = wl.normal(22, (T, N), 1.0, "bf16")
    bias = wl.normal(23, (M,), 0.02, "bf16")
    s_ref = orc.sumsq(W, R)
    k_ref, _ = orc.mask_rank(s_ref, (M // R) * N // 5, orc.SCOPE_MATRIX)
    cnt = k_ref.sum(axis=1)
    assert cnt.max() > 4 * max(cnt.min(), 1)            # the kept count per block really is skewed
    keep, _ = bsp.bsp_prune_mask(dev(s_ref), n_keep=(M // R) * N // 5, scope=bsp.SCOPE_MATRIX)
    assert np.array_equal(host(keep), k_ref)
    run_layer(X, W, bias, R, k_ref, 32, "bf16")


def test_determinism_run_to_run():
    d = wl.config4(tokens=512, shapes=[("attn_out", 1024, 1024)])[0]
    s_ref = orc.sumsq(d["W"], 16)
    k_ref, _ = orc.mask_rank(s_ref, d["n_keep"], orc.SCOPE_MATRIX)
    p = bsp.bsp_pack(dev(d["W"], "bf16"), 16, torch.from_numpy(k_ref).cuda(), 32)
    Xd, bd = dev(d["X"], "bf16"), dev(d["bias"], "bf16")
    y1 = bsp.bsp_linear(Xd, p, bd).clone()
    y2 = bsp.bsp_linear(Xd, p, bd)
    assert torch.equal(y1, y2)
    # the transposed product adds each cell's terms in one fixed order (steps in turn, a barrier between them)
    Ud = dev(wl.normal(55, (512, 1024), 1.0, "bf16"), "bf16")
    z1 = bsp.bsp_linear_transposed(Ud, p, bd).clone()
    z2 = bsp.bsp_linear_transposed(Ud, p, bd)
    assert torch.equal(z1, z2)
