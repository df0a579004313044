"""Pins of the CPU oracle against what the paper and the mathematics fix: closed forms,
brute force on tiny inputs, textbook special cases, library routines and invariants.
None of these tests touches the GPU library."""
import itertools
import math

import os

import numpy as np
import pytest
import torch

import bsp_workloads as wl
from oracle import bsp_oracle as orc

RNG = np.random.default_rng(1234)


def rand(shape, std=1.0):
    return (RNG.standard_normal(shape) * std).astype(np.float32)


# --------------------------------------------------------------------------- rounding
@pytest.mark.parametrize("code,tdt", [(orc.BF16, torch.bfloat16), (orc.F16, torch.float16)])
def test_round_matches_library_conversion(code, tdt):
    # float32 -> low precision through torch is a single RNE rounding of an exactly known value
    x = np.concatenate([rand(4000), rand(2000, 1e-3), rand(2000, 300.0),
                        np.array([0.0, -0.0, 1.0, 65504.0, 65520.0, 1e-8, 6e-8, 3e38], dtype=np.float32)])
    want = torch.from_numpy(x).to(tdt).to(torch.float64).numpy()
    got = orc.round_to(x.astype(np.float64), code)
    assert np.array_equal(want, got)


def test_round_ties_to_even():
    # bf16 has 8 significand bits: spacing 2^-7 in [1,2)
    assert orc.round_to(1.0 + 2.0 ** -8, orc.BF16) == 1.0              # tie -> even (down)
    assert orc.round_to(1.0 + 3 * 2.0 ** -8, orc.BF16) == 1.0 + 2.0 ** -6  # tie -> even (up)
    assert orc.round_to(1.0 + 2.0 ** -8 + 2.0 ** -40, orc.BF16) == 1.0 + 2.0 ** -7  # above tie
    # fp16: 11 bits, spacing 2^-10 in [1,2)
    assert orc.round_to(1.0 + 2.0 ** -11, orc.F16) == 1.0
    assert orc.round_to(1.0 + 3 * 2.0 ** -11, orc.F16) == 1.0 + 2.0 ** -9
    # a double that would round wrongly if it went through float first (double rounding)
    v = 1.0 + 2.0 ** -8 + 2.0 ** -30
    assert orc.round_to(v, orc.BF16) == 1.0 + 2.0 ** -7


# --------------------------------------------------------------------------- sums of squares
def test_sumsq_closed_forms():
    for R in (1, 2, 3, 8, 16, 32, 64):
        M, N = 4 * R, 7
        assert np.array_equal(orc.sumsq(np.ones((M, N), np.float32), R), np.full((4, N), R, np.float32))
    # one-hot: a single non-zero lands in exactly its own group, value w^2
    W = np.zeros((12, 5), np.float32)
    W[7, 3] = 1.5
    s = orc.sumsq(W, 4)
    want = np.zeros((3, 5), np.float32)
    want[1, 3] = 2.25
    assert np.array_equal(s, want)
    # R = 1: norm is |w|
    W = rand((6, 9))
    assert np.array_equal(orc.sumsq(W, 1), W * W)


def test_sumsq_power_of_two_scaling_is_exact():
    W = rand((32, 11), 0.02)
    assert np.array_equal(orc.sumsq(W * np.float32(8.0), 16), orc.sumsq(W, 16) * np.float32(64.0))


def test_sumsq_group_geometry_and_error_bound():
    # rows of a group are R consecutive rows of W at a fixed column; check against an independent
    # float64 evaluation with numpy reshapes on a non-square matrix
    M, N, R = 48, 20, 16
    W = rand((M, N), 0.02)
    want = (W.astype(np.float64).reshape(M // R, R, N) ** 2).sum(axis=1)
    exact = orc.sumsq_exact(W, R)
    assert np.allclose(exact, want, rtol=1e-14, atol=0)
    s = orc.sumsq(W, R).astype(np.float64)
    assert np.all(np.abs(s - exact) <= R * 2.0 ** -24 * exact)


def test_sumsq_canonical_order_is_ascending_fma_chain():
    # values chosen so that the fused chain, an unfused chain and a reversed chain all differ
    col = np.array([1.0 + 2.0 ** -12, 2.0 ** -13, 3.0, 1.0 - 2.0 ** -13], np.float32)
    W = col.reshape(4, 1)
    acc = 0.0  # exact rational arithmetic of "round(w*w + acc)" with float32 rounding, rows ascending
    from fractions import Fraction
    acc = Fraction(0)
    for w in col:
        acc = Fraction(float(np.float32(float(Fraction(float(w)) ** 2 + acc))))
    assert float(orc.sumsq(W, 4)[0, 0]) == float(acc)


# --------------------------------------------------------------------------- norm, reweighting
def test_norm_alpha_closed_forms():
    eps = 1e-6
    for R in (4, 16):
        s = np.full((2, 3), R, np.float32)
        norm, a_sq = orc.norm_alpha(s, eps, orc.ALPHA_SQNORM)
        _, a_n = orc.norm_alpha(s, eps, orc.ALPHA_NORM)
        assert np.allclose(norm, math.sqrt(R), rtol=1e-7)
        assert np.allclose(a_sq, 1.0 / (R + eps), rtol=1e-6)
        assert np.allclose(a_n, 1.0 / (math.sqrt(R) + eps), rtol=1e-6)   # Sec. 3.2, gamma update rule
    z = np.zeros((1, 1), np.float32)
    assert orc.norm_alpha(z, eps, orc.ALPHA_SQNORM)[1][0, 0] == np.float32(1.0) / np.float32(eps)
    assert orc.norm_alpha(z, eps, orc.ALPHA_NORM)[1][0, 0] == np.float32(1.0) / np.float32(eps)


def test_norm_alpha_against_float64():
    s = np.abs(rand((5, 40), 0.01)) + np.float32(1e-4)
    eps = 1e-6
    norm, a_sq = orc.norm_alpha(s, eps, orc.ALPHA_SQNORM)
    _, a_n = orc.norm_alpha(s, eps, orc.ALPHA_NORM)
    s64 = s.astype(np.float64)
    assert np.allclose(norm, np.sqrt(s64), rtol=2e-7)
    assert np.allclose(a_sq, 1 / (s64 + eps), rtol=3e-7)
    assert np.allclose(a_n, 1 / (np.sqrt(s64) + eps), rtol=3e-7)


# --------------------------------------------------------------------------- penalty, gradient
@pytest.mark.parametrize("mode", [orc.ALPHA_SQNORM, orc.ALPHA_NORM])
def test_penalty_gradient_is_derivative_of_penalty(mode):
    M, N, R, lam = 8, 5, 4, 0.37
    W = rand((M, N), 0.5)
    s = orc.sumsq(W, R)
    _, alpha = orc.norm_alpha(s, 1e-6, mode)
    G, pen = orc.penalty_grad(W, R, alpha, lam, mode)
    # central differences of the penalty value (alpha held fixed) at a few coordinates
    for (m, j) in [(0, 0), (3, 4), (5, 2), (7, 1)]:
        h = 1e-3
        Wp, Wm = W.copy(), W.copy()
        Wp[m, j] += h
        Wm[m, j] -= h
        pp = orc.penalty_grad(Wp, R, alpha, lam, mode)[1]
        pm = orc.penalty_grad(Wm, R, alpha, lam, mode)[1]
        fd = (pp - pm) / (float(Wp[m, j]) - float(Wm[m, j]))
        assert abs(fd - G[m, j]) <= 2e-4 * abs(fd) + 1e-7, (m, j, fd, G[m, j])


def test_penalty_value_closed_form_is_eq3():
    # all-ones weights: every group has norm sqrt(R); Eq. 3's term is lambda * sum_g gamma_g ||W_g||
    M, N, R, lam, eps = 8, 6, 4, 0.25, 1e-6
    W = np.ones((M, N), np.float32)
    _, gamma = orc.norm_alpha(orc.sumsq(W, R), eps, orc.ALPHA_NORM)
    G, pen = orc.penalty_grad(W, R, gamma, lam, orc.ALPHA_NORM)
    n_groups = (M // R) * N
    assert pen == pytest.approx(lam * n_groups * (1 / (2 + eps)) * 2.0, rel=1e-6)
    # gradient of gamma*||w|| wrt each of the R equal entries: gamma * w/||w|| = gamma / 2
    assert np.allclose(G, lam * (1 / (2 + eps)) / 2.0, rtol=1e-6)
    # squared form: alpha * w, penalty (lambda/2) * alpha * ||w||^2
    _, alpha = orc.norm_alpha(orc.sumsq(W, R), eps, orc.ALPHA_SQNORM)
    G, pen = orc.penalty_grad(W, R, alpha, lam, orc.ALPHA_SQNORM)
    assert np.allclose(G, lam / (4 + eps), rtol=1e-6)
    assert pen == pytest.approx(0.5 * lam * n_groups * 4 / (4 + eps), rel=1e-6)


def test_penalty_grad_zero_group_and_accumulate():
    W = rand((8, 4), 0.3)
    W[0:4, 2] = 0.0
    for mode in (orc.ALPHA_SQNORM, orc.ALPHA_NORM):
        _, alpha = orc.norm_alpha(orc.sumsq(W, 4), 1e-6, mode)
        G, _ = orc.penalty_grad(W, 4, alpha, 0.1, mode)
        assert np.all(G[0:4, 2] == 0.0) and np.all(np.isfinite(G))
        G0 = rand((8, 4))
        G1, _ = orc.penalty_grad(W, 4, alpha, 0.1, mode, G0=G0)
        assert np.allclose(G1, G0.astype(np.float64) + G, rtol=0, atol=5e-7)
    # gradient rounded to bf16 is the fp32 gradient rounded once
    _, alpha = orc.norm_alpha(orc.sumsq(W, 4), 1e-6, orc.ALPHA_SQNORM)
    G32, _ = orc.penalty_grad(W, 4, alpha, 0.1, orc.ALPHA_SQNORM)
    Gb, _ = orc.penalty_grad(W, 4, alpha, 0.1, orc.ALPHA_SQNORM, gdt=orc.BF16)
    assert np.array_equal(Gb, torch.from_numpy(G32).bfloat16().float().numpy())


# --------------------------------------------------------------------------- masks
def test_threshold_tie_is_pruned():
    # Alg. 1 zeroes a group whose norm is <= t_b
    s = np.array([[0.25, 0.2500001, 0.2499999, 0.0]], np.float32)
    keep = orc.mask_threshold(s, 0.5)
    assert keep.tolist() == [[0, 1, 0, 0]]
    assert orc.mask_threshold(s, -1.0).tolist() == [[1, 1, 1, 1]]
    assert orc.mask_threshold(s, 0.0).tolist() == [[1, 1, 1, 0]]


def test_threshold_compare_is_exact_in_the_squared_domain():
    # t*t is not representable in fp32: a float-rounded t^2 would flip this decision
    t = np.float32(0.1)
    t2 = float(t) * float(t)
    below = np.nextafter(np.float32(t2), np.float32(0))
    above = np.nextafter(below, np.float32(1))
    s = np.array([[below, above]], np.float32)
    want = [[int(float(below) > t2), int(float(above) > t2)]]
    assert orc.mask_threshold(s, float(t)).tolist() == want
    assert want == [[0, 1]]


def test_r1_is_elementwise_magnitude_pruning_and_b1_is_column_pruning():
    W = rand((16, 12))
    t = 0.7
    keep = orc.mask_threshold(orc.sumsq(W, 1), t)
    assert np.array_equal(keep, (np.abs(W.astype(np.float64)) > np.float32(t).astype(np.float64)).astype(np.uint8))
    keep = orc.mask_threshold(orc.sumsq(W, 16), 4.0)
    col_norm = np.linalg.norm(W.astype(np.float64), axis=0)
    assert np.array_equal(keep[0], (col_norm > 4.0).astype(np.uint8))
    assert 0 < keep.sum() < 12


def test_threshold_monotone():
    s = orc.sumsq(rand((32, 50), 0.02), 16)
    prev = None
    for t in (0.0, 0.05, 0.07, 0.08, 0.1, 1.0):
        keep = orc.mask_threshold(s, t)
        if prev is not None:
            assert np.all(keep <= prev)
        prev = keep
    assert prev.sum() == 0


@pytest.mark.parametrize("scope", [orc.SCOPE_BLOCK, orc.SCOPE_MATRIX])
def test_rank_mask_vs_brute_force(scope):
    B, N = 5, 9
    s = np.abs(rand((B, N)))
    s[1, 3] = s[1, 4]            # a tie inside one row
    s[2, :] = 0.5                # a row of equal values
    s[0, 0] = s[4, 8]            # a tie across rows
    n_scope = N if scope == orc.SCOPE_BLOCK else B * N
    for n_keep in [0, 1, 2, n_scope // 2, n_scope - 1, n_scope, n_scope + 3]:
        keep, t_used = orc.mask_rank(s, n_keep, scope)
        rows = [s[b] for b in range(B)] if scope == orc.SCOPE_BLOCK else [s.ravel()]
        got = [keep[b] for b in range(B)] if scope == orc.SCOPE_BLOCK else [keep.ravel()]
        for i, (v, k) in enumerate(zip(rows, got)):
            P = len(v) - n_keep
            if P <= 0:
                assert k.all() and t_used[i] == -np.inf
                continue
            thr = sorted(v.tolist())[P - 1]          # P-th smallest, plain python
            want = [int(x > thr) for x in v.tolist()]
            assert k.tolist() == want
            assert t_used[i] == np.float32(thr)
            assert k.sum() <= n_keep
            if k.any() and not k.all():
                assert v[k == 1].min() > v[k == 0].max()


def test_rank_mask_exact_count_when_distinct():
    s = np.abs(rand((8, 64))) + np.float32(1e-3)
    assert len(np.unique(s)) == s.size
    for n_keep in (0, 1, 17, 200, 512):
        assert orc.mask_rank(s, n_keep, orc.SCOPE_MATRIX)[0].sum() == n_keep
    for n_keep in (0, 1, 21, 64):
        keep, _ = orc.mask_rank(s, n_keep, orc.SCOPE_BLOCK)
        assert np.all(keep.sum(axis=1) == n_keep)


# --------------------------------------------------------------------------- packing
def unpack(p, vdt_values=True):
    """Independent inverse of the compact layout, written from its definition."""
    M, N, R = p["M"], p["N"], p["R"]
    Wd = np.zeros((M, N), np.float32)
    for b in range(M // R):
        base, kb = int(p["blk_ptr"][b]), int(p["blk_cnt"][b])
        kp = int(p["blk_ptr"][b + 1]) - base
        panel = p["vals"][R * base:R * (base + kp)].reshape(R, kp) if kp else np.zeros((R, 0), np.float32)
        for c in range(kb):
            Wd[b * R:(b + 1) * R, p["col_idx"][base + c]] = panel[:, c]
    return Wd


@pytest.mark.parametrize("k_align", [1, 16, 32])
@pytest.mark.parametrize("R", [1, 3, 8, 16])
def test_pack_round_trip_and_layout(R, k_align):
    M, N = 6 * R, 75
    W = rand((M, N), 0.02)
    keep = wl.bernoulli_keep_mask(7 + R, M // R, N, 0.4)
    keep[1, :] = 0                      # an empty block
    keep[2, :] = 1                      # a full block
    p = orc.pack(W, R, keep, k_align)
    assert np.array_equal(unpack(p), W * np.repeat(keep, R, axis=0))
    assert np.array_equal(p["blk_cnt"], keep.sum(axis=1))
    kp = -(-p["blk_cnt"] // k_align) * k_align
    assert p["blk_ptr"][0] == 0 and np.array_equal(np.diff(p["blk_ptr"]), kp)
    assert p["col_idx"].size == p["blk_ptr"][-1] and p["vals"].size == R * p["blk_ptr"][-1]
    for b in range(M // R):
        base, kb = p["blk_ptr"][b], p["blk_cnt"][b]
        idx = p["col_idx"][base:base + kp[b]]
        assert np.array_equal(idx[:kb], np.flatnonzero(keep[b]))       # ascending kept columns
        assert np.all(idx[kb:] == (idx[kb - 1] if kb else 0))          # pads repeat the last one
        panel = p["vals"][R * base:R * (base + kp[b])].reshape(R, kp[b])
        assert np.all(panel[:, kb:] == 0) and not np.signbit(panel[:, kb:]).any()


def test_pack_rounds_values_to_bf16():
    W = rand((16, 20), 0.02)
    keep = wl.bernoulli_keep_mask(3, 1, 20, 0.5)
    p32, pb = orc.pack(W, 16, keep, 1, orc.F32), orc.pack(W, 16, keep, 1, orc.BF16)
    assert np.array_equal(pb["vals"], torch.from_numpy(p32["vals"]).bfloat16().float().numpy())
    assert np.array_equal(pb["col_idx"], p32["col_idx"])


def golden(name):
    """Records of a fixture under tests/golden/: {key: [values as float lists, one per occurrence]}."""
    out = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", name)) as f:
        for line in f:
            line = line.split("#")[0].split()
            if line:
                out.setdefault(line[0], []).append([float(v) for v in line[1:]])
    return out


def test_compression_rate_and_storage_accounting():
    g = golden("sec4_storage_and_rates.txt")
    # Sec. 4.2 / 4.4: 1.428x <=> 30 % sparsity; 2.0x <=> 50 %; 5x <=> 80 % (the printed pairs)
    for sparsity, rate in g["rate_of_sparsity"]:
        kept = int(round(48 * 768 * (1.0 - sparsity)))
        assert orc.compression_rate(768, 768, 16, kept) == pytest.approx(rate, rel=1e-3)
    assert round(orc.compression_rate(100, 100, 10, 70 * 10), 3) == 1.429
    assert orc.compression_rate(768, 768, 16, 48 * 384) == 2.0
    assert orc.compression_rate(1000, 10, 10, 200) == 5.0
    # Sec. 4.4 worked example: 8x8 matrix, 4x4 blocks => groups of 4 weights, 16 groups, half kept: the values
    # and one index word per group against three words per non-zero in the COO format
    (m, n), (br, _), (sp,) = g["storage_example_matrix"][0], g["storage_example_block"][0], g["storage_example_sparsity"][0]
    m, n, br = int(m), int(n), int(br)
    W = rand((m, n)) + np.float32(3.0)
    keep = wl.random_keep_mask(1, m // br, n, int(n * (1.0 - sp)))
    p = orc.pack(W, br, keep, 1)
    nnz = int(np.count_nonzero(unpack(p)))
    n_groups = keep.size
    assert n_groups == g["storage_example_bsp_indices"][0][0]
    assert p["vals"].size == nnz and nnz + n_groups == g["storage_example_bsp_words"][0][0]
    assert 3 * nnz == g["storage_example_coo_words"][0][0]


# --------------------------------------------------------------------------- the layer
def brute_force_layer(X, W, keep, bias, R):
    """Triple python loop in exact rational arithmetic, then to float."""
    from fractions import Fraction
    T, N = X.shape
    M = W.shape[0]
    Y = np.zeros((T, M), np.float64)
    for t in range(T):
        for m in range(M):
            acc = Fraction(float(bias[m])) if bias is not None else Fraction(0)
            for j in range(N):
                if keep[m // R, j]:
                    acc += Fraction(float(X[t, j])) * Fraction(float(W[m, j]))
            Y[t, m] = float(acc)
    return Y


@pytest.mark.parametrize("R", [1, 2, 4, 8])
def test_linear_vs_exact_brute_force(R):
    T, M, N = 3, 8, 10
    X, W, bias = rand((T, N)), rand((M, N), 0.02), rand((M,), 0.02)
    keep = wl.bernoulli_keep_mask(R, M // R, N, 0.5)
    want = brute_force_layer(X, W, keep, bias, R)
    _, Yd = orc.linear_dense(X, W, keep, bias, R)
    assert np.allclose(Yd, want, rtol=0, atol=1e-15)
    p = orc.pack(W, R, keep, 1)
    Yp, Ypd = orc.linear_packed(X, p, bias)
    assert np.array_equal(Ypd, Yd)                       # bit for bit in double
    assert np.array_equal(Yp, Yd.astype(np.float32))
    # orientation: W is [out, in], Y = X W^T
    assert Yd.shape == (T, M)


@pytest.mark.parametrize("k_align", [1, 16, 32])
def test_linear_dense_equals_packed_bitwise_with_padding(k_align):
    T, M, N, R = 5, 32, 70, 16
    X, W, bias = rand((T, N)), rand((M, N), 0.02), rand((M,), 0.02)
    keep = wl.bernoulli_keep_mask(11, M // R, N, 0.3)
    _, Yd = orc.linear_dense(X, W, keep, bias, R)
    _, Ypd = orc.linear_packed(X, orc.pack(W, R, keep, k_align), bias)
    assert np.array_equal(Yd, Ypd)


def test_linear_keep_all_is_dense_gemm_and_keep_none_is_bias():
    T, M, N, R = 7, 32, 24, 16
    X, W, bias = rand((T, N)), rand((M, N), 0.02), rand((M,), 0.02)
    ones, zeros = np.ones((M // R, N), np.uint8), np.zeros((M // R, N), np.uint8)
    want = (torch.from_numpy(X).double() @ torch.from_numpy(W).double().T + torch.from_numpy(bias).double()).numpy()
    for k_align in (1, 16):
        Y, Yd = orc.linear_packed(X, orc.pack(W, R, ones, k_align), bias)
        assert np.allclose(Yd, want, rtol=1e-13, atol=1e-15)
        Y0, _ = orc.linear_packed(X, orc.pack(W, R, zeros, k_align), bias)
        assert np.array_equal(Y0, np.broadcast_to(bias, (T, M)))
    Y0, _ = orc.linear_packed(X, orc.pack(W, R, zeros, 1), None)
    assert np.all(Y0 == 0)


def test_linear_against_library_matmul_with_zeroed_weights():
    T, M, N, R = 9, 48, 40, 8
    X, W, bias = rand((T, N)), rand((M, N), 0.02), rand((M,), 0.02)
    keep = wl.bernoulli_keep_mask(5, M // R, N, 0.35)
    Wz = W.astype(np.float64) * np.repeat(keep, R, axis=0)
    want = (torch.from_numpy(X).double() @ torch.from_numpy(Wz).T + torch.from_numpy(bias).double()).numpy()
    _, Yd = orc.linear_packed(X, orc.pack(W, R, keep, 16), bias)
    assert np.allclose(Yd, want, rtol=1e-12, atol=1e-15)


def test_linear_additivity_permutation_and_block_locality():
    T, M, N, R = 4, 24, 30, 8
    X, W, bias = rand((T, N)), rand((M, N), 0.02), rand((M,), 0.02)
    m1 = wl.bernoulli_keep_mask(1, M // R, N, 0.3)
    m2 = wl.bernoulli_keep_mask(2, M // R, N, 0.3) & (1 - m1)
    y = lambda m, XX=X, WW=W: orc.linear_packed(XX, orc.pack(WW, R, m, 1), bias)[1]
    assert np.allclose(y(m1) + y(m2) - bias, y(m1 | m2), rtol=0, atol=1e-12)
    perm = RNG.permutation(N)
    assert np.allclose(y(m1[:, perm], X[:, perm], W[:, perm]), y(m1), rtol=0, atol=1e-13)
    W2, mk2 = W.copy(), m1.copy()
    W2[8:16] += 1.0
    mk2[1] = 1 - mk2[1]
    d = y(mk2, X, W2) != y(m1)
    assert d[:, 8:16].any() and not d[:, :8].any() and not d[:, 16:].any()


def test_linear_output_rounding_and_row_range():
    T, M, N, R = 6, 16, 33, 16
    X = wl.to_dtype_values(rand((T, N)), "bf16")
    W = wl.to_dtype_values(rand((M, N), 0.02), "bf16")
    bias = wl.to_dtype_values(rand((M,), 0.02), "bf16")
    p = orc.pack(W, R, wl.bernoulli_keep_mask(9, 1, N, 0.5), 16, orc.BF16)
    Y, Yd = orc.linear_packed(X, p, bias, ydt=orc.BF16)
    assert np.array_equal(Y.astype(np.float64), orc.round_to(Yd, orc.BF16))
    Ys, _ = orc.linear_packed(X, p, bias, ydt=orc.BF16, t0=2, t1=4)
    assert np.array_equal(Ys[2:4], Y[2:4]) and np.isnan(Ys[:2]).all() and np.isnan(Ys[4:]).all()
    Ymt, _ = orc.linear_packed(X, p, bias, ydt=orc.BF16, n_threads=4)
    assert np.array_equal(Ymt, Y)


# --------------------------------------------------------------------------- the transposed product
def brute_force_transposed(U, W, keep, bias, R):
    """Exact rational arithmetic: Z[t, j] = bias[j] + sum_m U[t, m] W[m, j] over the kept groups."""
    from fractions import Fraction
    T, M = U.shape
    N = W.shape[1]
    Z = np.zeros((T, N), np.float64)
    for t in range(T):
        for j in range(N):
            acc = Fraction(float(bias[j])) if bias is not None else Fraction(0)
            for m in range(M):
                if keep[m // R, j]:
                    acc += Fraction(float(U[t, m])) * Fraction(float(W[m, j]))
            Z[t, j] = float(acc)
    return Z


@pytest.mark.parametrize("R", [1, 2, 4, 8])
def test_linear_t_vs_exact_brute_force(R):
    T, M, N = 3, 8, 10
    U, W, bias = rand((T, M)), rand((M, N), 0.02), rand((N,), 0.02)
    keep = wl.bernoulli_keep_mask(R + 20, M // R, N, 0.5)
    want = brute_force_transposed(U, W, keep, bias, R)
    Z, Zd = orc.linear_t_dense(U, W, keep, bias, R)
    assert Zd.shape == (T, N)                            # orientation: U is [T, out], Z is [T, in]
    assert np.allclose(Zd, want, rtol=0, atol=1e-15)
    for k_align in (1, 8):
        Zp, Zpd = orc.linear_t_packed(U, orc.pack(W, R, keep, k_align), bias)
        assert np.array_equal(Zpd, Zd)                   # same order of the additions: bit for bit
        assert np.array_equal(Zp, Zd.astype(np.float32))


def test_linear_t_against_library_matmul_and_special_cases():
    T, M, N, R = 9, 48, 40, 8
    U, W, bias = rand((T, M)), rand((M, N), 0.02), rand((N,), 0.02)
    keep = wl.bernoulli_keep_mask(6, M // R, N, 0.35)
    Wz = W.astype(np.float64) * np.repeat(keep, R, axis=0)
    want = (torch.from_numpy(U).double() @ torch.from_numpy(Wz) + torch.from_numpy(bias).double()).numpy()
    _, Zd = orc.linear_t_packed(U, orc.pack(W, R, keep, 16), bias)
    assert np.allclose(Zd, want, rtol=1e-12, atol=1e-15)
    ones, zeros = np.ones_like(keep), np.zeros_like(keep)
    _, Zall = orc.linear_t_packed(U, orc.pack(W, R, ones, 1), None)
    assert np.allclose(Zall, (torch.from_numpy(U).double() @ torch.from_numpy(W).double()).numpy(), rtol=1e-12,
                       atol=1e-15)
    Z0, _ = orc.linear_t_packed(U, orc.pack(W, R, zeros, 16), bias)
    assert np.array_equal(Z0, np.broadcast_to(bias, (T, N)))
    # a column no block keeps receives the bias alone; a pad slot (k_align > 1) adds nothing to the last kept column
    k1 = keep.copy()
    k1[:, 7] = 0
    Z1, _ = orc.linear_t_packed(U, orc.pack(W, R, k1, 16), bias)
    assert np.array_equal(Z1[:, 7], np.broadcast_to(bias[7], (T,)))
    Uinf = U.copy()
    Uinf[0, 0] = np.inf                                  # would give inf * 0 = NaN if pads were multiplied in
    kone = np.zeros_like(keep)
    kone[0, 3] = 1
    Zi, _ = orc.linear_t_packed(Uinf, orc.pack(np.abs(W) + 1, R, kone, 16), None)
    assert np.isinf(Zi[0, 3]) and not np.isnan(Zi).any()


def test_linear_t_is_the_adjoint_of_the_layer():
    """<linear(X), U> = <X, linear_t(U)> without biases: the input gradient of the layer (chain rule), checked
    against the layer's own oracle and against torch's autograd on the dense masked product."""
    T, M, N, R = 6, 32, 28, 8
    X, U, W = rand((T, N)), rand((T, M)), rand((M, N), 0.05)
    keep = wl.bernoulli_keep_mask(3, M // R, N, 0.4)
    p = orc.pack(W, R, keep, 8)
    _, Yd = orc.linear_packed(X, p, None)
    _, Zd = orc.linear_t_packed(U, p, None)
    assert math.isclose(float((Yd * U).sum()), float((X * Zd).sum()), rel_tol=1e-12, abs_tol=1e-13)
    Xt = torch.from_numpy(X).double().requires_grad_(True)
    Wz = torch.from_numpy(W.astype(np.float64) * np.repeat(keep, R, axis=0))
    (Xt @ Wz.T).backward(torch.from_numpy(U).double())
    assert np.allclose(Zd, Xt.grad.numpy(), rtol=1e-12, atol=1e-15)
    # the other variant of Alg. 1: groups are row segments of column blocks of V = W^T; its layer is X' V^T
    V = np.ascontiguousarray(W.T)                       # [N, M]: V's column block b holds columns bR .. bR+R-1
    Vz = V.astype(np.float64) * np.repeat(keep, R, axis=0).T
    want = (torch.from_numpy(U).double() @ torch.from_numpy(Vz).T).numpy()
    assert np.allclose(Zd, want, rtol=1e-12, atol=1e-15)


def test_linear_t_rounding_row_range_and_threads():
    T, M, N, R = 6, 32, 33, 16
    U = wl.to_dtype_values(rand((T, M)), "bf16")
    W = wl.to_dtype_values(rand((M, N), 0.02), "bf16")
    bias = wl.to_dtype_values(rand((N,), 0.02), "bf16")
    p = orc.pack(W, R, wl.bernoulli_keep_mask(9, M // R, N, 0.5), 16, orc.BF16)
    Z, Zd = orc.linear_t_packed(U, p, bias, zdt=orc.BF16)
    assert np.array_equal(Z.astype(np.float64), orc.round_to(Zd, orc.BF16))
    Zs, _ = orc.linear_t_packed(U, p, bias, zdt=orc.BF16, t0=2, t1=4)
    assert np.array_equal(Zs[2:4], Z[2:4]) and np.isnan(Zs[:2]).all() and np.isnan(Zs[4:]).all()
    Zmt, _ = orc.linear_t_packed(U, p, bias, zdt=orc.BF16, n_threads=4)
    assert np.array_equal(Zmt, Z)


# --------------------------------------------------------------------------- end to end
def test_chain_on_base_attention_projection():
    """norms -> percentile mask -> pack -> layer equals the dense layer with the mask's zeros."""
    c = wl.config1(tokens=8)
    X, W, bias, R = c["X"], c["W"], c["bias"], c["R"]
    s = orc.sumsq(W, R)
    keep, _ = orc.mask_rank(s, 384, orc.SCOPE_BLOCK)
    assert np.all(keep.sum(axis=1) == 384)
    p = orc.pack(W, R, keep, 32)
    assert orc.compression_rate(768, 768, R, int(p["blk_cnt"].sum())) == 2.0
    Y, Yd = orc.linear_packed(X, p, bias)
    _, Yd_dense = orc.linear_dense(X, W, keep, bias, R)
    assert np.array_equal(Yd, Yd_dense)
    Wz = W.astype(np.float64) * np.repeat(keep, R, axis=0)
    want = (torch.from_numpy(X).double() @ torch.from_numpy(Wz).T + torch.from_numpy(bias).double()).numpy()
    assert np.allclose(Yd, want, rtol=1e-12, atol=1e-14)
    # the given random mask of the workload keeps exactly half of every block
    assert np.all(c["keep"].sum(axis=1) == 384)


# ---------------------------------------------------------------------------------- masked weights
def test_mask_weights_definition_and_invariants():
    # Alg. 1 sets a pruned group to zero; Alg. 2 re-applies W = W * Mask after every retraining update.
    rng = np.random.default_rng(12)
    R, B, N = 4, 5, 37
    W = rng.standard_normal((B * R, N)).astype(np.float32)
    W[3, 5] = -0.0                                       # a kept negative zero must stay as it is
    W[7, 9] = np.float32("nan")                          # and so must any bit pattern of a kept weight
    keep = (rng.random((B, N)) < 0.4).astype(np.uint8)
    keep[0, 5] = 1
    keep[1, 9] = 1
    keep[2, :] = 0
    keep[3, :] = 1
    Wm = orc.mask_weights(W, R, keep)
    big = np.repeat(keep, R, axis=0).astype(bool)        # the element mask of Alg. 2
    assert np.array_equal(Wm.view(np.uint32)[big], W.view(np.uint32)[big])          # kept: untouched, bit for bit
    assert np.all(Wm.view(np.uint32)[~big] == 0)                                    # pruned: +0 exactly
    assert np.array_equal(orc.mask_weights(Wm, R, keep).view(np.uint32), Wm.view(np.uint32))   # idempotent
    fin = np.isfinite(W)
    assert np.array_equal((W * big)[fin & big], Wm[fin & big])                      # W * Mask where that is defined
    # what survives is exactly what the group norms see and what the compact storage holds
    s = orc.sumsq(np.nan_to_num(Wm), R)
    assert np.all(s[keep == 0] == 0.0)
    W2 = np.nan_to_num(W)
    p1, p2 = orc.pack(W2, R, keep, 8), orc.pack(orc.mask_weights(W2, R, keep), R, keep, 8)
    assert np.array_equal(p1["col_idx"], p2["col_idx"]) and np.array_equal(p1["vals"].view(np.uint32), p2["vals"].view(np.uint32))
    # the element mask Alg. 2 would build from the pruned matrix reproduces the group mask on generic weights
    Wg = rng.standard_normal((B * R, N)).astype(np.float32)
    assert np.array_equal(orc.mask_weights(Wg, R, keep) != 0, big)
    # and the masked layer equals the dense layer on the masked weights
    X = rng.standard_normal((6, N)).astype(np.float32)
    Yd, _ = orc.linear_dense(X, orc.mask_weights(Wg, R, keep), np.ones_like(keep), None, R, ydt=orc.F32)
    Yp, _ = orc.linear_packed(X, orc.pack(Wg, R, keep, 1), None, ydt=orc.F32)
    assert np.allclose(Yd, Yp, rtol=0, atol=1e-5)


# ---------------------------------------------------------------------------------- the Adam update of Alg. 2
def _adam_f64(w, g, m, v, lr, b1, b2, eps, t):
    """Kingma & Ba, Algorithm 1, in double on the fp32 inputs and fp32 hyper-parameters."""
    b1, b2, lr, eps = (float(np.float32(x)) for x in (b1, b2, lr, eps))
    w, g, m, v = (np.asarray(a, np.float64) for a in (w, g, m, v))
    m = b1 * m + (1.0 - b1) * g
    v = b2 * v + (1.0 - b2) * g * g
    w = w - lr * (m / (1.0 - b1 ** t)) / (np.sqrt(v / (1.0 - b2 ** t)) + eps)
    return w, m, v


def test_adam_step_against_the_published_update_in_double():
    rng = np.random.default_rng(21)
    R, B, N = 4, 6, 29
    W = (rng.standard_normal((B * R, N)) * 0.05).astype(np.float32)
    lr, b1, b2, eps = 3e-5, 0.9, 0.999, 1e-8
    m = np.zeros_like(W)
    v = np.zeros_like(W)
    Wd, md, vd = W.astype(np.float64), m.astype(np.float64), v.astype(np.float64)
    for t in range(1, 8):                                # several steps, the state carried by both sides
        G = (rng.standard_normal(W.shape) * 1e-3).astype(np.float32)
        W, m, v = orc.adam_step(W, G, m, v, R, lr, b1, b2, eps, t)
        Wd, md, vd = _adam_f64(Wd, G, md, vd, lr, b1, b2, eps, t)
        # m is a signed sum (cancellation: absolute bound on its scale); v is a sum of non-negative terms
        assert np.allclose(m, md, rtol=0, atol=4e-7 * 5e-3) and np.allclose(v, vd, rtol=4e-6, atol=0)
        # each step rounds w once (half an ulp of |w| < 0.25) on a move of about lr = 3e-5
        assert np.allclose(W - Wd, 0, atol=t * (1.5e-8 + lr * 1e-5))


def test_adam_step_closed_forms_and_invariants():
    rng = np.random.default_rng(22)
    R, B, N = 8, 3, 17
    shape = (B * R, N)
    W0 = (rng.standard_normal(shape) * 0.05).astype(np.float32)
    G = (rng.standard_normal(shape) * 1e-2).astype(np.float32)
    z = np.zeros(shape, np.float32)
    lr = 2e-5
    # first step from zero moments: the bias corrections cancel, the move is lr * g / (|g| + eps)
    W1, m1, v1 = orc.adam_step(W0, G, z, z, R, lr, 0.9, 0.999, 1e-8, 1)
    want = W0.astype(np.float64) - lr * G.astype(np.float64) / (np.abs(G.astype(np.float64)) + 1e-8)
    assert np.allclose(W1, want, rtol=0, atol=lr * 2e-6 + 4e-9)
    assert np.allclose(m1, 0.1 * G.astype(np.float64), rtol=1e-6) and np.allclose(v1, 0.001 * G.astype(np.float64) ** 2, rtol=1e-5)
    # no gradient, no moments: nothing moves, bit for bit
    W2, m2, v2 = orc.adam_step(W0, z, z, z, R, lr, 0.9, 0.999, 1e-8, 5)
    assert np.array_equal(W2.view(np.uint32), W0.view(np.uint32)) and not m2.any() and not v2.any()
    # a constant gradient: every step moves each weight by lr against the gradient's sign (eps negligible)
    W, m, v = W0.copy(), z, z
    for t in range(1, 21):
        W, m, v = orc.adam_step(W, G, m, v, R, lr, 0.9, 0.999, 1e-12, t)
    assert np.allclose(W, W0.astype(np.float64) - 20 * lr * np.sign(G), rtol=0, atol=20 * lr * 1e-5 + 1e-7)
    # with eps = 0 the update does not see a rescaling of the gradients by a power of two
    Wa, ma, va = orc.adam_step(W0, G, z, z, R, lr, 0.9, 0.999, 0.0, 1)
    Wb, mb, vb = orc.adam_step(W0, 4 * G, z, z, R, lr, 0.9, 0.999, 0.0, 1)
    assert np.array_equal(Wa.view(np.uint32), Wb.view(np.uint32))
    assert np.array_equal(mb, 4 * ma) and np.array_equal(vb, 16 * va)
    # beta1 = beta2 = 0: no memory, the move is lr * sign(g) whatever the old moments were
    junk = np.abs(rng.standard_normal(shape)).astype(np.float32)
    Wc, mc, vc = orc.adam_step(W0, G, junk, junk, R, lr, 0.0, 0.0, 0.0, 3)
    assert np.array_equal(mc, G) and np.array_equal(vc, G * G)
    assert np.allclose(Wc, W0.astype(np.float64) - lr * np.sign(G), rtol=0, atol=lr * 1e-6 + 4e-9)


def test_adam_step_mask_and_regulariser():
    rng = np.random.default_rng(23)
    R, B, N = 4, 5, 23
    shape = (B * R, N)
    W0 = (rng.standard_normal(shape) * 0.05).astype(np.float32)
    W0[0:R, 2] = 0.0                                    # an all-zero group
    G = (rng.standard_normal(shape) * 1e-3).astype(np.float32)
    m0 = (rng.standard_normal(shape) * 1e-3).astype(np.float32)
    v0 = (rng.standard_normal(shape) ** 2 * 1e-6).astype(np.float32)
    keep = (rng.random((B, N)) < 0.3).astype(np.uint8)
    big = np.repeat(keep, R, axis=0).astype(bool)
    hp = dict(lr=3e-5, beta1=0.9, beta2=0.999, eps=1e-8, t=4)
    Wp, mp, vp = orc.adam_step(W0, G, m0, v0, R, **hp)
    # retraining: the update, then W = W * Mask; the moments are those of the unmasked update
    Wk, mk, vk = orc.adam_step(W0, G, m0, v0, R, keep=keep, **hp)
    assert np.array_equal(Wk.view(np.uint32), orc.mask_weights(Wp, R, keep).view(np.uint32))
    assert np.all(Wk.view(np.uint32)[~big] == 0) and np.array_equal(Wk[big], Wp[big])
    assert np.array_equal(mk, mp) and np.array_equal(vk, vp)
    # reweighted training: Adam on the mixed loss = Adam on G + gradient of the regulariser (Eq. 3, factors fixed)
    lam = 1e-3
    for mode in (orc.ALPHA_SQNORM, orc.ALPHA_NORM):
        _, alpha = orc.norm_alpha(orc.sumsq(W0, R), 1e-6, mode)
        Gmix, _ = orc.penalty_grad(W0, R, alpha, lam, mode, gdt=orc.F32, G0=G)
        assert not np.array_equal(Gmix, G)
        Wr, mr, vr = orc.adam_step(W0, G, m0, v0, R, alpha=alpha, lam=lam, mode=mode, **hp)
        Ws, ms, vs = orc.adam_step(W0, Gmix, m0, v0, R, **hp)
        for a, b in ((Wr, Ws), (mr, ms), (vr, vs)):
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
        # lambda = 0 leaves the plain update
        Wz, mz, vz = orc.adam_step(W0, G, m0, v0, R, alpha=alpha, lam=0.0, mode=mode, **hp)
        assert np.array_equal(Wz, Wp) and np.array_equal(mz, mp) and np.array_equal(vz, vp)
    # the regulariser pulls every weight of a non-zero group towards zero when there is no other gradient
    _, alpha = orc.norm_alpha(orc.sumsq(W0, R), 1e-6, orc.ALPHA_SQNORM)
    z = np.zeros(shape, np.float32)
    Wq, _, _ = orc.adam_step(W0, z, z, z, R, alpha=alpha, lam=lam, mode=orc.ALPHA_SQNORM, lr=1e-4, t=1)
    nz = W0 != 0
    assert np.all(np.abs(Wq[nz]) < np.abs(W0[nz])) and np.all(Wq[~nz] == 0)


# --------------------------------------------------------------------------- epilogue of a layer
def test_epilogue_gelu_is_the_exact_erf_form():
    y = np.concatenate([rand(2000, 2.0), np.linspace(-8, 8, 401).astype(np.float32)]).astype(np.float64)
    got = orc.epilogue(y, orc.ACT_GELU)[1]
    want = np.array([0.5 * v * (1.0 + math.erf(v / math.sqrt(2.0))) for v in y])   # the interpreter's own erf
    assert np.allclose(got, want, rtol=1e-14, atol=1e-300)
    # closed forms: gelu(0) = 0; gelu(1) = Phi(1), the textbook value of the normal distribution function;
    # gelu(x) - gelu(-x) = x (Phi(x) + Phi(-x) = 1); far out it is the identity / zero
    assert orc.epilogue(np.array([0.0]), orc.ACT_GELU)[1][0] == 0.0
    assert abs(orc.epilogue(np.array([1.0]), orc.ACT_GELU)[1][0] - 0.8413447460685429) < 1e-15
    pos, neg = orc.epilogue(np.abs(y), orc.ACT_GELU)[1], orc.epilogue(-np.abs(y), orc.ACT_GELU)[1]
    assert np.allclose(pos - neg, np.abs(y), rtol=1e-14, atol=1e-15)
    far = orc.epilogue(np.array([40.0, -40.0]), orc.ACT_GELU)[1]
    assert far[0] == 40.0 and far[1] == 0.0
    # not the tanh approximation: the two differ by about 1e-4 at x = 2
    tanh_form = 0.5 * 2.0 * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (2.0 + 0.044715 * 8.0)))
    assert abs(orc.epilogue(np.array([2.0]), orc.ACT_GELU)[1][0] - tanh_form) > 5e-5


def test_epilogue_order_residual_and_single_rounding():
    y, res = rand((7, 9), 1.5).astype(np.float64), wl.to_dtype_values(rand((7, 9)), "bf16")
    plain = orc.epilogue(y)[1]
    assert np.array_equal(plain, y)                                               # nothing asked: the sums themselves
    assert np.array_equal(orc.epilogue(y, residual=res)[1], y + res.astype(np.float64))
    both = orc.epilogue(y, orc.ACT_GELU, res)[1]
    assert np.array_equal(both, orc.epilogue(y, orc.ACT_GELU)[1] + res.astype(np.float64))   # activation, then residual
    assert not np.allclose(both, orc.epilogue(y + res, orc.ACT_GELU)[1])
    # one rounding, after the addition: 1 + 2^-8 is a tie in bf16 (-> 1), the residual 2^-20 lifts it above the tie
    one = np.array([1.0 + 2.0 ** -8]); r = np.array([2.0 ** -20], dtype=np.float32)
    assert orc.epilogue(one, residual=r, ydt=orc.BF16)[0][0] == np.float32(1.0 + 2.0 ** -7)
    assert orc.round_to(one, orc.BF16)[0] + r[0] != np.float32(1.0 + 2.0 ** -7)
    # rounded output == the layer's own rounding when nothing is asked
    d = wl.layer(5, 6, 8, 12, "bf16")
    keep = wl.bernoulli_keep_mask(6, 2, 12, 0.5)
    p = orc.pack(d["W"], 4, keep, 1, orc.BF16)
    Y, Yd = orc.linear_packed(d["X"], p, d["bias"], ydt=orc.BF16)
    assert np.array_equal(orc.linear_packed_fused(d["X"], p, d["bias"], ydt=orc.BF16)[0], Y)


# --------------------------------------------------------------------------- gradient of the kept weights
def test_dvals_exact_rational_brute_force_and_pads():
    from fractions import Fraction
    T, M, N, R = 5, 6, 7, 3
    X, dY, W = rand((T, N)), rand((T, M)), rand((M, N))
    keep = wl.bernoulli_keep_mask(3, M // R, N, 0.6)
    keep[1, :] = 0
    keep[1, 2] = 1
    for k_align in (1, 8):
        p = orc.pack(W, R, keep, k_align, orc.F32)
        D, Dd = orc.linear_dvals(X, dY, p)
        for b in range(M // R):
            base, kp, kb = int(p["blk_ptr"][b]), int(p["blk_ptr"][b + 1] - p["blk_ptr"][b]), int(p["blk_cnt"][b])
            for r in range(R):
                for c in range(kp):
                    at = R * base + r * kp + c
                    if c >= kb:
                        assert D[at] == 0.0 and not np.signbit(D[at]) and Dd[at] == 0.0   # a pad: exactly +0
                        continue
                    j = int(p["col_idx"][base + c])
                    want = sum(Fraction(float(dY[t, b * R + r])) * Fraction(float(X[t, j])) for t in range(T))
                    assert abs(Fraction(float(Dd[at])) - want) <= abs(want) * Fraction(1, 10 ** 14)
                    assert D[at] == np.float32(float(want))


def test_dvals_is_the_gradient_of_the_layer():
    T, M, N, R = 9, 8, 11, 4
    X, dY, W = rand((T, N)), rand((T, M)), rand((M, N))
    keep = wl.bernoulli_keep_mask(4, M // R, N, 0.5)
    p = orc.pack(W, R, keep, 8, orc.F32)
    D, Dd = orc.linear_dvals(X, dY, p)
    # torch's autograd on the dense masked product, gathered at the kept positions
    Wt = torch.tensor(W.astype(np.float64), requires_grad=True)
    mask = torch.tensor(np.repeat(keep, R, axis=0).astype(np.float64))
    (torch.tensor(dY.astype(np.float64)) * (torch.tensor(X.astype(np.float64)) @ (Wt * mask).T)).sum().backward()
    G = Wt.grad.numpy()
    ref = orc.pack(G.astype(np.float32), R, keep, 8, orc.F32)
    assert np.allclose(Dd, ref["vals"].astype(np.float64), rtol=1e-6, atol=1e-6)
    # adjointness: <dY, layer(X; V)> = <V, dvals> for any panel values V on the same pattern, pads included (they are 0)
    V = rand(ref["vals"].shape)
    for b in range(M // R):                                           # pads of V must be 0 for the layer to ignore them
        base, kp, kb = int(p["blk_ptr"][b]), int(p["blk_ptr"][b + 1] - p["blk_ptr"][b]), int(p["blk_cnt"][b])
        for r in range(R):
            V[R * base + r * kp + kb: R * base + (r + 1) * kp] = 0.0
    q = dict(p); q["vals"] = V
    _, Yd = orc.linear_packed(X, q, None)
    assert abs((dY.astype(np.float64) * Yd).sum() - (V.astype(np.float64) * Dd).sum()) < 1e-9
    # keep all: the dense product dY^T X, row-block by row-block
    pa = orc.pack(W, R, np.ones_like(keep), 1, orc.F32)
    Da = orc.linear_dvals(X, dY, pa)[1].reshape(M, N)
    assert np.allclose(Da, dY.astype(np.float64).T @ X.astype(np.float64), rtol=1e-13, atol=1e-13)
    # rounding to a 16-bit type is one rounding of the double sum
    Db, Dbd = orc.linear_dvals(X, dY, p, gdt=orc.BF16)
    assert np.array_equal(Db.astype(np.float64), orc.round_to(Dbd, orc.BF16))


# --------------------------------------------------------------------------- whole-block pruning (Table 4's comparison)
def test_tile_sumsq_and_whole_block_mask():
    B, N, R = 5, 24, 4
    W = rand((B * R, N), 0.02)
    s = orc.sumsq(W, R)
    assert np.array_equal(orc.tile_sumsq(s, 1), s)                                   # tiles of one column: the groups
    for Ct in (2, 4, 8, 24):
        ts = orc.tile_sumsq(s, Ct)
        # replay of the stated order in numpy fp32, and the plain definition in fp64
        want = np.zeros((B, N // Ct), dtype=np.float32)
        for c in range(Ct):
            want = (want + s[:, c::Ct]).astype(np.float32)
        assert np.array_equal(ts, want)
        tiles = (W.astype(np.float64) ** 2).reshape(B, R, N // Ct, Ct).sum(axis=(1, 3))
        assert np.allclose(ts, tiles, rtol=1e-5)
        tk, _ = orc.mask_rank(ts, ts.size // 2, orc.SCOPE_MATRIX)
        keep = orc.expand_tile_mask(tk, Ct)
        assert keep.shape == (B, N) and keep.sum() == Ct * tk.sum()
        assert np.array_equal(keep.reshape(B, N // Ct, Ct).min(axis=2), keep.reshape(B, N // Ct, Ct).max(axis=2))
        assert np.array_equal(keep[:, ::Ct], tk)
    # one tile per row-block: whole row-blocks go (the coarsest structure); kept tiles beat pruned ones
    ts = orc.tile_sumsq(s, N)
    tk, _ = orc.mask_rank(ts, 2, orc.SCOPE_MATRIX)
    assert tk.sum() == 2 and ts[tk == 1].min() > ts[tk == 0].max()
    ones = np.ones((2 * R, 8), np.float32)
    assert np.array_equal(orc.tile_sumsq(orc.sumsq(ones, R), 4), np.full((2, 2), 4.0 * R, np.float32))


# --------------------------------------------------------------------------- the other division: row segments
def test_rowseg_sumsq_is_the_column_group_sum_of_the_transposed_matrix():
    for (M, N, Cs) in ((6, 12, 3), (16, 64, 16), (5, 40, 8), (3, 7, 7), (4, 9, 1)):
        W = rand((M, N), 0.5)
        got = orc.rowseg_sumsq(W, Cs)
        # the same chain of fused multiply-adds, read along rows: bit for bit the pinned column-group sums of W^T
        assert np.array_equal(got, orc.sumsq(np.ascontiguousarray(W.T), Cs).T)
        assert np.allclose(got, (W.astype(np.float64) ** 2).reshape(M, N // Cs, Cs).sum(axis=2), rtol=1e-6)
    assert np.array_equal(orc.rowseg_sumsq(np.ones((2, 8), np.float32), 4), np.full((2, 2), 4.0, np.float32))
    one_hot = np.zeros((1, 8), np.float32); one_hot[0, 5] = -3.0
    assert np.array_equal(orc.rowseg_sumsq(one_hot, 4), np.array([[0.0, 9.0]], np.float32))
