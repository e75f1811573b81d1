"""Pins for the oracle's delta linear layer Y = X W_hat^T, W_hat = v (.) B + W_b (Eq. 1).

The pins are cases where the answer is known without running the oracle's own loop: v = 0
reduces to a library matmul, an all-ones B gives a rank-one closed form that tells row mode
from column mode and d_out from d_in, a constant v makes the two modes coincide (the scalar
1-bit delta of the paper's baseline), the delta term is linear in v, and small integer-valued
problems are enumerated exactly.
"""
import itertools

import numpy as np
import pytest

from oracle import pdelta_oracle as orc
from paper_2512_19720_amd import synth


def h(a):
    return np.asarray(a, dtype=np.float16)


def f64(a):
    return np.asarray(a).astype(np.float64)


def small_case(seed, M=5, d_out=24, d_in=96):
    rng = np.random.default_rng(seed)
    X = h(rng.standard_normal((M, d_in)))
    W_b = h(rng.standard_normal((d_out, d_in)) * 0.02)
    B = rng.integers(0, 2 ** 32, (d_out, d_in // 32), dtype=np.uint32)
    v_r = h(np.exp(rng.normal(np.log(1e-3), 0.5, d_out)))
    v_c = h(np.exp(rng.normal(np.log(1e-3), 0.5, d_in)))
    return X, W_b, B, v_r, v_c


def test_zero_scale_is_the_plain_matmul():
    X, W_b, B, v_r, v_c = small_case(1)
    want = f64(X) @ f64(W_b).T                                   # library routine
    for axis, v in ((orc.ROW, np.zeros_like(v_r)), (orc.COL, np.zeros_like(v_c))):
        got = orc.linear(X, W_b, B, v, axis)
        assert got.shape == (5, 24)
        assert np.allclose(got, want, rtol=1e-13, atol=1e-15)


def test_all_plus_one_mask_gives_the_rank_one_closed_form():
    X, W_b, _, v_r, v_c = small_case(2)
    ones = np.full((24, 3), 0xFFFFFFFF, np.uint32)
    base = f64(X) @ f64(W_b).T
    # row: Y = X W_b^T + rowsum(X) v_row^T          (one scale per OUTPUT feature)
    want_row = base + np.outer(f64(X).sum(axis=1), f64(v_r))
    assert np.allclose(orc.linear(X, W_b, ones, v_r, orc.ROW), want_row, rtol=1e-12, atol=1e-14)
    # col: Y = X W_b^T + (X v_col) 1^T              (one scale per INPUT feature)
    want_col = base + np.outer(f64(X) @ f64(v_c), np.ones(24))
    assert np.allclose(orc.linear(X, W_b, ones, v_c, orc.COL), want_col, rtol=1e-12, atol=1e-14)
    # all minus one flips the sign of the delta term only
    zeros = np.zeros((24, 3), np.uint32)
    assert np.allclose(orc.linear(X, W_b, zeros, v_r, orc.ROW), 2 * base - want_row, rtol=1e-12, atol=1e-14)


def test_single_entry_picks_the_right_bit_and_the_right_operands():
    # X = e_m-th row selects input i0; W_b = 0; only B[o0, i0] is -1: Y must be -v at (m, o0)
    d_out, d_in, M = 6, 64, 3
    i0, o0, m0 = 37, 4, 2
    X = np.zeros((M, d_in), np.float16)
    X[m0, i0] = 2.0
    W_b = np.zeros((d_out, d_in), np.float16)
    B = np.full((d_out, 2), 0xFFFFFFFF, np.uint32)
    B[o0, 1] ^= np.uint32(1 << (i0 - 32))
    v_r = h(np.arange(d_out) + 1.0)
    Y = orc.linear(X, W_b, B, v_r, orc.ROW)
    want = np.zeros((M, d_out))
    want[m0] = 2.0 * (np.arange(d_out) + 1.0)
    want[m0, o0] *= -1
    assert np.array_equal(Y, want)
    v_c = h(np.arange(d_in) + 1.0)
    Y = orc.linear(X, W_b, B, v_c, orc.COL)
    want = np.zeros((M, d_out))
    want[m0] = 2.0 * (i0 + 1.0)
    want[m0, o0] *= -1
    assert np.array_equal(Y, want)


def test_row_and_col_modes_agree_for_a_constant_scale():
    X, W_b, B, _, _ = small_case(3)
    c = np.float16(0.0017)
    Yr = orc.linear(X, W_b, B, np.full(24, c), orc.ROW)
    Yc = orc.linear(X, W_b, B, np.full(96, c), orc.COL)
    assert np.allclose(Yr, Yc, rtol=1e-13, atol=1e-16)
    # and both equal base + c * (X B^T) with B from unpack: the scalar 1-bit delta
    want = f64(X) @ f64(W_b).T + float(c) * (f64(X) @ orc.unpack(B, 96).T)
    assert np.allclose(Yr, want, rtol=1e-12, atol=1e-14)


def test_delta_term_is_linear_in_v():
    X, W_b, B, v_r, v_c = small_case(4)
    for axis, v in ((orc.ROW, v_r), (orc.COL, v_c)):
        v1 = h(f64(v) * 0 + 2.0 ** -10)
        v2 = h(np.round(f64(v) * 2 ** 14) / 2 ** 14)            # v1 + v2 exactly representable
        v12 = h(f64(v1) + f64(v2))
        assert np.array_equal(f64(v12), f64(v1) + f64(v2))
        Y0 = orc.linear(X, W_b, B, np.zeros_like(v), axis)
        d1 = orc.linear(X, W_b, B, v1, axis) - Y0
        d2 = orc.linear(X, W_b, B, v2, axis) - Y0
        d12 = orc.linear(X, W_b, B, v12, axis) - Y0
        assert np.allclose(d12, d1 + d2, rtol=1e-9, atol=1e-12)


def test_sign_product_identity_and_equivalence_with_the_merged_weights():
    X, W_b, B, v_r, v_c = small_case(5)
    Bd = orc.unpack(B, 96)
    P = (Bd + 1) / 2
    xb = f64(X) @ Bd.T
    assert np.allclose(xb, 2 * (f64(X) @ P.T) - f64(X).sum(axis=1, keepdims=True), atol=1e-12)
    # on-the-fly layer == plain layer with the merged weights (the paper's deployed path)
    for axis, v in ((orc.ROW, v_r), (orc.COL, v_c)):
        W_hat = orc.patch(W_b, B, v, axis)
        assert np.allclose(orc.linear(X, W_b, B, v, axis), f64(X) @ W_hat.T, rtol=1e-12, atol=1e-14)
    want_row = f64(X) @ f64(W_b).T + xb * f64(v_r)[None, :]
    want_col = f64(X) @ f64(W_b).T + (f64(X) * f64(v_c)[None, :]) @ Bd.T
    assert np.allclose(orc.linear(X, W_b, B, v_r, orc.ROW), want_row, rtol=1e-12, atol=1e-14)
    assert np.allclose(orc.linear(X, W_b, B, v_c, orc.COL), want_col, rtol=1e-12, atol=1e-14)


def test_brute_force_4_by_8_with_integer_values_is_exact():
    # Integer-valued X, W_b, v: every product and sum is an exact small integer in fp64, so the
    # result can be compared with ==.  Python integers do the arithmetic here.
    rng = np.random.default_rng(6)
    d_out, d_in, M = 4, 8, 2
    for trial in range(40):
        Xi = rng.integers(-4, 5, (M, d_in))
        Wi = rng.integers(-8, 9, (d_out, d_in))
        Bi = rng.integers(0, 2, (d_out, d_in)) * 2 - 1
        vr = rng.integers(-3, 4, d_out)
        vc = rng.integers(-3, 4, d_in)
        words = np.array([[sum(1 << i for i in range(d_in) if Bi[o, i] > 0)] for o in range(d_out)], np.uint32)
        for axis, v in ((orc.ROW, vr), (orc.COL, vc)):
            want = [[sum(int(Xi[m, i]) * (int(Wi[o, i]) + int(v[o] if axis == orc.ROW else v[i]) * int(Bi[o, i]))
                         for i in range(d_in)) for o in range(d_out)] for m in range(M)]
            got = orc.linear(h(Xi), h(Wi), words, h(v), axis)
            assert got.tolist() == [[float(x) for x in r] for r in want]


def test_every_sign_pattern_of_one_8_wide_row():
    X = h([[1, 2, 4, 8, 16, 32, 64, 128]])
    W_b = np.zeros((1, 8), np.float16)
    for pattern in range(256):
        got = orc.linear(X, W_b, np.array([[pattern]], np.uint32), h([1.0]), orc.ROW)
        assert got[0, 0] == 2 * pattern - 255          # sum_{set} x - sum_{clear} x


def test_linear_at_matches_the_full_product():
    X, W_b, B, v_r, v_c = small_case(7, M=7, d_out=40, d_in=128)
    rng = np.random.default_rng(0)
    m_idx, o_idx = rng.integers(0, 7, 50), rng.integers(0, 40, 50)
    for axis, v in ((orc.ROW, v_r), (orc.COL, v_c)):
        Y = orc.linear(X, W_b, B, v, axis)
        ya = orc.linear_at(X, W_b, B, v, axis, m_idx, o_idx)
        assert np.allclose(ya, Y[m_idx, o_idx], rtol=1e-12, atol=1e-15)
    # and pin it independently too: v = 0 -> plain dot products
    ya = orc.linear_at(X, W_b, B, np.zeros_like(v_r), orc.ROW, m_idx, o_idx)
    want = np.einsum("sk,sk->s", f64(X)[m_idx], f64(W_b)[o_idx])
    assert np.allclose(ya, want, rtol=1e-12, atol=1e-15)
    with pytest.raises(ValueError):
        orc.linear_at(X, W_b, B, v_r, orc.ROW, [7], [0])


def test_bf16_operands_are_decoded_as_bf16():
    rng = np.random.default_rng(12)
    X = synth.f32_to_bf16_bits(rng.standard_normal((3, 64)).astype(np.float32))
    W = synth.f32_to_bf16_bits((rng.standard_normal((5, 64)) * 0.02).astype(np.float32))
    B = rng.integers(0, 2 ** 32, (5, 2), dtype=np.uint32)
    v = h(rng.random(5) * 1e-3)
    Xd, Wd = f64(synth.bf16_bits_to_f32(X)), f64(synth.bf16_bits_to_f32(W))
    want = Xd @ (Wd + f64(v)[:, None] * orc.unpack(B, 64)).T
    assert np.allclose(orc.linear(X, W, B, v, orc.ROW, orc.BF16), want, rtol=1e-12, atol=1e-15)


def test_config0_shape_runs_in_well_under_a_second():
    import time
    L = synth.layer_host(256, 512, 4, synth.F16, "row", synth.seed_for(0))
    B, v_row, _ = orc.pack(L["dW"], np.zeros_like(L["dW"]))
    t0 = time.time()
    Y = orc.linear(L["X"], L["W_b"], B, v_row, orc.ROW)
    assert time.time() - t0 < 1.0
    assert Y.shape == (4, 256) and np.isfinite(Y).all()
    # RMS(Y) ~ sqrt(d_in) * 0.02 for N(0,1) inputs against N(0, 0.02^2) weights
    assert 0.3 < np.sqrt((Y ** 2).mean()) < 0.65


def test_variants_reduce_to_the_single_layer_and_to_brute_force():
    # identical variants: the R requests are the R tokens of one ordinary layer
    rng = np.random.default_rng(21)
    d_out, d_in, R = 24, 96, 5
    X = rng.standard_normal((R, d_in)).astype(np.float16)
    W_b = (rng.standard_normal((d_out, d_in)) * 0.05).astype(np.float16)
    Bs = [rng.integers(0, 2 ** 32, (d_out, d_in // 32), dtype=np.uint32) for _ in range(R)]
    v_rows = [(rng.random(d_out) * 0.01).astype(np.float16) for _ in range(R)]
    v_cols = [(rng.random(d_in) * 0.01).astype(np.float16) for _ in range(R)]
    same = orc.linear_variants(X, W_b, [Bs[0]] * R, [v_rows[0]] * R, orc.ROW)
    assert np.array_equal(same, orc.linear(X, W_b, Bs[0], v_rows[0], orc.ROW))
    # distinct variants against the definition written out with numpy on unpacked signs
    for axis, vs in ((orc.ROW, v_rows), (orc.COL, v_cols)):
        got = orc.linear_variants(X, W_b, Bs, vs, axis)
        for r in range(R):
            S = orc.unpack(Bs[r], d_in)
            v = vs[r].astype(np.float64)
            W_hat = W_b.astype(np.float64) + (v[:, None] * S if axis == orc.ROW else v[None, :] * S)
            want = X[r].astype(np.float64) @ W_hat.T
            assert np.allclose(got[r], want, rtol=1e-12, atol=1e-12)
    # a request's result does not depend on the other requests
    alone = orc.linear_variants(X[2:3], W_b, [Bs[2]], [v_cols[2]], orc.COL)
    assert np.array_equal(alone[0], orc.linear_variants(X, W_b, Bs, v_cols, orc.COL)[2])


def test_grad_v_is_the_slope_of_the_layer_in_v_and_matches_brute_force():
    # Y is linear in v, so for L(v) = sum(dY * Y(v)) the gradient is an exact finite difference:
    # dL/dv[a] = L(v + e_a) - L(v).  Integer-valued v keeps v + 1 representable in fp16.
    rng = np.random.default_rng(31)
    M, d_out, d_in = 7, 12, 64
    X = rng.standard_normal((M, d_in)).astype(np.float16)
    dY = rng.standard_normal((M, d_out)).astype(np.float16)
    W_b = (rng.standard_normal((d_out, d_in)) * 0.05).astype(np.float16)
    B = rng.integers(0, 2 ** 32, (d_out, d_in // 32), dtype=np.uint32)
    S = orc.unpack(B, d_in)
    X64, dY64 = X.astype(np.float64), dY.astype(np.float64)
    for axis, n in ((orc.ROW, d_out), (orc.COL, d_in)):
        g = orc.grad_v(X, dY, B, axis)
        v = rng.integers(-3, 4, n).astype(np.float16)
        base = float((dY64 * orc.linear(X, W_b, B, v, axis)).sum())
        for a in (0, 1, n // 2, n - 1):
            bumped = v.copy()
            bumped[a] += np.float16(1.0)
            slope = float((dY64 * orc.linear(X, W_b, B, bumped, axis)).sum()) - base
            assert abs(slope - g[a]) <= 1e-9 * max(1.0, abs(g[a])), (axis, a)
        # the formula written out with numpy on the unpacked signs
        want = ((X64 @ S.T) * dY64).sum(0) if axis == orc.ROW else ((dY64 @ S) * X64).sum(0)
        assert np.allclose(g, want, rtol=1e-12, atol=1e-12)
    # swapping the roles of the two modes needs the transposed sign matrix: with B = all ones
    # both gradients reduce to sums that are easy to state
    ones = np.full((d_out, d_in // 32), 0xFFFFFFFF, dtype=np.uint32)
    assert np.allclose(orc.grad_v(X, dY, ones, orc.ROW), (X64.sum(1)[:, None] * dY64).sum(0), atol=1e-12)
    assert np.allclose(orc.grad_v(X, dY, ones, orc.COL), (dY64.sum(1)[:, None] * X64).sum(0), atol=1e-12)
