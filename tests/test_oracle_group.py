"""Pins for the oracle's blockwise ("per-group") and scalar scale functions and for the
per-request axis of linear_variants.

Blockwise scales are Eq. 1 with v constant over blocks (one scale per output row and group of g
consecutive inputs, or one per group shared by all rows); the paper names them as its first
extension (Conclusion) and its comparison baseline is the one-scalar case (Experiments).  The
pins are what those definitions fix without running the oracle's own loops: the reductions to
row mode (g = d_in), to column mode (g = 1, shared rows) and to a constant scale, bit for bit
against the per-axis functions (which have their own pins); exact rational block means rounded
by brute-force search; the least-squares property of mean|dW| per block; deltas built as
v (.) B recovered exactly; integer-valued brute force compared with ==.
"""
from fractions import Fraction

import numpy as np
import pytest

from oracle import pdelta_oracle as orc
from test_oracle_pack import h, rne_f16_search


def random_layer(seed, d_out=12, d_in=96, M=5):
    rng = np.random.default_rng(seed)
    X = h(rng.standard_normal((M, d_in)))
    W_b = h(rng.standard_normal((d_out, d_in)) * 0.02)
    dW = h(rng.standard_normal((d_out, d_in)) * np.exp(rng.normal(np.log(1e-3), 0.5, (d_out, 1))))
    return X, W_b, dW


def test_group_equal_to_d_in_is_row_mode_bit_for_bit():
    X, W_b, dW = random_layer(1)
    zero = np.zeros_like(dW)
    B, v_row, _ = orc.pack(dW, zero)
    Bg, vg = orc.pack_group(dW, zero, 96)
    assert np.array_equal(Bg, B) and vg.shape == (12, 1) and np.array_equal(vg[:, 0], v_row)
    assert np.array_equal(orc.patch_group(W_b, B, vg, 96), orc.patch(W_b, B, v_row, orc.ROW))
    assert np.array_equal(orc.patch_group_round(W_b, B, vg, 96), orc.patch_round(W_b, B, v_row, orc.ROW))
    assert np.array_equal(orc.linear_group(X, W_b, B, vg, 96), orc.linear(X, W_b, B, v_row, orc.ROW))


def test_group_of_one_shared_by_the_rows_is_column_mode_bit_for_bit():
    X, W_b, dW = random_layer(2)
    zero = np.zeros_like(dW)
    B, _, v_col = orc.pack(dW, zero)
    Bg, vg = orc.pack_group(dW, zero, 1, shared_rows=True)
    assert np.array_equal(Bg, B) and vg.shape == (1, 96) and np.array_equal(vg[0], v_col)
    assert np.array_equal(orc.patch_group(W_b, B, vg, 1), orc.patch(W_b, B, v_col, orc.COL))
    assert np.array_equal(orc.linear_group(X, W_b, B, vg, 1), orc.linear(X, W_b, B, v_col, orc.COL))


def test_one_scalar_is_a_constant_vector_in_either_per_axis_mode():
    X, W_b, dW = random_layer(3)
    B, _, _ = orc.pack(dW, np.zeros_like(dW))
    c = np.float16(0.0017)
    scalar = np.full((1, 1), c).view(np.uint16)
    want_row = orc.linear(X, W_b, B, np.full(12, c), orc.ROW)
    want_col = orc.linear(X, W_b, B, np.full(96, c), orc.COL)
    got = orc.linear_group(X, W_b, B, scalar, 96)
    assert np.array_equal(got, want_row) and np.array_equal(got, want_col)
    # and a constant block scale of any block size gives the same matrix again
    for g in (2, 8, 32, 48):
        assert np.array_equal(orc.patch_group(W_b, B, np.full((12, 96 // g), c).view(np.uint16), g),
                              orc.patch_group(W_b, B, scalar, 96))
    # the scalar's initial value: the mean of |dW| over the whole matrix, rounded once
    _, alpha = orc.pack_group(dW, np.zeros_like(dW), 96, shared_rows=True)
    total = sum(abs(Fraction(float(x))) for x in dW.ravel())
    assert alpha.shape == (1, 1) and int(alpha[0, 0]) == rne_f16_search(total / dW.size)


@pytest.mark.parametrize("shared", [False, True])
def test_block_means_equal_exact_rational_means_rounded_once(shared):
    rng = np.random.default_rng(5)
    for (d_out, d_in), g in (((3, 8), 4), ((4, 12), 3), ((5, 64), 32), ((2, 96), 16)):
        W_f = h(rng.standard_normal((d_out, d_in)) * 0.02)
        W_b = h(rng.standard_normal((d_out, d_in)) * 0.02)
        W_f[0, 0] = W_b[0, 0]
        _, v = orc.pack_group(W_f, W_b, g, shared_rows=shared)
        F = [[abs(Fraction(float(a)) - Fraction(float(b))) for a, b in zip(ra, rb)] for ra, rb in zip(W_f, W_b)]
        for r in range(v.shape[0]):
            rows = range(d_out) if shared else [r]
            for k in range(d_in // g):
                s = sum(F[o][i] for o in rows for i in range(k * g, (k + 1) * g))
                assert int(v[r, k]) == rne_f16_search(s / (len(rows) * g)), (d_out, d_in, g, r, k)


def test_block_scales_tell_rows_from_groups():
    # magnitude depends on (row, group) only: each block's scale is its own magnitude
    mag = np.array([[1.0, 2.0, 4.0], [8.0, 16.0, 32.0]])
    dW = h(np.repeat(mag, 32, axis=1))
    _, v = orc.pack_group(dW, np.zeros_like(dW), 32)
    assert v.view(np.float16).tolist() == mag.tolist()
    _, v = orc.pack_group(dW, np.zeros_like(dW), 32, shared_rows=True)
    assert v.view(np.float16).tolist() == [[4.5, 9.0, 18.0]]
    # patching with distinct block scales puts each scale on its own block and nowhere else
    B = np.full((2, 3), 0xFFFFFFFF, dtype=np.uint32)
    W = orc.patch_group(np.zeros((2, 96), np.float16), B, h(mag), 32)
    assert np.array_equal(W, np.repeat(mag, 32, axis=1))


def test_block_mean_is_the_least_squares_scale_of_its_block():
    rng = np.random.default_rng(9)
    dW = h(rng.standard_normal((4, 128)) * np.exp(rng.normal(np.log(1e-3), 0.5, (4, 4))).repeat(32, axis=1))
    B, v = orc.pack_group(dW, np.zeros_like(dW), 32)
    S, d = orc.unpack(B, 128), dW.astype(np.float64)
    s0 = v.view(np.float16).astype(np.float64)
    for o in range(4):
        for k in range(4):
            blk = slice(32 * k, 32 * k + 32)
            res = lambda s: np.sum((d[o, blk] - s * S[o, blk]) ** 2)
            ulp = float(np.spacing(np.float16(s0[o, k])))
            assert res(s0[o, k]) <= res(s0[o, k] + ulp) and res(s0[o, k]) <= res(s0[o, k] - ulp)
            assert res(s0[o, k]) < res(s0[o, k] * 1.05) and res(s0[o, k]) < res(s0[o, k] * 0.95)


def test_delta_built_as_block_scale_times_sign_is_recovered_exactly():
    rng = np.random.default_rng(21)
    d_out, d_in, g = 6, 128, 32
    S = np.where(rng.random((d_out, d_in)) < 0.5, -1.0, 1.0)
    v = h(np.exp(rng.normal(np.log(1e-3), 0.5, (d_out, d_in // g))))
    dW = h(np.repeat(v.astype(np.float64), g, axis=1) * S)
    B, vg = orc.pack_group(dW, np.zeros_like(dW), g)
    assert np.array_equal(orc.unpack(B, d_in), S) and np.array_equal(vg, v.view(np.uint16))
    # merging a delta onto a base it is exactly representable on gives the fine-tuned matrix back
    # (base on a grid of 1/64, block scales on a grid of 1/1024: every sum fits fp16 exactly)
    W_b = h(rng.integers(-8, 8, (d_out, d_in)) / 64.0)
    v2 = h(rng.integers(1, 9, (d_out, d_in // g)) / 1024.0)
    dW2 = np.repeat(v2.astype(np.float64), g, axis=1) * S
    W_f = h(W_b.astype(np.float64) + dW2)
    assert np.array_equal(W_f.astype(np.float64), W_b.astype(np.float64) + dW2)
    B, vg = orc.pack_group(W_f, W_b, g)
    assert np.array_equal(vg, v2.view(np.uint16))
    assert np.array_equal(orc.patch_group_round(W_b, B, vg, g), W_f.view(np.uint16))


@pytest.mark.parametrize("g,shared", [(4, False), (2, False), (8, False), (4, True), (1, True)])
def test_integer_brute_force_4_by_8(g, shared):
    rng = np.random.default_rng(100 + g)
    X = rng.integers(-4, 5, (3, 8)).astype(np.float16)
    W_b = rng.integers(-4, 5, (4, 8)).astype(np.float16)
    S = np.where(rng.random((4, 8)) < 0.5, -1, 1)
    v = rng.integers(0, 6, (1 if shared else 4, 8 // g)).astype(np.float16)
    B, _, _ = orc.pack(S.astype(np.float16), np.zeros((4, 8), np.float16))
    want = np.zeros((3, 4))
    for m in range(3):
        for o in range(4):
            for i in range(8):
                scale = int(v[0 if shared else o, i // g])
                want[m, o] += int(X[m, i]) * (int(W_b[o, i]) + scale * int(S[o, i]))
    assert np.array_equal(orc.linear_group(X, W_b, B, v, g), want)
    mi, oi = np.array([0, 2, 1]), np.array([3, 0, 2])
    assert np.array_equal(orc.linear_group_at(X, W_b, B, v, g, mi, oi), want[mi, oi])


def test_linear_group_at_and_patch_round_follow_the_full_functions():
    X, W_b, dW = random_layer(8, d_out=10, d_in=64, M=4)
    B, v = orc.pack_group(dW, np.zeros_like(dW), 16)
    Y = orc.linear_group(X, W_b, B, v, 16)
    mi, oi = np.array([0, 3, 1, 2]), np.array([9, 0, 4, 4])
    assert np.array_equal(orc.linear_group_at(X, W_b, B, v, 16, mi, oi), Y[mi, oi])
    assert np.array_equal(orc.patch_group_round(W_b, B, v, 16), orc.rne(orc.patch_group(W_b, B, v, 16)))
    # merged weights multiply to the same layer (the paper's merged deployment is the same function)
    assert np.allclose(Y, X.astype(np.float64) @ orc.patch_group(W_b, B, v, 16).T, rtol=1e-13, atol=1e-13)


def test_bad_group_arguments_are_rejected():
    X, W_b, dW = random_layer(4)
    with pytest.raises(ValueError):
        orc.pack_group(dW, np.zeros_like(dW), 7)
    B, v = orc.pack_group(dW, np.zeros_like(dW), 32)
    with pytest.raises(ValueError):
        orc.linear_group(X, W_b, B, v, 16)                       # v has the wrong number of groups
    with pytest.raises(ValueError):
        orc.linear_group(X, W_b, B, v[:5], 32)                   # neither d_out rows nor one


def test_variants_with_one_axis_per_request():
    rng = np.random.default_rng(17)
    R, d_out, d_in = 5, 8, 64
    X = h(rng.standard_normal((R, d_in)))
    W_b = h(rng.standard_normal((d_out, d_in)) * 0.05)
    Bs = [rng.integers(0, 2 ** 32, (d_out, d_in // 32), dtype=np.uint32) for _ in range(R)]
    axes = [orc.ROW, orc.COL, orc.COL, orc.ROW, orc.COL]
    vs = [h(rng.random(d_out if a == orc.ROW else d_in) * 0.01) for a in axes]
    got = orc.linear_variants(X, W_b, Bs, vs, axes)
    for r in range(R):
        S = orc.unpack(Bs[r], d_in)
        v = vs[r].astype(np.float64)
        W_hat = W_b.astype(np.float64) + (v[:, None] * S if axes[r] == orc.ROW else v[None, :] * S)
        assert np.allclose(got[r], X[r].astype(np.float64) @ W_hat.T, rtol=1e-12, atol=1e-12)
        assert np.array_equal(got[r], orc.linear(X[r:r + 1], W_b, Bs[r], vs[r], axes[r])[0])
    # one axis for all requests is the same as a list that repeats it
    rows = [r for r in range(R) if axes[r] == orc.COL]
    sub = orc.linear_variants(X[rows], W_b, [Bs[r] for r in rows], [vs[r] for r in rows], orc.COL)
    assert np.array_equal(sub, got[rows])
    with pytest.raises(ValueError):
        orc.linear_variants(X, W_b, Bs, vs, axes[:3])
