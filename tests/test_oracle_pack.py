"""Pins for the oracle's sign / pack / unpack / scale-init / patch functions.

Nothing here recomputes the oracle's formula in the oracle's way.  The pins are: hand-written
words, an exhaustive sweep of 8-wide sign patterns, exact rational means rounded by brute-force
search over all fp16 values, the least-squares property that makes mean|dW| the right initial
scale, deltas built as v (.) B that must be recovered exactly, and the storage-size claim of
the paper (one bit per weight plus one fp16 vector: Section 2, Table "Checkpoint sizes").
"""
import bisect
from fractions import Fraction

import numpy as np
import pytest

from oracle import pdelta_oracle as orc
from paper_2512_19720_amd import synth


def h(a):
    return np.asarray(a, dtype=np.float16)


_F16_TABLE = None


def rne_f16_search(x: Fraction) -> int:
    """fp16 RNE of a non-negative rational by brute force over every finite fp16 value."""
    global _F16_TABLE
    if _F16_TABLE is None:
        bits = np.arange(0x7C00, dtype=np.uint16)
        _F16_TABLE = [Fraction(float(v)) for v in bits.view(np.float16).astype(np.float64)]
    keys = _F16_TABLE                      # monotone in the bit pattern for non-negative values
    j = bisect.bisect_left(keys, x)
    if j < len(keys) and keys[j] == x:
        return j
    assert 0 < j < len(keys)
    dlo, dhi = x - keys[j - 1], keys[j] - x
    if dlo != dhi:
        return j - 1 if dlo < dhi else j
    return j - 1 if (j - 1) % 2 == 0 else j


# ---- sign and bit order -----------------------------------------------------------------------

def test_hand_written_words():
    d = 2.0 ** -10
    z = np.zeros((1, 32), np.float16)
    alt = h([[d if i % 2 == 0 else -d for i in range(32)]])
    B, _, _ = orc.pack(alt, z)
    assert B.tolist() == [[0x55555555]]            # even input indices positive -> even bits set
    last_neg = h([[d] * 31 + [-d]])
    assert orc.pack(last_neg, z)[0].tolist() == [[0x7FFFFFFF]]
    first_neg = h([[-d] + [d] * 31])
    assert orc.pack(first_neg, z)[0].tolist() == [[0xFFFFFFFE]]   # LSB is input index 0
    w = h(np.linspace(-1, 1, 32)[None, :])
    assert orc.pack(w, w)[0].tolist() == [[0xFFFFFFFF]]            # W_f == W_b: sign(0) -> +1
    assert orc.pack(z, h(np.full((1, 32), d)))[0].tolist() == [[0]]  # W_f < W_b everywhere


def test_words_follow_the_input_axis_and_rows_are_separate():
    # entry (o, i) negative only at (1, 40): word [1][1], bit 8
    W = np.full((3, 64), 1.0, np.float16)
    W[1, 40] = -1.0
    B, _, _ = orc.pack(W, np.zeros_like(W))
    want = np.full((3, 2), 0xFFFFFFFF, np.uint32)
    want[1, 1] = 0xFFFFFFFF ^ (1 << 8)
    assert np.array_equal(B, want)


def test_sign_of_zero_minus_zero_and_subnormals():
    W_f = np.array([[0x0000, 0x8000, 0x0001, 0x8001, 0x0000, 0x8000, 0x0001, 0x0002]], np.uint16)
    W_b = np.array([[0x8000, 0x0000, 0x0000, 0x0000, 0x0000, 0x8000, 0x0002, 0x0001]], np.uint16)
    #               +0 vs -0 -0 vs +0  tiny>0   tiny<0   equal    equal   1ulp<2ulp 2ulp>1ulp
    B, v_row, _ = orc.pack(W_f, W_b)
    assert B.tolist() == [[0b10110111]]
    # mean |dW| = (0+0+1+1+0+0+1+1) * 2^-24 / 8 = 2^-25: a tie between 0 and the smallest
    # subnormal, which goes to the even one (0)
    assert v_row.tolist() == [0]


def test_exhaustive_8_wide_rows_at_each_of_4_positions():
    mags = h([0.5, 2.0 ** -24, 3.0, 2.0 ** -14, 7.0, 0.001, 1.0, 60000.0])
    for row in range(4):
        for pattern in range(256):
            bits = [(pattern >> i) & 1 for i in range(8)]
            W = np.full((4, 8), 1.0, np.float16)
            W[row] = [m if b else -m for m, b in zip(mags, bits)]
            B, _, _ = orc.pack(W, np.zeros_like(W))
            want = [[0xFF]] * 4
            want[row] = [pattern]
            assert B.tolist() == want
            U = orc.unpack(B, 8)
            assert np.array_equal(U[row], np.where(np.array(bits) == 1, 1.0, -1.0))
            assert np.all(U[[r for r in range(4) if r != row]] == 1.0)


@pytest.mark.parametrize("shape", [(5, 32), (3, 96), (7, 40), (2, 31), (1, 1)])
def test_round_trip_against_numpy_where(shape):
    rng = np.random.default_rng(shape[0] * 100 + shape[1])
    dW = h(rng.standard_normal(shape) * 1e-3)
    dW[rng.random(shape) < 0.1] = 0.0
    base = h(rng.standard_normal(shape) * 0.02)
    B, _, _ = orc.pack(dW, np.zeros_like(dW))
    assert B.shape == (shape[0], (shape[1] + 31) // 32)
    want = np.where(dW.astype(np.float64) < 0, -1.0, 1.0)
    assert np.array_equal(orc.unpack(B, shape[1]), want)
    # sign is decided by comparing the stored values, not by a rounded subtraction
    W_f = h(base.astype(np.float32) + dW.astype(np.float32))
    B2, _, _ = orc.pack(W_f, base)
    want2 = np.where(W_f.astype(np.float64) < base.astype(np.float64), -1.0, 1.0)
    assert np.array_equal(orc.unpack(B2, shape[1]), want2)
    # padding bits of a ragged last word are zero
    if shape[1] % 32:
        assert np.all(B[:, -1] >> np.uint32(shape[1] % 32) == 0)


def test_bf16_inputs_are_compared_as_bf16():
    rng = np.random.default_rng(5)
    a = synth.f32_to_bf16_bits(rng.standard_normal((4, 64)).astype(np.float32))
    b = synth.f32_to_bf16_bits(rng.standard_normal((4, 64)).astype(np.float32))
    B, v_row, v_col = orc.pack(a, b, orc.BF16)
    fa, fb = synth.bf16_bits_to_f32(a).astype(np.float64), synth.bf16_bits_to_f32(b).astype(np.float64)
    assert np.array_equal(orc.unpack(B, 64), np.where(fa < fb, -1.0, 1.0))
    assert np.array_equal(v_row, np.abs(fa - fb).mean(axis=1).astype(np.float16).view(np.uint16))
    assert np.array_equal(v_col, np.abs(fa - fb).mean(axis=0).astype(np.float16).view(np.uint16))


def test_storage_is_one_bit_per_weight_plus_one_fp16_vector():
    d_out, d_in = 48, 256
    dW = h(np.ones((d_out, d_in)))
    B, v_row, v_col = orc.pack(dW, np.zeros_like(dW))
    assert B.nbytes == d_out * d_in // 8                 # 1/16 of the fp16 matrix
    assert B.nbytes * 16 == dW.nbytes
    assert v_row.nbytes == 2 * d_out and v_col.nbytes == 2 * d_in
    # Llama-3.1-8B projections: 32 blocks of q,o (4096x4096), k,v (1024x4096), gate,up,down
    # (14336x4096).  Their sign bits, the per-axis fp16 vectors, and the embeddings and head
    # that stay in fp16 must land on the size the paper prints for this model
    # (tests/golden/checkpoint_sizes.txt, from the paper's checkpoint-size table).
    import os
    golden = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "checkpoint_sizes.txt")):
        if line.strip() and not line.startswith("#"):
            model, artifact, mb, ratio = line.split()
            golden[(model, artifact)] = (float(mb), float(ratio))
    printed_mb, printed_ratio = golden[("Llama-3.1-8B-Instruct", "vector")]
    shapes = 32 * [(4096, 4096)] * 2 + 32 * [(1024, 4096)] * 2 + 32 * [(14336, 4096)] * 2 + 32 * [(4096, 14336)]
    sign_bytes = sum(o * i // 8 for o, i in shapes)
    vector_bytes = sum(2 * max(o, i) for o, i in shapes)            # at most one fp16 per row or column
    fp16_rest = 2 * 128256 * 4096 * 2                               # embeddings and head
    total_mb = (sign_bytes + vector_bytes + fp16_rest) / 1e6
    assert abs(total_mb - printed_mb) / printed_mb < 0.01
    full_fp16_mb = (2 * sum(o * i for o, i in shapes) + fp16_rest) / 1e6
    assert abs(full_fp16_mb / total_mb - printed_ratio) / printed_ratio < 0.03


# ---- scale initialisation ----------------------------------------------------------------------

def test_scales_equal_exact_rational_means_rounded_once():
    rng = np.random.default_rng(3)
    for shape in [(3, 5), (4, 8), (6, 33), (2, 64)]:
        W_f = h(rng.standard_normal(shape) * 0.02)
        W_b = h(rng.standard_normal(shape) * 0.02)
        W_f[0, 0] = W_b[0, 0]
        _, v_row, v_col = orc.pack(W_f, W_b)
        F = [[abs(Fraction(float(a)) - Fraction(float(b))) for a, b in zip(ra, rb)]
             for ra, rb in zip(W_f, W_b)]
        want_row = [rne_f16_search(sum(r) / shape[1]) for r in F]
        want_col = [rne_f16_search(sum(F[o][i] for o in range(shape[0])) / shape[0])
                    for i in range(shape[1])]
        assert v_row.tolist() == want_row
        assert v_col.tolist() == want_col


def test_row_scale_has_d_out_entries_and_col_scale_d_in():
    dW = h(np.outer([1.0, 2.0, 4.0], np.ones(64)))            # magnitude depends on the row only
    _, v_row, v_col = orc.pack(dW, np.zeros_like(dW))
    assert v_row.view(np.float16).tolist() == [1.0, 2.0, 4.0]
    assert np.all(v_col.view(np.float16) == np.float16(7.0 / 3.0))
    dW = h(np.outer(np.ones(3), np.arange(64) + 1.0))          # ... on the column only
    _, v_row, v_col = orc.pack(dW, np.zeros_like(dW))
    assert np.array_equal(v_col.view(np.float16), h(np.arange(64) + 1.0))
    assert np.all(v_row.view(np.float16) == np.float16(32.5))


def test_mean_abs_is_the_least_squares_scale_for_a_sign_matrix():
    # argmin_s || dW_row - s * B_row ||^2 = mean |dW_row|: moving s either way raises the residual
    rng = np.random.default_rng(9)
    dW = h(rng.standard_normal((6, 128)) * np.exp(rng.normal(np.log(1e-3), 0.5, (6, 1))))
    B, v_row, _ = orc.pack(dW, np.zeros_like(dW))
    Bd = orc.unpack(B, 128)
    d = dW.astype(np.float64)
    s0 = v_row.view(np.float16).astype(np.float64)
    for o in range(6):
        ulp = np.spacing(np.float16(s0[o])).astype(np.float64)
        res = lambda s: np.sum((d[o] - s * Bd[o]) ** 2)
        assert res(s0[o]) <= res(s0[o] + ulp) and res(s0[o]) <= res(s0[o] - ulp)
        assert res(s0[o]) < res(s0[o] * 1.05) and res(s0[o]) < res(s0[o] * 0.95)


def test_delta_built_as_v_times_b_is_recovered_exactly():
    rng = np.random.default_rng(21)
    d_out, d_in = 12, 96
    Bd = np.where(rng.random((d_out, d_in)) < 0.5, -1.0, 1.0)
    v_r = h(np.exp(rng.normal(np.log(1e-3), 0.5, d_out)))
    dW = h(v_r.astype(np.float64)[:, None] * Bd)                # exactly representable
    B, v_row, _ = orc.pack(dW, np.zeros_like(dW))
    assert np.array_equal(orc.unpack(B, d_in), Bd)
    assert np.array_equal(v_row, v_r.view(np.uint16))
    v_c = h(np.exp(rng.normal(np.log(1e-3), 0.5, d_in)))
    dW = h(v_c.astype(np.float64)[None, :] * Bd)
    B, _, v_col = orc.pack(dW, np.zeros_like(dW))
    assert np.array_equal(orc.unpack(B, d_in), Bd)
    assert np.array_equal(v_col, v_c.view(np.uint16))
    # a constant magnitude is both the row and the column mean
    c = np.float16(0.00123)
    B, v_row, v_col = orc.pack(h(np.float64(c) * Bd), np.zeros((d_out, d_in), np.float16))
    assert np.all(v_row == c.view(np.uint16)) and np.all(v_col == c.view(np.uint16))


def test_generated_deltas_give_sigma_times_sqrt_2_over_pi():
    L = synth.layer_host(64, 4096, 1, synth.F16, "row", synth.seed_for(0, 99))
    _, v_row, _ = orc.pack(L["dW"], np.zeros_like(L["dW"]))
    v = v_row.view(np.float16).astype(np.float64)
    rms = np.sqrt((L["dW"].view(np.float16).astype(np.float64) ** 2).mean(axis=1))
    # E|N(0,s^2)| = s * sqrt(2/pi); 4096 samples per row -> ~1.2 % standard error
    assert np.allclose(v / rms, np.sqrt(2 / np.pi), rtol=0.06)


# ---- patch --------------------------------------------------------------------------------------

def test_patch_special_cases():
    rng = np.random.default_rng(33)
    d_out, d_in = 9, 64
    W_b = h(rng.standard_normal((d_out, d_in)) * 0.02)
    Bd = np.where(rng.random((d_out, d_in)) < 0.5, -1.0, 1.0)
    B, _, _ = orc.pack(h(Bd), np.zeros((d_out, d_in), np.float16))
    zero_r, zero_c = np.zeros(d_out, np.float16), np.zeros(d_in, np.float16)
    # v = 0 leaves the base untouched
    assert np.array_equal(orc.patch(W_b, B, zero_r, orc.ROW), W_b.astype(np.float64))
    assert np.array_equal(orc.patch_round(W_b, B, zero_c, orc.COL), W_b.view(np.uint16))
    # W_b = 0, v = 1 returns B itself
    assert np.array_equal(orc.patch(np.zeros_like(W_b), B, np.ones(d_out, np.float16), orc.ROW), Bd)
    assert np.array_equal(orc.patch(np.zeros_like(W_b), B, np.ones(d_in, np.float16), orc.COL), Bd)
    # row mode scales whole rows, col mode whole columns (non-square on purpose)
    v_r = h(np.arange(d_out) + 1.0)
    v_c = h(np.arange(d_in) + 1.0)
    assert np.array_equal(orc.patch(np.zeros_like(W_b), B, v_r, orc.ROW), Bd * (np.arange(d_out) + 1.0)[:, None])
    assert np.array_equal(orc.patch(np.zeros_like(W_b), B, v_c, orc.COL), Bd * (np.arange(d_in) + 1.0)[None, :])
    with pytest.raises(ValueError):
        orc.patch(W_b, B, v_r, orc.COL)           # wrong length for the axis


def test_patch_restores_a_fine_tuned_matrix_built_from_exact_pieces():
    # W_b on a coarse grid (multiples of 2^-8, |w| < 0.5) and v on a fine one (multiples of
    # 2^-14 below 2^-7): every W_b +- v fits fp16's 11 significant bits... only when the sum
    # stays within one binade's precision, so build it to be so and check representability.
    rng = np.random.default_rng(4)
    d_out, d_in = 8, 64
    W_b = h(rng.integers(-32, 32, (d_out, d_in)) / 64.0)                  # multiples of 2^-6
    v_r = h(rng.integers(1, 8, d_out) / 1024.0)                           # multiples of 2^-10
    Bd = np.where(rng.random((d_out, d_in)) < 0.5, -1.0, 1.0)
    W_f64 = W_b.astype(np.float64) + v_r.astype(np.float64)[:, None] * Bd
    W_f = h(W_f64)
    assert np.array_equal(W_f.astype(np.float64), W_f64)                  # representable
    B, v_row, _ = orc.pack(W_f, W_b)
    assert np.array_equal(v_row, v_r.view(np.uint16))
    assert np.array_equal(orc.patch_round(W_b, B, v_row, orc.ROW), W_f.view(np.uint16))
    assert np.array_equal(orc.patch(W_b, B, v_row, orc.ROW), W_f64)


def test_patch_round_rounds_the_exact_sum_once():
    rng = np.random.default_rng(8)
    d_out, d_in = 6, 32
    W_b = h(rng.standard_normal((d_out, d_in)) * 0.02)
    v_c = h(np.exp(rng.normal(np.log(1e-3), 0.5, d_in)))
    B = rng.integers(0, 2 ** 32, (d_out, 1), dtype=np.uint32)
    got = orc.patch_round(W_b, B, v_c, orc.COL)
    for o in range(d_out):
        for i in range(d_in):
            b = 1 if (int(B[o, 0]) >> i) & 1 else -1
            exact = Fraction(float(W_b[o, i])) + b * Fraction(float(v_c[i]))
            want = rne_f16_search(abs(exact)) | (0x8000 if exact < 0 else 0)
            assert int(got[o, i]) == want


def test_swapping_the_models_flips_every_untied_sign_and_keeps_the_scales():
    rng = np.random.default_rng(41)
    W_f = h(rng.standard_normal((9, 96)) * 0.02)
    W_b = h(rng.standard_normal((9, 96)) * 0.02)
    W_f[:, :7] = W_b[:, :7]                                        # ties stay +1 both ways
    B1, r1, c1 = orc.pack(W_f, W_b)
    B2, r2, c2 = orc.pack(W_b, W_f)
    U1, U2 = orc.unpack(B1, 96), orc.unpack(B2, 96)
    tied = W_f.view(np.float16) == W_b.view(np.float16)
    assert np.array_equal(U1[~tied], -U2[~tied]) and np.all(U1[tied] == 1.0) and np.all(U2[tied] == 1.0)
    assert np.array_equal(r1, r2) and np.array_equal(c1, c2)       # |W_f - W_b| is symmetric


def test_scaling_both_models_by_a_power_of_two_scales_the_scales_exactly():
    rng = np.random.default_rng(42)
    W_f = (rng.standard_normal((6, 64)) * 0.02).astype(np.float16)
    W_b = (rng.standard_normal((6, 64)) * 0.02).astype(np.float16)
    B1, r1, c1 = orc.pack(W_f.view(np.uint16), W_b.view(np.uint16))
    B2, r2, c2 = orc.pack((W_f * np.float16(8)).view(np.uint16), (W_b * np.float16(8)).view(np.uint16))
    assert np.array_equal(B1, B2)
    assert np.array_equal(r2.view(np.float16), r1.view(np.float16) * np.float16(8))
    assert np.array_equal(c2.view(np.float16), c1.view(np.float16) * np.float16(8))


def test_rows_and_columns_are_independent():
    # changing one entry changes its own word, its row scale and its column scale, nothing else
    rng = np.random.default_rng(43)
    W_f = h(rng.standard_normal((5, 64)) * 0.02)
    W_b = h(rng.standard_normal((5, 64)) * 0.02)
    B1, r1, c1 = orc.pack(W_f, W_b)
    W_f2 = W_f.copy()
    W_f2[3, 40] = h(np.array([W_b.view(np.float16)[3, 40] - np.float16(0.5)]))[0]
    B2, r2, c2 = orc.pack(W_f2, W_b)
    diff_words = np.argwhere(B1 != B2)
    assert all(tuple(d) == (3, 1) for d in diff_words)             # entry (3, 40) lives in word [3][1]
    assert (orc.unpack(B2, 64)[3, 40]) == -1.0
    assert np.array_equal(np.delete(r1, 3), np.delete(r2, 3)) and r1[3] != r2[3]
    assert np.array_equal(np.delete(c1, 40), np.delete(c2, 40)) and c1[40] != c2[40]
