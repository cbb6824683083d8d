"""Pins for the CPU oracle: everything here is checked against something other
than the oracle itself -- hand-evaluated values of Eq. 1, exact rational
arithmetic, invariants Eq. 1 fixes, brute force over tiny matrices, closed
forms.  A dropped term, wrong sign, wrong group axis or transposed operand in
oracle/ fails at least one of these.  (CPU only.)
"""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import c_oracle

WIDTHS = (2, 3, 4, 6, 8)
C = 8
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "slice_eq1_examples.txt")
ALL_Q = np.arange(256, dtype=np.uint8)

SLICERS = [pytest.param(oracle.slice_codes, id="numpy"),
           pytest.param(c_oracle.slice_codes, id="c")]


# ----------------------------------------------------------------- Eq. 1 pins
def _golden_rows():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.split("#")[0].split()
            if line:
                rows.append([int(v) for v in line])
    return rows


@pytest.mark.parametrize("slicer", SLICERS)
def test_slice_hand_evaluated_examples(slicer):
    rows = _golden_rows()
    assert len(rows) >= 7
    for q, *expected in rows:
        got = [int(slicer(np.array([q], dtype=np.uint8), C, r)[0]) for r in WIDTHS]
        assert got == expected, (q, got, expected)


def _eq1_exact(q: int, c: int, r: int) -> int:
    """Eq. 1 in exact rationals: floor(q/2^(c-r) + 1/2), clamp, rescale."""
    v = Fraction(q, 2 ** (c - r)) + Fraction(1, 2)
    t = v.numerator // v.denominator
    t = max(0, min(t, 2 ** r - 1))
    return t * 2 ** (c - r)


@pytest.mark.parametrize("slicer", SLICERS)
@pytest.mark.parametrize("c", [8, 6, 4])
def test_slice_exhaustive_vs_exact_rationals(slicer, c):
    q = np.arange(2 ** c, dtype=np.uint8)
    for r in range(1, c + 1):
        got = slicer(q, c, r)
        want = np.array([_eq1_exact(int(v), c, r) for v in q], dtype=np.uint8)
        assert np.array_equal(got, want), (c, r)


@pytest.mark.parametrize("slicer", SLICERS)
def test_slice_invariants(slicer):
    for r in range(1, C + 1):
        S = slicer(ALL_Q, C, r).astype(int)
        step = 2 ** (C - r)
        h = step // 2
        if r == C:
            assert np.array_equal(S, ALL_Q.astype(int))          # identity at r = c
        assert np.all(np.diff(S) >= 0)                            # monotone in the code
        assert np.all(S % step == 0)                              # on the 2^(c-r) grid
        assert S.min() == 0 and S.max() == 2 ** C - step          # range of an r-bit model
        assert len(np.unique(S)) == 2 ** r                        # every level reachable
        err = ALL_Q.astype(int) - S
        clamped = ALL_Q.astype(int) >= 2 ** C - h if h else np.zeros(256, bool)
        if h:
            assert np.all(err[~clamped] >= -h) and np.all(err[~clamped] <= h - 1)
            assert np.all(err[clamped] >= h) and np.all(err[clamped] <= 2 * h - 1)
        # a sliced code is a fixed point of slicing
        assert np.array_equal(slicer(S.astype(np.uint8), C, r).astype(int), S)


def test_slice_tie_codes_round_up():
    # q = (2j+1) * 2^(c-r-1) sits exactly between two levels: Section 3.1 pushes it up.
    for r in (2, 3, 4, 6):
        h = 2 ** (C - r - 1)
        for j in range(2 ** r - 1):
            q = (2 * j + 1) * h
            assert int(oracle.slice_codes(np.array([q], np.uint8), C, r)[0]) == (j + 1) * 2 * h


def test_slice_is_not_a_bit_prefix_and_not_nested():
    # Rounding carries, so S(q,r) is not "the top r bits" and slicing twice differs
    # from slicing once (q=8: 4 bits -> 1, then 3 bits -> 1; directly 3 bits -> 0).
    S4 = oracle.slice_codes(ALL_Q, C, 4)
    assert np.any(S4 != (ALL_Q & 0xF0))
    t43 = oracle.sliced_index(S4, C, 3)
    t3 = oracle.sliced_index(ALL_Q, C, 3)
    assert int(t43[8]) == 1 and int(t3[8]) == 0


def test_sliced_index_is_S_shifted():
    for r in WIDTHS:
        t = oracle.sliced_index(ALL_Q, C, r).astype(int)
        S = oracle.slice_codes(ALL_Q, C, r).astype(int)
        assert np.array_equal(t * 2 ** (C - r), S) and t.max() == 2 ** r - 1


def test_slice_rejects_bad_widths():
    for c, r in [(8, 0), (8, 9), (9, 4), (4, 5)]:
        with pytest.raises(ValueError):
            oracle.slice_codes(ALL_Q[:4], c, r)


# ---------------------------------------------------- dequant + linear pins
def _f(v):  # exact rational value of a float16/float
    return Fraction(float(v))


def _linear_exact(x, parent, scales, zeros, c, r, group):
    """Brute force in exact rationals, one term at a time."""
    M, K = x.shape
    N = parent.shape[0]
    y = [[Fraction(0)] * N for _ in range(M)]
    for m in range(M):
        for n in range(N):
            acc = Fraction(0)
            for k in range(K):
                g = k // group
                S = _eq1_exact(int(parent[n, k]), c, r)
                acc += _f(x[m, k]) * _f(scales[n, g]) * (S - _f(zeros[n, g]))
            y[m][n] = acc
    return np.array([[float(v) for v in row] for row in y])


def _tiny(seed, M, N, K, group):
    rng = np.random.default_rng(seed)
    G = K // group
    return dict(
        x=rng.standard_normal((M, K)).astype(np.float16),
        parent=rng.integers(0, 256, (N, K), dtype=np.uint8),
        scales=rng.uniform(1e-3, 2e-2, (N, G)).astype(np.float16),
        zeros=rng.uniform(0, 255, (N, G)).astype(np.float16),
    )


@pytest.mark.parametrize("r", WIDTHS)
@pytest.mark.parametrize("shape", [(1, 3, 8, 4), (2, 5, 12, 4), (3, 2, 16, 8)])
def test_linear_brute_force_exact_rationals(r, shape):
    M, N, K, group = shape
    t = _tiny(100 + r, M, N, K, group)
    want = _linear_exact(t["x"], t["parent"], t["scales"], t["zeros"], C, r, group)
    got = oracle.linear(t["x"], t["parent"], t["scales"], t["zeros"], C, r, group)
    assert got.shape == (M, N)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)
    got_c, used = c_oracle.linear(t["x"], t["parent"], t["scales"], t["zeros"], C, r, group)
    assert used >= 1
    np.testing.assert_allclose(got_c, want, rtol=1e-12, atol=1e-12)


def test_linear_enumerates_every_code_at_every_position():
    # N=1, K=2 (group 1 and group 2): all 256 codes at each position, one at a time.
    x = np.array([[1.5, -0.25]], dtype=np.float16)
    s = np.array([[0.5, 2.0]], dtype=np.float16)
    z = np.array([[3.0, 100.5]], dtype=np.float16)
    for r in WIDTHS:
        for pos, q in itertools.product(range(2), range(256)):
            parent = np.array([[7, 200]], dtype=np.uint8)
            parent[0, pos] = q
            S = [_eq1_exact(int(v), C, r) for v in parent[0]]
            want = 1.5 * 0.5 * (S[0] - 3.0) + (-0.25) * 2.0 * (S[1] - 100.5)
            got = oracle.linear(x, parent, s, z, C, r, 1)[0, 0]
            assert got == pytest.approx(want, abs=1e-12)


def test_one_hot_weight_picks_one_input_and_one_output():
    # Every weight dequantises to 0 (code == zero) except W[n0,k0]: catches a
    # transposed operand, a wrong group axis and an off-by-one group index.
    N, K, group = 6, 16, 4
    G = K // group
    zeros = np.full((N, G), 64.0, dtype=np.float16)
    scales = (np.arange(N * G).reshape(N, G) + 1).astype(np.float16)
    x = (np.arange(K) + 1).astype(np.float16)[None, :]
    for n0, k0 in [(0, 0), (2, 5), (5, 15), (3, 8)]:
        parent = np.full((N, K), 64, dtype=np.uint8)
        parent[n0, k0] = 192
        for r in WIDTHS:            # 64 and 192 are on every grid, so slicing keeps them
            y = oracle.linear(x, parent, scales, zeros, C, r, group)
            want = np.zeros((1, N))
            want[0, n0] = float(x[0, k0]) * float(scales[n0, k0 // group]) * 128.0
            np.testing.assert_array_equal(y, want)


def test_constant_code_closed_form():
    # all codes equal q0, scale s, zero z  =>  y[n] = s * (S(q0) - z) * sum(x)
    t = _tiny(7, 2, 4, 32, 8)
    for r in WIDTHS:
        for q0 in (0, 9, 100, 250):
            parent = np.full((4, 32), q0, dtype=np.uint8)
            s = np.full((4, 4), 0.25, dtype=np.float16)
            z = np.full((4, 4), 17.0, dtype=np.float16)
            y = oracle.linear(t["x"], parent, s, z, C, r, 8)
            S0 = _eq1_exact(q0, C, r)
            want = 0.25 * (S0 - 17.0) * t["x"].astype(np.float64).sum(axis=1)
            np.testing.assert_allclose(y, np.repeat(want[:, None], 4, axis=1), rtol=1e-13, atol=1e-13)


def test_group_factorisation_identity():
    # sum_k x s (S - z) = sum_g s_g (sum_{k in g} x S - z_g sum_{k in g} x), loops written here.
    t = _tiny(11, 2, 5, 24, 8)
    for r in WIDTHS:
        y = oracle.linear(t["x"], t["parent"], t["scales"], t["zeros"], C, r, 8)
        x = t["x"].astype(np.float64)
        want = np.zeros((2, 5))
        for m in range(2):
            for n in range(5):
                for g in range(3):
                    ks = range(8 * g, 8 * g + 8)
                    xs = sum(x[m, k] * _eq1_exact(int(t["parent"][n, k]), C, r) for k in ks)
                    sx = sum(x[m, k] for k in ks)
                    want[m, n] += float(t["scales"][n, g]) * (xs - float(t["zeros"][n, g]) * sx)
        np.testing.assert_allclose(y, want, rtol=1e-11, atol=1e-11)


def test_r8_is_the_textbook_affine_dequant_matmul():
    # At r = c the layer is the ordinary 8-bit group-quantised linear: einsum over
    # an explicitly expanded (repeat) scale/zero, a different route from reshape.
    t = _tiny(3, 3, 7, 64, 16)
    s = np.repeat(t["scales"].astype(np.float64), 16, axis=1)
    z = np.repeat(t["zeros"].astype(np.float64), 16, axis=1)
    w = s * (t["parent"].astype(np.float64) - z)
    want = np.einsum("mk,nk->mn", t["x"].astype(np.float64), w)
    got = oracle.linear(t["x"], t["parent"], t["scales"], t["zeros"], C, 8, 16)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


def test_linear_is_linear_in_x_and_rows_are_independent():
    t = _tiny(5, 2, 6, 32, 8)
    a = oracle.linear(t["x"][:1], t["parent"], t["scales"], t["zeros"], C, 3, 8)
    b = oracle.linear(t["x"][1:], t["parent"], t["scales"], t["zeros"], C, 3, 8)
    both = oracle.linear(t["x"], t["parent"], t["scales"], t["zeros"], C, 3, 8)
    np.testing.assert_allclose(np.vstack([a, b]), both, rtol=1e-13)
    x2 = (t["x"].astype(np.float32) * 2).astype(np.float16)        # exact doubling
    d = oracle.linear(x2, t["parent"], t["scales"], t["zeros"], C, 3, 8)
    np.testing.assert_allclose(d, 2 * both, rtol=1e-13)
    rows = [4, 1]
    sub = oracle.linear_rows(t["x"], t["parent"], t["scales"], t["zeros"], C, 3, 8, rows)
    np.testing.assert_array_equal(sub, both[:, rows])


def test_symmetric_case_zero_is_half_range():
    # Section 5 setup quantises symmetrically: zero = 2^(c-1) for every group.
    t = _tiny(9, 1, 4, 32, 8)
    z = np.full_like(t["zeros"], 128.0)
    y = oracle.linear(t["x"], t["parent"], t["scales"], z, C, 4, 8)
    want = _linear_exact(t["x"], t["parent"], t["scales"], z, C, 4, 8)
    np.testing.assert_allclose(y, want, rtol=1e-12, atol=1e-12)


def test_numpy_and_c_oracles_agree_on_a_multi_group_layer():
    from paper_2602_03537_amd import synth
    L = synth.make_layer(96, 384, M=2, seed=[0, 42])
    for r in WIDTHS:
        a = oracle.linear(L["x"], L["parent"], L["scales"], L["zeros"], C, r, 128)
        b, _ = c_oracle.linear(L["x"], L["parent"], L["scales"], L["zeros"], C, r, 128)
        np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-12)


def test_linear_stack_uses_each_layers_own_width():
    ts = [_tiny(20 + i, 1, 3, 16, 8) for i in range(3)]
    for t, r in zip(ts, (2, 6, 4)):
        t["r"] = r
    ys = oracle.linear_stack(ts, C, 8)
    for t, y in zip(ts, ys):
        want = _linear_exact(t["x"], t["parent"], t["scales"], t["zeros"], C, t["r"], 8)
        np.testing.assert_allclose(y, want, rtol=1e-12, atol=1e-12)
