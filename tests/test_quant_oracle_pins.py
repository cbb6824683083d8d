"""Pins of the Algorithm 1 oracle (oracle/mq_quant_oracle.py) against things other than itself:
hand-evaluated cases, the special cases that reduce to round-to-nearest and to a closed form per
slice interval, and invariants of the objective.  CPU only."""
import os

import numpy as np
import pytest

import oracle

C = 8
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "alg1_hand_cases.txt")


def _one(w, s, z, widths, lam, dtype=np.float64):
    """Algorithm 1 on single weights w (1-D) sharing one scale and zero-offset."""
    w = np.atleast_1d(np.asarray(w, dtype=np.float64))
    W = np.zeros((1, 128 * ((w.size + 127) // 128)), dtype=np.float64)
    W[0, :w.size] = w
    G = W.shape[1] // 128
    q = oracle.quant_matgptq(W, np.full((1, G), s), np.full((1, G), z), C, widths, lam, 128, dtype)
    return q[0, :w.size]


def test_hand_evaluated_cases():
    n = 0
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        case, s, z, widths, lam, w, q = line.split()
        widths = [int(v) for v in widths.split(",")]
        lam = [float(v) for v in lam.split(",")]
        for dtype in (np.float64, np.float32):
            got = _one([float(w)], float(s), float(z), widths, lam, dtype)[0]
            assert got == int(q), (case, dtype)
        n += 1
    assert n == 12


def test_single_master_width_is_round_to_nearest():
    # R = {c}: the objective is (w - s(q - z))^2, minimised by the integer nearest to w/s + z, clipped
    rng = np.random.default_rng(1)
    s, z = 0.0123, 117.0
    k = rng.integers(-20, 280, 4000)                       # beyond both ends of the code range
    d = rng.uniform(-0.45, 0.45, k.size)                   # away from ties
    w = s * (k + d - z)
    want = np.clip(np.rint(w / s + z), 0, 255).astype(np.uint8)
    assert np.array_equal(_one(w, s, z, [8], [1.0]), want)
    assert np.array_equal(_one(w, s, z, [8], [0.37]), want)           # a positive weight changes nothing here


@pytest.mark.parametrize("r", [1, 2, 3, 4, 6, 7])
def test_single_low_width_picks_the_lowest_code_of_the_nearest_grid_point(r):
    # R = {r}: E depends on q only through S(q, r); all codes that slice to the nearest grid point tie,
    # and the smallest of them is q = max(0, t * step - step/2) for grid index t (round half up in Eq. 1)
    rng = np.random.default_rng(r)
    step = 1 << (C - r)
    s, z = 0.02, 0.0
    t = rng.integers(0, 1 << r, 500)
    d = rng.uniform(-0.4, 0.4, t.size)
    w = s * (t + d) * step
    want = np.maximum(0, t * step - step // 2).astype(np.uint8)
    assert np.array_equal(_one(w, s, z, [r], [1.0]), want)


def _interval_closed_form(wp, r, lam_r, lam_c):
    """R = {r, c}, unit scale, zero offset 0: on each interval of q where S(q, r) is constant the best q is
    the integer nearest to wp inside the interval; the answer is the best interval's.  Exact in float64
    for the inputs used (multiples of 1/8)."""
    step = 1 << (C - r)
    best = None
    for t in range(1 << r):
        lo = max(0, t * step - step // 2)
        hi = 255 if t == (1 << r) - 1 else t * step + step // 2 - 1
        q = int(min(max(np.floor(wp + 0.5), lo), hi))
        if abs(q - wp) == 0.5 and q - 1 >= lo and q > wp:      # nearest-integer tie inside: the smaller code
            q -= 1
        e = lam_r * (wp - t * step) ** 2 + lam_c * (wp - q) ** 2
        if best is None or e < best[0]:
            best = (e, q)
    return best[1]


@pytest.mark.parametrize("r,lam", [(2, (1.0, 1.0)), (3, (0.5, 1.0)), (4, (1.0, 0.125)), (6, (4.0, 1.0))])
def test_two_widths_against_interval_closed_form(r, lam):
    wp = np.arange(-64, 2700, 3) / 8.0 - 3.0               # multiples of 1/8 across and beyond the range
    wp = wp[np.abs(wp * 2 - np.rint(wp * 2)) > 0]          # no exact .5 (ties between intervals are not unique)
    got = _one(wp, 1.0, 0.0, [r, 8], list(lam))
    want = np.array([_interval_closed_form(v, r, lam[0], lam[1]) for v in wp], dtype=np.uint8)
    assert np.array_equal(got, want)


def test_invariants_of_the_objective():
    rng = np.random.default_rng(5)
    s, z = 0.031, 96.0
    w = s * (rng.uniform(70, 180, 3000) - z)
    widths, lam = [3, 4, 8], [1.0, 0.5, 0.1]
    q = _one(w, s, z, widths, lam)
    # scaling every lambda by a power of two scales E exactly: same codes, also in binary32
    assert np.array_equal(_one(w, s, z, widths, [4 * v for v in lam]), q)
    assert np.array_equal(_one(w, s, z, widths, lam, np.float32), _one(w, s, z, widths, [4 * v for v in lam], np.float32))
    # the order in which R is written does not matter
    assert np.array_equal(_one(w, s, z, [8, 3, 4], [0.1, 1.0, 0.5]), q)
    # a shift of w by the coarsest slicing step (32 codes at r = 3) shifts the code by the same, away from the clamps
    assert np.array_equal(_one(w + s * 32, s, z, widths, lam), q + 32)
    # the code is non-decreasing in w
    order = np.argsort(w)
    assert np.all(np.diff(q[order].astype(int)) >= 0)
    # a width with lambda 0 is the same as leaving it out
    assert np.array_equal(_one(w, s, z, [2, 3, 4, 8], [0.0, 1.0, 0.5, 0.1]), q)
    # unlike round-to-nearest: some codes differ from the nearest integer, none by more than the coarsest half step
    rtn = np.clip(np.rint(w / s + z), 0, 255)
    assert 0 < np.count_nonzero(q != rtn) < q.size and np.abs(q - rtn).max() <= 16


def test_chosen_code_beats_every_other_candidate_under_the_pinned_slice_and_dequant():
    # optimality, evaluated with the slice and de-quantisation functions that the linear-layer pins cover
    rng = np.random.default_rng(7)
    N, K = 3, 256
    scales = rng.uniform(0.01, 0.05, (N, 2)).astype(np.float16)
    zeros = rng.integers(100, 156, (N, 2)).astype(np.float16)
    W = (rng.standard_normal((N, K)) * 1.2).astype(np.float32)
    widths, lam = [2, 4, 8], [0.3, 1.0, 2.0]
    q = oracle.quant_matgptq(W, scales, zeros, C, widths, lam, 128, np.float64)

    def total(codes):
        e = np.zeros((N, K))
        for r, l in zip(widths, lam):
            e += l * (W.astype(np.float64) - oracle.dequant(oracle.slice_codes(codes, C, r), scales, zeros, 128)) ** 2
        return e

    e_best = total(q)
    for cand in range(256):
        e = total(np.full((N, K), cand, np.uint8))
        assert np.all(e_best <= e)
        assert np.all((e > e_best) | (q <= cand))              # among equal errors the smallest code was taken


def test_binary32_and_binary64_agree_except_at_near_ties():
    rng = np.random.default_rng(9)
    N, K = 8, 512
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    scales = np.full((N, 4), 0.0005, np.float16)
    zeros = np.full((N, 4), 128, np.float16)
    q32 = oracle.quant_matgptq(W, scales, zeros, C, [3, 4, 8], [1, 1, 1], 128, np.float32)
    q64 = oracle.quant_matgptq(W, scales, zeros, C, [3, 4, 8], [1, 1, 1], 128, np.float64)
    diff = q32 != q64
    assert diff.mean() < 1e-3
    if diff.any():                                           # where they differ the two errors are equal to rounding
        E = oracle.quant_errors(W, scales, zeros, C, [3, 4, 8], [1, 1, 1], 128, np.float64)
        n, k = np.nonzero(diff)
        a, b = E[q32[n, k], n, k], E[q64[n, k], n, k]
        assert np.all(np.abs(a - b) <= 1e-5 * b)


# ------------------------------------------------------------------ the column loop (Algorithm 2 of the appendix)
def _hessian_factor(K, seed, samples=None):
    """H = 2 X X^T + damping (the appendix' definition), U = upper Cholesky factor of H^-1 (numpy, float64)."""
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((K, samples or 4 * K)) * (1.0 + 3.0 * rng.random((K, 1)))   # uneven feature scales
    X[:, :] += 0.5 * X[rng.permutation(K), :]                                            # correlated features
    H = 2.0 * X @ X.T
    H += 0.01 * np.mean(np.diag(H)) * np.eye(K)
    Hinv = np.linalg.inv(H)
    return H, Hinv, np.linalg.cholesky(Hinv).T


def _layer(N, K, seed):
    from paper_2602_03537_amd import synth
    W = synth.make_weights(N, K, seed).astype(np.float32)
    _, s, z = synth.quantize_parent(W)
    return W, s, z


def _mean_dequant(Q, s, z, widths):
    return np.mean([oracle.dequant(oracle.slice_codes(Q, C, r), s, z, 128) for r in widths], axis=0)


def test_column_loop_with_a_diagonal_factor_is_algorithm_1_per_column():
    W, s, z = _layer(16, 256, [80])
    U = np.diag(np.random.default_rng(80).uniform(0.5, 2.0, 256))
    widths, lam = [3, 4, 8], [1.0, 0.5, 0.1]
    for dtype in (np.float32, np.float64):
        Q, E = oracle.matgptq_quantize(W, U, s, z, C, widths, lam, 128, 128, dtype)
        assert np.array_equal(Q, oracle.quant_matgptq(W, s, z, C, widths, lam, 128, dtype))
    want = (W.astype(np.float64) - _mean_dequant(Q, s, z, widths)) / np.diag(U)[None, :]
    assert np.allclose(E, want, rtol=1e-12, atol=1e-15)


def test_column_loop_telescopes_original_minus_quantised_equals_E_times_U():
    # every update the loop applied, summed up: W - mean_r dequant(S(Q, r)) = E @ U (U upper triangular).
    # A wrong sign, index range, transposed factor or missing division by the diagonal breaks this.
    W, s, z = _layer(12, 384, [81])
    _, _, U = _hessian_factor(384, 81)
    for widths, lam in (([8], [1.0]), ([3, 4, 8], [1.0, 1.0, 1.0]), ([2, 6], [0.5, 2.0])):
        Q, E = oracle.matgptq_quantize(W, U, s, z, C, widths, lam, 128, 128, np.float64)
        lhs = W.astype(np.float64) - _mean_dequant(Q, s, z, widths)
        assert np.abs(lhs - E @ U).max() <= 1e-12 * max(1.0, np.abs(lhs).max())
        assert np.abs(E @ U - E @ np.triu(U)).max() == 0.0


def test_column_loop_does_not_depend_on_the_block_size_bit_for_bit():
    W, s, z = _layer(8, 256, [82])
    _, _, U = _hessian_factor(256, 82)
    ref = oracle.matgptq_quantize(W, U, s, z, C, [3, 4, 8], [1, 1, 1], 128, 128, np.float32)
    for block in (32, 64, 256):
        got = oracle.matgptq_quantize(W, U, s, z, C, [3, 4, 8], [1, 1, 1], 128, block, np.float32)
        assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])


def _obs_row_solver(w, Hinv, s, z, widths, lam):
    """The same quantiser in its other textbook form: optimal-brain-surgeon updates with the explicit inverse
    Hessian, eliminating one coordinate at a time (no Cholesky factor).  One row, float64."""
    w = w.astype(np.float64).copy()
    Hi = Hinv.copy()
    K = w.size
    q = np.zeros(K, dtype=np.uint8)
    for j in range(K):
        g = j // 128
        qj = oracle.quant_matgptq(np.array([[w[j]]]), [[s[g]]], [[z[g]]], C, widths, lam, 1, np.float64)[0, 0]
        q[j] = qj
        deq = np.mean([float(s[g]) * (float(oracle.slice_codes(np.array([qj], np.uint8), C, r)[0]) - float(z[g]))
                       for r in widths])
        d = (w[j] - deq) / Hi[j, j]
        w[j + 1:] -= d * Hi[j, j + 1:]
        Hi[j + 1:, j + 1:] -= np.outer(Hi[j + 1:, j], Hi[j, j + 1:]) / Hi[j, j]
    return q


@pytest.mark.parametrize("widths,lam", [([8], [1.0]), ([3, 4, 8], [1.0, 1.0, 1.0])])
def test_column_loop_against_the_explicit_inverse_formulation(widths, lam):
    W, s, z = _layer(3, 256, [83])
    _, Hinv, U = _hessian_factor(256, 83)
    Q, _ = oracle.matgptq_quantize(W, U, s, z, C, widths, lam, 128, 128, np.float64)
    for n in range(3):
        assert np.array_equal(Q[n], _obs_row_solver(W[n], Hinv, s[n], z[n], widths, lam)), n


def test_column_loop_lowers_the_hessian_weighted_error_of_plain_rounding():
    W, s, z = _layer(16, 256, [84])
    H, _, U = _hessian_factor(256, 84)
    Q, _ = oracle.matgptq_quantize(W, U, s, z, C, [8], [1.0], 128, 128, np.float64)
    rtn = oracle.quant_matgptq(W, s, z, C, [8], [1.0], 128, np.float64)

    def loss(codes):
        d = W.astype(np.float64) - oracle.dequant(codes, s, z, 128)
        return np.trace(d @ H @ d.T)
    assert loss(Q) < 0.8 * loss(rtn)
    # and with several target widths the summed loss over those widths drops against Algorithm 1 without propagation
    widths = [3, 4, 8]
    Qm, _ = oracle.matgptq_quantize(W, U, s, z, C, widths, [1, 1, 1], 128, 128, np.float64)
    Q1 = oracle.quant_matgptq(W, s, z, C, widths, [1, 1, 1], 128, np.float64)

    def loss_mean(codes):
        d = W.astype(np.float64) - _mean_dequant(codes, s, z, widths)
        return np.trace(d @ H @ d.T)
    assert loss_mean(Qm) < loss_mean(Q1)
