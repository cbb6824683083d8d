"""CPU checks of the bar in tests/tolerance.py: the reading for outputs too short for a relative-L2 norm.

The two one-row layers below are the inputs on which a randomized sweep of the library missed relative-L2 <= 1e-3
at batch 1 (the outputs are single values of 2.1e-3 and -6.6e-4 left over from terms of root-sum-square 0.7 and
0.45).  Here the kernel's arithmetic is imitated in numpy binary32 (factored form, one group after the other, fp16
result) to show that the reading accepts what fp32 accumulation can deliver and still rejects a planted mistake."""
import numpy as np
import pytest

import oracle
from paper_2602_03537_amd import synth
import tolerance

CANCELLING = [(1, 1280, 3, 972345906), (1, 512, 4, 649105576)]


def fp32_factored(L, r, order=1):
    """y as an fp32 machine adding the factored form group by group would get it, rounded to fp16"""
    S = oracle.slice_codes(L["parent"], 8, r).astype(np.float32)
    x = L["x"].astype(np.float32)
    s, z = L["scales"].astype(np.float32), L["zeros"].astype(np.float32)
    M, K = x.shape
    N = S.shape[0]
    y = np.zeros((M, N), np.float32)
    for g in list(range(K // 128))[::order]:
        sl = slice(g * 128, (g + 1) * 128)
        for m in range(M):
            d = np.zeros(N, np.float32)
            xg = np.float32(0)
            for k in range(128):
                d = d + x[m, sl][k] * S[:, sl][:, k]
                xg = np.float32(xg + x[m, sl][k])
            y[m] = y[m] + s[:, g] * (d - z[:, g] * xg)
    return y.astype(np.float16).astype(np.float64)


@pytest.mark.parametrize("N,K,r,seed", CANCELLING)
def test_cancelling_one_row_outputs_are_judged_by_their_terms(N, K, r, seed):
    L = synth.make_layer(N, K, M=1, seed=[seed])
    ref = oracle.linear(L["x"], L["parent"], L["scales"], L["zeros"], 8, r, 128)
    a, B = tolerance.term_scales(L["x"], L["parent"], L["scales"], L["zeros"], 8, r, 128)
    assert abs(ref[0, 0]) < 5e-3 * a[0, 0]                    # the terms cancel to well below their scale
    for order in (1, -1):
        y = fp32_factored(L, r, order)
        assert tolerance.failure(y, ref, (a, B)) is None
    assert tolerance.failure(ref, ref) is not None             # a short output is never judged without its terms
    # planted mistakes the size of one weight's contribution, or of one group's zero-offset, are still caught
    w = oracle.dequant(oracle.slice_codes(L["parent"], 8, r), L["scales"], L["zeros"], 128)
    k = int(np.argmax(np.abs(L["x"][0].astype(np.float64) * w[0])))
    dropped = ref - L["x"][0, k].astype(np.float64) * w[0, k]
    assert tolerance.failure(dropped, ref, (a, B)) is not None
    zoff = ref + L["scales"][0, 0].astype(np.float64) * L["x"][0, :128].astype(np.float64).sum()   # zero-offset off by one
    assert tolerance.failure(zoff, ref, (a, B)) is not None


def test_long_outputs_keep_the_literal_bar():
    L = synth.make_layer(64, 256, M=1, seed=[5])
    ref = oracle.linear(L["x"], L["parent"], L["scales"], L["zeros"], 8, 4, 128)
    assert tolerance.failure(ref.astype(np.float16).astype(np.float64), ref) is None
    assert tolerance.failure(ref * (1 + 2e-3), ref) is not None           # relative-L2 2e-3
    bad = ref.copy()
    bad[0, 3] += 3e-2
    assert tolerance.failure(bad, ref) is not None                        # max-abs
    nan = ref.copy()
    nan[0, 0] = np.nan
    assert tolerance.failure(nan, ref) is not None
    assert tolerance.failure(ref[:, :10], ref) is not None                # shape


def test_term_scales_against_a_loop():
    L = synth.make_random_codes_layer(3, 256, M=2, seed=[6])
    a, B = tolerance.term_scales(L["x"], L["parent"], L["scales"], L["zeros"], 8, 3, 128)
    S = oracle.slice_codes(L["parent"], 8, 3).astype(float)
    x = L["x"].astype(float)
    s, z = L["scales"].astype(float), L["zeros"].astype(float)
    for m in range(2):
        for n in range(3):
            aa = bb = 0.0
            for k in range(256):
                g = k // 128
                aa += (x[m, k] * s[n, g] * (S[n, k] - z[n, g])) ** 2
                bb += s[n, g] * (abs(x[m, k]) * S[n, k] + z[n, g] * abs(x[m, k]))
            assert np.isclose(a[m, n], aa ** 0.5) and np.isclose(B[m, n], bb)
