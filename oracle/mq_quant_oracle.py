"""Plain CPU oracle of the cross-bit-width quantiser (Algorithm 1 of the paper,
"Generate Q^c given weight matrix W, target bit-widths R, and weights lambda_R").

TEST INFRASTRUCTURE ONLY (see package docstring).  The steps are the
algorithm's, in its order, on whole arrays:

  1. candidates 0 .. Q_max = 2^c - 1 along a new first axis (initQ);
  2. E = 0;  for every target width r:
         E = E + lambda_r * (W - dequant(S(candidates, r)))^2
     with S = Eq. 1 (Section 2) and dequant = scale * (S - zero) using the scale
     and zero-offset of the master width c for every r (Section 3.2, item 1);
  3. per weight, the candidate with the smallest E.

Readings taken where the paper is silent:
  * precision: an argmin is decided in floating point, so the precision and the
    order of the operations are part of the definition.  Here: IEEE binary32,
    every operation rounded on its own (no fused multiply-add), in the order
        t = S - zero;  D = scale * t;  e = W - D;  p = e * e;  E = E + lambda_r * p
    `dtype=np.float64` runs the same steps in binary64 (used by the pins, on
    inputs whose minima are well separated).
  * order of the sum over R: ascending r (the paper writes "for r in R" over a set).
  * ties: the smallest candidate (first minimum along the candidate axis).
  * lambda_r == 0 is the same as r not in R (adding +0 changes nothing).

Pins: tests/test_quant_oracle_pins.py -- R = {c} is round-to-nearest; R = {r} is
the lowest code whose slice is the nearest r-bit grid point; R = {r, c} against
an interval-by-interval closed form; hand-evaluated cases in
tests/golden/alg1_hand_cases.txt; invariants (scaling of lambda, shift by the
coarsest step, monotonicity in w, optimality against every other candidate).
"""
from __future__ import annotations

import numpy as np

from .mq_oracle import slice_codes

__all__ = ["quant_matgptq", "quant_errors"]


def _group_params(scales, zeros, N, K, group, dtype):
    if group <= 0 or K % group:
        raise ValueError("group must divide K")
    G = K // group
    s = np.asarray(scales).astype(dtype)
    z = np.asarray(zeros).astype(dtype)
    if s.shape != (N, G) or z.shape != (N, G):
        raise ValueError("scales/zeros must be [N, K/group]")
    return np.repeat(s, group, axis=1), np.repeat(z, group, axis=1)


def quant_errors(W, scales, zeros, c: int, widths, lam, group: int, dtype=np.float32) -> np.ndarray:
    """E[q, n, k] of Algorithm 1 for every candidate q (steps 1 and 2 above)."""
    W = np.asarray(W)
    if W.ndim != 2:
        raise ValueError("W must be [N, K]")
    widths = [int(r) for r in widths]
    lam = [float(x) for x in lam]
    if len(widths) != len(lam) or not widths or len(set(widths)) != len(widths):
        raise ValueError("one lambda per distinct width")
    N, K = W.shape
    Wd = W.astype(dtype)
    s, z = _group_params(scales, zeros, N, K, group, dtype)
    cand = np.arange(1 << c, dtype=np.uint8)                      # initQ
    E = np.zeros((1 << c, N, K), dtype=dtype)
    for r, l in sorted(zip(widths, lam)):
        S = slice_codes(cand, c, r).astype(dtype)                 # Eq. 1 on every candidate
        t = S[:, None, None] - z[None, :, :]
        D = s[None, :, :] * t                                     # dequant
        e = Wd[None, :, :] - D
        p = e * e
        E = E + dtype(l) * p
    return E


def quant_matgptq(W, scales, zeros, c: int, widths, lam, group: int, dtype=np.float32) -> np.ndarray:
    """Algorithm 1: uint8 [N, K] parent codes Q^c minimising the lambda-weighted
    squared error over the target widths.  Rows are processed in slabs only to
    bound memory (each weight is independent of every other)."""
    W = np.asarray(W)
    N, K = W.shape
    out = np.empty((N, K), dtype=np.uint8)
    rows = max(1, (1 << 22) // max(K, 1))
    sc, zr = np.asarray(scales), np.asarray(zeros)
    for r0 in range(0, N, rows):
        r1 = min(N, r0 + rows)
        E = quant_errors(W[r0:r1], sc[r0:r1], zr[r0:r1], c, widths, lam, group, dtype)
        out[r0:r1] = np.argmin(E, axis=0).astype(np.uint8)        # first minimum = smallest candidate
    return out
