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

Also here: the MatGPTQ column loop (Algorithm 2 of the appendix), `matgptq_quantize`, whose
readings are listed in its docstring.

Pins: tests/test_quant_oracle_pins.py -- R = {c} is round-to-nearest; R = {r} is
the lowest code whose slice is the nearest r-bit grid point; R = {r, c} against
an interval-by-interval closed form; hand-evaluated cases in
tests/golden/alg1_hand_cases.txt; invariants (scaling of lambda, shift by the
coarsest step, monotonicity in w, optimality against every other candidate).
Column loop: an identity factor reduces it to Algorithm 1 per column; the telescoping identity
W - mean_r dequant(S(Q, r)) = E @ U; independence of the block size; R = {c} against an
independently written textbook GPTQ row solver; lower Hessian-weighted error than plain rounding.
"""
from __future__ import annotations

import numpy as np

from .mq_oracle import slice_codes

__all__ = ["quant_matgptq", "quant_errors", "matgptq_quantize"]


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


def matgptq_quantize(W, U, scales, zeros, c: int, widths, lam, group: int, block: int = 128,
                     dtype=np.float32):
    """Algorithm 2 of the paper's appendix ("Quantize W given inverse Hessian ..."), the MatGPTQ
    column loop, from the point where `U`, the upper-triangular Cholesky factor of H^-1 (the
    listing's "H^-1 <- Cholesky(H^-1)^T"), is given.

    For blocks of `block` columns, column by column j:
        Q[:, j]   = Algorithm 1 on the current W[:, j]
        E[:, j-i] = (1/|R|) * sum_{r in R} (W[:, j] - dequant(S(Q[:, j], r))) / U[j, j]
        W[:, j+1 : i+block] -= E[:, j-i] (outer) U[j, j+1 : i+block]        (update inside the block)
    then  W[:, i+block:] -= E @ U[i:i+block, i+block:]                      (update of the rest).

    Readings taken where the listing is silent, garbled or abbreviated:
      * the error is taken against the de-quantised slices (the listing prints S(Q, r) bare, which
        is in code units, not weight units);
      * scale and zero-offset per group are inputs, fixed before the loop ("static groups");
      * the in-block update starts at column j+1 (U is upper triangular and column j itself is
        not used again; the listing's index range starts at the block's first column);
      * precision and order, because the codes that follow depend on every rounding: `dtype`
        throughout, each operation rounded on its own; the error sum runs over r ascending as
        ((w - D_r1) + (w - D_r2)) + ..., then `/ |R|`, then `/ U[j, j]`; an update is
        w = w - (E * U[j, k]); the update of the rest is applied as the same rank-1 updates in
        ascending j (so the block size changes nothing, bit for bit); |R| counts lambda_r != 0.
      * the weights lambda_r enter Algorithm 1 only; the propagated error is the plain mean over R.

    W: [N, K];  U: [K, K];  returns (Q uint8 [N, K], E [N, K] with E[:, j] the propagated error).
    """
    W = np.array(W, dtype=dtype)                      # working copy, updated in place
    U = np.asarray(U).astype(dtype)
    N, K = W.shape
    if U.shape != (K, K):
        raise ValueError("U must be [K, K]")
    if K % block or block % 1:
        raise ValueError("block must divide K")
    pairs = sorted((int(r), float(l)) for r, l in zip(widths, lam) if float(l) != 0.0)
    if not pairs:
        raise ValueError("no target width")
    rs = [r for r, _ in pairs]
    ls = [l for _, l in pairs]
    s_full, z_full = _group_params(scales, zeros, N, K, group, dtype)
    Q = np.zeros((N, K), dtype=np.uint8)
    Eall = np.zeros((N, K), dtype=dtype)
    nR = dtype(len(rs))
    for i in range(0, K, block):
        E = np.zeros((N, block), dtype=dtype)
        for j in range(i, i + block):
            g = j // group
            sc = np.asarray(scales)[:, g:g + 1]
            zr = np.asarray(zeros)[:, g:g + 1]
            w = W[:, j]
            # Algorithm 1 on this column (a one-column matrix whose single group has the column's scale and zero)
            q = quant_matgptq(w[:, None], sc, zr, c, rs, ls, 1, dtype)[:, 0]
            Q[:, j] = q
            acc = None
            for r in rs:
                S = slice_codes(q, c, r).astype(dtype)
                t = S - z_full[:, j]
                D = s_full[:, j] * t
                d = w - D
                acc = d if acc is None else acc + d
            err = (acc / nR) / U[j, j]
            E[:, j - i] = err
            for k in range(j + 1, i + block):
                W[:, k] = W[:, k] - err * U[j, k]
        for jj in range(block):                        # E @ U[i:i+block, i+block:], one rank-1 term at a time
            W[:, i + block:] = W[:, i + block:] - E[:, jj:jj + 1] * U[i + jj:i + jj + 1, i + block:]
        Eall[:, i:i + block] = E
    return Q, Eall
