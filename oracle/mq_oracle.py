"""Plain CPU oracle: MSB slicing, group dequantisation, linear layer.

TEST INFRASTRUCTURE ONLY (see package docstring).  Written from the paper's
definitions, in the paper's order, with no blocking, fusion or reordering:

  1. slice   -- Eq. 1 (Section 2, "Matryoshka Quantization"):
                S(q^c, r) = clamp(round(q^c / 2^(c-r)), 0, 2^r - 1) * 2^(c-r)
  2. dequant -- Section 3.2, item 1: scale and zero-offset are those of the
                master width c and are reused unchanged for every r; weights
                are grouped contiguously along the input dimension.
                w = scale * (S - zero)
  3. linear  -- Section 4: X and the de-quantised W_D are fp16 values, the
                product is accumulated in a wider type.  torch.nn.Linear
                convention: W is [N_out, K_in], y = x @ W^T.

Readings taken where the paper is silent:
  * rounding mode of Eq. 1: round half up.  Section 3.1 ("Slicing") says the
    r-th bit is decided by the (r+1)-th bit alone and that values are pushed
    into the higher bucket, which is what adding half and flooring does.
    A half-to-even reading would change the codes q = (2j+1) * 2^(c-r-1) with
    j even.
  * r == c: Eq. 1 divides by 1, i.e. the identity.
  * dequantisation formula is the standard affine one; the zero-offset lives
    in c-bit units and is not rescaled with r.
  * the arithmetic here is float64 throughout (inputs are fp16/uint8 values,
    so every product is exact and only the summation rounds, at 2^-53).

Pins: tests/test_oracle_pins.py (exhaustive enumeration of Eq. 1 against exact
rational arithmetic, hand-evaluated values of Eq. 1 in tests/golden/, the
invariants Eq. 1 fixes, brute-force exact-rational linear layers on tiny
matrices, one-hot/closed-form cases).  Parity of the *accuracy* of a sliced
model against full-precision weights is not a property of this path: parity
unpinned, and not needed.
"""
from __future__ import annotations

import numpy as np

__all__ = ["slice_codes", "sliced_index", "dequant", "linear", "linear_rows",
           "linear_stack"]


def _check_widths(c: int, r: int) -> None:
    if not (1 <= c <= 8):
        raise ValueError(f"master width c={c} outside 1..8")
    if not (1 <= r <= c):
        raise ValueError(f"slice width r={r} outside 1..c={c}")


def sliced_index(q, c: int, r: int) -> np.ndarray:
    """r-bit integer t = clamp(round_half_up(q / 2^(c-r)), 0, 2^r - 1).

    This is the clamp(...) factor of Eq. 1 before the rescale by 2^(c-r).
    """
    _check_widths(c, r)
    q = np.asarray(q)
    if q.dtype != np.uint8:
        raise TypeError("parent codes must be uint8")
    if q.size and int(q.max()) > (1 << c) - 1:
        raise ValueError("parent code exceeds 2^c - 1")
    step = 1 << (c - r)                       # 2^(c-r)
    qi = q.astype(np.int64)
    # round half up of qi/step, in integers: floor((2*qi + step) / (2*step))
    t = (2 * qi + step) // (2 * step)
    t = np.clip(t, 0, (1 << r) - 1)
    return t.astype(np.uint8)


def slice_codes(q, c: int, r: int) -> np.ndarray:
    """Eq. 1: S(q^c, r), a c-bit code on the 2^(c-r) grid (uint8)."""
    t = sliced_index(q, c, r).astype(np.int64)
    return (t * (1 << (c - r))).astype(np.uint8)


def dequant(S, scales, zeros, group: int) -> np.ndarray:
    """w[n,k] = scales[n, k//group] * (S[n,k] - zeros[n, k//group]) in float64.

    S: uint8 [N, K];  scales, zeros: [N, K/group] (fp16 values).
    """
    S = np.asarray(S)
    N, K = S.shape
    if group <= 0 or K % group:
        raise ValueError("group must divide K")
    G = K // group
    s = np.asarray(scales, dtype=np.float64)
    z = np.asarray(zeros, dtype=np.float64)
    if s.shape != (N, G) or z.shape != (N, G):
        raise ValueError("scales/zeros must be [N, K/group]")
    Sg = S.astype(np.float64).reshape(N, G, group)
    w = s[:, :, None] * (Sg - z[:, :, None])
    return w.reshape(N, K)


def linear(x, parent, scales, zeros, c: int, r: int, group: int) -> np.ndarray:
    """y = x @ dequant(slice(parent))^T, float64 [M, N].

    x: [M, K] fp16 values; parent: uint8 [N, K] c-bit codes.
    """
    x = np.asarray(x, dtype=np.float64)
    if x.ndim != 2:
        raise ValueError("x must be [M, K]")
    S = slice_codes(parent, c, r)
    w = dequant(S, scales, zeros, group)
    if x.shape[1] != w.shape[1]:
        raise ValueError("x and W disagree on K")
    return x @ w.T


def linear_rows(x, parent, scales, zeros, c: int, r: int, group: int, rows) -> np.ndarray:
    """Same as linear() but only for the output features listed in rows: [M, len(rows)]."""
    rows = np.asarray(rows, dtype=np.int64)
    return linear(x, np.asarray(parent)[rows], np.asarray(scales)[rows],
                  np.asarray(zeros)[rows], c, r, group)


def linear_stack(layers, c: int, group: int):
    """Section 3.3 / 5.5: each layer carries its own bit-width r.

    layers: iterable of dicts with keys x, parent, scales, zeros, r.
    Layers are independent (each has its own input); returns a list of y.
    """
    return [linear(L["x"], L["parent"], L["scales"], L["zeros"], c, int(L["r"]), group)
            for L in layers]
