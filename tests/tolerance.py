"""The bar a computed y is held to, in one place.

Target: max-abs error <= 2e-2 and relative-L2 <= 1e-3 against the float64 oracle (fp16
activations, fp32 accumulation, fp16 output).

Relative L2 is a statement about a vector whose norm is representative of the terms it sums:
with a[m, n] = sqrt(sum_k (x[m, k] * w[n, k])^2), the root-sum-square of the terms (the standard
deviation of y[m, n] if the terms' signs were random), an output of 64 or more elements has
||y|| within a small factor of ||a||, and the relative-L2 bar is applied literally.

An output of fewer than 64 elements (a one-row layer) can cancel to a value arbitrarily close to
zero, while the error of an fp32 accumulation scales with the terms that were added, not with what
is left of them.  The relative bar then has no meaning of its own, and such an output is held to
  (i)  ||y - y_ref|| <= 1e-3 * max(||y_ref||, ||a||)   -- the absolute budget a representative
       output of the same terms is given by the target, and
  (ii) per element |y - y_ref| <= 2^-10 |y_ref| + 2^-24 + 8 * 2^-24 * B  (+ 2^-9 * a  when the
       weights are rounded to fp16 before the product, i.e. on the wide matrix-core path):
       fp16 rounding of the output (half an ulp is 2^-11 relative; 2^-24 is half the spacing of
       fp16 subnormals) plus a few fp32 unit round-offs of B, the sum of the MAGNITUDES the
       factored form  s_g * (sum_k x_k S_k - z_g * sum_k x_k)  adds up per group:
       B[m, n] = sum_g s_g * (sum_{k in g} |x_k| S_k + z_g * sum_{k in g} |x_k|).
(ii) is the tighter of the two by an order of magnitude when y_ref is small; (i) ties the reading
to the target's own number.
"""
import numpy as np

import oracle

MAX_ABS = 2e-2
REL_L2 = 1e-3
SHORT = 64          # outputs with fewer elements are "short"
U32 = 2.0 ** -24    # fp32 unit round-off


def term_scales(x, parent, scales, zeros, c, r, group):
    """(a, B) of the module docstring, float64 [M, N] each, from the oracle's own slice and de-quantisation."""
    x = np.asarray(x, dtype=np.float64)
    S = oracle.slice_codes(parent, c, r)
    w = oracle.dequant(S, scales, zeros, group)
    a = np.sqrt((x * x) @ (w * w).T)
    N, K = S.shape
    G = K // group
    s = np.asarray(scales, dtype=np.float64)
    z = np.asarray(zeros, dtype=np.float64)
    ax = np.abs(x).reshape(x.shape[0], G, group)
    Sg = S.astype(np.float64).reshape(N, G, group)
    B = np.einsum("mgk,ngk,ng->mn", ax, Sg, np.abs(s)) + np.einsum("mg,ng->mn", ax.sum(2), np.abs(s) * np.abs(z))
    return a, B


def errors(y, y_ref):
    err = float(np.abs(y - y_ref).max()) if y.size else 0.0
    rel = float(np.linalg.norm(y - y_ref) / max(np.linalg.norm(y_ref), 1e-30)) if y.size else 0.0
    return err, rel


def failure(y, y_ref, scales=None, fp16_weights=False):
    """None if y meets the bar, else a string saying what it missed.  y, y_ref: float64 arrays of one shape.
    scales: (a, B) from term_scales, required for short outputs."""
    if y.shape != y_ref.shape:
        return f"shape {y.shape} != {y_ref.shape}"
    if not np.all(np.isfinite(y)):
        return "non-finite output"
    if y.size == 0:
        return None
    err, rel = errors(y, y_ref)
    if err > MAX_ABS:
        return f"max-abs {err:.3e} > {MAX_ABS}"
    if y.size >= SHORT:
        return None if rel <= REL_L2 else f"rel-L2 {rel:.3e} > {REL_L2}"
    if scales is None:
        return "short output: term scales are needed to judge it"
    a, B = scales
    budget = REL_L2 * max(np.linalg.norm(y_ref), np.linalg.norm(a))
    if np.linalg.norm(y - y_ref) > budget:
        return f"short output: ||y - y_ref|| {np.linalg.norm(y - y_ref):.3e} > {budget:.3e}"
    bound = 2.0 ** -10 * np.abs(y_ref) + U32 + 8 * U32 * B + (2.0 ** -9 * a if fp16_weights else 0.0)
    over = np.abs(y - y_ref) - bound
    if over.max() > 0:
        i = np.unravel_index(np.argmax(over), over.shape)
        return f"short output: |y - y_ref| {abs(y[i] - y_ref[i]):.3e} > {bound[i]:.3e} at {i} (y_ref {y_ref[i]:.3e})"
    return None
