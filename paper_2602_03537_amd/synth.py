"""Seeded synthetic inputs: parent checkpoints, activations, per-layer bit-widths.

This module only *creates inputs* (an 8-bit parent by per-group asymmetric
min-max round-to-nearest, Gaussian activations, a bit-width vector).  It holds
none of the method's arithmetic (no slicing, no packing, no dequantisation, no
matmul) so that the CPU oracle and the HIP path can both be fed from it without
sharing any code of their own.

Stand-ins: the paper runs on Llama/Qwen/Phi checkpoints quantised with MatGPTQ
and on bit-width vectors found by its evolutionary search (Sections 3.3, 5.5);
neither exists here, so layers have the Llama shapes with Gaussian weights and
the bit-width vector is drawn by seed to a parameter-weighted mean.
"""
from __future__ import annotations

import numpy as np

GROUP = 128
C_BITS = 8
WIDTHS = (2, 3, 4, 6, 8)

# (name, N_out, K_in) of one decoder block's linears
LLAMA2_7B_BLOCK = (
    ("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096), ("o", 4096, 4096),
    ("gate", 11008, 4096), ("up", 11008, 4096), ("down", 4096, 11008),
)
LLAMA3_70B_BLOCK = (
    ("q", 8192, 8192), ("k", 1024, 8192), ("v", 1024, 8192), ("o", 8192, 8192),
    ("gate", 28672, 8192), ("up", 28672, 8192), ("down", 8192, 28672),
)
LLAMA2_7B_LAYERS = 32
LLAMA3_70B_LAYERS = 80


def _rng(seed):
    return np.random.default_rng(seed)


def make_weights(N: int, K: int, seed, std: float = 0.02) -> np.ndarray:
    return (_rng(seed).standard_normal((N, K), dtype=np.float32) * np.float32(std))


def quantize_parent(W: np.ndarray, group: int = GROUP):
    """Per-group asymmetric min-max RTN to 8-bit codes (input creation only).

    Returns (codes uint8 [N,K], scales fp16 [N,G], zeros fp16 [N,G]).
    """
    N, K = W.shape
    assert K % group == 0
    G = K // group
    Wg = W.reshape(N, G, group).astype(np.float32)
    lo = Wg.min(axis=2)
    hi = Wg.max(axis=2)
    s = ((hi - lo) / np.float32(255.0)).astype(np.float16)
    s = np.where((hi == lo) | (s == 0), np.float16(1.0), s).astype(np.float16)
    s32 = s.astype(np.float32)
    z = np.clip(np.rint(-lo / s32), 0, 255).astype(np.float16)
    q = np.clip(np.rint(Wg / s32[:, :, None]) + z.astype(np.float32)[:, :, None], 0, 255)
    return q.astype(np.uint8).reshape(N, K), s, z


def make_x(M: int, K: int, seed) -> np.ndarray:
    return _rng(seed).standard_normal((M, K), dtype=np.float32).astype(np.float16)


def make_layer(N: int, K: int, M: int = 1, seed=0, group: int = GROUP) -> dict:
    """One linear layer's inputs: x, parent codes, scales, zeros (numpy, host)."""
    ss = np.random.SeedSequence(seed)
    sw, sx = ss.spawn(2)
    W = make_weights(N, K, sw)
    parent, scales, zeros = quantize_parent(W, group)
    x = make_x(M, K, sx)
    return {"x": x, "parent": parent, "scales": scales, "zeros": zeros,
            "N": N, "K": K, "M": M, "group": group}


def make_random_codes_layer(N: int, K: int, M: int = 1, seed=0, group: int = GROUP) -> dict:
    """Uniform random codes / scales / fractional zeros: an adversarial input
    that does not come from a quantiser (exercises every code value)."""
    rng = _rng(seed)
    G = K // group
    parent = rng.integers(0, 256, size=(N, K), dtype=np.uint8)
    scales = (rng.uniform(1e-4, 2e-3, size=(N, G))).astype(np.float16)
    zeros = (rng.uniform(0.0, 255.0, size=(N, G))).astype(np.float16)
    x = rng.standard_normal((M, K), dtype=np.float32).astype(np.float16)
    return {"x": x, "parent": parent, "scales": scales, "zeros": zeros,
            "N": N, "K": K, "M": M, "group": group}


_P_FOR_TARGET = {
    3.5: (0.27, 0.35, 0.23, 0.10, 0.05),
    4.0: (0.15, 0.30, 0.30, 0.15, 0.10),
}


def draw_bitwidths(sizes, target_mean: float, seed: int = 0, tol: float = 0.02):
    """One width from WIDTHS per linear, parameter-weighted mean within tol of
    target_mean.  Draw i.i.d., then move seeded-random linears one level toward
    the target until the mean fits.  Returns (widths int array, achieved mean)."""
    sizes = np.asarray(sizes, dtype=np.float64)
    rng = _rng([seed, 0xB175])
    p = _P_FOR_TARGET.get(float(target_mean))
    if p is None:
        p = (0.2,) * 5
    idx = rng.choice(len(WIDTHS), size=len(sizes), p=p)
    widths = np.array(WIDTHS)

    def mean():
        return float((widths[idx] * sizes).sum() / sizes.sum())

    for _ in range(100000):
        m = mean()
        if abs(m - target_mean) <= tol:
            break
        j = int(rng.integers(len(sizes)))
        if m > target_mean and idx[j] > 0:
            idx[j] -= 1
        elif m < target_mean and idx[j] < len(WIDTHS) - 1:
            idx[j] += 1
    return widths[idx].astype(np.int32), mean()


def stack_shapes(block, n_layers: int):
    """[(layer, name, N, K)] for a decoder stack."""
    return [(l, name, N, K) for l in range(n_layers) for (name, N, K) in block]


# ---------------------------------------------------------------- on-device generation
def make_layer_device(N: int, K: int, M: int = 1, seed: int = 0, device="cuda", group: int = GROUP,
                      want_x: bool = True) -> dict:
    """Same recipe as make_layer but generated on the GPU with a seeded torch.Generator (for
    stacks whose 8-bit parent does not fit in host memory).  Input creation only: plain
    torch ops, no slicing / packing / de-quantisation / matmul of the method."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    G = K // group
    parent = torch.empty((N, K), dtype=torch.uint8, device=device)
    scales = torch.empty((N, G), dtype=torch.float16, device=device)
    zeros = torch.empty((N, G), dtype=torch.float16, device=device)
    rows = max(1, min(N, (1 << 26) // K))          # <= 256 MB of fp32 at a time
    for r0 in range(0, N, rows):
        r1 = min(N, r0 + rows)
        W = torch.randn((r1 - r0, G, group), generator=g, device=device, dtype=torch.float32) * 0.02
        lo = W.amin(dim=2)
        hi = W.amax(dim=2)
        s = ((hi - lo) / 255.0).to(torch.float16)
        s = torch.where((hi == lo) | (s == 0), torch.ones_like(s), s)
        s32 = s.float()
        z = torch.clamp(torch.round(-lo / s32), 0, 255).to(torch.float16)
        q = torch.clamp(torch.round(W / s32[:, :, None]) + z.float()[:, :, None], 0, 255)
        parent[r0:r1] = q.to(torch.uint8).reshape(r1 - r0, K)
        scales[r0:r1] = s
        zeros[r0:r1] = z
        del W, q
    out = {"parent": parent, "scales": scales, "zeros": zeros, "N": N, "K": K, "M": M, "group": group}
    if want_x:
        out["x"] = torch.randn((M, K), generator=g, device=device, dtype=torch.float32).to(torch.float16)
    return out
