"""Helpers shared by the GPU parity tests: device transfer, the tolerance check, one layer end to end."""
import numpy as np
import pytest

import oracle
import paper_2602_03537_amd as mq
from paper_2602_03537_amd import synth
import tolerance

torch = pytest.importorskip("torch")

WIDTHS = (2, 3, 4, 6, 8)
C = 8
DEV = "cuda"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def check_y(y_gpu, y_ref, what="", layer=None, r=None):
    """y against the oracle's y_ref at the bar of tests/tolerance.py.  An output of fewer than 64 elements needs
    `layer` (host dict with x, parent, scales, zeros for exactly the rows and batch rows of y_ref) and its width."""
    yg = y_gpu.detach().cpu().numpy().astype(np.float64)
    scales = None
    if y_ref.size < tolerance.SHORT and layer is not None:
        scales = tolerance.term_scales(layer["x"][:yg.shape[0]], layer["parent"], layer["scales"], layer["zeros"], C,
                                       int(r), 128)
    msg = tolerance.failure(yg, y_ref, scales, fp16_weights=yg.shape[0] > 16)
    assert msg is None, f"{what}: {msg}"


def check_layer(y_gpu, L, r, what=""):
    """The whole output of host layer L at width r (batch = rows of y_gpu)."""
    M = y_gpu.shape[0]
    ref = oracle.linear(L["x"][:M], L["parent"], L["scales"], L["zeros"], C, int(r), 128)
    check_y(y_gpu, ref, what, layer=L, r=r)


def run_linear(L, r, M=None):
    """host layer dict -> y (device tensor) through slice, pack, meta, linear."""
    N, K = L["parent"].shape
    lay = mq.prepare_layer(dev(L["parent"]), dev(L["scales"]), dev(L["zeros"]), r)
    x = dev(L["x"] if M is None else L["x"][:M])
    ws = mq.new_workspace(x.shape[0], N, K, r)
    y = mq.mq_linear(x, lay["packed_W"], lay["scales_t"], lay["zeros_t"], N, K, r, 128, ws)
    torch.cuda.synchronize()
    return y
