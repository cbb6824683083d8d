"""GPU test of mq_linear_noalloc (the entry point for callers that cannot allocate): called through the C-ABI on
outputs and inputs that exist beforehand, compared with mq_linear on the same layer and with the oracle, on calls in a
row whose shapes differ (the static scratch array keeps the previous call's contents, laid out for another shape)."""
import ctypes

import numpy as np
import pytest

import paper_2602_03537_amd as mq
from paper_2602_03537_amd import synth
from gpu_util import DEV, check_layer, dev

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _noalloc(x, lay, N, K, r, y):
    """straight through ctypes: nothing but pointers and sizes crosses"""
    st = mq.lib().mq_linear_noalloc(x.data_ptr(), x.shape[0], lay["packed_W"].data_ptr(), lay["scales_t"].data_ptr(),
                                    lay["zeros_t"].data_ptr(), N, K, r, 128, y.data_ptr(),
                                    ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert st == 0, mq.STATUS.get(st, st)


# first a big input, then smaller ones: (N, K, M, r).  4096 x 11008 splits K over several workgroups, 8192 x 28672
# runs the persistent schedule with hand-over between shares, M = 8 and 16 the matrix-core path with prepared activations
SEQUENCES = [
    [(4096, 11008, 1, 3), (512, 512, 1, 4)],
    [(8192, 28672, 2, 4), (200, 1280, 2, 2), (1, 128, 1, 8)],
    [(4096, 4096, 16, 6), (130, 384, 8, 3), (4096, 4096, 4, 2)],
]


@pytest.mark.parametrize("seq", SEQUENCES, ids=["gemv", "stream_k", "mfma"])
def test_noalloc_matches_mq_linear_on_calls_in_a_row(seq):
    for (N, K, M, r) in seq:
        print(f"noalloc N={N} K={K} M={M} r={r}", flush=True)
        L = synth.make_layer(N, K, M=M, seed=[110, N, K, M])
        lay = mq.prepare_layer(dev(L["parent"]), dev(L["scales"]), dev(L["zeros"]), r)
        x = dev(L["x"])
        want = mq.mq_linear(x, lay["packed_W"], lay["scales_t"], lay["zeros_t"], N, K, r, 128, mq.new_workspace(M, N, K, r))
        buf = torch.full((M * N + 128,), float("nan"), dtype=torch.float16, device=DEV)
        y = buf[64:64 + M * N].view(M, N)
        for rep in range(2):
            y.fill_(float("nan"))
            torch.cuda.synchronize()
            free0 = torch.cuda.mem_get_info()[0]
            _noalloc(x, lay, N, K, r, y)
            torch.cuda.synchronize()
            assert rep == 0 or torch.cuda.mem_get_info()[0] == free0      # no device memory came or went
            assert torch.isnan(buf[:64]).all() and torch.isnan(buf[64 + M * N:]).all()
            # same kernels, possibly other split-K shares: equal to fp32 summation order, i.e. within an fp16 ulp or so
            assert torch.allclose(y.float(), want.float(), rtol=2e-3, atol=1e-4), (N, K, M, r, rep)
            if N * K <= 4096 * 11008:
                check_layer(y, L, r, f"noalloc {N}x{K} M={M} r={r} rep {rep}")
    # a sampled-row oracle check of the largest case
    N, K, M, r = seq[0]
    if N * K > 4096 * 11008:
        import oracle
        from gpu_util import check_y
        L = synth.make_layer(N, K, M=M, seed=[110, N, K, M])
        lay = mq.prepare_layer(dev(L["parent"]), dev(L["scales"]), dev(L["zeros"]), r)
        y = torch.empty((M, N), dtype=torch.float16, device=DEV)
        _noalloc(dev(L["x"]), lay, N, K, r, y)
        rows = np.unique(np.random.default_rng(111).integers(0, N, 96))
        ref = oracle.linear_rows(L["x"], L["parent"], L["scales"], L["zeros"], 8, r, 128, rows)
        check_y(y[:, torch.from_numpy(rows).to(DEV)], ref, "noalloc sampled rows")


def test_noalloc_refuses_what_does_not_fit():
    L = synth.make_layer(64, 128, M=32, seed=[112])
    lay = mq.prepare_layer(dev(L["parent"]), dev(L["scales"]), dev(L["zeros"]), 4)
    y = torch.empty((32, 64), dtype=torch.float16, device=DEV)
    with pytest.raises(mq.MqError) as e:
        mq.mq_linear_noalloc(dev(L["x"]), lay["packed_W"], lay["scales_t"], lay["zeros_t"], 64, 128, 4, 128, y)
    assert e.value.status == 8                                 # M > 16: unsupported
    # a shape whose counters and prepared activations leave no room for the partial sums: refused before any launch
    st = mq.lib().mq_linear_noalloc(0x10000, 16, 0x10000, 0x10000, 0x10000, 64, 128 * 4096, 6, 128, 0x10000, None)
    assert st == 6
    with pytest.raises(mq.MqError):
        mq.mq_linear_noalloc(dev(L["x"])[:1], lay["packed_W"], lay["scales_t"], lay["zeros_t"], 64, 128, 5, 128, y)


def test_noalloc_under_graph_capture():
    N, K, M, r = 4096, 4096, 1, 4
    L = synth.make_layer(N, K, M=M, seed=[113])
    lay = mq.prepare_layer(dev(L["parent"]), dev(L["scales"]), dev(L["zeros"]), r)
    x = dev(L["x"])
    y = torch.empty((M, N), dtype=torch.float16, device=DEV)
    _noalloc(x, lay, N, K, r, y)                               # first call on the device, outside capture
    torch.cuda.synchronize()
    want = y.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            mq.mq_linear_noalloc(x, lay["packed_W"], lay["scales_t"], lay["zeros_t"], N, K, r, 128, y, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        y.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, want), rep
