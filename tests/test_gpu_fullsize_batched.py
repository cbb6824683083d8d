"""GPU parity at full size for the batched regime (Section 4, the matrix-core kernel): both Llama-3-70B MLP shapes
at the batches where the wide kernel runs in its real launch shape (several chunks per pass, two passes at M = 256,
256 workgroups, long split-K hand-over chains on the down-projection), and a Llama-3-70B-shaped stack at M = 32, 64 and 96.
The oracle computes sampled output rows (rows are independent); all of y is checked to be finite."""
import numpy as np
import pytest

import oracle
import paper_2602_03537_amd as mq
from paper_2602_03537_amd import synth
from gpu_util import C, DEV, check_layer, check_y, dev

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("shape", [(28672, 8192), (8192, 28672)], ids=["up", "down"])
def test_llama3_70b_mlp_shapes_at_m64_m256_sampled_rows(shape):
    N, K = shape
    Mmax = 256
    L = synth.make_layer(N, K, M=Mmax, seed=[52, N, K])
    rng = np.random.default_rng([53, N])
    # first/last rows of row blocks and of the 256-row super-tiles, plus a random sample
    rows = np.unique(np.concatenate([[0, 63, 64, 255, 256, N - 257, N - 256, N - 1], rng.integers(0, N, 88)]))
    rt = torch.from_numpy(rows).to(DEV)
    p, s, z, x = dev(L["parent"]), dev(L["scales"]), dev(L["zeros"]), dev(L["x"])
    for r in (3, 4, 8):
        lay = mq.prepare_layer(p, s, z, r)
        for M in (64, 256):
            print(f"70B {shape} r={r} M={M}", flush=True)
            ws = mq.new_workspace(M, N, K, r)
            y = mq.mq_linear(x[:M], lay["packed_W"], lay["scales_t"], lay["zeros_t"], N, K, r, 128, ws)
            torch.cuda.synchronize()
            assert torch.isfinite(y).all()
            ref = oracle.linear_rows(L["x"][:M], L["parent"], L["scales"], L["zeros"], C, r, 128, rows)
            check_y(y[:, rt], ref, f"70B {shape} r={r} M={M}")
            y2 = mq.mq_linear(x[:M], lay["packed_W"], lay["scales_t"], lay["zeros_t"], N, K, r, 128, ws)
            torch.cuda.synchronize()
            assert torch.equal(y, y2)                      # fixed summation order: the same bits again
        del lay


def test_llama3_70b_down_projection_small_batches_sampled_rows():
    # the down-projection (224 groups: the longest split-K chains) on the vector-ALU and narrow matrix-core paths
    N, K = 8192, 28672
    L = synth.make_layer(N, K, M=16, seed=[54])
    rng = np.random.default_rng(55)
    rows = np.unique(np.concatenate([[0, 63, 64, N - 1], rng.integers(0, N, 124)]))
    rt = torch.from_numpy(rows).to(DEV)
    p, s, z = dev(L["parent"]), dev(L["scales"]), dev(L["zeros"])
    for r in (3, 4, 8):
        lay = mq.prepare_layer(p, s, z, r)
        for M in (1, 4, 16):
            print(f"70B down r={r} M={M}", flush=True)
            ws = mq.new_workspace(M, N, K, r)
            y = mq.mq_linear(dev(L["x"][:M]), lay["packed_W"], lay["scales_t"], lay["zeros_t"], N, K, r, 128, ws)
            torch.cuda.synchronize()
            assert torch.isfinite(y).all()
            ref = oracle.linear_rows(L["x"][:M], L["parent"], L["scales"], L["zeros"], C, r, 128, rows)
            sub = dict(x=L["x"][:M], parent=L["parent"][rows], scales=L["scales"][rows], zeros=L["zeros"][rows])
            check_y(y[:, rt], ref, f"70B down r={r} M={M}", sub, r)


@pytest.mark.parametrize("M", [32, 64, 96])
def test_llama3_70b_shaped_stack_three_blocks(M):
    # 21 linears at the real shapes, widths by seed, one persistent launch on the wide matrix-core path: one and two
    # chunks per pass (two workgroups per compute unit, accumulators in vector registers) and three (one per unit)
    n_blocks = 3
    shapes = synth.stack_shapes(synth.LLAMA3_70B_BLOCK, n_blocks)
    widths, _ = synth.draw_bitwidths([N * K for (_, _, N, K) in shapes], 4.0, seed=6, tol=0.3)
    gen, layers = [], []
    for i, ((_, _, N, K), r) in enumerate(zip(shapes, widths)):
        G = synth.make_layer_device(N, K, M, seed=600000 + i, device=DEV)
        lay = mq.prepare_layer(G["parent"], G["scales"], G["zeros"], int(r))
        lay.update(x=G["x"], y=torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV))
        gen.append(G)
        layers.append(lay)
    plan = mq.mq_stack_plan(layers, M)
    mq.mq_linear_stack(plan)
    torch.cuda.synchronize()
    rng = np.random.default_rng(56)
    for i, (G, lay) in enumerate(zip(gen, layers)):
        assert torch.isfinite(lay["y"]).all(), i
        N = lay["N"]
        rows = np.unique(np.concatenate([[0, N - 1], rng.integers(0, N, 30)]))
        rt = torch.from_numpy(rows).to(DEV)
        sub = dict(x=G["x"].cpu().numpy(), parent=G["parent"][rt].cpu().numpy(), scales=G["scales"][rt].cpu().numpy(),
                   zeros=G["zeros"][rt].cpu().numpy())
        check_layer(lay["y"][:, rt], sub, lay["r"], f"70B stack M={M} linear {i} r={lay['r']}")
    first = [lay["y"].clone() for lay in layers]
    mq.mq_linear_stack(plan)
    torch.cuda.synchronize()
    assert all(torch.equal(a, lay["y"]) for a, lay in zip(first, layers))
