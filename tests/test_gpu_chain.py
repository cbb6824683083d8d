"""GPU parity tests of chained small stacks (MQ_X_AFTER_EARLIER): layers of ONE launch that read what earlier
layers of the same launch write.  Every layer is checked on its own against the CPU oracle, which is given the
activations the GPU actually produced for it (the fp16 output of the earlier layers), so that the bar of a single
layer applies to each link of the chain and errors do not pile up in the comparison."""
import numpy as np
import pytest

import oracle
import paper_2602_03537_amd as mq
from paper_2602_03537_amd import synth
from gpu_util import C, DEV, check_y, dev

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _prepared(N, K, r, seed, from_parent=False):
    L = synth.make_layer(N, K, M=1, seed=seed)
    if from_parent:
        lay = mq.prepare_layer(dev(L["parent"]), dev(L["scales"]), dev(L["zeros"]), 8)
        lay.update(r=r, from_parent=1)
    else:
        lay = mq.prepare_layer(dev(L["parent"]), dev(L["scales"]), dev(L["zeros"]), r)
    return L, lay


def _check_link(L, lay, r, x_gpu, what):
    xin = x_gpu.detach().cpu().numpy()                      # fp16, as the layer read it
    ref = oracle.linear(xin, L["parent"], L["scales"], L["zeros"], C, r, 128)
    check_y(lay["y"], ref, what, layer=dict(L, x=xin), r=r)


@pytest.mark.parametrize("M", [1, 2, 3])
@pytest.mark.parametrize("from_parent", [False, True])
def test_chain_of_three_layers_in_one_launch(M, from_parent):
    # x -> y0 -> y1 -> y2: widths and K-slice counts differ per link; ragged last layer
    shapes_r = [(384, 512, 4), (640, 384, 2), (200, 640, 6)]
    x0 = dev(synth.make_x(M, 512, [201, M]))
    host, layers, xs = [], [], [x0]
    for i, (N, K, r) in enumerate(shapes_r):
        L, lay = _prepared(N, K, r, [201, M, i], from_parent)
        y = torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV)
        lay.update(x=xs[-1], y=y, flags=mq.MQ_X_AFTER_EARLIER if i else 0)
        xs.append(y)
        host.append(L)
        layers.append(lay)
    plan = mq.mq_stack_plan(layers, M)
    for rep in range(3):                                    # the stage counters zero themselves
        for lay in layers:
            lay["y"].fill_(float("nan"))
        mq.mq_linear_stack(plan)
        torch.cuda.synchronize()
        for i, (L, lay) in enumerate(zip(host, layers)):
            assert torch.isfinite(lay["y"]).all(), (rep, i)
            _check_link(L, lay, shapes_r[i][2], xs[i], f"chain M={M} parent={from_parent} rep {rep} link {i}")


def test_chain_equals_the_same_layers_launched_one_by_one():
    # the waits change when a layer runs, not what it computes: bit-identical to three launches in stream order
    M = 2
    shapes_r = [(512, 256, 3), (256, 512, 8), (384, 256, 4)]
    x0 = dev(synth.make_x(M, 256, [202]))
    layers, xs = [], [x0]
    for i, (N, K, r) in enumerate(shapes_r):
        _, lay = _prepared(N, K, r, [202, i])
        y = torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV)
        lay.update(x=xs[-1], y=y, flags=mq.MQ_X_AFTER_EARLIER if i else 0)
        xs.append(y)
        layers.append(lay)
    mq.mq_linear_stack(mq.mq_stack_plan(layers, M))
    torch.cuda.synchronize()
    chained = [lay["y"].clone() for lay in layers]
    for lay in layers:
        lay["y"].fill_(float("nan"))
    for lay in layers:                                      # one stack of one layer each, no flag
        mq.mq_linear_stack(mq.mq_stack_plan([dict(lay, flags=0)], M))
    torch.cuda.synchronize()
    for i, (lay, want) in enumerate(zip(layers, chained)):
        assert torch.equal(lay["y"], want), i


def test_chain_with_two_outputs_side_by_side_as_one_input_and_a_layer_that_does_not_wait():
    # stage 0: A and B write the two halves of one buffer; stage 1: Cc reads the whole buffer (waits for both), D reads
    # the caller's x and does not wait; stage 2: E reads Cc's output.  M = 1, where [y_A | y_B] is a plain row.
    x0 = dev(synth.make_x(1, 512, [203]))
    buf = torch.full((1, 640), float("nan"), dtype=torch.float16, device=DEV)
    spec = [("A", 256, 512, 4, x0, buf[:, :256], 0), ("B", 384, 512, 2, x0, buf[:, 256:], 0),
            ("Cc", 384, 640, 3, buf, None, mq.MQ_X_AFTER_EARLIER), ("D", 130, 512, 8, x0, None, 0),
            ("E", 70, 384, 6, None, None, mq.MQ_X_AFTER_EARLIER)]
    host, layers = [], []
    for i, (name, N, K, r, x, y, flags) in enumerate(spec):
        L, lay = _prepared(N, K, r, [203, i])
        if y is None:
            y = torch.full((1, N), float("nan"), dtype=torch.float16, device=DEV)
        if x is None:
            x = layers[2]["y"]
        lay.update(x=x, y=y, flags=flags)
        host.append(L)
        layers.append(lay)
    plan = mq.mq_stack_plan(layers, 1)
    for rep in range(2):
        buf.fill_(float("nan"))
        for lay in layers[2:]:
            lay["y"].fill_(float("nan"))
        mq.mq_linear_stack(plan)
        torch.cuda.synchronize()
        for i, (L, lay) in enumerate(zip(host, layers)):
            _check_link(L, lay, spec[i][3], lay["x"], f"fan-in rep {rep} layer {spec[i][0]}")


def test_chain_at_llama2_7b_width_sampled_rows_and_inside_a_hip_graph():
    # three 4096 x 4096 links at M = 1 (6144 tiles, the launch shape shrunk to what the device holds at one time),
    # eager twice, then recorded into a HIP graph and replayed: every replay gives the eager bits
    M, widths = 1, (3, 4, 8)
    x0 = dev(synth.make_x(M, 4096, [204]))
    gens, layers, xs = [], [], [x0]
    for i, r in enumerate(widths):
        G = synth.make_layer_device(4096, 4096, M, seed=2040 + i, device=DEV)
        lay = mq.prepare_layer(G["parent"], G["scales"], G["zeros"], r)
        y = torch.full((M, 4096), float("nan"), dtype=torch.float16, device=DEV)
        lay.update(x=xs[-1], y=y, flags=mq.MQ_X_AFTER_EARLIER if i else 0)
        xs.append(y)
        gens.append(G)
        layers.append(lay)
    plan = mq.mq_stack_plan(layers, M)
    rows = np.unique(np.concatenate([[0, 63, 64, 4095], np.random.default_rng(204).integers(0, 4096, 124)]))
    ridx = torch.from_numpy(rows).to(DEV)
    for rep in range(2):
        for lay in layers:
            lay["y"].fill_(float("nan"))
        mq.mq_linear_stack(plan)
        torch.cuda.synchronize()
        for i, (G, lay) in enumerate(zip(gens, layers)):
            assert torch.isfinite(lay["y"]).all(), (rep, i)
            ref = oracle.linear(xs[i].cpu().numpy(), G["parent"][ridx].cpu().numpy(), G["scales"][ridx].cpu().numpy(),
                                G["zeros"][ridx].cpu().numpy(), C, widths[i], 128)
            check_y(lay["y"][:, ridx], ref, f"7B-width chain rep {rep} link {i}")
    want = [lay["y"].clone() for lay in layers]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            mq.mq_linear_stack(plan, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        for lay in layers:
            lay["y"].fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for i, (lay, w) in enumerate(zip(layers, want)):
            assert torch.equal(lay["y"], w), (rep, i)


def test_chain_is_refused_where_no_launch_can_wait():
    L, lay = _prepared(256, 256, 4, [205])
    x = dev(synth.make_x(8, 256, [205]))
    mk = lambda M, flags: dict(lay, x=x[:M], y=torch.empty((M, 256), dtype=torch.float16, device=DEV), flags=flags)  # noqa: E731
    with pytest.raises(mq.MqError):                          # the first layer has nothing to wait for
        mq.mq_stack_plan([mk(1, mq.MQ_X_AFTER_EARLIER), mk(1, 0)], 1)
    with pytest.raises(mq.MqError):                          # matrix-core batches run as a persistent launch
        mq.mq_stack_plan([mk(8, 0), mk(8, mq.MQ_X_AFTER_EARLIER)], 8)
    with pytest.raises(mq.MqError):                          # more than 16 layers: persistent launch as well
        mq.mq_stack_plan([mk(1, 0)] + [mk(1, mq.MQ_X_AFTER_EARLIER)] * 16, 1)
    with pytest.raises(mq.MqError):                          # batch 4 is switched off for chained stacks
        mq.mq_stack_plan([mk(4, 0), mk(4, mq.MQ_X_AFTER_EARLIER)], 4)
    mq.mq_stack_plan([mk(1, 0), mk(1, mq.MQ_X_AFTER_EARLIER)], 1)   # the same layers, chained properly
