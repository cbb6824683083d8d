"""GPU parity tests: every call goes through the C-ABI library (ctypes binding)
and is compared with the CPU oracle on the same seeded inputs.

Bars: integer work (slice, pack, unpack) bit-exact; y within max-abs 2e-2 and
relative-L2 1e-3 of the float64 oracle (fp16 activations, fp32 accumulation,
fp16 output)."""
import numpy as np
import pytest

import oracle
import paper_2602_03537_amd as mq
from paper_2602_03537_amd import synth
from layout_ref import pack_ref, meta_ref
import tolerance
from gpu_util import C, DEV, WIDTHS, check_layer, check_y, dev, run_linear

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


# ------------------------------------------------------------------ slice
def test_slice_every_code_every_width_bit_exact():
    q = np.arange(256, dtype=np.uint8)
    for c in (8, 6, 4, 1):
        qc = (q & ((1 << c) - 1)).astype(np.uint8)
        for r in range(1, c + 1):
            got = mq.mq_slice_codes(dev(qc), c, r).cpu().numpy()
            assert np.array_equal(got, oracle.slice_codes(qc, c, r)), (c, r)


@pytest.mark.parametrize("n", [0, 1, 15, 16, 17, 4097, 1_000_003])
def test_slice_ragged_lengths_and_unaligned_views(n):
    rng = np.random.default_rng(n)
    q = rng.integers(0, 256, n + 3, dtype=np.uint8)
    buf = dev(q)
    for off in (0, 1):                      # off=1: pointer not 16-byte aligned
        src = buf[off:off + n]
        out = torch.full((n + 2,), 0xAB, dtype=torch.uint8, device=DEV)
        mq.mq_slice_codes(src, C, 3, out=out[1:1 + n])
        torch.cuda.synchronize()
        o = out.cpu().numpy()
        assert o[0] == 0xAB and o[-1] == 0xAB                      # guard bytes untouched
        assert np.array_equal(o[1:1 + n], oracle.slice_codes(q[off:off + n], C, 3))


def test_slice_in_place():
    q = np.random.default_rng(1).integers(0, 256, 5000, dtype=np.uint8)
    t = dev(q)
    mq.mq_slice_codes(t, C, 4, out=t)
    assert np.array_equal(t.cpu().numpy(), oracle.slice_codes(q, C, 4))


# ------------------------------------------------------------------ pack
def _patterns(N, K, r, rng):
    step = 1 << (8 - r)
    top = ((1 << r) - 1) * step
    yield "random", (rng.integers(0, 1 << r, (N, K)) * step).astype(np.uint8)
    yield "zeros", np.zeros((N, K), np.uint8)
    yield "max", np.full((N, K), top, np.uint8)
    alt = np.zeros((N, K), np.uint8)
    alt[:, ::2] = top
    yield "alternating", alt
    ramp = ((np.arange(N)[:, None] * 7 + np.arange(K)[None, :]) % (1 << r) * step).astype(np.uint8)
    yield "ramp", ramp


@pytest.mark.parametrize("r", WIDTHS)
@pytest.mark.parametrize("shape", [(64, 128), (130, 384), (1, 128), (200, 1280)])
def test_pack_matches_documented_layout_and_round_trips(r, shape):
    N, K = shape
    rng = np.random.default_rng([r, N, K])
    for name, S in _patterns(N, K, r, rng):
        packed = mq.mq_pack(dev(S), C, r)
        ref = pack_ref(S, r)
        assert packed.numel() == mq.mq_packed_bytes(N, K, r) == ref.size
        assert np.array_equal(packed.cpu().numpy(), ref), (name, r, shape)
        back = mq.mq_unpack(packed, N, K, C, r)
        assert np.array_equal(back.cpu().numpy(), S), (name, r, shape)


@pytest.mark.parametrize("r", (2, 3, 6))
def test_pack_one_hot_positions(r):
    # a single non-zero code moves to exactly one place; every position of a group is visited
    N, K = 64, 256
    top = ((1 << r) - 1) << (8 - r)
    for k in list(range(0, 128, 7)) + [127, 128, 255]:
        S = np.zeros((N, K), np.uint8)
        S[k % N, k] = top
        packed = mq.mq_pack(dev(S), C, r)
        assert np.array_equal(packed.cpu().numpy(), pack_ref(S, r)), k
        assert np.array_equal(mq.mq_unpack(packed, N, K, C, r).cpu().numpy(), S), k


def test_pack_ignores_low_bits_of_off_grid_codes():
    rng = np.random.default_rng(5)
    q = rng.integers(0, 256, (64, 128), dtype=np.uint8)
    for r in WIDTHS:
        a = mq.mq_pack(dev(q), C, r).cpu().numpy()
        b = mq.mq_pack(dev((q >> (8 - r) << (8 - r)).astype(np.uint8)), C, r).cpu().numpy()
        assert np.array_equal(a, b)


def test_pack_meta_tiling():
    rng = np.random.default_rng(2)
    for N, K in [(64, 128), (200, 1280), (1, 256)]:
        s = rng.uniform(1e-4, 1e-2, (N, K // 128)).astype(np.float16)
        z = rng.integers(0, 256, (N, K // 128)).astype(np.float16)
        st, zt = mq.mq_pack_meta(dev(s), dev(z), K)
        assert np.array_equal(st.cpu().numpy(), meta_ref(s))
        assert np.array_equal(zt.cpu().numpy(), meta_ref(z))


def test_slice_then_pack_of_parent_equals_pack_of_oracle_slice():
    L = synth.make_layer(192, 512, seed=[0, 9])
    for r in WIDTHS:
        S = mq.mq_slice_codes(dev(L["parent"]), C, r)
        assert np.array_equal(mq.mq_pack(S, C, r).cpu().numpy(), pack_ref(oracle.slice_codes(L["parent"], C, r), r))


# ------------------------------------------------------------------ linear
def test_linear_config_512x512_r4_seed0():
    # smallest configuration: K=512, N=512, M=1, group 128, r=4, seed 0
    L = synth.make_layer(512, 512, M=1, seed=0)
    y = run_linear(L, 4)
    check_layer(y, L, 4, "config 512x512")


@pytest.mark.parametrize("r", WIDTHS)
@pytest.mark.parametrize("shape", [(64, 128), (1, 128), (63, 256), (130, 384), (200, 1280), (448, 2048)])
def test_linear_matches_oracle_multi_tile_and_ragged(r, shape):
    N, K = shape
    L = synth.make_layer(N, K, M=1, seed=[1, N, K])
    y = run_linear(L, r)
    check_layer(y, L, r, f"{shape} r={r}")


@pytest.mark.parametrize("r", WIDTHS)
@pytest.mark.parametrize("M", [2, 3, 4])
def test_linear_small_batches(r, M):
    L = synth.make_layer(200, 768, M=M, seed=[2, M])
    y = run_linear(L, r)
    check_layer(y, L, r, f"M={M} r={r}")


@pytest.mark.parametrize("r", WIDTHS)
def test_linear_uniform_random_codes_and_fractional_zeros(r):
    # not a quantiser's output: every code value, non-integer zero-offsets
    L = synth.make_random_codes_layer(192, 640, M=2, seed=[3, r])
    y = run_linear(L, r)
    check_layer(y, L, r, f"random codes r={r}")


def test_linear_symmetric_zero_offsets():
    # Section 5's setup is symmetric quantisation: zero = 2^(c-1) everywhere
    L = synth.make_layer(128, 512, M=1, seed=[4])
    L["zeros"] = np.full_like(L["zeros"], 128.0)
    for r in WIDTHS:
        check_layer(run_linear(L, r), L, r, f"sym r={r}")


def test_linear_degenerate_inputs():
    L = synth.make_layer(128, 256, M=1, seed=[5])
    zero_x = dict(L, x=np.zeros_like(L["x"]))
    assert torch.count_nonzero(run_linear(zero_x, 3)) == 0
    # extreme codes only (0 and 255): clamp region of Eq. 1 at every width
    ext = dict(L, parent=np.where(L["parent"] > 127, 255, 0).astype(np.uint8))
    for r in WIDTHS:
        check_layer(run_linear(ext, r), ext, r, f"extreme r={r}")
    # large activations (outliers) keep the fp16-subnormal arithmetic exact
    big = dict(L, x=(L["x"].astype(np.float32) * 64).astype(np.float16), scales=(L["scales"] / 64).astype(np.float16))
    check_layer(run_linear(big, 2), big, 2, "big x")


def test_linear_r8_equals_plain_8bit_layer_and_low_widths_differ():
    L = synth.make_layer(128, 512, M=1, seed=[6])
    y8 = run_linear(L, 8).cpu().numpy().astype(np.float64)
    w = np.repeat(L["scales"].astype(np.float64), 128, 1) * (L["parent"].astype(np.float64)
                                                              - np.repeat(L["zeros"].astype(np.float64), 128, 1))
    ref8 = L["x"].astype(np.float64) @ w.T
    assert np.abs(y8 - ref8).max() <= tolerance.MAX_ABS
    y2 = run_linear(L, 2).cpu().numpy().astype(np.float64)
    assert np.abs(y2 - ref8).max() > 10 * tolerance.MAX_ABS          # the 2-bit slice is a different model


def test_linear_is_deterministic_and_leaves_guard_bands_alone():
    N, K, r = 200, 1280, 3
    L = synth.make_layer(N, K, M=2, seed=[7])
    lay = mq.prepare_layer(dev(L["parent"]), dev(L["scales"]), dev(L["zeros"]), r)
    x = dev(L["x"])
    ws = mq.new_workspace(2, N, K, r)
    buf = torch.full((2 * N + 128,), float("nan"), dtype=torch.float16, device=DEV)
    y = buf[64:64 + 2 * N].view(2, N)
    outs = []
    for _ in range(3):
        y.fill_(float("nan"))
        mq.mq_linear(x, lay["packed_W"], lay["scales_t"], lay["zeros_t"], N, K, r, 128, ws, y=y)
        torch.cuda.synchronize()
        outs.append(y.clone())
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])
    assert torch.isnan(buf[:64]).all() and torch.isnan(buf[64 + 2 * N:]).all()
    check_layer(outs[0], L, r, "guard")


def test_linear_workspace_is_reusable_across_shapes():
    # counters are left at zero by every call, so one workspace serves many layers
    ws = mq.new_workspace(1, 4096, 4096, 8)
    for (N, K, r) in [(4096, 512, 4), (200, 1280, 2), (512, 512, 6), (4096, 512, 3)]:
        L = synth.make_layer(N, K, M=1, seed=[8, N, K, r])
        lay = mq.prepare_layer(dev(L["parent"]), dev(L["scales"]), dev(L["zeros"]), r)
        y = mq.mq_linear(dev(L["x"]), lay["packed_W"], lay["scales_t"], lay["zeros_t"], N, K, r, 128, ws)
        check_layer(y, L, r, f"reuse {N}x{K} r={r}")


def test_linear_rejects_oversized_batch_loudly():
    L = synth.make_layer(64, 128, M=1, seed=[9])
    lay = mq.prepare_layer(dev(L["parent"]), dev(L["scales"]), dev(L["zeros"]), 4)
    x = torch.zeros((300, 128), dtype=torch.float16, device=DEV)
    ws = mq.new_workspace(1, 64, 128, 4)
    with pytest.raises(mq.MqError):
        mq.mq_linear(x, lay["packed_W"], lay["scales_t"], lay["zeros_t"], 64, 128, 4, 128, ws)
    small_ws = torch.empty(mq.mq_workspace_bytes(8, 64, 128, 4) - 256, dtype=torch.uint8, device=DEV)   # one line short
    with pytest.raises(mq.MqError):
        mq.mq_linear(x[:8], lay["packed_W"], lay["scales_t"], lay["zeros_t"], 64, 128, 4, 128, small_ws)


# ------------------------------------------------------------------ matrix-core path (M > 4)
@pytest.mark.parametrize("r", WIDTHS)
@pytest.mark.parametrize("M", [5, 8, 16])
def test_linear_mfma_one_chunk(r, M):
    L = synth.make_layer(200, 768, M=M, seed=[40, M])
    y = run_linear(L, r)
    check_layer(y, L, r, f"mfma M={M} r={r}")


@pytest.mark.parametrize("r", WIDTHS)
@pytest.mark.parametrize("shape_m", [(64, 128, 17), (130, 384, 33), (63, 256, 64), (257, 1280, 20), (448, 2048, 256),
                                     (1, 128, 7), (1027, 512, 12)])
def test_linear_mfma_chunks_ragged_rows_and_columns(r, shape_m):
    # several 16-column chunks, a ragged last chunk, N not a multiple of 64 or of 4
    N, K, M = shape_m
    L = synth.make_layer(N, K, M=M, seed=[41, N, K, M])
    y = run_linear(L, r)
    check_layer(y, L, r, f"mfma {shape_m} r={r}")


@pytest.mark.parametrize("r", WIDTHS)
def test_linear_mfma_uniform_random_codes_and_fractional_zeros(r):
    L = synth.make_random_codes_layer(192, 640, M=24, seed=[42, r])
    y = run_linear(L, r)
    check_layer(y, L, r, f"mfma random codes r={r}")


def test_linear_mfma_deterministic_guard_bands_and_matches_alu_path():
    N, K, r, M = 200, 1280, 3, 8
    L = synth.make_layer(N, K, M=M, seed=[43])
    lay = mq.prepare_layer(dev(L["parent"]), dev(L["scales"]), dev(L["zeros"]), r)
    x = dev(L["x"])
    ws = mq.new_workspace(M, N, K, r)
    buf = torch.full((M * N + 128,), float("nan"), dtype=torch.float16, device=DEV)
    y = buf[64:64 + M * N].view(M, N)
    outs = []
    for _ in range(3):
        y.fill_(float("nan"))
        mq.mq_linear(x, lay["packed_W"], lay["scales_t"], lay["zeros_t"], N, K, r, 128, ws, y=y)
        torch.cuda.synchronize()
        outs.append(y.clone())
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])
    assert torch.isnan(buf[:64]).all() and torch.isnan(buf[64 + M * N:]).all()
    check_layer(outs[0], L, r, "mfma guard")
    # the same rows through the vector-ALU path (M=4 at a time) agree to fp16 rounding of the same fp32 sums
    ws4 = mq.new_workspace(4, N, K, r)
    y4 = torch.cat([mq.mq_linear(x[i:i + 4], lay["packed_W"], lay["scales_t"], lay["zeros_t"], N, K, r, 128, ws4)
                    for i in (0, 4)])
    assert (outs[0].float() - y4.float()).abs().max() <= 2e-2


@pytest.mark.parametrize("M", [8, 20])
def test_stack_mfma_mixed_widths(M):
    shapes_r = [(256, 512, 2), (64, 128, 8), (200, 1280, 3), (512, 256, 6), (130, 384, 4), (1024, 1024, 3)]
    host, layers = _stack(shapes_r, M=M, seed=44)
    plan = mq.mq_stack_plan(layers, M)
    for rep in range(2):
        for lay in layers:
            lay["y"].fill_(float("nan"))
        mq.mq_linear_stack(plan)
        torch.cuda.synchronize()
        for i, (lay, ref) in enumerate(zip(layers, oracle.linear_stack(host, C, 128))):
            check_y(lay["y"], ref, f"mfma stack layer {i} rep {rep}", host[i], host[i]["r"])


# ------------------------------------------------------------------ wide matrix-core path (M > 16)
@pytest.mark.parametrize("r", WIDTHS)
@pytest.mark.parametrize("shape_m", [(320, 640, 32), (256, 384, 40), (700, 1152, 96), (192, 512, 129), (130, 768, 160),
                                     (1, 256, 31), (520, 256, 250)])
def test_linear_wide_chunk_counts_passes_and_ragged_edges(r, shape_m):
    # 1..4 chunks of 32 columns per pass, one and two passes (padded chunk counts: 129 -> 3+3, 160 -> 3+3, 250 -> 4+4),
    # fewer rows than the four row blocks of a workgroup, N not a multiple of 64, several groups per share
    N, K, M = shape_m
    L = synth.make_layer(N, K, M=M, seed=[47, N, K, M])
    y = run_linear(L, r)
    check_layer(y, L, r, f"wide {shape_m} r={r}")


@pytest.mark.parametrize("r", WIDTHS)
def test_linear_wide_uniform_random_codes_and_fractional_zeros(r):
    # every code value, zeros with fraction bits: the fp16 step 2^(8-r)*code - zero of this path rounds then
    L = synth.make_random_codes_layer(320, 1024, M=72, seed=[48, r])
    y = run_linear(L, r)
    check_layer(y, L, r, f"wide random codes r={r}")


def test_linear_wide_split_k_hand_over_deterministic_with_guard_bands():
    # long K, few row blocks: every row block is shared by several workgroups
    N, K, r, M = 256, 28672, 4, 48
    L = synth.make_layer(N, K, M=M, seed=[49])
    lay = mq.prepare_layer(dev(L["parent"]), dev(L["scales"]), dev(L["zeros"]), r)
    x = dev(L["x"])
    ws = mq.new_workspace(M, N, K, r)
    buf = torch.full((M * N + 128,), float("nan"), dtype=torch.float16, device=DEV)
    y = buf[64:64 + M * N].view(M, N)
    outs = []
    for _ in range(3):
        y.fill_(float("nan"))
        mq.mq_linear(x, lay["packed_W"], lay["scales_t"], lay["zeros_t"], N, K, r, 128, ws, y=y)
        torch.cuda.synchronize()
        outs.append(y.clone())
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])
    assert torch.isnan(buf[:64]).all() and torch.isnan(buf[64 + M * N:]).all()
    check_layer(outs[0], L, r, "wide split-K")


@pytest.mark.parametrize("M", [40, 200])
def test_stack_wide_mixed_widths(M):
    shapes_r = [(256, 512, 2), (64, 128, 8), (200, 1280, 3), (512, 256, 6), (130, 384, 4), (1024, 1024, 3), (320, 2048, 8)]
    host, layers = _stack(shapes_r, M=M, seed=50)
    plan = mq.mq_stack_plan(layers, M)
    for rep in range(2):
        for lay in layers:
            lay["y"].fill_(float("nan"))
        mq.mq_linear_stack(plan)
        torch.cuda.synchronize()
        for i, (lay, ref) in enumerate(zip(layers, oracle.linear_stack(host, C, 128))):
            check_y(lay["y"], ref, f"wide stack layer {i} rep {rep}", host[i], host[i]["r"])


def test_linear_wide_rejects_misaligned_meta():
    L = synth.make_layer(64, 128, M=32, seed=[51])
    lay = mq.prepare_layer(dev(L["parent"]), dev(L["scales"]), dev(L["zeros"]), 4)
    ws = mq.new_workspace(32, 64, 128, 4)
    shifted = torch.empty(lay["scales_t"].numel() + 4, dtype=torch.float16, device=DEV)[4:]  # 8-byte, not 16-byte aligned
    shifted.copy_(lay["scales_t"].flatten())
    with pytest.raises(mq.MqError):
        mq.mq_linear(dev(L["x"]), lay["packed_W"], shifted, lay["zeros_t"], 64, 128, 4, 128, ws)


def test_linear_llama3_70b_mlp_shape_batched_sampled_rows():
    # batched regime on the 8192 -> 28672 up-projection shape; rows sampled for the oracle
    N, K = 28672, 8192
    L = synth.make_layer(N, K, M=16, seed=[45])
    rng = np.random.default_rng(46)
    rows = np.unique(np.concatenate([[0, 63, 64, N - 1], rng.integers(0, N, 124)]))
    p, s, z = dev(L["parent"]), dev(L["scales"]), dev(L["zeros"])
    for r in (3, 4, 8):
        lay = mq.prepare_layer(p, s, z, r)
        for M in (1, 4, 16):
            ws = mq.new_workspace(M, N, K, r)
            y = mq.mq_linear(dev(L["x"][:M]), lay["packed_W"], lay["scales_t"], lay["zeros_t"], N, K, r, 128, ws)
            ref = oracle.linear_rows(L["x"][:M], L["parent"], L["scales"], L["zeros"], C, r, 128, rows)
            check_y(y[:, torch.from_numpy(rows).to(DEV)], ref, f"70B up r={r} M={M}")
            assert torch.isfinite(y).all()


# ------------------------------------------------ full-size layers, sampled rows
LLAMA7B = [(4096, 4096), (11008, 4096), (4096, 11008)]


@pytest.mark.parametrize("shape", LLAMA7B)
def test_linear_llama2_7b_shapes_sampled_rows(shape):
    N, K = shape
    L = synth.make_layer(N, K, M=1, seed=[0, N, K])
    rng = np.random.default_rng([11, N])
    rows = np.unique(np.concatenate([[0, 63, 64, N - 1], rng.integers(0, N, 252)]))
    p, s, z, x = dev(L["parent"]), dev(L["scales"]), dev(L["zeros"]), dev(L["x"])
    for r in WIDTHS:
        lay = mq.prepare_layer(p, s, z, r)
        ws = mq.new_workspace(1, N, K, r)
        y = mq.mq_linear(x, lay["packed_W"], lay["scales_t"], lay["zeros_t"], N, K, r, 128, ws)
        ref = oracle.linear_rows(L["x"], L["parent"], L["scales"], L["zeros"], C, r, 128, rows)
        check_y(y[:, torch.from_numpy(rows).to(DEV)], ref, f"{shape} r={r}")
        # the sliced codes of the whole matrix, bit-exact
        S = mq.mq_unpack(lay["packed_W"], N, K, C, r).cpu().numpy()
        assert np.array_equal(S, oracle.slice_codes(L["parent"], C, r))
        assert torch.isfinite(y).all()


# ------------------------------------------------------------------ stack
def _stack(shapes_r, M=1, seed=0):  # noqa: E302
    host, layers = [], []
    for i, (N, K, r) in enumerate(shapes_r):
        L = synth.make_layer(N, K, M=M, seed=[seed, i, N, K])
        lay = mq.prepare_layer(dev(L["parent"]), dev(L["scales"]), dev(L["zeros"]), r)
        lay.update(x=dev(L["x"]), y=torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV))
        host.append(dict(L, r=r))
        layers.append(lay)
    return host, layers


@pytest.mark.parametrize("M", [1, 2, 3, 4])
def test_stack_mixed_widths_matches_oracle(M):
    shapes_r = [(256, 512, 2), (64, 128, 8), (200, 1280, 3), (512, 256, 6), (130, 384, 4), (1024, 1024, 3),
                (63, 128, 2), (320, 640, 8)]
    host, layers = _stack(shapes_r, M=M, seed=21)
    plan = mq.mq_stack_plan(layers, M)
    for rep in range(2):                               # the plan is reusable (counters self-reset)
        for lay in layers:
            lay["y"].fill_(float("nan"))
        mq.mq_linear_stack(plan)
        torch.cuda.synchronize()
        refs = oracle.linear_stack(host, C, 128)
        for i, (lay, ref) in enumerate(zip(layers, refs)):
            check_y(lay["y"], ref, f"stack layer {i} rep {rep}", host[i], host[i]["r"])


def test_stack_equals_layer_by_layer_calls_bit_for_bit_when_unsplit():
    # one tile per layer: no split-K anywhere, so stack and single calls do identical arithmetic
    shapes_r = [(64, 128, r) for r in WIDTHS]
    host, layers = _stack(shapes_r, seed=22)
    plan = mq.mq_stack_plan(layers, 1)
    mq.mq_linear_stack(plan)
    torch.cuda.synchronize()
    for lay in layers:
        ws = mq.new_workspace(1, lay["N"], lay["K"], lay["r"])
        y = mq.mq_linear(lay["x"], lay["packed_W"], lay["scales_t"], lay["zeros_t"], lay["N"], lay["K"], lay["r"],
                         128, ws)
        assert torch.equal(y, lay["y"])


def test_stack_llama2_7b_block_mixed_widths_sampled_rows():
    # two decoder blocks (14 linears) at the real shapes, widths drawn by seed
    shapes = [(N, K) for _ in range(2) for (_, N, K) in synth.LLAMA2_7B_BLOCK]
    widths, _ = synth.draw_bitwidths([N * K for N, K in shapes], 3.5, seed=3, tol=0.5)
    base = {}
    host, layers = [], []
    for i, ((N, K), r) in enumerate(zip(shapes, widths)):
        if (N, K) not in base:
            base[(N, K)] = synth.make_layer(N, K, M=1, seed=[31, N, K])
        L = dict(base[(N, K)])
        L["x"] = synth.make_x(1, K, [32, i])
        lay = mq.prepare_layer(dev(L["parent"]), dev(L["scales"]), dev(L["zeros"]), int(r))
        lay.update(x=dev(L["x"]), y=torch.full((1, N), float("nan"), dtype=torch.float16, device=DEV))
        host.append(dict(L, r=int(r)))
        layers.append(lay)
    plan = mq.mq_stack_plan(layers, 1)
    mq.mq_linear_stack(plan)
    torch.cuda.synchronize()
    rng = np.random.default_rng(33)
    for i, (L, lay) in enumerate(zip(host, layers)):
        N = lay["N"]
        rows = np.unique(np.concatenate([[0, N - 1], rng.integers(0, N, 62)]))
        ref = oracle.linear_rows(L["x"], L["parent"], L["scales"], L["zeros"], C, L["r"], 128, rows)
        sub = dict(L, parent=L["parent"][rows], scales=L["scales"][rows], zeros=L["zeros"][rows])
        check_y(lay["y"][:, torch.from_numpy(rows).to(DEV)], ref, f"block linear {i} r={L['r']}", sub, L["r"])
        assert torch.isfinite(lay["y"]).all()


# ------------------------------------------------ full-size stacks (generated on the device)
def _device_stack(block, n_blocks, target_bits, M, seed):
    shapes = synth.stack_shapes(block, n_blocks)
    widths, mean = synth.draw_bitwidths([N * K for (_, _, N, K) in shapes], target_bits, seed=seed)
    gen, layers = [], []
    for i, ((_, _, N, K), r) in enumerate(zip(shapes, widths)):
        L = synth.make_layer_device(N, K, M, seed=seed * 100000 + i, device=DEV)
        lay = mq.prepare_layer(L["parent"], L["scales"], L["zeros"], int(r))
        lay.update(x=L["x"], y=torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV))
        gen.append(L)
        layers.append(lay)
    return shapes, widths, mean, gen, layers


def _check_sampled(gen, layers, idx, n_rows, rng, what):
    L, lay = gen[idx], layers[idx]
    N = lay["N"]
    rows = np.unique(np.concatenate([[0, N - 1], rng.integers(0, N, n_rows - 2)]))
    rt = torch.from_numpy(rows).to(DEV)
    sub = dict(x=L["x"].cpu().numpy(), parent=L["parent"][rt].cpu().numpy(), scales=L["scales"][rt].cpu().numpy(),
               zeros=L["zeros"][rt].cpu().numpy())
    check_layer(lay["y"][:, rt], sub, lay["r"], f"{what} linear {idx} r={lay['r']}")


def test_stack_llama2_7b_full_mixed_widths_mean_3p5():
    # all 32 blocks x 7 linears, widths by seed with parameter-weighted mean 3.5, batch 1
    shapes, widths, mean, gen, layers = _device_stack(synth.LLAMA2_7B_BLOCK, synth.LLAMA2_7B_LAYERS, 3.5, 1, seed=4)
    assert len(layers) == 224 and abs(mean - 3.5) <= 0.02
    plan = mq.mq_stack_plan(layers, 1)
    mq.mq_linear_stack(plan)
    torch.cuda.synchronize()
    rng = np.random.default_rng(404)
    for i in range(len(layers)):
        assert torch.isfinite(layers[i]["y"]).all(), i
        _check_sampled(gen, layers, i, 64 if i < 7 or i >= 217 else 8, rng, "7B stack")
    first = [lay["y"].clone() for lay in layers[:14]]
    mq.mq_linear_stack(plan)                                   # replay: same bits
    torch.cuda.synchronize()
    assert all(torch.equal(a, lay["y"]) for a, lay in zip(first, layers[:14]))


@pytest.mark.parametrize("M", [1, 8])
def test_stack_llama3_70b_full_mixed_widths_mean_4(M):
    # 80 blocks x 7 linears (68.45 G weights): the 8-bit parent stays resident next to the packed slices
    shapes, widths, mean, gen, layers = _device_stack(synth.LLAMA3_70B_BLOCK, synth.LLAMA3_70B_LAYERS, 4.0, M, seed=5)
    assert len(layers) == 560 and abs(mean - 4.0) <= 0.02
    assert sum(int(L["parent"].numel()) for L in gen) == 68_451_041_280
    plan = mq.mq_stack_plan(layers, M)
    mq.mq_linear_stack(plan)
    torch.cuda.synchronize()
    rng = np.random.default_rng(505 + M)
    for i in range(len(layers)):
        block = i // 7
        assert torch.isfinite(layers[i]["y"]).all(), i
        _check_sampled(gen, layers, i, 64 if block in (0, 39, 79) else 6, rng, f"70B stack M={M}")
    del gen, layers, plan
    torch.cuda.empty_cache()


# ------------------------------------------------------------------ run-time re-slicing of a resident parent
def _resident(L):
    """host layer -> (8-bit pack of the unsliced parent, tiled scales, tiled zeros) on the device."""
    N, K = L["parent"].shape
    p8 = mq.mq_pack(dev(L["parent"]), C, 8)
    st, zt = mq.mq_pack_meta(dev(L["scales"]), dev(L["zeros"]), K, 128)
    return p8, st, zt


def _every_code_parent(N, K, rng):
    """all 256 code values next to each other, rounding ties and the clamp region of Eq. 1 in every row"""
    q = (np.arange(N)[:, None] * 37 + np.arange(K)[None, :]) % 256
    q[rng.integers(0, N, N // 2 + 1), rng.integers(0, K, N // 2 + 1)] = 255
    return q.astype(np.uint8)


@pytest.mark.parametrize("r", WIDTHS)
@pytest.mark.parametrize("shape", [(64, 128), (1, 128), (130, 384), (200, 1280), (448, 2048)])
def test_slice_pack_and_reslice_bit_exact(r, shape):
    N, K = shape
    rng = np.random.default_rng([60, r, N, K])
    for name, parent in (("uniform", rng.integers(0, 256, (N, K), dtype=np.uint8)),
                         ("every code", _every_code_parent(N, K, rng)),
                         ("quantiser", synth.make_layer(N, K, seed=[60, N, K])["parent"])):
        ref = pack_ref(oracle.slice_codes(parent, C, r), r)
        fused = mq.mq_slice_pack(dev(parent), C, r)
        assert np.array_equal(fused.cpu().numpy(), ref), ("slice_pack", name, r, shape)
        p8 = mq.mq_pack(dev(parent), C, 8)
        out = torch.full((ref.size + 32,), 0xAB, dtype=torch.uint8, device=DEV)
        mq.mq_reslice(p8, N, K, C, r, out=out[16:16 + ref.size])
        torch.cuda.synchronize()
        o = out.cpu().numpy()
        assert np.array_equal(o[16:16 + ref.size], ref), ("reslice", name, r, shape)
        assert (o[:16] == 0xAB).all() and (o[16 + ref.size:] == 0xAB).all()     # guard bytes untouched


def test_reslice_rejects_bad_arguments_loudly():
    parent = np.zeros((64, 128), np.uint8)
    p8 = mq.mq_pack(dev(parent), C, 8)
    with pytest.raises(mq.MqError):
        mq.mq_reslice(p8, 64, 128, C, 5)                          # width without a layout
    with pytest.raises(mq.MqError):
        mq.mq_reslice(p8, 64, 128, 7, 4)                          # c != 8
    with pytest.raises(mq.MqError):
        mq.mq_reslice(p8, 64, 128, C, 4, out=p8[:4096])           # in place is not supported
    with pytest.raises(mq.MqError):
        mq.mq_reslice(p8, 64, 128, C, 4, out=torch.empty(100, dtype=torch.uint8, device=DEV))
    with pytest.raises(mq.MqError):
        mq.mq_slice_pack(dev(parent), C, 4, out=torch.empty(100, dtype=torch.uint8, device=DEV))


@pytest.mark.parametrize("r", WIDTHS)
@pytest.mark.parametrize("shape_m", [(64, 128, 1), (1, 128, 1), (130, 384, 2), (200, 1280, 3), (448, 2048, 4),
                                     (4096, 512, 1), (512, 14336, 1)])
def test_linear_from_parent_matches_oracle_and_the_repacked_layer(r, shape_m):
    # (4096, 512) runs the low-latency kernel unsplit, (512, 14336) the stream-K kernel with hand-over
    N, K, M = shape_m
    L = synth.make_layer(N, K, M=M, seed=[61, N, K])
    p8, st, zt = _resident(L)
    x = dev(L["x"])
    ws = mq.new_workspace(M, N, K, 8)
    y = mq.mq_linear_from_parent(x, p8, st, zt, N, K, r, 128, ws)
    torch.cuda.synchronize()
    check_layer(y, L, r, f"from parent {shape_m} r={r}")
    # the re-packed layer computes the same sums in another order: equal to fp32 rounding
    pr = mq.mq_reslice(p8, N, K, C, r)
    y2 = mq.mq_linear(x, pr, st, zt, N, K, r, 128, mq.new_workspace(M, N, K, r))
    assert torch.allclose(y.float(), y2.float(), rtol=2e-3, atol=2e-3)


@pytest.mark.parametrize("r", WIDTHS)
def test_linear_from_parent_every_code_and_fractional_zeros(r):
    L = synth.make_random_codes_layer(192, 640, M=2, seed=[62, r])
    L["parent"] = _every_code_parent(192, 640, np.random.default_rng(62))
    p8, st, zt = _resident(L)
    y = mq.mq_linear_from_parent(dev(L["x"]), p8, st, zt, 192, 640, r, 128, mq.new_workspace(2, 192, 640, 8))
    check_layer(y, L, r, f"every code r={r}")


def test_linear_from_parent_batch_above_four_is_refused():
    L = synth.make_layer(64, 128, M=8, seed=[63])
    p8, st, zt = _resident(L)
    with pytest.raises(mq.MqError) as e:
        mq.mq_linear_from_parent(dev(L["x"]), p8, st, zt, 64, 128, 4, 128, mq.new_workspace(8, 64, 128, 8))
    assert e.value.status == 8


@pytest.mark.parametrize("M", [1, 3])
def test_stack_from_parent_mixed_widths(M):
    shapes_r = [(256, 512, 2), (64, 128, 8), (200, 1280, 3), (512, 256, 6), (130, 384, 4), (1024, 1024, 3),
                (63, 128, 2), (320, 640, 8)]
    host, layers = [], []
    for i, (N, K, r) in enumerate(shapes_r):
        L = synth.make_layer(N, K, M=M, seed=[64, i, N, K])
        p8, st, zt = _resident(L)
        layers.append(dict(packed_W=p8, scales_t=st, zeros_t=zt, N=N, K=K, r=r, from_parent=1, x=dev(L["x"]),
                           y=torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV)))
        host.append(dict(L, r=r))
    plan = mq.mq_stack_plan(layers, M)
    refs = oracle.linear_stack(host, C, 128)
    for rep in range(2):
        for lay in layers:
            lay["y"].fill_(float("nan"))
        mq.mq_linear_stack(plan)
        torch.cuda.synchronize()
        for i, (lay, ref) in enumerate(zip(layers, refs)):
            check_y(lay["y"], ref, f"from-parent stack layer {i} rep {rep}", host[i], host[i]["r"])
    # a different budget from the same resident parents: only the plan changes
    for lay, hl in zip(layers, host):
        lay["r"] = hl["r"] = 4
    plan4 = mq.mq_stack_plan(layers, M)
    mq.mq_linear_stack(plan4)
    torch.cuda.synchronize()
    for i, (lay, ref) in enumerate(zip(layers, oracle.linear_stack(host, C, 128))):
        check_y(lay["y"], ref, f"from-parent stack at 4 bits, layer {i}", host[i], 4)
    mixed = [dict(l) for l in layers]
    mixed[1]["from_parent"] = 0
    with pytest.raises(mq.MqError):
        mq.mq_stack_plan(mixed, M)


def test_from_parent_llama3_70b_down_projection_sampled_rows_and_full_reslice():
    # 8192 x 28672: more tiles than the low-latency kernel takes, so the stream-K kernel with hand-over runs
    N, K = 8192, 28672
    L = synth.make_layer(N, K, M=2, seed=[65])
    rng = np.random.default_rng(66)
    rows = np.unique(np.concatenate([[0, 63, 64, N - 1], rng.integers(0, N, 124)]))
    p8, st, zt = _resident(L)
    for M in (1, 2):
        ws = mq.new_workspace(M, N, K, 8)
        for r in (2, 3, 6):
            y = mq.mq_linear_from_parent(dev(L["x"][:M]), p8, st, zt, N, K, r, 128, ws)
            ref = oracle.linear_rows(L["x"][:M], L["parent"], L["scales"], L["zeros"], C, r, 128, rows)
            check_y(y[:, torch.from_numpy(rows).to(DEV)], ref, f"from parent 70B down r={r} M={M}")
            assert torch.isfinite(y).all()
    for r in (3, 4):                 # the whole re-sliced matrix, bit for bit, through the inverse of the pack
        S = mq.mq_unpack(mq.mq_reslice(p8, N, K, C, r), N, K, C, r).cpu().numpy()
        assert np.array_equal(S, oracle.slice_codes(L["parent"], C, r))


# ------------------------------------------------------------------ Algorithm 1: cross-bit-width choice of the parent code
def _quant_inputs(N, K, seed, std=0.02):
    """weights, and the min-max scale / zero-offset of the seeded recipe (fp16), on the host"""
    W = synth.make_weights(N, K, seed, std)
    _, s, z = synth.quantize_parent(W)
    return W.astype(np.float32), s, z


QUANT_SETS = [((8,), (1.0,)), ((3, 4, 8), (1.0, 1.0, 1.0)), ((3, 4, 8), (1.0, 0.5, 0.1)),
              ((2, 3, 4, 6, 8), (0.1, 0.5, 1.0, 1.0, 0.25)), ((2, 5, 7), (1.0, 2.0, 0.5)), ((4,), (1.0,)),
              ((1, 2, 3, 4, 5, 6, 7, 8), (1.0,) * 8)]


@pytest.mark.parametrize("widths,lam", QUANT_SETS)
@pytest.mark.parametrize("shape", [(64, 128), (3, 256), (130, 384), (257, 1280)])
def test_quant_matgptq_whole_matrix_bit_exact(widths, lam, shape):
    N, K = shape
    W, s, z = _quant_inputs(N, K, [70, N, K])
    W[0, :8] = [10.0, -10.0, 0.0, W[0, 3], 1e-30, -1e-30, 3.0, -3.0]       # far outside the grid, zero, tiny
    ref = oracle.quant_matgptq(W, s, z, C, widths, lam, 128, np.float32)
    got = mq.mq_quant_matgptq(dev(W), dev(s), dev(z), widths, lam)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), ref), (widths, lam, shape)


def test_quant_matgptq_differs_from_plain_rounding_and_serves_the_low_widths_better():
    # what the step is for: against round-to-nearest at 8 bits, the summed error over the target widths drops
    N, K = 128, 512
    W, s, z = _quant_inputs(N, K, [71])
    widths, lam = (3, 4, 8), (1.0, 1.0, 1.0)
    q = mq.mq_quant_matgptq(dev(W), dev(s), dev(z), widths, lam).cpu().numpy()
    rtn = mq.mq_quant_matgptq(dev(W), dev(s), dev(z), (8,), (1.0,)).cpu().numpy()
    recipe = synth.quantize_parent(W)[0].astype(int)                        # R = {8} is plain rounding to nearest:
    assert np.abs(rtn.astype(int) - recipe).max() <= 1                      # the recipe's codes up to rounding ties
    assert np.count_nonzero(rtn != recipe) < 1e-3 * rtn.size
    assert 0 < np.count_nonzero(q != rtn) < q.size

    def total(codes):
        return sum(((W - oracle.dequant(oracle.slice_codes(codes, C, r), s, z, 128)) ** 2).sum() for r in widths)
    assert total(q) < total(rtn)


@pytest.mark.parametrize("ncols,col0", [(1, 0), (1, 131), (5, 126), (128, 256), (4, 124), (132, 4)])
def test_quant_matgptq_column_slabs_strides_and_guard_bytes(ncols, col0):
    # the column-at-a-time and block-at-a-time calls of the GPTQ loop: a strided view of W, codes into a strided view
    N, K = 100, 512
    W, s, z = _quant_inputs(N, K, [72, ncols, col0])
    widths, lam = (3, 4, 8), (1.0, 0.5, 0.1)
    ref = oracle.quant_matgptq(W, s, z, C, widths, lam, 128, np.float32)[:, col0:col0 + ncols]
    Wd = dev(W)
    out = torch.full((N, K + 8), 0xAB, dtype=torch.uint8, device=DEV)
    for view_off in (0, 4, 3):              # 3: the codes land on an address that rules out four columns per lane
        out.fill_(0xAB)
        dst = out[:, view_off + col0: view_off + col0 + ncols]
        mq.mq_quant_matgptq(Wd[:, col0:col0 + ncols], dev(s), dev(z), widths, lam, K=K, col0=col0, out=dst)
        torch.cuda.synchronize()
        o = out.cpu().numpy()
        assert np.array_equal(o[:, view_off + col0: view_off + col0 + ncols], ref), (ncols, col0, view_off)
        o[:, view_off + col0: view_off + col0 + ncols] = 0xAB
        assert (o == 0xAB).all()                                           # nothing else was written


def test_quant_matgptq_fractional_zero_offsets_constant_groups_and_ties():
    N, K = 64, 256
    rng = np.random.default_rng(73)
    W = (rng.standard_normal((N, K)) * 0.05).astype(np.float32)
    s = rng.uniform(2e-4, 2e-3, (N, 2)).astype(np.float16)
    z = rng.uniform(0, 255, (N, 2)).astype(np.float16)                     # not integers
    W[1] = 0.0
    s[1], z[1] = 1.0, 0.0                                                  # constant group: unit scale
    W[2, :128] = (np.arange(128) + 0.5).astype(np.float32)                 # exact ties between neighbours at r = 8
    s[2], z[2] = 1.0, 0.0
    for widths, lam in QUANT_SETS[:4]:
        ref = oracle.quant_matgptq(W, s, z, C, widths, lam, 128, np.float32)
        got = mq.mq_quant_matgptq(dev(W), dev(s), dev(z), widths, lam).cpu().numpy()
        assert np.array_equal(got, ref), (widths, lam)
    assert np.array_equal(mq.mq_quant_matgptq(dev(W), dev(s), dev(z), (8,), (1.0,)).cpu().numpy()[2, :128],
                          np.arange(128))                                  # the smaller code wins the tie


def test_quant_matgptq_llama2_7b_layer_sampled_rows():
    N, K = 4096, 4096
    L = synth.make_layer_device(N, K, 1, seed=74, device=DEV)
    g = torch.Generator(device=DEV)
    g.manual_seed(75)
    W = torch.randn((N, K), generator=g, device=DEV, dtype=torch.float32) * 0.02
    widths, lam = (3, 4, 8), (1.0, 1.0, 1.0)
    q = mq.mq_quant_matgptq(W, L["scales"], L["zeros"], widths, lam)
    rows = np.unique(np.concatenate([[0, 63, 64, N - 1], np.random.default_rng(76).integers(0, N, 28)]))
    ridx = torch.from_numpy(rows).to(DEV)
    ref = oracle.quant_matgptq(W[ridx].cpu().numpy(), L["scales"][ridx].cpu().numpy(), L["zeros"][ridx].cpu().numpy(),
                               C, widths, lam, 128, np.float32)
    assert np.array_equal(q[ridx].cpu().numpy(), ref)


def test_quant_matgptq_rejects_bad_arguments_loudly():
    W, s, z = _quant_inputs(64, 128, [77])
    Wd, sd, zd = dev(W), dev(s), dev(z)
    for widths, lam in [((8,), (0.0,)), ((3, 8), (1.0, -1.0)), ((4,), (float("nan"),)), ((9,), (1.0,))]:
        with pytest.raises(mq.MqError):
            mq.mq_quant_matgptq(Wd, sd, zd, widths, lam)
    with pytest.raises(mq.MqError):
        mq.mq_quant_matgptq(Wd, sd, zd, (8,), (1.0,), c=7)
    with pytest.raises(mq.MqError):
        mq.mq_quant_matgptq(Wd[:, :8], sd, zd, (8,), (1.0,), K=128, col0=124)        # slab runs past the last column


# ------------------------------------------------------------------ Algorithm 2: the MatGPTQ column loop
def _cholesky_factor(K, seed):
    """U, the upper Cholesky factor of (2 X X^T + damping)^-1 for seeded correlated features (numpy float64 -> float32)."""
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((K, 4 * K)) * (1.0 + 3.0 * rng.random((K, 1)))
    X += 0.5 * X[rng.permutation(K), :]
    H = 2.0 * X @ X.T
    H += 0.01 * np.mean(np.diag(H)) * np.eye(K)
    return np.linalg.cholesky(np.linalg.inv(H)).T.astype(np.float32)


@pytest.mark.parametrize("widths,lam", [((8,), (1.0,)), ((3, 4, 8), (1.0, 1.0, 1.0)), ((3, 4, 8), (1.0, 0.5, 0.1)),
                                        ((2, 3, 4, 6, 8), (1.0,) * 5), ((2, 5), (1.0, 2.0))])
@pytest.mark.parametrize("shape_block", [(64, 256, 128), (70, 384, 128), (3, 256, 32), (130, 256, 64), (16, 128, 16)])
def test_matgptq_column_loop_bit_exact(widths, lam, shape_block):
    N, K, block = shape_block
    W, s, z = _quant_inputs(N, K, [90, N, K])
    U = _cholesky_factor(K, [90, K])
    ref, _ = oracle.matgptq_quantize(W, U, s, z, C, widths, lam, 128, block, np.float32)
    Wd = dev(W.copy())
    got = mq.mq_matgptq_quantize(Wd, dev(U), dev(s), dev(z), widths, lam, block=block)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), ref), (widths, lam, shape_block)


def test_matgptq_column_loop_block_size_changes_nothing_and_beats_plain_rounding():
    N, K = 96, 512
    W, s, z = _quant_inputs(N, K, [91])
    rng = np.random.default_rng(91)
    X = rng.standard_normal((K, 4 * K)) * (1.0 + 3.0 * rng.random((K, 1)))
    H = 2.0 * X @ X.T
    H += 0.01 * np.mean(np.diag(H)) * np.eye(K)
    U = np.linalg.cholesky(np.linalg.inv(H)).T.astype(np.float32)
    widths, lam = (3, 4, 8), (1.0, 1.0, 1.0)
    outs = [mq.mq_matgptq_quantize(dev(W.copy()), dev(U), dev(s), dev(z), widths, lam, block=b).cpu().numpy()
            for b in (16, 32, 64, 128)]
    for o in outs[1:]:
        assert np.array_equal(o, outs[0])
    q1 = mq.mq_quant_matgptq(dev(W), dev(s), dev(z), widths, lam).cpu().numpy()       # no error propagation

    def loss(codes):
        d = W.astype(np.float64) - np.mean([oracle.dequant(oracle.slice_codes(codes, C, r), s, z, 128) for r in widths], 0)
        return np.trace(d @ H @ d.T)
    assert loss(outs[0]) < loss(q1)


def test_matgptq_column_loop_strided_buffers_and_guard_bytes():
    N, K = 40, 256
    W, s, z = _quant_inputs(N, K, [92])
    U = _cholesky_factor(K, [92])
    ref, _ = oracle.matgptq_quantize(W, U, s, z, C, (3, 4, 8), (1, 1, 1), 128, 128, np.float32)
    Wbuf = torch.full((N, K + 24), float("nan"), dtype=torch.float32, device=DEV)
    Wbuf[:, 8:8 + K] = dev(W)
    Ubuf = torch.full((K, K + 8), float("nan"), dtype=torch.float32, device=DEV)
    Ubuf[:, :K] = dev(U)
    Qbuf = torch.full((N, K + 16), 0xAB, dtype=torch.uint8, device=DEV)
    mq.mq_matgptq_quantize(Wbuf[:, 8:8 + K], Ubuf[:, :K], dev(s), dev(z), (3, 4, 8), (1, 1, 1), out=Qbuf[:, 4:4 + K])
    torch.cuda.synchronize()
    q = Qbuf.cpu().numpy()
    assert np.array_equal(q[:, 4:4 + K], ref)
    assert (q[:, :4] == 0xAB).all() and (q[:, 4 + K:] == 0xAB).all()
    assert torch.isnan(Wbuf[:, :8]).all() and torch.isnan(Wbuf[:, 8 + K:]).all()      # the loop stays inside W
    # odd strides and a base address that rules out 16-byte accesses: the one-column-per-lane update
    Wodd = torch.full((N, K + 3), float("nan"), dtype=torch.float32, device=DEV)
    Wodd[:, 1:1 + K] = dev(W)
    Uodd = torch.full((K, K + 1), float("nan"), dtype=torch.float32, device=DEV)
    Uodd[:, :K] = dev(U)
    q2 = mq.mq_matgptq_quantize(Wodd[:, 1:1 + K], Uodd[:, :K], dev(s), dev(z), (3, 4, 8), (1, 1, 1), block=32)
    torch.cuda.synchronize()
    assert np.array_equal(q2.cpu().numpy(), ref)
    assert torch.isnan(Wodd[:, :1]).all() and torch.isnan(Wodd[:, 1 + K:]).all()


def test_matgptq_column_loop_llama_width_sampled_rows():
    # K = 4096 (32 blocks of 128 columns), rows are independent so the oracle runs on a sample of them
    N, K = 512, 4096
    g = torch.Generator(device=DEV)
    g.manual_seed(93)
    W = torch.randn((N, K), generator=g, device=DEV, dtype=torch.float32) * 0.02
    L = synth.make_layer_device(N, K, 1, seed=93, device=DEV, want_x=False)
    X = torch.randn((K, 2 * K), generator=g, device=DEV, dtype=torch.float32) * (1.0 + 3.0 * torch.rand((K, 1), generator=g, device=DEV))
    H = (2.0 * X @ X.T).double()
    H += 0.01 * H.diagonal().mean() * torch.eye(K, device=DEV, dtype=torch.float64)
    U = torch.linalg.cholesky(torch.linalg.inv(H)).T.contiguous().float()
    rows = np.array([0, 63, 64, 311, N - 1])
    ridx = torch.from_numpy(rows).to(DEV)
    Wh, sh, zh = W[ridx].cpu().numpy(), L["scales"][ridx].cpu().numpy(), L["zeros"][ridx].cpu().numpy()
    q = mq.mq_matgptq_quantize(W.clone(), U, L["scales"], L["zeros"], (3, 4, 8), (1.0, 1.0, 1.0))
    torch.cuda.synchronize()
    ref, _ = oracle.matgptq_quantize(Wh, U.cpu().numpy(), sh, zh, C, (3, 4, 8), (1.0, 1.0, 1.0), 128, 128, np.float32)
    assert np.array_equal(q[ridx].cpu().numpy(), ref)


def test_matgptq_column_loop_rejects_bad_arguments_loudly():
    W, s, z = _quant_inputs(64, 256, [94])
    U = _cholesky_factor(256, [94])
    Wd, Ud, sd, zd = dev(W), dev(U), dev(s), dev(z)
    with pytest.raises(mq.MqError):
        mq.mq_matgptq_quantize(Wd, Ud, sd, zd, (8,), (1.0,), block=48)
    with pytest.raises(mq.MqError):
        mq.mq_matgptq_quantize(Wd, Ud, sd, zd, (8,), (0.0,))
    with pytest.raises(ValueError):
        mq.mq_matgptq_quantize(Wd, Ud[:, :128], sd, zd, (8,), (1.0,))                 # factor narrower than K
    with pytest.raises(mq.MqError):
        mq.mq_matgptq_quantize(Wd, Ud, sd, zd, (8,), (1.0,), c=4)


@pytest.mark.parametrize("N,K", [(4096, 256), (4100, 128), (16384, 128), (16390, 256)])   # 64, 16, 16, 4 lanes per row
def test_matgptq_column_loop_many_rows_sampled(N, K):
    # with more rows fewer lanes share a row (16, then 4): the same codes, checked on sampled rows
    W, s, z = _quant_inputs(N, K, [95, N, K])
    U = _cholesky_factor(K, [95, K])
    rows = np.unique(np.concatenate([[0, 1, 3, 4, 15, 16, 63, 64, N - 2, N - 1],
                                     np.random.default_rng(N).integers(0, N, 22)]))
    for widths, lam in (((3, 4, 8), (1.0, 1.0, 1.0)), ((2, 3, 4, 6, 8), (0.1, 0.5, 1.0, 1.0, 0.25))):
        q = mq.mq_matgptq_quantize(dev(W.copy()), dev(U), dev(s), dev(z), widths, lam).cpu().numpy()
        ref, _ = oracle.matgptq_quantize(W[rows], U, s[rows], z[rows], C, widths, lam, 128, 128, np.float32)
        assert np.array_equal(q[rows], ref), (N, K, widths)


def test_reslice_many_layers_in_few_launches_bit_exact():
    # 37 layers of mixed shapes and widths (three launches of 16, 16 and 5 jobs), each checked against the
    # independent packer applied to the oracle's slice; guard bytes around every output
    rng = np.random.default_rng(97)
    shapes = [(64, 128), (130, 384), (1, 128), (200, 1280), (448, 256), (63, 512)]
    jobs, refs, bufs = [], [], []
    for i in range(37):
        N, K = shapes[i % len(shapes)]
        r = WIDTHS[int(rng.integers(0, 5))]
        parent = rng.integers(0, 256, (N, K), dtype=np.uint8)
        ref = pack_ref(oracle.slice_codes(parent, C, r), r)
        buf = torch.full((ref.size + 32,), 0xAB, dtype=torch.uint8, device=DEV)
        jobs.append(dict(packed_parent=mq.mq_pack(dev(parent), C, 8), N=N, K=K, r=r, out=buf[16:16 + ref.size]))
        refs.append(ref)
        bufs.append(buf)
    mq.mq_reslice_many(jobs)
    torch.cuda.synchronize()
    for i, (buf, ref) in enumerate(zip(bufs, refs)):
        o = buf.cpu().numpy()
        assert np.array_equal(o[16:16 + ref.size], ref), i
        assert (o[:16] == 0xAB).all() and (o[16 + ref.size:] == 0xAB).all(), i
    bad = [dict(jobs[0]), dict(jobs[1], r=5)]
    with pytest.raises(mq.MqError):
        mq.mq_reslice_many(bad)
    with pytest.raises(mq.MqError):
        mq.mq_reslice_many([dict(jobs[0], out=jobs[0]["packed_parent"][:jobs[0]["out"].numel()])])   # in place


@pytest.mark.parametrize("M", [1, 4, 8])
def test_stack_shared_input_fusions_qkv_and_gate_up(M):
    # decode-shaped fusions: the linears that read the same activations (q/k/v; gate/up) as one launch each
    rng = np.random.default_rng([98, M])
    x = synth.make_x(M, 512, [98, M])
    xd = dev(x)
    for shapes_r in ([(512, 512, 4), (128, 512, 2), (128, 512, 8)], [(1376, 512, 3), (1376, 512, 6)]):
        host, layers = [], []
        for i, (N, K, r) in enumerate(shapes_r):
            L = synth.make_layer(N, K, M=M, seed=[98, M, i, N])
            lay = mq.prepare_layer(dev(L["parent"]), dev(L["scales"]), dev(L["zeros"]), r)
            lay.update(x=xd, y=torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV))    # one x for all
            layers.append(lay)
            host.append(dict(L, x=x, r=r))
        mq.mq_linear_stack(mq.mq_stack_plan(layers, M))
        torch.cuda.synchronize()
        for i, (lay, ref) in enumerate(zip(layers, oracle.linear_stack(host, C, 128))):
            check_y(lay["y"], ref, f"shared input M={M} layer {i}", host[i], host[i]["r"])


@pytest.mark.parametrize("M", [1, 3])
def test_stack_shared_input_fusions_at_llama2_7b_size_sampled_rows(M):
    # the real q/k/v and gate/up launches of a Llama-2-7B block: more workgroups than the device holds at one time
    # unless the plan shrinks the launch shape (waves per workgroup, then K slices), which is what runs here
    x = synth.make_x(M, 4096, [97, M])
    xd = dev(x)
    for shapes_r in ([(4096, 4096, 3), (4096, 4096, 4), (4096, 4096, 8)], [(11008, 4096, 6), (11008, 4096, 2)]):
        host, layers = [], []
        for i, (N, K, r) in enumerate(shapes_r):
            L = synth.make_layer_device(N, K, M, seed=970 + 10 * M + i, device=DEV)
            lay = mq.prepare_layer(L["parent"], L["scales"], L["zeros"], r)
            lay.update(x=xd, y=torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV))
            layers.append(lay)
            host.append((L, N, r))
        plan = mq.mq_stack_plan(layers, M)
        for rep in range(2):                                     # counters reset themselves
            for lay in layers:
                lay["y"].fill_(float("nan"))
            mq.mq_linear_stack(plan)
            torch.cuda.synchronize()
            for i, (lay, (L, N, r)) in enumerate(zip(layers, host)):
                assert torch.isfinite(lay["y"]).all()
                rows = np.unique(np.concatenate([[0, 63, 64, N - 1], np.random.default_rng([97, i]).integers(0, N, 124)]))
                ridx = torch.from_numpy(rows).to(DEV)
                ref = oracle.linear(x, L["parent"][ridx].cpu().numpy(), L["scales"][ridx].cpu().numpy(),
                                    L["zeros"][ridx].cpu().numpy(), C, r, 128)
                check_y(lay["y"][:, ridx], ref, f"7B-size shared input M={M} layer {i} r={r} rep {rep}")


# ------------------------------------------------------------------ boundary conventions
@pytest.mark.parametrize("shape_m_r", [(512, 512, 1, 4), (200, 1280, 3, 3), (130, 384, 8, 6), (320, 640, 40, 2), (1, 256, 1, 8)])
def test_linear_plain_on_row_major_scales_and_zeros(shape_m_r):
    # the call shape of the paper's kernel interface: the quantiser's own [N, K/128] arrays go straight in
    N, K, M, r = shape_m_r
    L = synth.make_layer(N, K, M=M, seed=[99, N, K, M])
    packed = mq.mq_slice_pack(dev(L["parent"]), C, r)
    ws = torch.empty(mq.mq_linear_plain_workspace_bytes(M, N, K, r), dtype=torch.uint8, device=DEV)
    mq.mq_workspace_init(ws)
    for _ in range(2):                                           # the workspace is reusable
        y = mq.mq_linear_plain(dev(L["x"]), packed, dev(L["scales"]), dev(L["zeros"]), N, K, r, 128, ws)
        torch.cuda.synchronize()
        check_layer(y, L, r, f"plain {shape_m_r}")
    st, zt = mq.mq_pack_meta(dev(L["scales"]), dev(L["zeros"]), K)
    y2 = mq.mq_linear(dev(L["x"]), packed, st, zt, N, K, r, 128, mq.new_workspace(M, N, K, r))
    assert torch.equal(y, y2)                                    # the same kernels on the same tiles


def test_stack_replanned_in_the_same_workspace_and_host_arrays_reused_at_once():
    # the plan header lives with the caller: planning again into the same device workspace simply replaces it, and
    # the host layer table may be overwritten as soon as mq_stack_plan has returned (nothing is waited for)
    hostA, layersA = _stack([(256, 512, 2), (200, 1280, 3), (64, 128, 8), (1024, 1024, 3)], M=2, seed=101)
    hostB, layersB = _stack([(130, 384, 4), (512, 256, 6)], M=2, seed=102)
    planA = mq.mq_stack_plan(layersA, 2)
    mq.mq_linear_stack(planA)
    torch.cuda.synchronize()
    for i, (lay, L) in enumerate(zip(layersA, hostA)):
        check_layer(lay["y"], L, L["r"], f"first plan layer {i}")
    planB = mq.mq_stack_plan(layersB, 2, ws=planA.ws)            # same address, another stack
    mq.mq_linear_stack(planB)
    torch.cuda.synchronize()
    for i, (lay, L) in enumerate(zip(layersB, hostB)):
        check_layer(lay["y"], L, L["r"], f"second plan layer {i}")
    # many stacks planned back to back from ONE host array that is rewritten between the calls
    import ctypes
    n = 40
    arr = (mq.MqLayer * n)()
    handles, wss, ys = [], [], []
    base = layersA[1]
    for rep in range(3):
        for i in range(n):
            y = torch.full((2, base["N"]), float("nan"), dtype=torch.float16, device=DEV)
            ys.append(y)
            arr[i] = mq.MqLayer(base["packed_W"].data_ptr(), base["scales_t"].data_ptr(), base["zeros_t"].data_ptr(),
                                base["x"].data_ptr(), y.data_ptr(), base["N"], base["K"], base["r"], 128, 0, 0)
        nbytes = mq.lib().mq_stack_workspace_bytes(ctypes.cast(arr, ctypes.c_void_p), n, 2)
        ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
        h = mq.MqPlan()
        st = mq.lib().mq_stack_plan(ctypes.cast(arr, ctypes.c_void_p), n, 2, ws.data_ptr(), nbytes, ctypes.byref(h),
                                    ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        assert st == 0
        ctypes.memset(arr, 0xFF, ctypes.sizeof(arr))             # the table is gone before anything has run
        handles.append(h)
        wss.append(ws)
    for h in handles:
        assert mq.lib().mq_linear_stack(ctypes.byref(h), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)) == 0
    torch.cuda.synchronize()
    for y in ys:
        assert torch.equal(y, ys[0])
    check_layer(ys[0], hostA[1], hostA[1]["r"], "stack of 40 from a rewritten host table")


def test_stack_plan_and_run_inside_a_hip_graph():
    # neither call copies, synchronises or allocates: both can be recorded, and every replay gives the eager bits
    host, layers = _stack([(256, 512, 2), (200, 1280, 3), (64, 128, 8), (512, 256, 6)], M=1, seed=103)
    eager = mq.mq_stack_plan(layers, 1)
    mq.mq_linear_stack(eager)
    torch.cuda.synchronize()
    want = [lay["y"].clone() for lay in layers]
    ws = torch.empty_like(eager.ws)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            plan = mq.mq_stack_plan(layers, 1, ws=ws, stream=side)
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


def test_read_probe_xors_every_word_once():
    rng = np.random.default_rng(120)
    for nbytes in (16, 1024, 8 * 64 * 16 * 3 + 48, 5_000_000 // 16 * 16):
        a = rng.integers(0, 256, nbytes, dtype=np.uint8)
        out = torch.zeros(1, dtype=torch.int32, device=DEV)
        mq.mq_read_probe(dev(a), out)
        torch.cuda.synchronize()
        want = np.bitwise_xor.reduce(a.view(np.uint32))
        assert np.uint32(out.cpu().numpy().view(np.uint32)[0]) == want, nbytes


# ------------------------------------------------------------------ symmetric layers (no zero-offset array)
@pytest.mark.parametrize("r", WIDTHS)
@pytest.mark.parametrize("shape_m", [(200, 768, 1), (130, 384, 3), (512, 4096, 4), (257, 1280, 8), (448, 2048, 16),
                                     (320, 640, 40), (700, 1152, 200), (1, 256, 1),
                                     # more than 1024 tiles: the constant lines a symmetric layer reads are used many times over
                                     (2304, 4096, 1), (2304, 4096, 8), (2240, 4224, 24)])
def test_symmetric_layer_without_zero_offsets(r, shape_m):
    # zeros_t = NULL means every zero-offset is 128 (the paper's own setting): the oracle gets an array of 128s,
    # and the library's result equals, bit for bit, what it computes from such an array
    N, K, M = shape_m
    L = synth.make_layer(N, K, M=M, seed=[130, N, K, M])
    L["zeros"] = np.full_like(L["zeros"], 128.0)
    lay = mq.prepare_layer(dev(L["parent"]), dev(L["scales"]), None, r)
    assert lay["zeros_t"] is None
    x = dev(L["x"])
    ws = mq.new_workspace(M, N, K, r)
    y = mq.mq_linear(x, lay["packed_W"], lay["scales_t"], None, N, K, r, 128, ws)
    torch.cuda.synchronize()
    check_layer(y, L, r, f"symmetric {shape_m} r={r}")
    full = mq.prepare_layer(dev(L["parent"]), dev(L["scales"]), dev(L["zeros"]), r)
    y2 = mq.mq_linear(x, full["packed_W"], full["scales_t"], full["zeros_t"], N, K, r, 128, ws)
    assert torch.equal(y, y2)


@pytest.mark.parametrize("M", [1, 8, 40])
def test_symmetric_stack_from_parent_and_plain(M):
    shapes_r = [(256, 512, 2), (64, 128, 8), (200, 1280, 3), (512, 256, 6), (130, 384, 4), (1024, 1024, 3)]
    host, layers = [], []
    for i, (N, K, r) in enumerate(shapes_r):
        L = synth.make_layer(N, K, M=M, seed=[131, i, N, K])
        L["zeros"] = np.full_like(L["zeros"], 128.0)
        sym = i % 2 == 0                                   # symmetric and asymmetric layers in one stack
        lay = mq.prepare_layer(dev(L["parent"]), dev(L["scales"]), None if sym else dev(L["zeros"]), r)
        lay.update(x=dev(L["x"]), y=torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV))
        host.append(dict(L, r=r))
        layers.append(lay)
    plan = mq.mq_stack_plan(layers, M)
    mq.mq_linear_stack(plan)
    torch.cuda.synchronize()
    for i, (lay, L) in enumerate(zip(layers, host)):
        check_layer(lay["y"], L, L["r"], f"symmetric stack M={M} layer {i}")
    L = host[2]
    N, K = L["parent"].shape
    packed = mq.mq_slice_pack(dev(L["parent"]), C, 3)
    ws = torch.empty(mq.mq_linear_plain_workspace_bytes(M, N, K, 3), dtype=torch.uint8, device=DEV)
    mq.mq_workspace_init(ws)
    y = mq.mq_linear_plain(dev(L["x"]), packed, dev(L["scales"]), None, N, K, 3, 128, ws)
    check_layer(y, L, 3, f"symmetric plain M={M}")
    if M <= 4:
        p8 = mq.mq_pack(dev(L["parent"]), C, 8)
        st, _ = mq.mq_pack_meta(dev(L["scales"]), None, K)
        y = mq.mq_linear_from_parent(dev(L["x"]), p8, st, None, N, K, 3, 128, mq.new_workspace(M, N, K, 8))
        check_layer(y, L, 3, f"symmetric from parent M={M}")


# ------------------------------------------------------------------ bf16 activations and outputs
def _bf16_round(a):
    """float64 array -> nearest-even bfloat16 values, as float64"""
    b = np.asarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    b = (b + 0x7FFF + ((b >> 16) & 1)) >> 16 << 16
    return b.astype(np.uint32).view(np.float32).astype(np.float64)


@pytest.mark.parametrize("r", WIDTHS)
@pytest.mark.parametrize("shape_m", [(200, 768, 1), (130, 384, 3), (512, 2048, 4), (257, 1280, 8), (448, 2048, 16),
                                     (320, 640, 40), (700, 1152, 200)])
def test_bf16_activations_and_outputs(r, shape_m):
    N, K, M = shape_m
    L = synth.make_layer(N, K, M=M, seed=[140, N, K, M])
    xb = torch.from_numpy(L["x"].astype(np.float32)).to(torch.bfloat16)         # bf16 activations (rounded once, here)
    Lb = dict(L, x=xb.to(torch.float16).numpy())                                # the same values: all inside the fp16 range
    assert np.array_equal(Lb["x"].astype(np.float32), xb.float().numpy())
    lay = mq.prepare_layer(dev(L["parent"]), dev(L["scales"]), dev(L["zeros"]), r)
    ws = mq.new_workspace(M, N, K, r)
    # bf16 in, fp16 out (a stack of one layer with MQ_X_BF16): the fp16 bar, and the bits of the same values given as fp16
    y16 = torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV)
    plan = mq.mq_stack_plan([dict(lay, x=xb.to(DEV), y=y16, flags=mq.MQ_X_BF16)], M)
    mq.mq_linear_stack(plan)
    torch.cuda.synchronize()
    check_layer(y16, Lb, r, f"bf16 x {shape_m} r={r}")
    y16b = torch.empty_like(y16)
    mq.mq_linear_stack(mq.mq_stack_plan([dict(lay, x=dev(Lb["x"]), y=y16b)], M))
    torch.cuda.synchronize()
    assert torch.equal(y16, y16b)
    # bf16 in, bf16 out: one bf16 rounding of the fp32 sums
    yb = mq.mq_linear_bf16(xb.to(DEV), lay["packed_W"], lay["scales_t"], lay["zeros_t"], N, K, r, 128, ws)
    torch.cuda.synchronize()
    assert yb.dtype == torch.bfloat16 and torch.isfinite(yb).all()
    ref = oracle.linear(Lb["x"], L["parent"], L["scales"], L["zeros"], C, r, 128)
    got = yb.float().cpu().numpy().astype(np.float64)
    # within one bf16 spacing of the exact result (half a spacing from rounding, the rest from the fp32 sums), and
    # exactly the rounding of a value within the fp16-output bar
    assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 3e-3), f"bf16 y {shape_m} r={r}"
    assert np.linalg.norm(got - ref) <= 2.5e-3 * np.linalg.norm(ref)
    assert np.array_equal(got, _bf16_round(got))


@pytest.mark.parametrize("M", [2, 8, 40, 100])
def test_bf16_flags_in_a_mixed_stack(M):
    # vector ALUs, narrow matrix-core kernel, wide kernel with two workgroups per compute unit and with one
    shapes_r = [(256, 512, 2), (64, 128, 8), (200, 1280, 3), (512, 256, 6)]
    host, layers = [], []
    for i, (N, K, r) in enumerate(shapes_r):
        L = synth.make_layer(N, K, M=M, seed=[141, i])
        xb = torch.from_numpy(L["x"].astype(np.float32)).to(torch.bfloat16)
        flags = (0, mq.MQ_X_BF16, mq.MQ_Y_BF16, mq.MQ_X_BF16 | mq.MQ_Y_BF16)[i]
        lay = mq.prepare_layer(dev(L["parent"]), dev(L["scales"]), dev(L["zeros"]), r)
        xin = xb.to(DEV) if flags & mq.MQ_X_BF16 else dev(L["x"])
        y = torch.full((M, N), float("nan"), dtype=torch.bfloat16 if flags & mq.MQ_Y_BF16 else torch.float16, device=DEV)
        lay.update(x=xin, y=y, flags=flags)
        layers.append(lay)
        host.append(dict(L, x=xb.to(torch.float16).numpy() if flags & mq.MQ_X_BF16 else L["x"], r=r, flags=flags))
    mq.mq_linear_stack(mq.mq_stack_plan(layers, M))
    torch.cuda.synchronize()
    for i, (lay, L) in enumerate(zip(layers, host)):
        ref = oracle.linear(L["x"], L["parent"], L["scales"], L["zeros"], C, L["r"], 128)
        got = lay["y"].float().cpu().numpy().astype(np.float64)
        if L["flags"] & mq.MQ_Y_BF16:
            assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 3e-3), (M, i)
        else:
            check_layer(lay["y"], L, L["r"], f"mixed flags M={M} layer {i}")
