"""CPU-only checks: the C-ABI library loads and exports everything include/mq.h
declares, host-side size arithmetic, every argument-validation path (which
returns before anything is enqueued, so no GPU is touched), the synthetic input
recipe, and the reference layout used by the GPU pack test."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2602_03537_amd as mq
from paper_2602_03537_amd import synth
from layout_ref import FIELDS, pack_ref, meta_ref

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "mq.h")
FAKE = 0x10000  # a non-null, 256-byte aligned "device pointer" that is never dereferenced


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mq_[a-z_]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    L = mq.lib()
    names = declared_symbols()
    assert {"mq_pack", "mq_slice_codes", "mq_linear", "mq_linear_stack", "mq_unpack", "mq_pack_meta",
            "mq_stack_plan", "mq_workspace_init"} <= set(names)
    for n in names:
        assert hasattr(L, n), n
    assert mq.mq_version() >= 1


def test_binding_exposes_the_same_names():
    for n in declared_symbols():
        assert hasattr(mq, n), n


def test_status_strings():
    for code, name in mq.STATUS.items():
        assert mq.mq_status_str(code) not in ("", "unknown status"), name
    assert mq.mq_status_str(99) == "unknown status"


@pytest.mark.parametrize("r", [2, 3, 4, 6, 8])
def test_packed_bytes_is_exactly_r_bits_per_weight(r):
    assert mq.mq_packed_bytes(4096, 4096, r) == 4096 * 4096 * r // 8
    assert mq.mq_packed_bytes(11008, 4096, r) == 11008 * 4096 * r // 8
    assert mq.mq_packed_bytes(100, 256, r) == 128 * 256 * r // 8       # rows pad to 64
    assert mq.mq_packed_bytes(1, 128, r) == 64 * 128 * r // 8


def test_size_queries_reject_bad_arguments():
    assert mq.mq_packed_bytes(64, 128, 5) == 0
    assert mq.mq_packed_bytes(64, 100, 4) == 0
    assert mq.mq_packed_bytes(0, 128, 4) == 0
    assert mq.mq_meta_bytes(64, 256, 64) == 0
    assert mq.mq_meta_bytes(100, 256, 128) == 128 * 2 * 2
    assert mq.mq_workspace_bytes(0, 64, 128, 4) == 0
    assert mq.mq_workspace_bytes(257, 64, 128, 4) == 0
    assert mq.mq_workspace_bytes(1, 4096, 4096, 4) > 0
    assert mq.mq_workspace_bytes(2, 4096, 4096, 4) >= mq.mq_workspace_bytes(1, 4096, 4096, 4)
    assert mq.mq_workspace_bytes(64, 4096, 4096, 4) > mq.mq_workspace_bytes(16, 4096, 4096, 4)   # prepared activations


def _st(name):
    return {v: k for k, v in mq.STATUS.items()}[name]


def test_slice_validation():
    L = mq.lib()
    assert L.mq_slice_codes(None, 16, 8, 4, FAKE, None) == _st("MQ_ERR_NULL")
    assert L.mq_slice_codes(FAKE, 16, 8, 4, None, None) == _st("MQ_ERR_NULL")
    assert L.mq_slice_codes(None, 0, 8, 4, None, None) == _st("MQ_OK")        # empty input: no-op
    for c, r in [(8, 0), (8, 9), (9, 4), (4, 5), (0, 0)]:
        assert L.mq_slice_codes(FAKE, 16, c, r, FAKE, None) == _st("MQ_ERR_BAD_R")
    assert L.mq_slice_codes(FAKE, -1, 8, 4, FAKE, None) == _st("MQ_ERR_BAD_SHAPE")


def test_pack_validation():
    L = mq.lib()
    big = 1 << 30
    assert L.mq_pack(None, 64, 128, 8, 4, FAKE, big, None) == _st("MQ_ERR_NULL")
    assert L.mq_pack(FAKE, 64, 128, 8, 4, None, big, None) == _st("MQ_ERR_NULL")
    assert L.mq_pack(FAKE, 64, 128, 8, 5, FAKE, big, None) == _st("MQ_ERR_BAD_R")
    assert L.mq_pack(FAKE, 64, 128, 8, 1, FAKE, big, None) == _st("MQ_ERR_BAD_R")
    assert L.mq_pack(FAKE, 64, 128, 7, 4, FAKE, big, None) == _st("MQ_ERR_BAD_R")
    assert L.mq_pack(FAKE, 0, 128, 8, 4, FAKE, big, None) == _st("MQ_ERR_BAD_SHAPE")
    assert L.mq_pack(FAKE, 64, 100, 8, 4, FAKE, big, None) == _st("MQ_ERR_BAD_GROUP")
    assert L.mq_pack(FAKE, 64, 128, 8, 4, FAKE + 4, big, None) == _st("MQ_ERR_ALIGN")
    assert L.mq_pack(FAKE, 64, 128, 8, 4, FAKE, 64 * 128 // 2 - 1, None) == _st("MQ_ERR_BUF_TOO_SMALL")
    assert L.mq_unpack(None, 64, 128, 8, 4, FAKE, None) == _st("MQ_ERR_NULL")
    assert L.mq_unpack(FAKE, 64, 128, 8, 7, FAKE, None) == _st("MQ_ERR_BAD_R")
    assert L.mq_unpack(FAKE + 8, 64, 128, 8, 4, FAKE, None) == _st("MQ_ERR_ALIGN")
    assert L.mq_pack_meta(FAKE, FAKE, 64, 256, 64, FAKE, FAKE, big, None) == _st("MQ_ERR_BAD_GROUP")
    assert L.mq_pack_meta(FAKE, None, 64, 256, 128, FAKE, FAKE, big, None) == _st("MQ_ERR_NULL")    # zeros without ...
    assert L.mq_pack_meta(FAKE, FAKE, 64, 256, 128, FAKE, None, big, None) == _st("MQ_ERR_NULL")    # ... or with only one side
    assert L.mq_pack_meta(FAKE, None, 64, 256, 128, FAKE, None, 10, None) == _st("MQ_ERR_BUF_TOO_SMALL")   # symmetric: judged on
    assert L.mq_pack_meta(FAKE, FAKE, 64, 256, 128, FAKE, FAKE, 10, None) == _st("MQ_ERR_BUF_TOO_SMALL")
    assert L.mq_pack_meta(FAKE, FAKE + 1, 64, 256, 128, FAKE, FAKE, big, None) == _st("MQ_ERR_ALIGN")


def test_reslice_validation():
    L = mq.lib()
    big = 1 << 30
    for fn in (L.mq_slice_pack, L.mq_reslice):
        assert fn(None, 64, 128, 8, 4, FAKE + (1 << 20), big, None) == _st("MQ_ERR_NULL")
        assert fn(FAKE, 64, 128, 8, 4, None, big, None) == _st("MQ_ERR_NULL")
        assert fn(FAKE, 64, 128, 8, 5, FAKE + (1 << 20), big, None) == _st("MQ_ERR_BAD_R")
        assert fn(FAKE, 64, 128, 7, 4, FAKE + (1 << 20), big, None) == _st("MQ_ERR_BAD_R")
        assert fn(FAKE, 0, 128, 8, 4, FAKE + (1 << 20), big, None) == _st("MQ_ERR_BAD_SHAPE")
        assert fn(FAKE, 64, 100, 8, 4, FAKE + (1 << 20), big, None) == _st("MQ_ERR_BAD_GROUP")
        assert fn(FAKE, 64, 128, 8, 4, FAKE + (1 << 20) + 4, big, None) == _st("MQ_ERR_ALIGN")
        assert fn(FAKE, 64, 128, 8, 4, FAKE + (1 << 20), 64 * 128 // 2 - 1, None) == _st("MQ_ERR_BUF_TOO_SMALL")
    assert L.mq_reslice(FAKE + 8, 64, 128, 8, 4, FAKE + (1 << 20), big, None) == _st("MQ_ERR_ALIGN")
    # output overlapping the resident parent (8192 bytes here) is refused, adjacent buffers are not an overlap
    assert L.mq_reslice(FAKE, 64, 128, 8, 4, FAKE, big, None) == _st("MQ_ERR_UNSUPPORTED")
    assert L.mq_reslice(FAKE, 64, 128, 8, 4, FAKE + 8176, big, None) == _st("MQ_ERR_UNSUPPORTED")
    assert L.mq_reslice(FAKE + 4096, 64, 128, 8, 4, FAKE + 16, big, None) == _st("MQ_ERR_UNSUPPORTED")


def test_reslice_many_validation():
    # every call below fails validation: nothing is ever launched with these fake pointers
    L = mq.lib()
    jobs = (mq.MqResliceJob * 2)()
    jobs[0] = mq.MqResliceJob(FAKE, FAKE + (1 << 20), 1 << 30, 64, 128, 4, 0)
    jobs[1] = mq.MqResliceJob(FAKE, FAKE + (2 << 20), 1 << 30, 64, 128, 3, 0)
    p = ctypes.cast(jobs, ctypes.c_void_p)
    assert L.mq_reslice_many(None, 2, 8, None) == _st("MQ_ERR_NULL")
    assert L.mq_reslice_many(p, 0, 8, None) == _st("MQ_ERR_BAD_SHAPE")
    assert L.mq_reslice_many(p, 2, 7, None) == _st("MQ_ERR_BAD_R")
    jobs[1].r = 5
    assert L.mq_reslice_many(p, 2, 8, None) == _st("MQ_ERR_BAD_R")
    jobs[1].r = 3
    jobs[1].packed = None
    assert L.mq_reslice_many(p, 2, 8, None) == _st("MQ_ERR_NULL")
    jobs[1].packed = FAKE + (2 << 20) + 8
    assert L.mq_reslice_many(p, 2, 8, None) == _st("MQ_ERR_ALIGN")
    jobs[1].packed = FAKE + (2 << 20)
    jobs[1].packed_bytes = 100
    assert L.mq_reslice_many(p, 2, 8, None) == _st("MQ_ERR_BUF_TOO_SMALL")
    jobs[1].packed_bytes = 1 << 30
    jobs[1].K = 100
    assert L.mq_reslice_many(p, 2, 8, None) == _st("MQ_ERR_BAD_GROUP")
    jobs[1].K = 128
    jobs[1].packed = FAKE + 4096                    # inside its own parent
    assert L.mq_reslice_many(p, 2, 8, None) == _st("MQ_ERR_UNSUPPORTED")


def test_linear_from_parent_validation():
    # every call below fails validation: nothing is ever launched with these fake pointers
    L = mq.lib()
    args = lambda **kw: _linear_args(**kw)  # noqa: E731
    assert L.mq_linear_from_parent(*args(M=5)) == _st("MQ_ERR_UNSUPPORTED")
    assert L.mq_linear_from_parent(*args(M=256)) == _st("MQ_ERR_UNSUPPORTED")
    assert L.mq_linear_from_parent(*args(M=257)) == _st("MQ_ERR_BAD_SHAPE")
    assert L.mq_linear_from_parent(*args(r=5)) == _st("MQ_ERR_BAD_R")
    assert L.mq_linear_from_parent(*args(W=None)) == _st("MQ_ERR_NULL")
    assert L.mq_linear_from_parent(*args(W=FAKE + 8)) == _st("MQ_ERR_ALIGN")
    # the workspace is that of the 8-bit layout whatever r is
    need = L.mq_workspace_bytes(1, 64, 128, 8)
    assert L.mq_linear_from_parent(*args(r=2, wsb=need - 1)) == _st("MQ_ERR_BUF_TOO_SMALL")


def test_quant_validation():
    # every call below fails validation: nothing is ever launched with these fake pointers
    L = mq.lib()
    lam = (ctypes.c_float * 8)(0, 0, 1, 1, 0, 0, 0, 1)
    lp = ctypes.cast(lam, ctypes.c_void_p)

    def call(W=FAKE, ldw=128, N=64, ncols=128, col0=0, s=FAKE, z=FAKE, K=128, group=128, c=8, lam=lp, Q=FAKE, ldq=128):
        return L.mq_quant_matgptq(W, ldw, N, ncols, col0, s, z, K, group, c, lam, Q, ldq, None)
    for k in ("W", "s", "z", "lam", "Q"):
        assert call(**{k: None}) == _st("MQ_ERR_NULL"), k
    assert call(c=7) == _st("MQ_ERR_BAD_R")
    for bad in ((0,) * 8, (0, 0, -1, 0, 0, 0, 0, 1), (0, 0, float("nan"), 0, 0, 0, 0, 1), (float("inf"),) * 8):
        arr = (ctypes.c_float * 8)(*bad)
        assert call(lam=ctypes.cast(arr, ctypes.c_void_p)) == _st("MQ_ERR_BAD_R"), bad
    assert call(N=0) == _st("MQ_ERR_BAD_SHAPE")
    assert call(K=100) == _st("MQ_ERR_BAD_GROUP")
    assert call(group=64) == _st("MQ_ERR_BAD_GROUP")
    assert call(ncols=0) == _st("MQ_ERR_BAD_SHAPE")
    assert call(ncols=8, col0=124) == _st("MQ_ERR_BAD_SHAPE")
    assert call(col0=-4, ncols=4) == _st("MQ_ERR_BAD_SHAPE")
    assert call(ldw=100) == _st("MQ_ERR_BAD_SHAPE")
    assert call(ldq=100) == _st("MQ_ERR_BAD_SHAPE")
    assert call(W=FAKE + 2) == _st("MQ_ERR_ALIGN")
    assert call(s=FAKE + 1) == _st("MQ_ERR_ALIGN")


def test_matgptq_loop_validation():
    # every call below fails validation: nothing is ever launched with these fake pointers
    L = mq.lib()
    lam = (ctypes.c_float * 8)(0, 0, 1, 1, 0, 0, 0, 1)
    lp = ctypes.cast(lam, ctypes.c_void_p)
    assert L.mq_matgptq_workspace_bytes(4096, 128) == 4096 * 128 * 4
    assert L.mq_matgptq_workspace_bytes(4096, 48) == 0 and L.mq_matgptq_workspace_bytes(0, 128) == 0

    def call(W=FAKE, ldw=256, N=64, K=256, U=FAKE, ldu=256, s=FAKE, z=FAKE, group=128, c=8, lam=lp, block=128, Q=FAKE,
             ldq=256, ws=FAKE, wsb=1 << 30):
        return L.mq_matgptq_quantize(W, ldw, N, K, U, ldu, s, z, group, c, lam, block, Q, ldq, ws, wsb, None)
    for k in ("W", "U", "s", "z", "lam", "Q", "ws"):
        assert call(**{k: None}) == _st("MQ_ERR_NULL"), k
    assert call(c=7) == _st("MQ_ERR_BAD_R")
    zero = (ctypes.c_float * 8)()
    assert call(lam=ctypes.cast(zero, ctypes.c_void_p)) == _st("MQ_ERR_BAD_R")
    assert call(block=48) == _st("MQ_ERR_BAD_SHAPE")
    assert call(K=200) == _st("MQ_ERR_BAD_GROUP")
    assert call(ldw=128) == _st("MQ_ERR_BAD_SHAPE")
    assert call(ldu=128) == _st("MQ_ERR_BAD_SHAPE")
    assert call(ldq=255) == _st("MQ_ERR_BAD_SHAPE")
    assert call(U=FAKE + 2) == _st("MQ_ERR_ALIGN")
    assert call(wsb=64 * 128 * 4 - 1) == _st("MQ_ERR_BUF_TOO_SMALL")


def _linear_args(**kw):
    a = dict(x=FAKE, M=1, W=FAKE, st=FAKE, zt=FAKE, N=64, K=128, r=4, group=128, y=FAKE, ws=FAKE, wsb=1 << 30)
    a.update(kw)
    return (a["x"], a["M"], a["W"], a["st"], a["zt"], a["N"], a["K"], a["r"], a["group"], a["y"], a["ws"], a["wsb"], None)


def _linear(L, **kw):
    a = dict(x=FAKE, M=1, W=FAKE, st=FAKE, zt=FAKE, N=64, K=128, r=4, group=128, y=FAKE, ws=FAKE, wsb=1 << 30)
    a.update(kw)
    return L.mq_linear(a["x"], a["M"], a["W"], a["st"], a["zt"], a["N"], a["K"], a["r"], a["group"], a["y"],
                       a["ws"], a["wsb"], None)


def test_linear_validation():
    L = mq.lib()
    for k in ("x", "W", "st", "y", "ws"):
        assert _linear(L, **{k: None}) == _st("MQ_ERR_NULL"), k
    # zeros_t == NULL is the symmetric layer (every zero-offset 128), not an error: such a call is judged like any
    # other (here it stops at the next check, the misaligned workspace, so nothing is launched)
    assert _linear(L, zt=None, ws=FAKE + 64) == _st("MQ_ERR_ALIGN")
    assert _linear(L, r=5) == _st("MQ_ERR_BAD_R")
    assert _linear(L, r=1) == _st("MQ_ERR_BAD_R")
    assert _linear(L, M=0) == _st("MQ_ERR_BAD_SHAPE")
    assert _linear(L, M=257) == _st("MQ_ERR_BAD_SHAPE")
    assert _linear(L, N=0) == _st("MQ_ERR_BAD_SHAPE")
    assert _linear(L, K=0) == _st("MQ_ERR_BAD_SHAPE")
    assert _linear(L, K=192) == _st("MQ_ERR_BAD_GROUP")
    assert _linear(L, group=64) == _st("MQ_ERR_BAD_GROUP")
    assert _linear(L, W=FAKE + 8) == _st("MQ_ERR_ALIGN")
    assert _linear(L, x=FAKE + 2) == _st("MQ_ERR_ALIGN")
    assert _linear(L, ws=FAKE + 64) == _st("MQ_ERR_ALIGN")
    assert _linear(L, wsb=128) == _st("MQ_ERR_BUF_TOO_SMALL")


def test_workspace_and_stack_validation():
    L = mq.lib()
    assert L.mq_workspace_init(None, 1024, None) == _st("MQ_ERR_NULL")
    assert L.mq_workspace_init(FAKE + 16, 1024, None) == _st("MQ_ERR_ALIGN")
    assert L.mq_workspace_init(FAKE, 8, None) == _st("MQ_ERR_BUF_TOO_SMALL")
    lay = (mq.MqLayer * 2)()
    lay[0] = mq.MqLayer(FAKE, FAKE, FAKE, FAKE, FAKE, 64, 128, 4, 128)
    lay[1] = mq.MqLayer(FAKE, FAKE, FAKE, FAKE, FAKE, 64, 128, 3, 128)
    p = ctypes.cast(lay, ctypes.c_void_p)
    need = L.mq_stack_workspace_bytes(p, 2, 1)
    assert need > 0
    assert L.mq_stack_workspace_bytes(p, 0, 1) == 0
    assert L.mq_stack_workspace_bytes(None, 2, 1) == 0
    h = mq.MqPlan()
    hp = ctypes.byref(h)
    assert L.mq_stack_plan(None, 2, 1, FAKE, need, hp, None) == _st("MQ_ERR_NULL")
    assert L.mq_stack_plan(p, 2, 1, None, need, hp, None) == _st("MQ_ERR_NULL")
    assert L.mq_stack_plan(p, 2, 1, FAKE, need, None, None) == _st("MQ_ERR_NULL")
    assert L.mq_stack_plan(p, 0, 1, FAKE, need, hp, None) == _st("MQ_ERR_BAD_SHAPE")
    assert L.mq_stack_plan(p, 2, 1, FAKE + 32, need, hp, None) == _st("MQ_ERR_ALIGN")
    assert L.mq_stack_plan(p, 2, 1, FAKE, need - 1, hp, None) == _st("MQ_ERR_BUF_TOO_SMALL")
    lay[1].r = 5
    assert L.mq_stack_plan(p, 2, 1, FAKE, need, hp, None) == _st("MQ_ERR_BAD_R")
    lay[1].r = 3
    lay[1].x = None
    assert L.mq_stack_plan(p, 2, 1, FAKE, need, hp, None) == _st("MQ_ERR_NULL")
    assert L.mq_linear_stack(None, None) == _st("MQ_ERR_NULL")
    lay[1].x = FAKE
    lay[1].from_parent = 1                        # layers of one stack must agree
    assert L.mq_stack_plan(p, 2, 1, FAKE, need, hp, None) == _st("MQ_ERR_UNSUPPORTED")
    lay[0].from_parent = 1
    assert L.mq_stack_plan(p, 2, 8, FAKE, 1 << 40, hp, None) == _st("MQ_ERR_UNSUPPORTED")   # batch above the ALU path
    lay[0].from_parent = lay[1].from_parent = 2
    assert L.mq_stack_plan(p, 2, 1, FAKE, need, hp, None) == _st("MQ_ERR_UNSUPPORTED")
    lay[0].from_parent = lay[1].from_parent = 0
    lay[1].flags = 8                              # only MQ_X_BF16 | MQ_Y_BF16 | MQ_X_AFTER_EARLIER are flags
    assert L.mq_stack_plan(p, 2, 1, FAKE, need, hp, None) == _st("MQ_ERR_UNSUPPORTED")
    # a layer that waits for earlier layers: not the first one, not on bf16 activations, only in a stack that is
    # launched for latency (M <= 4, at most 16 layers), never on its own
    lay[1].flags = 0
    lay[0].flags = mq.MQ_X_AFTER_EARLIER
    assert L.mq_stack_plan(p, 2, 1, FAKE, need, hp, None) == _st("MQ_ERR_UNSUPPORTED")
    lay[0].flags = 0
    lay[1].flags = mq.MQ_X_AFTER_EARLIER | mq.MQ_X_BF16
    assert L.mq_stack_plan(p, 2, 1, FAKE, need, hp, None) == _st("MQ_ERR_UNSUPPORTED")
    lay[1].flags = mq.MQ_X_AFTER_EARLIER
    assert L.mq_stack_plan(p, 2, 8, FAKE, 1 << 40, hp, None) == _st("MQ_ERR_UNSUPPORTED")
    assert L.mq_stack_plan(p, 2, 4, FAKE, 1 << 40, hp, None) == _st("MQ_ERR_UNSUPPORTED")   # chained: M <= 3
    many = (mq.MqLayer * 17)()
    for i in range(17):
        many[i] = mq.MqLayer(FAKE, FAKE, FAKE, FAKE, FAKE, 64, 128, 4, 128, 0, mq.MQ_X_AFTER_EARLIER if i == 5 else 0)
    assert L.mq_stack_plan(ctypes.cast(many, ctypes.c_void_p), 17, 1, FAKE, 1 << 40, hp, None) == _st("MQ_ERR_UNSUPPORTED")
    assert L.mq_stack_plan(p, 2, 1, FAKE, need - 1, hp, None) == _st("MQ_ERR_BUF_TOO_SMALL")   # a valid chain: judged on
    lay[1].flags = mq.MQ_X_BF16 | mq.MQ_Y_BF16
    assert L.mq_stack_plan(p, 2, 1, FAKE, need - 1, hp, None) == _st("MQ_ERR_BUF_TOO_SMALL")   # valid flags: judged on
    assert L.mq_linear_bf16(None, 1, FAKE, FAKE, FAKE, 64, 128, 4, 128, FAKE, FAKE, 1 << 30, None) == _st("MQ_ERR_NULL")
    assert L.mq_linear_bf16(FAKE, 1, FAKE, FAKE, FAKE, 64, 128, 5, 128, FAKE, FAKE, 1 << 30, None) == _st("MQ_ERR_BAD_R")
    assert bytes(h) == bytes(ctypes.sizeof(h))    # a refused plan leaves the caller's header untouched


def test_stack_run_refuses_a_header_that_no_plan_filled():
    # mq_linear_stack takes everything it knows from the caller's host header and checks it before any launch:
    # zeroes, garbage and a copy with one field changed are "not a plan", not a launch on whatever the bytes say
    L = mq.lib()
    h = mq.MqPlan()
    assert L.mq_linear_stack(ctypes.byref(h), None) == _st("MQ_ERR_BAD_SHAPE")
    rng = np.random.default_rng(0)
    for _ in range(20):
        for i in range(272):
            h.opaque[i] = int(rng.integers(0, 1 << 63))
        assert L.mq_linear_stack(ctypes.byref(h), None) == _st("MQ_ERR_BAD_SHAPE")
    h.opaque[0] = 0x4d51504c414e3038              # the right magic alone is not enough
    assert L.mq_linear_stack(ctypes.byref(h), None) == _st("MQ_ERR_BAD_SHAPE")


def test_header_states_the_conventions_the_library_keeps():
    text = " ".join(open(HEADER).read().replace("*", " ").split())
    for phrase in ("never allocates or frees", "never synchronises", "keeps no state of its own",
                   "neither read nor cleared"):
        assert phrase in text, phrase
    # and the sources hold none of the calls that would break them
    csrc = os.path.join(ROOT, "paper_2602_03537_amd", "csrc")
    banned = ("hipMalloc", "hipFree", "hipMemcpy", "hipMemset", "hipStreamSynchronize", "hipDeviceSynchronize",
              "hipGetLastError", "hipEventSynchronize", "unordered_map", "std::map")
    for name in sorted(os.listdir(csrc)):
        if not name.endswith((".hip", ".h")):
            continue
        src = open(os.path.join(csrc, name)).read()
        code = re.sub(r"//[^\n]*|/\*.*?\*/", "", src, flags=re.S)
        for b in banned:
            assert b not in code, (name, b)


def test_slice_rejects_partial_overlap():
    L = mq.lib()
    assert L.mq_slice_codes(FAKE, 100, 8, 4, FAKE + 50, None) == _st("MQ_ERR_UNSUPPORTED")
    assert L.mq_slice_codes(FAKE + 50, 100, 8, 4, FAKE, None) == _st("MQ_ERR_UNSUPPORTED")


def test_linear_plain_validation():
    L = mq.lib()
    need = L.mq_linear_plain_workspace_bytes(1, 64, 128, 4)
    assert need >= L.mq_workspace_bytes(1, 64, 128, 4) + 2 * L.mq_meta_bytes(64, 128, 128)
    assert L.mq_linear_plain_workspace_bytes(1, 64, 100, 4) == 0 and L.mq_linear_plain_workspace_bytes(1, 64, 128, 5) == 0

    def call(x=FAKE, M=1, W=FAKE, s=FAKE, z=FAKE, N=64, K=128, r=4, group=128, y=FAKE, ws=FAKE, wsb=None):
        return L.mq_linear_plain(x, M, W, s, z, N, K, r, group, y, ws, need if wsb is None else wsb, None)
    assert call(s=None) == _st("MQ_ERR_NULL") and call(ws=None) == _st("MQ_ERR_NULL")
    assert call(z=None, wsb=need - 1) == _st("MQ_ERR_BUF_TOO_SMALL")      # zeros == NULL: symmetric layer, judged on
    assert call(x=None) == _st("MQ_ERR_NULL") and call(W=None) == _st("MQ_ERR_NULL") and call(y=None) == _st("MQ_ERR_NULL")
    assert call(r=5) == _st("MQ_ERR_BAD_R")
    assert call(M=0) == _st("MQ_ERR_BAD_SHAPE") and call(M=257) == _st("MQ_ERR_BAD_SHAPE")
    assert call(K=192) == _st("MQ_ERR_BAD_GROUP") and call(group=64) == _st("MQ_ERR_BAD_GROUP")
    assert call(ws=FAKE + 64) == _st("MQ_ERR_ALIGN") and call(W=FAKE + 8) == _st("MQ_ERR_ALIGN")
    assert call(wsb=need - 1) == _st("MQ_ERR_BUF_TOO_SMALL")


# ------------------------------------------------------------ input recipe
def test_parent_quantiser_recipe():
    L = synth.make_layer(96, 512, M=2, seed=0)
    assert L["parent"].dtype == np.uint8 and L["scales"].dtype == np.float16 and L["zeros"].dtype == np.float16
    assert L["parent"].shape == (96, 512) and L["scales"].shape == (96, 4) and L["x"].shape == (2, 512)
    # min-max RTN: every group reaches (within one step) both ends of the code range
    g = L["parent"].reshape(96, 4, 128)
    assert g.min(axis=2).max() <= 1 and g.min(axis=2).min() == 0
    assert g.max(axis=2).min() >= 254
    z = L["zeros"].astype(np.float64)
    assert np.all(z == np.rint(z)) and z.min() >= 0 and z.max() <= 255
    L2 = synth.make_layer(96, 512, M=2, seed=0)
    assert np.array_equal(L["parent"], L2["parent"]) and np.array_equal(L["x"], L2["x"])
    L3 = synth.make_layer(96, 512, M=2, seed=1)
    assert not np.array_equal(L["parent"], L3["parent"])


def test_constant_group_gets_unit_scale():
    W = np.zeros((2, 128), dtype=np.float32)
    q, s, z = synth.quantize_parent(W)
    assert np.all(s == 1.0) and np.all(q == z.astype(np.uint8)[:, :, None].repeat(128, 2).reshape(2, 128))


@pytest.mark.parametrize("target", [3.5, 4.0])
def test_bitwidth_vector_hits_parameter_weighted_mean(target):
    block = synth.LLAMA2_7B_BLOCK if target == 3.5 else synth.LLAMA3_70B_BLOCK
    nl = 32 if target == 3.5 else 80
    sizes = [N * K for (_, _, N, K) in synth.stack_shapes(block, nl)]
    w, mean = synth.draw_bitwidths(sizes, target, seed=0)
    assert len(w) == 7 * nl and set(np.unique(w)) <= {2, 3, 4, 6, 8}
    assert abs(mean - target) <= 0.02
    assert abs(float((w * np.array(sizes)).sum() / np.sum(sizes)) - mean) < 1e-12
    w2, _ = synth.draw_bitwidths(sizes, target, seed=0)
    assert np.array_equal(w, w2)
    assert len(set(w.tolist())) >= 4


# ------------------------------------------------------------ reference layout
@pytest.mark.parametrize("r", [2, 3, 4, 6, 8])
def test_reference_layout_uses_every_bit_exactly_once(r):
    ud, ppu, fields = FIELDS[r]
    assert ppu * 2 * r == ud * 32 and (4 * r) % ud == 0
    used = [0] * ud
    for p, fl in fields.items():
        bits = 0
        for (dw, pos, nb, b0) in fl:
            m = ((1 << nb) - 1) << pos
            assert used[dw] & m == 0
            used[dw] |= m
            cb = ((1 << nb) - 1) << b0
            assert bits & cb == 0
            bits |= cb
        assert bits == (1 << r) - 1
    assert all(u == 0xFFFF for u in used)


@pytest.mark.parametrize("r", [2, 3, 4, 6, 8])
def test_reference_pack_is_injective_and_sized(r):
    rng = np.random.default_rng(r)
    S = (rng.integers(0, 1 << r, (70, 256)).astype(np.uint8) << (8 - r)).astype(np.uint8)
    a = pack_ref(S, r)
    assert a.size == mq.mq_packed_bytes(70, 256, r)
    assert int(np.unpackbits(a).sum()) == int(np.unpackbits((S >> (8 - r)).astype(np.uint8)).sum())
    S2 = S.copy()
    S2[37, 200] ^= 1 << (8 - r)
    b = pack_ref(S2, r)
    assert np.count_nonzero(np.unpackbits(a ^ b)) == 1          # one code bit -> one packed bit


def test_reference_meta_tiling():
    a = np.arange(70 * 3, dtype=np.float16).reshape(70, 3)
    t = meta_ref(a).reshape(2, 3, 64)
    assert t[0, 1, 5] == a[5, 1] and t[1, 2, 5] == a[69, 2] and t[1, 0, 6] == 0
