"""Thin ctypes binding of libmq (include/mq.h).  Argument marshalling only:
PyTorch supplies device memory and streams, every step runs in the library's
HIP kernels.  There is no fallback: if libmq.so is missing, calls raise.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

__all__ = [
    "MqError", "lib", "lib_path", "MQ_ROW_BLOCK", "MQ_GROUP", "MQ_MAX_M", "STATUS",
    "mq_status_str", "mq_version", "mq_packed_bytes", "mq_meta_bytes", "mq_workspace_bytes",
    "mq_workspace_init", "mq_slice_codes", "mq_pack", "mq_unpack", "mq_pack_meta", "mq_linear",
    "mq_slice_pack", "mq_reslice", "mq_reslice_many", "MqResliceJob", "mq_linear_from_parent", "mq_quant_matgptq",
    "mq_matgptq_workspace_bytes", "mq_matgptq_quantize",
    "mq_stack_workspace_bytes", "mq_stack_plan", "mq_linear_stack", "MqLayer", "MqPlan", "StackPlan",
    "mq_read_probe", "mq_linear_bf16", "MQ_X_BF16", "MQ_Y_BF16", "MQ_X_AFTER_EARLIER", "mq_linear_plain", "mq_linear_plain_workspace_bytes", "mq_linear_noalloc", "MQ_NOALLOC_SCRATCH_BYTES",
    "new_workspace", "prepare_layer",
]

MQ_ROW_BLOCK = 64
MQ_GROUP = 128
MQ_MAX_M = 256
MQ_NOALLOC_SCRATCH_BYTES = 8 << 20
MQ_X_BF16 = 1
MQ_Y_BF16 = 2
MQ_X_AFTER_EARLIER = 4
STATUS = {
    0: "MQ_OK", 1: "MQ_ERR_NULL", 2: "MQ_ERR_BAD_R", 3: "MQ_ERR_BAD_SHAPE", 4: "MQ_ERR_BAD_GROUP",
    5: "MQ_ERR_ALIGN", 6: "MQ_ERR_BUF_TOO_SMALL", 7: "MQ_ERR_HIP", 8: "MQ_ERR_UNSUPPORTED",
}

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmq.so")
_lib = None


class MqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {STATUS.get(status, status)} ({mq_status_str(status)})")


class MqLayer(ctypes.Structure):
    """mq_layer of include/mq.h."""
    _fields_ = [
        ("packed_W", ctypes.c_void_p), ("scales_t", ctypes.c_void_p), ("zeros_t", ctypes.c_void_p),
        ("x", ctypes.c_void_p), ("y", ctypes.c_void_p),
        ("N", ctypes.c_int64), ("K", ctypes.c_int64), ("r", ctypes.c_int32), ("group", ctypes.c_int32),
        ("from_parent", ctypes.c_int32), ("flags", ctypes.c_int32),
    ]


class MqPlan(ctypes.Structure):
    """mq_plan of include/mq.h: the host-side header of a planned stack (opaque)."""
    _fields_ = [("opaque", ctypes.c_uint64 * 272)]


class StackPlan:
    """A planned stack as Python holds it: the host header and the device workspace it names (kept alive here)."""
    __slots__ = ("handle", "ws")

    def __init__(self, handle: MqPlan, ws):
        self.handle = handle
        self.ws = ws


class MqResliceJob(ctypes.Structure):
    """mq_reslice_job of include/mq.h."""
    _fields_ = [
        ("packed_parent", ctypes.c_void_p), ("packed", ctypes.c_void_p), ("packed_bytes", ctypes.c_size_t),
        ("N", ctypes.c_int64), ("K", ctypes.c_int64), ("r", ctypes.c_int32), ("reserved", ctypes.c_int32),
    ]


def lib_path() -> str:
    return _LIB_PATH


def lib():
    """The loaded C-ABI library.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2602_03537_amd.build` "
            "(there is no CPU or PyTorch fallback)")
    # PyTorch ships its own copy of the HIP runtime (same soname).  It must be in the
    # process before libmq.so is loaded, so that both use ONE runtime: streams and
    # device pointers made by torch are then valid for the library's launches.
    import torch  # noqa: F401
    L = ctypes.CDLL(_LIB_PATH)
    vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t
    sig = {
        "mq_status_str": (ctypes.c_char_p, [i32]),
        "mq_version": (i32, []),
        "mq_packed_bytes": (sz, [i64, i64, i32]),
        "mq_meta_bytes": (sz, [i64, i64, i32]),
        "mq_workspace_bytes": (sz, [i64, i64, i64, i32]),
        "mq_workspace_init": (i32, [vp, sz, vp]),
        "mq_slice_codes": (i32, [vp, i64, i32, i32, vp, vp]),
        "mq_pack": (i32, [vp, i64, i64, i32, i32, vp, sz, vp]),
        "mq_unpack": (i32, [vp, i64, i64, i32, i32, vp, vp]),
        "mq_pack_meta": (i32, [vp, vp, i64, i64, i32, vp, vp, sz, vp]),
        "mq_linear": (i32, [vp, i64, vp, vp, vp, i64, i64, i32, i32, vp, vp, sz, vp]),
        "mq_slice_pack": (i32, [vp, i64, i64, i32, i32, vp, sz, vp]),
        "mq_reslice": (i32, [vp, i64, i64, i32, i32, vp, sz, vp]),
        "mq_reslice_many": (i32, [vp, i32, i32, vp]),
        "mq_linear_from_parent": (i32, [vp, i64, vp, vp, vp, i64, i64, i32, i32, vp, vp, sz, vp]),
        "mq_quant_matgptq": (i32, [vp, i64, i64, i64, i64, vp, vp, i64, i32, i32, vp, vp, i64, vp]),
        "mq_matgptq_workspace_bytes": (sz, [i64, i32]),
        "mq_matgptq_quantize": (i32, [vp, i64, i64, i64, vp, i64, vp, vp, i32, i32, vp, i32, vp, i64, vp, sz, vp]),
        "mq_stack_workspace_bytes": (sz, [vp, i32, i64]),
        "mq_stack_plan": (i32, [vp, i32, i64, vp, sz, vp, vp]),
        "mq_linear_stack": (i32, [vp, vp]),
        "mq_read_probe": (i32, [vp, sz, vp, vp]),
        "mq_linear_bf16": (i32, [vp, i64, vp, vp, vp, i64, i64, i32, i32, vp, vp, sz, vp]),
        "mq_linear_noalloc": (i32, [vp, i64, vp, vp, vp, i64, i64, i32, i32, vp, vp]),
        "mq_linear_plain_workspace_bytes": (sz, [i64, i64, i64, i32]),
        "mq_linear_plain": (i32, [vp, i64, vp, vp, vp, i64, i64, i32, i32, vp, vp, sz, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype = res
        fn.argtypes = args
    _lib = L
    return L


def _stream(stream=None):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _check(status: int, where: str) -> None:
    if status != 0:
        raise MqError(status, where)


# ----------------------------------------------------------------- host-only
def mq_status_str(status: int) -> str:
    return lib().mq_status_str(int(status)).decode()


def mq_version() -> int:
    return lib().mq_version()


def mq_packed_bytes(N: int, K: int, r: int) -> int:
    return lib().mq_packed_bytes(N, K, r)


def mq_meta_bytes(N: int, K: int, group: int = MQ_GROUP) -> int:
    return lib().mq_meta_bytes(N, K, group)


def mq_workspace_bytes(M: int, N: int, K: int, r: int) -> int:
    return lib().mq_workspace_bytes(M, N, K, r)


# ----------------------------------------------------------------- device calls
def mq_workspace_init(ws, stream=None) -> None:
    _check(lib().mq_workspace_init(_ptr(ws), ws.numel() * ws.element_size(), _stream(stream)), "mq_workspace_init")


def new_workspace(M: int, N: int, K: int, r: int, device="cuda"):
    """Allocate (torch) and initialise a workspace for mq_linear."""
    import torch
    nbytes = mq_workspace_bytes(M, N, K, r)
    if nbytes == 0:
        raise MqError(3, "mq_workspace_bytes")
    ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
    mq_workspace_init(ws)
    return ws


def mq_slice_codes(parent, c: int, r: int, out=None, stream=None):
    import torch
    if out is None:
        out = torch.empty_like(parent)
    _check(lib().mq_slice_codes(_ptr(parent), parent.numel(), c, r, _ptr(out), _stream(stream)), "mq_slice_codes")
    return out


def mq_pack(S, c: int, r: int, out=None, stream=None):
    import torch
    N, K = S.shape
    if out is None:
        nbytes = mq_packed_bytes(N, K, r)
        out = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=S.device)
    _check(lib().mq_pack(_ptr(S), N, K, c, r, _ptr(out), out.numel(), _stream(stream)), "mq_pack")
    return out


def mq_unpack(packed, N: int, K: int, c: int, r: int, out=None, stream=None):
    import torch
    if out is None:
        out = torch.empty((N, K), dtype=torch.uint8, device=packed.device)
    _check(lib().mq_unpack(_ptr(packed), N, K, c, r, _ptr(out), _stream(stream)), "mq_unpack")
    return out


def mq_pack_meta(scales, zeros, K: int, group: int = MQ_GROUP, stream=None):
    """zeros=None: symmetric layer; returns (scales_t, None)."""
    import torch
    N = scales.shape[0]
    nbytes = mq_meta_bytes(N, K, group)
    st = torch.empty(max(nbytes // 2, 1), dtype=torch.float16, device=scales.device)
    zt = None if zeros is None else torch.empty(max(nbytes // 2, 1), dtype=torch.float16, device=scales.device)
    _check(lib().mq_pack_meta(_ptr(scales), _ptr(zeros), N, K, group, _ptr(st), _ptr(zt), nbytes, _stream(stream)),
           "mq_pack_meta")
    return st, zt


def mq_linear(x, packed_W, scales_t, zeros_t, N: int, K: int, r: int, group: int, ws, y=None, stream=None):
    import torch
    M = x.shape[0]
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=x.device)
    _check(lib().mq_linear(_ptr(x), M, _ptr(packed_W), _ptr(scales_t), _ptr(zeros_t), N, K, r, group, _ptr(y),
                           _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)), "mq_linear")
    return y


def mq_read_probe(buf, out, stream=None) -> None:
    """xor of all 32-bit words of buf (uint8 tensor, a multiple of 16 bytes) is xor-ed into out (one int32/uint32)."""
    _check(lib().mq_read_probe(_ptr(buf), buf.numel() * buf.element_size(), _ptr(out), _stream(stream)), "mq_read_probe")


def mq_linear_bf16(x, packed_W, scales_t, zeros_t, N: int, K: int, r: int, group: int, ws, y=None, stream=None):
    """mq_linear on bfloat16 activations (torch.bfloat16 [M, K]) with a bfloat16 result."""
    import torch
    M = x.shape[0]
    if y is None:
        y = torch.empty((M, N), dtype=torch.bfloat16, device=x.device)
    _check(lib().mq_linear_bf16(_ptr(x), M, _ptr(packed_W), _ptr(scales_t), _ptr(zeros_t), N, K, r, group, _ptr(y),
                                _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)), "mq_linear_bf16")
    return y


def mq_linear_noalloc(x, packed_W, scales_t, zeros_t, N: int, K: int, r: int, group: int, y, stream=None):
    """mq_linear without a workspace: the library's static scratch array serves.  y must be given (this wrapper
    allocates nothing either)."""
    _check(lib().mq_linear_noalloc(_ptr(x), x.shape[0], _ptr(packed_W), _ptr(scales_t), _ptr(zeros_t), N, K, r, group,
                                   _ptr(y), _stream(stream)), "mq_linear_noalloc")
    return y


def mq_linear_plain_workspace_bytes(M: int, N: int, K: int, r: int) -> int:
    return lib().mq_linear_plain_workspace_bytes(M, N, K, r)


def mq_linear_plain(x, packed_W, scales, zeros, N: int, K: int, r: int, group: int, ws, y=None, stream=None):
    """mq_linear on the quantiser's own [N, K/group] scales and zero-offsets (re-tiled into ws by the call)."""
    import torch
    M = x.shape[0]
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=x.device)
    _check(lib().mq_linear_plain(_ptr(x), M, _ptr(packed_W), _ptr(scales), _ptr(zeros), N, K, r, group, _ptr(y),
                                 _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)), "mq_linear_plain")
    return y


def mq_slice_pack(parent, c: int, r: int, out=None, stream=None):
    """Row-major 8-bit parent -> r-bit pack (Eq. 1 and the pack in one kernel)."""
    import torch
    N, K = parent.shape
    if out is None:
        out = torch.empty(max(mq_packed_bytes(N, K, r), 16), dtype=torch.uint8, device=parent.device)
    _check(lib().mq_slice_pack(_ptr(parent), N, K, c, r, _ptr(out), out.numel(), _stream(stream)), "mq_slice_pack")
    return out


def mq_reslice(packed_parent, N: int, K: int, c: int, r: int, out=None, stream=None):
    """Resident 8-bit pack of the parent -> r-bit pack."""
    import torch
    if out is None:
        out = torch.empty(max(mq_packed_bytes(N, K, r), 16), dtype=torch.uint8, device=packed_parent.device)
    _check(lib().mq_reslice(_ptr(packed_parent), N, K, c, r, _ptr(out), out.numel(), _stream(stream)), "mq_reslice")
    return out


def mq_reslice_many(jobs: Sequence[dict], c: int = 8, stream=None):
    """jobs: dicts with packed_parent (tensor), N, K, r and optionally out (tensor).  Returns the output tensors."""
    import torch
    arr = (MqResliceJob * len(jobs))()
    outs = []
    for i, J in enumerate(jobs):
        out = J.get("out")
        if out is None:
            out = torch.empty(max(mq_packed_bytes(J["N"], J["K"], J["r"]), 16), dtype=torch.uint8,
                              device=J["packed_parent"].device)
        outs.append(out)
        arr[i] = MqResliceJob(_ptr(J["packed_parent"]), _ptr(out), out.numel(), J["N"], J["K"], J["r"], 0)
    _check(lib().mq_reslice_many(ctypes.cast(arr, ctypes.c_void_p), len(jobs), c, _stream(stream)), "mq_reslice_many")
    return outs


def mq_linear_from_parent(x, packed_parent, scales_t, zeros_t, N: int, K: int, r: int, group: int, ws, y=None,
                          stream=None):
    import torch
    M = x.shape[0]
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=x.device)
    _check(lib().mq_linear_from_parent(_ptr(x), M, _ptr(packed_parent), _ptr(scales_t), _ptr(zeros_t), N, K, r, group,
                                       _ptr(y), _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)),
           "mq_linear_from_parent")
    return y


def mq_quant_matgptq(W, scales, zeros, widths, lam, K: Optional[int] = None, col0: int = 0, c: int = 8,
                     group: int = MQ_GROUP, out=None, stream=None):
    """Algorithm 1 on W (fp32 [N, ncols], possibly a column slab / strided view of a [N, K] layer).
    widths / lam: the target widths R and their lambda_r.  Returns uint8 codes [N, ncols]."""
    import torch
    N, ncols = W.shape
    K = ncols if K is None else K
    if W.stride(1) != 1:
        raise ValueError("columns of W must be contiguous")
    if out is None:
        out = torch.empty((N, ncols), dtype=torch.uint8, device=W.device)
    lam8 = (ctypes.c_float * 8)()
    for r, l in zip(widths, lam):
        if not 1 <= int(r) <= 8:
            raise MqError(2, "mq_quant_matgptq")
        lam8[int(r) - 1] = float(l)
    _check(lib().mq_quant_matgptq(_ptr(W), W.stride(0), N, ncols, col0, _ptr(scales), _ptr(zeros), K, group, c,
                                  ctypes.cast(lam8, ctypes.c_void_p), _ptr(out), out.stride(0), _stream(stream)),
           "mq_quant_matgptq")
    return out


def _lambda8(widths, lam, where):
    lam8 = (ctypes.c_float * 8)()
    for r, l in zip(widths, lam):
        if not 1 <= int(r) <= 8:
            raise MqError(2, where)
        lam8[int(r) - 1] = float(l)
    return lam8


def mq_matgptq_workspace_bytes(N: int, block: int = 128) -> int:
    return lib().mq_matgptq_workspace_bytes(N, block)


def mq_matgptq_quantize(W, U, scales, zeros, widths, lam, block: int = 128, c: int = 8, group: int = MQ_GROUP,
                        out=None, stream=None):
    """The MatGPTQ column loop on W (fp32 [N, K], OVERWRITTEN) given U, the upper Cholesky factor of H^-1.
    Returns the uint8 parent codes [N, K]."""
    import torch
    N, K = W.shape
    if W.stride(1) != 1 or U.stride(1) != 1:
        raise ValueError("rows of W and U must be contiguous")
    if tuple(U.shape) != (K, K):
        raise ValueError("U must be [K, K]")
    if out is None:
        out = torch.empty((N, K), dtype=torch.uint8, device=W.device)
    nbytes = mq_matgptq_workspace_bytes(N, block)
    ws = torch.empty(max(nbytes, 4), dtype=torch.uint8, device=W.device)
    if stream is not None:
        ws.record_stream(stream)       # scratch of launches that are still running when this returns
    lam8 = _lambda8(widths, lam, "mq_matgptq_quantize")
    _check(lib().mq_matgptq_quantize(_ptr(W), W.stride(0), N, K, _ptr(U), U.stride(0), _ptr(scales), _ptr(zeros), group,
                                     c, ctypes.cast(lam8, ctypes.c_void_p), block, _ptr(out), out.stride(0), _ptr(ws),
                                     nbytes, _stream(stream)), "mq_matgptq_quantize")
    return out


def _layer_array(layers: Sequence[dict]):
    arr = (MqLayer * len(layers))()
    for i, L in enumerate(layers):
        arr[i] = MqLayer(_ptr(L["packed_W"]), _ptr(L["scales_t"]), _ptr(L["zeros_t"]), _ptr(L["x"]), _ptr(L["y"]),
                         L["N"], L["K"], L["r"], L.get("group", MQ_GROUP), int(L.get("from_parent", 0)),
                         int(L.get("flags", 0)))
    return arr


def mq_stack_workspace_bytes(layers: Sequence[dict], M: int) -> int:
    arr = _layer_array(layers)
    return lib().mq_stack_workspace_bytes(ctypes.cast(arr, ctypes.c_void_p), len(layers), M)


def mq_stack_plan(layers: Sequence[dict], M: int, device="cuda", stream=None, ws=None) -> StackPlan:
    """layers: dicts with packed_W, scales_t, zeros_t, x, y (tensors), N, K, r.  Returns a StackPlan (host header +
    the device workspace, allocated here with torch unless `ws` is given)."""
    import torch
    arr = _layer_array(layers)
    nbytes = lib().mq_stack_workspace_bytes(ctypes.cast(arr, ctypes.c_void_p), len(layers), M)
    if nbytes == 0:
        raise MqError(3, "mq_stack_workspace_bytes")
    if ws is None:
        ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
    handle = MqPlan()
    _check(lib().mq_stack_plan(ctypes.cast(arr, ctypes.c_void_p), len(layers), M, _ptr(ws),
                               ws.numel() * ws.element_size(), ctypes.byref(handle), _stream(stream)), "mq_stack_plan")
    return StackPlan(handle, ws)


def mq_linear_stack(plan: StackPlan, stream=None) -> None:
    _check(lib().mq_linear_stack(ctypes.byref(plan.handle), _stream(stream)), "mq_linear_stack")


# ----------------------------------------------------------------- convenience
def prepare_layer(parent, scales, zeros, r: int, c: int = 8, group: int = MQ_GROUP) -> dict:
    """parent/scales/zeros device tensors -> packed layer (slice, pack, meta), all on the GPU.
    zeros=None: symmetric layer (zeros_t is None in the result)."""
    N, K = parent.shape
    S = mq_slice_codes(parent, c, r)
    packed = mq_pack(S, c, r)
    st, zt = mq_pack_meta(scales, zeros, K, group)
    return {"packed_W": packed, "scales_t": st, "zeros_t": zt, "N": N, "K": K, "r": r, "group": group}
