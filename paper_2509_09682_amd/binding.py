"""ctypes binding of libcce_neg.so: argument marshalling only, every step runs in the HIP kernels.

Tensors are torch CUDA tensors used as device allocations; kernels are enqueued on torch's current stream.
There is no CPU fallback: a missing library or a missing GPU raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libcce_neg.so")

CCE_OK = 0
CCE_ERR_NULL, CCE_ERR_SHAPE, CCE_ERR_DTYPE, CCE_ERR_INDEX = 1, 2, 3, 4
CCE_ERR_WORKSPACE, CCE_ERR_UNSUPPORTED, CCE_ERR_HIP = 5, 6, 7
CCE_F32, CCE_BF16 = 0, 1
CCE_NEG_SHARED, CCE_NEG_PER_POSITION, CCE_NEG_FULL = 0, 1, 2
CCE_ALGO_AUTO, CCE_ALGO_GATHER, CCE_ALGO_TILE = 0, 1, 2
CCE_SAMPLER_UNIFORM, CCE_SAMPLER_ALIAS = 1, 2

EXPORTS = (
    "cce_neg_workspace_bytes", "cce_neg_workspace_init", "cce_neg_forward", "cce_neg_backward",
    "cce_neg_index_status", "cce_status_string", "cce_neg_profile_enable", "cce_neg_profile_read",
    "cce_neg_sample", "cce_neg_forward_sampled", "cce_neg_backward_sampled", "cce_neg_forward_noalloc",
)


class CceDesc(ctypes.Structure):
    _fields_ = [
        ("N", ctypes.c_int64), ("V", ctypes.c_int64), ("d", ctypes.c_int32), ("K", ctypes.c_int32),
        ("in_dtype", ctypes.c_int32), ("dH_dtype", ctypes.c_int32), ("neg_mode", ctypes.c_int32),
        ("mask_target_collisions", ctypes.c_int32), ("validate_indices", ctypes.c_int32), ("algo", ctypes.c_int32),
        ("reuse_forward_prep", ctypes.c_int32), ("filter_eps", ctypes.c_float), ("fuse_dH", ctypes.c_int32),
    ]


class CceSampler(ctypes.Structure):
    _fields_ = [
        ("kind", ctypes.c_int32), ("stream", ctypes.c_uint32), ("seed", ctypes.c_uint64),
        ("alias_thresh", ctypes.c_void_p), ("alias_id", ctypes.c_void_p),
    ]


class CceError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


_lib = None


def lib() -> ctypes.CDLL:
    """Load the HIP library; raises if it has not been built (python -m paper_2509_09682_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: build it with `python -m paper_2509_09682_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32p = ctypes.c_void_p, ctypes.c_void_p
        L.cce_neg_workspace_bytes.restype = ctypes.c_size_t
        L.cce_neg_workspace_bytes.argtypes = [ctypes.POINTER(CceDesc)]
        L.cce_neg_workspace_init.restype = ctypes.c_int
        L.cce_neg_workspace_init.argtypes = [vp, ctypes.c_size_t, vp]
        L.cce_neg_forward.restype = ctypes.c_int
        L.cce_neg_forward.argtypes = [ctypes.POINTER(CceDesc), vp, vp, i32p, i32p, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.cce_neg_forward_noalloc.restype = ctypes.c_int
        L.cce_neg_forward_noalloc.argtypes = [ctypes.POINTER(CceDesc), vp, vp, i32p, i32p, vp, vp, vp, vp]
        L.cce_neg_backward.restype = ctypes.c_int
        L.cce_neg_backward.argtypes = [ctypes.POINTER(CceDesc), vp, vp, i32p, i32p, vp, vp, vp, vp, vp, vp,
                                       ctypes.c_size_t, vp]
        L.cce_neg_sample.restype = ctypes.c_int
        L.cce_neg_sample.argtypes = [ctypes.POINTER(CceDesc), ctypes.POINTER(CceSampler), i32p, vp]
        L.cce_neg_forward_sampled.restype = ctypes.c_int
        L.cce_neg_forward_sampled.argtypes = [ctypes.POINTER(CceDesc), ctypes.POINTER(CceSampler), vp, vp, i32p, vp, vp, vp,
                                              vp, ctypes.c_size_t, vp]
        L.cce_neg_backward_sampled.restype = ctypes.c_int
        L.cce_neg_backward_sampled.argtypes = [ctypes.POINTER(CceDesc), ctypes.POINTER(CceSampler), vp, vp, i32p, vp, vp, vp,
                                               vp, vp, vp, ctypes.c_size_t, vp]
        L.cce_neg_index_status.restype = ctypes.c_int
        L.cce_neg_index_status.argtypes = [vp, ctypes.c_size_t, vp]
        L.cce_neg_profile_enable.restype = ctypes.c_int
        L.cce_neg_profile_enable.argtypes = [ctypes.c_int32]
        L.cce_neg_profile_read.restype = ctypes.c_int32
        L.cce_neg_profile_read.argtypes = [ctypes.c_int32, ctypes.c_char_p, ctypes.POINTER(ctypes.c_float),
                                           ctypes.POINTER(ctypes.c_int32)]
        L.cce_status_string.restype = ctypes.c_char_p
        L.cce_status_string.argtypes = [ctypes.c_int]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().cce_status_string(int(status)).decode()


def make_desc(N: int, V: int, d: int, K: int, in_dtype: int, neg_mode: int, *, dH_dtype: Optional[int] = None,
              mask_target_collisions: int = 1, validate_indices: int = 0, algo: int = CCE_ALGO_AUTO,
              reuse_forward_prep: int = 0, filter_eps: float = 0.0, fuse_dH: int = 0) -> CceDesc:
    return CceDesc(int(N), int(V), int(d), int(K), int(in_dtype), int(CCE_F32 if dH_dtype is None else dH_dtype),
                   int(neg_mode), int(mask_target_collisions), int(validate_indices), int(algo), int(reuse_forward_prep),
                   float(filter_eps), int(fuse_dH))


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors handed to the CCE- library must be contiguous CUDA tensors")
    return ctypes.c_void_p(t.data_ptr())


_BF16_CARRIERS = (torch.bfloat16, torch.int16, torch.uint16)   # bf16 values, or their bit patterns in a 16-bit integer tensor


def _want(name: str, t: Optional[torch.Tensor], dtypes, numel: int, *, optional: bool = False) -> None:
    """Raises before any launch unless tensor `name` has one of `dtypes` and exactly `numel` elements."""
    if t is None:
        if optional:
            return
        raise ValueError(f"{name} is required")
    if t.dtype not in dtypes:
        raise TypeError(f"{name} must have dtype {' or '.join(str(x) for x in dtypes)}, got {t.dtype} "
                        "(the kernels read the raw bytes: no conversion happens at this boundary)")
    if t.numel() != numel:
        raise ValueError(f"{name} must hold {numel} elements for this descriptor, got {tuple(t.shape)}")


def check_step_args(desc: CceDesc, H, E, tgt, neg, mask, *, sampled: bool = False, loss=None, lse=None, grad_loss=None,
                    dH=None, dE=None) -> None:
    """Dtype and size checks of the tensors of a forward or backward call against the descriptor.

    The C ABI takes plain pointers and trusts the sizes in the descriptor, so a torch.long index tensor, a short mask
    or a per-position `neg` of another shape would be read as garbage or out of bounds; they are refused here.
    """
    if desc.neg_mode not in (CCE_NEG_SHARED, CCE_NEG_PER_POSITION, CCE_NEG_FULL):
        raise ValueError(f"unknown neg_mode {desc.neg_mode}")
    elem = (torch.float32,) if desc.in_dtype == CCE_F32 else _BF16_CARRIERS
    N, V, d, K = int(desc.N), int(desc.V), int(desc.d), int(desc.K)
    _want("H", H, elem, N * d)
    _want("E", E, elem, V * d)
    _want("tgt", tgt, (torch.int32,), N)
    if not sampled and desc.neg_mode != CCE_NEG_FULL and K > 0:
        _want("neg", neg, (torch.int32,), K if desc.neg_mode == CCE_NEG_SHARED else N * K)
        if desc.neg_mode == CCE_NEG_PER_POSITION and neg.dim() == 2 and tuple(neg.shape) != (N, K):
            raise ValueError(f"per-position neg must be [N, K] = [{N}, {K}], got {tuple(neg.shape)}")
    _want("mask", mask, (torch.uint8, torch.bool), N, optional=True)
    _want("loss", loss, (torch.float32,), N, optional=True)
    _want("lse", lse, (torch.float32,), N, optional=True)
    _want("grad_loss", grad_loss, (torch.float32,), N, optional=True)
    _want("dH", dH, (torch.float32,) if desc.dH_dtype == CCE_F32 else _BF16_CARRIERS, N * d, optional=True)
    _want("dE", dE, (torch.float32,), V * d, optional=True)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def cce_neg_workspace_bytes(desc: CceDesc) -> int:
    return int(lib().cce_neg_workspace_bytes(ctypes.byref(desc)))


def cce_neg_workspace_init(workspace: torch.Tensor) -> None:
    st = lib().cce_neg_workspace_init(_ptr(workspace), workspace.numel() * workspace.element_size(), _stream())
    if st != CCE_OK:
        raise CceError(st, "cce_neg_workspace_init")


def new_workspace(desc: CceDesc, device="cuda") -> torch.Tensor:
    n = cce_neg_workspace_bytes(desc)
    if n == 0:
        raise CceError(CCE_ERR_SHAPE, "cce_neg_workspace_bytes")
    ws = torch.empty(n, dtype=torch.uint8, device=device)
    cce_neg_workspace_init(ws)
    return ws


def cce_neg_forward(desc: CceDesc, H, E, tgt, neg, mask, loss, lse, workspace, *, check: bool = True) -> int:
    check_step_args(desc, H, E, tgt, neg, mask, loss=loss, lse=lse)
    st = lib().cce_neg_forward(ctypes.byref(desc), _ptr(H), _ptr(E), _ptr(tgt), _ptr(neg), _ptr(mask), _ptr(loss),
                               _ptr(lse), _ptr(workspace),
                               0 if workspace is None else workspace.numel() * workspace.element_size(), _stream())
    if check and st != CCE_OK:
        raise CceError(st, "cce_neg_forward")
    return st


def cce_neg_forward_noalloc(desc: CceDesc, H, E, tgt, neg, mask, loss, lse, *, check: bool = True) -> int:
    """cce_neg_forward on the library's own fixed scratch array: no workspace, no allocation (see include/cce_neg.h)."""
    check_step_args(desc, H, E, tgt, neg, mask, loss=loss, lse=lse)
    st = lib().cce_neg_forward_noalloc(ctypes.byref(desc), _ptr(H), _ptr(E), _ptr(tgt), _ptr(neg), _ptr(mask), _ptr(loss),
                                       _ptr(lse), _stream())
    if check and st != CCE_OK:
        raise CceError(st, "cce_neg_forward_noalloc")
    return st


def cce_neg_backward(desc: CceDesc, H, E, tgt, neg, mask, lse, grad_loss, dH, dE, workspace, *, check: bool = True) -> int:
    check_step_args(desc, H, E, tgt, neg, mask, lse=lse, grad_loss=grad_loss, dH=dH, dE=dE)
    st = lib().cce_neg_backward(ctypes.byref(desc), _ptr(H), _ptr(E), _ptr(tgt), _ptr(neg), _ptr(mask), _ptr(lse),
                                _ptr(grad_loss), _ptr(dH), _ptr(dE), _ptr(workspace),
                                0 if workspace is None else workspace.numel() * workspace.element_size(), _stream())
    if check and st != CCE_OK:
        raise CceError(st, "cce_neg_backward")
    return st


def make_sampler(kind: int, seed: int, stream: int = 0, alias_thresh: Optional[torch.Tensor] = None,
                 alias_id: Optional[torch.Tensor] = None) -> CceSampler:
    """alias_thresh: CUDA tensor of V 32-bit words (the uint32 thresholds, any 4-byte dtype); alias_id: CUDA int32 [V].
    The sampler only borrows the pointers: keep the tensors alive while it is in use."""
    s = CceSampler(int(kind), int(stream) & 0xFFFFFFFF, int(seed) & 0xFFFFFFFFFFFFFFFF, None, None)
    if alias_thresh is not None:
        s.alias_thresh = _ptr(alias_thresh).value
    if alias_id is not None:
        s.alias_id = _ptr(alias_id).value
    return s


def cce_neg_sample(desc: CceDesc, sampler: CceSampler, neg_out, *, check: bool = True) -> int:
    st = lib().cce_neg_sample(ctypes.byref(desc), ctypes.byref(sampler), _ptr(neg_out), _stream())
    if check and st != CCE_OK:
        raise CceError(st, "cce_neg_sample")
    return st


def cce_neg_forward_sampled(desc: CceDesc, sampler: CceSampler, H, E, tgt, mask, loss, lse, workspace, *,
                            check: bool = True) -> int:
    check_step_args(desc, H, E, tgt, None, mask, sampled=True, loss=loss, lse=lse)
    st = lib().cce_neg_forward_sampled(ctypes.byref(desc), ctypes.byref(sampler), _ptr(H), _ptr(E), _ptr(tgt), _ptr(mask),
                                       _ptr(loss), _ptr(lse), _ptr(workspace),
                                       0 if workspace is None else workspace.numel() * workspace.element_size(), _stream())
    if check and st != CCE_OK:
        raise CceError(st, "cce_neg_forward_sampled")
    return st


def cce_neg_backward_sampled(desc: CceDesc, sampler: CceSampler, H, E, tgt, mask, lse, grad_loss, dH, dE, workspace, *,
                             check: bool = True) -> int:
    check_step_args(desc, H, E, tgt, None, mask, sampled=True, lse=lse, grad_loss=grad_loss, dH=dH, dE=dE)
    st = lib().cce_neg_backward_sampled(ctypes.byref(desc), ctypes.byref(sampler), _ptr(H), _ptr(E), _ptr(tgt), _ptr(mask),
                                        _ptr(lse), _ptr(grad_loss), _ptr(dH), _ptr(dE), _ptr(workspace),
                                        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream())
    if check and st != CCE_OK:
        raise CceError(st, "cce_neg_backward_sampled")
    return st


def cce_neg_index_status(workspace: torch.Tensor) -> int:
    return int(lib().cce_neg_index_status(_ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


def cce_neg_profile_enable(enable: bool) -> None:
    lib().cce_neg_profile_enable(1 if enable else 0)


def cce_neg_profile_read(max_families: int = 16) -> dict:
    """{family: (total_ms, launches)} since the last read; waits for the recorded events."""
    names = ctypes.create_string_buffer(32 * max_families)
    ms = (ctypes.c_float * max_families)()
    cnt = (ctypes.c_int32 * max_families)()
    n = lib().cce_neg_profile_read(max_families, names, ms, cnt)
    out = {}
    for i in range(n):
        out[names.raw[32 * i:32 * (i + 1)].split(b"\0", 1)[0].decode()] = (float(ms[i]), int(cnt[i]))
    return out
