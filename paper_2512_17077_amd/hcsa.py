"""Thin ctypes binding over libdllm_hcsa.so (include/dllm_hcsa.h).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  Tensors are torch tensors on the GPU, used for device memory and the
current stream; nothing here computes.  If the library has not been built,
loading raises -- there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdllm_hcsa.so")
LIB_PATH_CHECKED = os.path.join(_HERE, "libdllm_hcsa_checked.so")   # built with the device-side precondition checks

DLLM_OK = 0
DLLM_ERR_INVALID_ARG = -1
DLLM_ERR_UNSUPPORTED = -2
DLLM_ERR_WORKSPACE = -3
DLLM_ERR_DEVICE = -4
DLLM_F32, DLLM_BF16 = 0, 1
DLLM_SEQ_SPARSE, DLLM_SEQ_DENSE = 0, 1
DLLM_SELECT_FORM_AUTO, DLLM_SELECT_FORM_TWO_LAUNCHES, DLLM_SELECT_FORM_ONE_LAUNCH = 0, 1, 2

EXPORTS = [
    "dllm_hcsa_select_workspace", "dllm_hcsa_select", "dllm_hcsa_select_ex", "dllm_hcsa_select_static",
    "dllm_hcsa_set_select_form", "dllm_hcsa_select_form_of",
    "dllm_hcsa_attend_workspace", "dllm_hcsa_attend",
    "dllm_dense_refresh_attend_workspace", "dllm_dense_refresh_attend",
    "dllm_hcsa_pack", "dllm_hcsa_precondition_errors",
    "dllm_last_error", "dllm_hcsa_version",
]
DLLM_CHECK_CU_Q, DLLM_CHECK_CU_KV, DLLM_CHECK_CU_K, DLLM_CHECK_K_OVER_L, DLLM_CHECK_FORCED, DLLM_CHECK_IDX = 1, 2, 4, 8, 16, 32


class DllmBatch(ctypes.Structure):
    """Mirror of `dllm_batch`."""
    _fields_ = [
        ("dtype", ctypes.c_int),
        ("batch", ctypes.c_int32),
        ("n_q_heads", ctypes.c_int32),
        ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("q", ctypes.c_void_p),
        ("k", ctypes.c_void_p),
        ("v", ctypes.c_void_p),
        ("q_stride_tok", ctypes.c_int64),
        ("q_stride_head", ctypes.c_int64),
        ("kv_stride_tok", ctypes.c_int64),
        ("kv_stride_head", ctypes.c_int64),
        ("cu_q", ctypes.c_void_p),
        ("cu_kv", ctypes.c_void_p),
        ("total_q", ctypes.c_int32),
        ("total_kv", ctypes.c_int32),
        ("max_q", ctypes.c_int32),
        ("max_kv", ctypes.c_int32),
        ("softmax_scale", ctypes.c_float),
    ]


class DllmError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"dllm status {status}: {message}")
        self.status = status


_lib = None


def lib() -> ctypes.CDLL:
    """Open the built library (once).  A missing build is an error."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2512_17077_amd.build` "
                "(there is no CPU or PyTorch fallback for this library)")
        L = ctypes.CDLL(LIB_PATH)
        P, vp, i32, sz = ctypes.POINTER(DllmBatch), ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        L.dllm_hcsa_select_workspace.restype = sz
        L.dllm_hcsa_select_workspace.argtypes = [P, i32]
        L.dllm_hcsa_select.restype = ctypes.c_int
        L.dllm_hcsa_select.argtypes = [P, vp, i32, i32, i32, vp, vp, sz, vp]
        L.dllm_hcsa_select_ex.restype = ctypes.c_int
        L.dllm_hcsa_select_ex.argtypes = [P, vp, i32, i32, i32, i32, i32, vp, vp, sz, vp]
        L.dllm_hcsa_set_select_form.restype = i32
        L.dllm_hcsa_set_select_form.argtypes = [i32]
        L.dllm_hcsa_select_form_of.restype = i32
        L.dllm_hcsa_select_form_of.argtypes = [P, i32, i32]
        L.dllm_hcsa_select_static.restype = ctypes.c_int
        L.dllm_hcsa_select_static.argtypes = [P, vp, i32, i32, i32, i32, i32, vp, vp]
        L.dllm_hcsa_attend_workspace.restype = sz
        L.dllm_hcsa_attend_workspace.argtypes = [P, i32]
        L.dllm_hcsa_attend.restype = ctypes.c_int
        L.dllm_hcsa_attend.argtypes = [P, vp, vp, i32, i32, vp, vp, vp, sz, vp]
        L.dllm_dense_refresh_attend_workspace.restype = sz
        L.dllm_dense_refresh_attend_workspace.argtypes = [P]
        L.dllm_dense_refresh_attend.restype = ctypes.c_int
        L.dllm_dense_refresh_attend.argtypes = [P, vp, vp, sz, vp]
        L.dllm_hcsa_pack.restype = ctypes.c_int
        L.dllm_hcsa_pack.argtypes = [P, vp, vp, i32, i32, vp, vp, vp]
        L.dllm_hcsa_precondition_errors.restype = ctypes.c_int
        L.dllm_hcsa_precondition_errors.argtypes = [vp, ctypes.POINTER(ctypes.c_uint32)]
        L.dllm_last_error.restype = ctypes.c_char_p
        L.dllm_last_error.argtypes = []
        L.dllm_hcsa_version.restype = i32
        L.dllm_hcsa_version.argtypes = []
        _lib = L
    return _lib


def use_checked_library(on: bool = True):
    """Switch this binding to the library built with the device-side precondition checks (or back).  The
    checked library must have been built (paper_2512_17077_amd.build does both)."""
    global _lib, LIB_PATH
    _lib = None
    LIB_PATH = LIB_PATH_CHECKED if on else os.path.join(_HERE, "libdllm_hcsa.so")


def dllm_hcsa_precondition_errors(stream=None) -> int:
    """Fetch and clear the error word of the checked library (raises DLLM_ERR_UNSUPPORTED in the release one)."""
    out = ctypes.c_uint32(0)
    _raise(lib().dllm_hcsa_precondition_errors(_stream(stream), ctypes.byref(out)))
    return int(out.value)


def last_error() -> str:
    return lib().dllm_last_error().decode()


def _raise(status: int):
    if status != DLLM_OK:
        raise DllmError(status, last_error())


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def make_batch(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, cu_q: torch.Tensor, cu_kv: torch.Tensor,
               max_q: int, max_kv: int, softmax_scale: float) -> DllmBatch:
    """Describe packed q [total_q,Hq,D], k/v [total_kv,Hkv,D] (last dim contiguous) to the library."""
    assert q.dim() == 3 and k.dim() == 3 and v.dim() == 3
    assert q.stride(2) == 1 and k.stride(2) == 1 and v.stride(2) == 1
    assert k.shape == v.shape and k.stride() == v.stride() and q.dtype == k.dtype == v.dtype
    assert cu_q.dtype == torch.int32 and cu_kv.dtype == torch.int32
    dt = {torch.float32: DLLM_F32, torch.bfloat16: DLLM_BF16}[q.dtype]
    b = DllmBatch()
    b.dtype = dt
    b.batch = cu_q.numel() - 1
    b.n_q_heads, b.n_kv_heads, b.head_dim = q.shape[1], k.shape[1], q.shape[2]
    b.q, b.k, b.v = q.data_ptr(), k.data_ptr(), v.data_ptr()
    b.q_stride_tok, b.q_stride_head = q.stride(0), q.stride(1)
    b.kv_stride_tok, b.kv_stride_head = k.stride(0), k.stride(1)
    b.cu_q, b.cu_kv = cu_q.data_ptr(), cu_kv.data_ptr()
    b.total_q, b.total_kv = q.shape[0], k.shape[0]
    b.max_q, b.max_kv = int(max_q), int(max_kv)
    b.softmax_scale = float(softmax_scale)
    return b


def _workspace(nbytes: int, device) -> Optional[torch.Tensor]:
    if nbytes == 0:
        return None
    return torch.empty(nbytes, dtype=torch.uint8, device=device)   # torch allocations are >= 256-byte aligned


def dllm_hcsa_select_workspace(batch: DllmBatch, max_k: int) -> int:
    return int(lib().dllm_hcsa_select_workspace(ctypes.byref(batch), int(max_k)))


def dllm_hcsa_select(batch: DllmBatch, cu_k: torch.Tensor, total_k: int, max_k: int, idx_out: torch.Tensor,
                     pool_w: int = 1, workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Per-head top-k selection; fills idx_out [Hq, total_k] (int32, device)."""
    if workspace is None:
        workspace = _workspace(dllm_hcsa_select_workspace(batch, max_k), idx_out.device)
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _raise(lib().dllm_hcsa_select(ctypes.byref(batch), _ptr(cu_k), int(total_k), int(max_k), int(pool_w),
                                  _ptr(idx_out), _ptr(workspace), nbytes, _stream(stream)))
    return idx_out


def dllm_hcsa_select_ex(batch: DllmBatch, cu_k: torch.Tensor, total_k: int, max_k: int, idx_out: torch.Tensor,
                        pool_w: int = 1, forced_tail: int = 0, head_sum: bool = False,
                        workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Selection with the block's own positions always kept and / or one list shared by all heads."""
    if workspace is None:
        workspace = _workspace(dllm_hcsa_select_workspace(batch, max_k), idx_out.device)
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _raise(lib().dllm_hcsa_select_ex(ctypes.byref(batch), _ptr(cu_k), int(total_k), int(max_k), int(pool_w),
                                     int(forced_tail), int(bool(head_sum)), _ptr(idx_out), _ptr(workspace), nbytes,
                                     _stream(stream)))
    return idx_out


DLLM_SELECT_STATIC_BYTES = 32 << 20


def dllm_hcsa_select_form_of(batch: DllmBatch, pool_w: int = 1, head_sum: bool = False) -> int:
    """Which of its two forms a selection call on this batch takes under the current setting (DLLM_SELECT_FORM_*)."""
    form = int(lib().dllm_hcsa_select_form_of(ctypes.byref(batch), int(pool_w), int(bool(head_sum))))
    if form < 0:
        raise ValueError(last_error())
    return form


def dllm_hcsa_set_select_form(form: int) -> int:
    """Process-wide choice between the two forms of selection (DLLM_SELECT_FORM_*); returns the previous one."""
    prev = int(lib().dllm_hcsa_set_select_form(int(form)))
    if prev < 0:
        raise ValueError(f"select form {form} is none of DLLM_SELECT_FORM_AUTO/TWO_LAUNCHES/ONE_LAUNCH")
    return prev


def dllm_hcsa_select_static(batch: DllmBatch, cu_k: torch.Tensor, total_k: int, max_k: int, idx_out: torch.Tensor,
                            pool_w: int = 1, forced_tail: int = 0, head_sum: bool = False, stream=None) -> torch.Tensor:
    """dllm_hcsa_select_ex on the library's built-in scratch buffer: no workspace, nothing allocated."""
    _raise(lib().dllm_hcsa_select_static(ctypes.byref(batch), _ptr(cu_k), int(total_k), int(max_k), int(pool_w),
                                         int(forced_tail), int(bool(head_sum)), _ptr(idx_out), _stream(stream)))
    return idx_out


def dllm_hcsa_attend_workspace(batch: DllmBatch, max_k: int) -> int:
    return int(lib().dllm_hcsa_attend_workspace(ctypes.byref(batch), int(max_k)))


def dllm_hcsa_attend(batch: DllmBatch, idx: Optional[torch.Tensor], cu_k: Optional[torch.Tensor], total_k: int,
                     max_k: int, seq_mode: Optional[torch.Tensor], o: torch.Tensor,
                     workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Attention over kept rows (and over all rows for sequences flagged dense); fills o."""
    if workspace is None:
        workspace = _workspace(dllm_hcsa_attend_workspace(batch, max_k), o.device)
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _raise(lib().dllm_hcsa_attend(ctypes.byref(batch), _ptr(idx), _ptr(cu_k), int(total_k), int(max_k),
                                  _ptr(seq_mode), _ptr(o), _ptr(workspace), nbytes, _stream(stream)))
    return o


def dllm_dense_refresh_attend_workspace(batch: DllmBatch) -> int:
    return int(lib().dllm_dense_refresh_attend_workspace(ctypes.byref(batch)))


def dllm_dense_refresh_attend(batch: DllmBatch, o: torch.Tensor, workspace: Optional[torch.Tensor] = None,
                              stream=None) -> torch.Tensor:
    """Dense bidirectional attention of every sequence; fills o."""
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _raise(lib().dllm_dense_refresh_attend(ctypes.byref(batch), _ptr(o), _ptr(workspace), nbytes, _stream(stream)))
    return o


def dllm_hcsa_pack(batch: DllmBatch, idx: torch.Tensor, cu_k: torch.Tensor, total_k: int, max_k: int,
                   k_packed: torch.Tensor, v_packed: torch.Tensor, stream=None):
    """Copy every head's kept rows into k_packed / v_packed [Hq, total_k, D]."""
    _raise(lib().dllm_hcsa_pack(ctypes.byref(batch), _ptr(idx), _ptr(cu_k), int(total_k), int(max_k),
                                _ptr(k_packed), _ptr(v_packed), _stream(stream)))
    return k_packed, v_packed


def make_packed_batch(q: torch.Tensor, k_packed: torch.Tensor, v_packed: torch.Tensor, cu_q: torch.Tensor,
                      cu_k: torch.Tensor, max_q: int, max_k: int, softmax_scale: float) -> DllmBatch:
    """Describe packed buffers [Hq, total_k, D] as the K/V operand of an attend call: one KV head per
    query head, rows of a head contiguous, sequence b owning list positions cu_k[b] .. cu_k[b+1]-1."""
    assert k_packed.dim() == 3 and k_packed.is_contiguous() and v_packed.is_contiguous()
    return make_batch(q, k_packed.transpose(0, 1), v_packed.transpose(0, 1), cu_q, cu_k, max_q, max_k, softmax_scale)
