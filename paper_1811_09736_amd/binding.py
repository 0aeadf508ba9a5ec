"""Thin ctypes binding over the C ABI of libtcr.so (include/tcr.h).

Argument marshalling only: device pointers, sizes and the stream handle are passed
through; every step of the computation runs in the HIP kernels.  PyTorch supplies
device memory and streams, nothing else.  If the library has not been built the
import of this module fails -- there is no CPU fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

from .build import LIB_PATH

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP = range(5)
OP_SEGMENTED_REDUCE, OP_SEGMENTED_SCAN, OP_REDUCE, OP_SCAN, OP_IRREGULAR_REDUCE, OP_IRREGULAR_SCAN = range(6)
OP_SEGMENTED_MOMENTS, OP_IRREGULAR_MOMENTS = 6, 7          # tcr_workspace_bytes only

SCAN_EXCLUSIVE, OUT_F16, ACC_F16 = 1, 2, 4

EXPORTS = (
    "tcr_segmented_reduce", "tcr_segmented_scan", "tcr_segmented_scan_ex", "tcr_scan_ex", "tcr_reduce", "tcr_scan",
    "tcr_irregular_reduce", "tcr_irregular_scan", "tcr_irregular_scan_ex", "tcr_irregular_moments", "tcr_autotune", "tcr_autotune_irregular", "tcr_tuning_export", "tcr_tuning_import",
    "tcr_workspace_bytes", "tcr_set_workspace", "tcr_segmented_moments",
    "tcr_set_variant", "tcr_segmented_scan_noalloc",
    "tcr_kernel_name", "tcr_check_device_flags", "tcr_release", "tcr_release_stream", "tcr_status_string", "tcr_last_hip_error",
)


class TcrError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _lib.tcr_status_string(status).decode()
        if status == ERR_HIP:
            msg += " (" + _lib.tcr_last_hip_error().decode() + ")"
        super().__init__(f"{where}: {msg}")


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, u64, fp = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p
    lib.tcr_segmented_reduce.argtypes = [vp, fp, u64, u64, vp]
    lib.tcr_segmented_scan.argtypes = [vp, fp, u64, u64, vp]
    lib.tcr_segmented_scan_ex.argtypes = [vp, vp, u64, u64, ctypes.c_uint32, vp]
    lib.tcr_scan_ex.argtypes = [vp, vp, u64, ctypes.c_uint32, vp]
    lib.tcr_segmented_scan_ex.restype = ctypes.c_int
    lib.tcr_scan_ex.restype = ctypes.c_int
    lib.tcr_irregular_reduce.argtypes = [vp, vp, fp, u64, u64, vp]
    lib.tcr_irregular_scan.argtypes = [vp, vp, fp, u64, u64, vp]
    lib.tcr_irregular_scan_ex.argtypes = [vp, vp, vp, u64, u64, ctypes.c_uint32, vp]
    lib.tcr_irregular_scan_ex.restype = ctypes.c_int
    lib.tcr_irregular_moments.argtypes = [vp, vp, fp, fp, u64, u64, vp]
    lib.tcr_irregular_moments.restype = ctypes.c_int
    lib.tcr_irregular_reduce.restype = ctypes.c_int
    lib.tcr_irregular_scan.restype = ctypes.c_int
    lib.tcr_reduce.argtypes = [vp, fp, u64, vp]
    lib.tcr_scan.argtypes = [vp, fp, u64, vp]
    for name in ("tcr_segmented_reduce", "tcr_segmented_scan", "tcr_reduce", "tcr_scan"):
        getattr(lib, name).restype = ctypes.c_int
    lib.tcr_segmented_scan_noalloc.argtypes = [vp, fp, u64, u64, vp]
    lib.tcr_segmented_scan_noalloc.restype = ctypes.c_int
    lib.tcr_autotune.argtypes = [ctypes.c_int, vp, fp, u64, u64, vp]
    lib.tcr_autotune.restype = ctypes.c_int
    lib.tcr_autotune_irregular.argtypes = [ctypes.c_int, vp, vp, fp, u64, u64, vp]
    lib.tcr_autotune_irregular.restype = ctypes.c_int
    lib.tcr_tuning_export.argtypes = [ctypes.c_char_p, u64]
    lib.tcr_tuning_export.restype = u64
    lib.tcr_tuning_import.argtypes = [ctypes.c_char_p]
    lib.tcr_tuning_import.restype = ctypes.c_int
    lib.tcr_segmented_moments.argtypes = [vp, fp, fp, u64, u64, vp]
    lib.tcr_segmented_moments.restype = ctypes.c_int
    lib.tcr_workspace_bytes.argtypes = [ctypes.c_int, u64, u64]
    lib.tcr_workspace_bytes.restype = u64
    lib.tcr_set_workspace.argtypes = [vp, u64]
    lib.tcr_set_workspace.restype = ctypes.c_int
    lib.tcr_set_variant.argtypes = [ctypes.c_char_p, ctypes.c_char_p]
    lib.tcr_set_variant.restype = ctypes.c_int
    lib.tcr_kernel_name.argtypes = [ctypes.c_int, u64, u64]
    lib.tcr_kernel_name.restype = ctypes.c_char_p
    lib.tcr_check_device_flags.argtypes = [vp]
    lib.tcr_check_device_flags.restype = ctypes.c_int
    lib.tcr_release.argtypes = []
    lib.tcr_release.restype = None
    lib.tcr_release_stream.argtypes = [vp]
    lib.tcr_release_stream.restype = ctypes.c_int
    lib.tcr_status_string.argtypes = [ctypes.c_int]
    lib.tcr_status_string.restype = ctypes.c_char_p
    lib.tcr_last_hip_error.argtypes = []
    lib.tcr_last_hip_error.restype = ctypes.c_char_p
    return lib


_lib = _load()


def _stream_handle(stream: Optional[torch.cuda.Stream]) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def _check_input(x: torch.Tensor) -> None:
    if not (x.is_cuda and x.dtype == torch.float16 and x.dim() == 1 and x.is_contiguous()):
        raise TypeError("input must be a contiguous 1-D float16 CUDA tensor")


def _check_output(out: torch.Tensor, numel: int, like: torch.Tensor) -> None:
    if not (out.is_cuda and out.dtype == torch.float32 and out.is_contiguous() and out.numel() == numel
            and out.device == like.device):
        raise TypeError(f"out must be a contiguous float32 CUDA tensor of {numel} elements on the input's device")


def segmented_reduce(x: torch.Tensor, seg_len: int, out: Optional[torch.Tensor] = None,
                     stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """tcr_segmented_reduce: out[s] = sum of x[s*seg_len : (s+1)*seg_len]."""
    _check_input(x)
    n = x.numel()
    if seg_len <= 0 or n % seg_len:
        raise TcrError(ERR_INVALID_ARG, "tcr_segmented_reduce")
    if out is None:
        out = torch.empty(n // seg_len, dtype=torch.float32, device=x.device)
    _check_output(out, n // seg_len, x)
    with torch.cuda.device(x.device):
        st = _lib.tcr_segmented_reduce(x.data_ptr(), out.data_ptr(), n, seg_len, _stream_handle(stream))
    if st != OK:
        raise TcrError(st, "tcr_segmented_reduce")
    return out


def segmented_scan(x: torch.Tensor, seg_len: int, out: Optional[torch.Tensor] = None,
                   stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """tcr_segmented_scan: inclusive running sums restarting every seg_len elements."""
    _check_input(x)
    n = x.numel()
    if seg_len <= 0 or n % seg_len:
        raise TcrError(ERR_INVALID_ARG, "tcr_segmented_scan")
    if out is None:
        out = torch.empty(n, dtype=torch.float32, device=x.device)
    _check_output(out, n, x)
    with torch.cuda.device(x.device):
        st = _lib.tcr_segmented_scan(x.data_ptr(), out.data_ptr(), n, seg_len, _stream_handle(stream))
    if st != OK:
        raise TcrError(st, "tcr_segmented_scan")
    return out


def segmented_scan_noalloc(x: torch.Tensor, seg_len: int, out: torch.Tensor,
                           stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """tcr_segmented_scan_noalloc: tcr_segmented_scan on the library's fixed device scratch (the caller passes `out`)."""
    _check_input(x)
    n = x.numel()
    if seg_len <= 0 or n % seg_len:
        raise TcrError(ERR_INVALID_ARG, "tcr_segmented_scan_noalloc")
    _check_output(out, n, x)
    with torch.cuda.device(x.device):
        st = _lib.tcr_segmented_scan_noalloc(x.data_ptr(), out.data_ptr(), n, seg_len, _stream_handle(stream))
    if st != OK:
        raise TcrError(st, "tcr_segmented_scan_noalloc")
    return out


def segmented_scan_ex(x: torch.Tensor, seg_len: int, flags: int, out: Optional[torch.Tensor] = None,
                      stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """tcr_segmented_scan_ex: flags = SCAN_EXCLUSIVE | OUT_F16 (float16 output tensor when OUT_F16 is set)."""
    _check_input(x)
    n = x.numel()
    if seg_len <= 0 or n % seg_len:
        raise TcrError(ERR_INVALID_ARG, "tcr_segmented_scan_ex")
    dtype = torch.float16 if flags & OUT_F16 else torch.float32
    if out is None:
        out = torch.empty(n, dtype=dtype, device=x.device)
    if not (out.is_cuda and out.dtype == dtype and out.is_contiguous() and out.numel() == n and out.device == x.device):
        raise TypeError(f"out must be a contiguous {dtype} CUDA tensor of {n} elements on the input's device")
    with torch.cuda.device(x.device):
        st = _lib.tcr_segmented_scan_ex(x.data_ptr(), out.data_ptr(), n, seg_len, flags, _stream_handle(stream))
    if st != OK:
        raise TcrError(st, "tcr_segmented_scan_ex")
    return out


def scan_ex(x: torch.Tensor, flags: int, out: Optional[torch.Tensor] = None,
            stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """tcr_scan_ex: the full scan with flags = SCAN_EXCLUSIVE | OUT_F16."""
    _check_input(x)
    n = x.numel()
    dtype = torch.float16 if flags & OUT_F16 else torch.float32
    if out is None:
        out = torch.empty(n, dtype=dtype, device=x.device)
    if not (out.is_cuda and out.dtype == dtype and out.is_contiguous() and out.numel() == n and out.device == x.device):
        raise TypeError(f"out must be a contiguous {dtype} CUDA tensor of {n} elements on the input's device")
    with torch.cuda.device(x.device):
        st = _lib.tcr_scan_ex(x.data_ptr(), out.data_ptr(), n, flags, _stream_handle(stream))
    if st != OK:
        raise TcrError(st, "tcr_scan_ex")
    return out


def _check_offsets(x: torch.Tensor, offsets: torch.Tensor) -> int:
    if not (offsets.is_cuda and offsets.dtype == torch.int64 and offsets.dim() == 1 and offsets.is_contiguous()
            and offsets.numel() >= 1 and offsets.device == x.device):
        raise TypeError("offsets must be a contiguous 1-D int64 CUDA tensor of nseg + 1 entries on the input's device")
    return offsets.numel() - 1


def irregular_reduce(x: torch.Tensor, offsets: torch.Tensor, out: Optional[torch.Tensor] = None,
                     stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """tcr_irregular_reduce: out[s] = sum of x[offsets[s]:offsets[s+1]]."""
    if not (x.is_cuda and x.dtype == torch.float16 and x.dim() == 1 and x.is_contiguous()):
        raise TypeError("input must be a contiguous 1-D float16 CUDA tensor")
    nseg = _check_offsets(x, offsets)
    if out is None:
        out = torch.empty(nseg, dtype=torch.float32, device=x.device)
    _check_output(out, nseg, x)
    with torch.cuda.device(x.device):
        st = _lib.tcr_irregular_reduce(x.data_ptr(), offsets.data_ptr(), out.data_ptr(), x.numel(), nseg, _stream_handle(stream))
    if st != OK:
        raise TcrError(st, "tcr_irregular_reduce")
    return out


def irregular_scan(x: torch.Tensor, offsets: torch.Tensor, out: Optional[torch.Tensor] = None,
                   stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """tcr_irregular_scan: inclusive running sums restarting at every offsets[s]; out is indexed like x."""
    if not (x.is_cuda and x.dtype == torch.float16 and x.dim() == 1 and x.is_contiguous()):
        raise TypeError("input must be a contiguous 1-D float16 CUDA tensor")
    nseg = _check_offsets(x, offsets)
    if out is None:
        out = torch.zeros(x.numel(), dtype=torch.float32, device=x.device)
    _check_output(out, x.numel(), x)
    with torch.cuda.device(x.device):
        st = _lib.tcr_irregular_scan(x.data_ptr(), offsets.data_ptr(), out.data_ptr(), x.numel(), nseg, _stream_handle(stream))
    if st != OK:
        raise TcrError(st, "tcr_irregular_scan")
    return out


def irregular_moments(x: torch.Tensor, offsets: torch.Tensor, stream: Optional[torch.cuda.Stream] = None):
    """tcr_irregular_moments: (sum, sum of squares) of x[offsets[s]:offsets[s+1]] for every s."""
    if not (x.is_cuda and x.dtype == torch.float16 and x.dim() == 1 and x.is_contiguous()):
        raise TypeError("input must be a contiguous 1-D float16 CUDA tensor")
    nseg = _check_offsets(x, offsets)
    a = torch.empty(nseg, dtype=torch.float32, device=x.device)
    q = torch.empty(nseg, dtype=torch.float32, device=x.device)
    with torch.cuda.device(x.device):
        st = _lib.tcr_irregular_moments(x.data_ptr(), offsets.data_ptr(), a.data_ptr(), q.data_ptr(), x.numel(), nseg,
                                        _stream_handle(stream))
    if st != OK:
        raise TcrError(st, "tcr_irregular_moments")
    return a, q


def irregular_scan_ex(x: torch.Tensor, offsets: torch.Tensor, flags: int, out: Optional[torch.Tensor] = None,
                      stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """tcr_irregular_scan_ex: the irregular scan with SCAN_EXCLUSIVE / OUT_F16 flags."""
    if not (x.is_cuda and x.dtype == torch.float16 and x.dim() == 1 and x.is_contiguous()):
        raise TypeError("input must be a contiguous 1-D float16 CUDA tensor")
    nseg = _check_offsets(x, offsets)
    dtype = torch.float16 if flags & OUT_F16 else torch.float32
    if out is None:
        out = torch.zeros(x.numel(), dtype=dtype, device=x.device)
    if not (out.is_cuda and out.dtype == dtype and out.is_contiguous() and out.numel() == x.numel() and out.device == x.device):
        raise TypeError(f"out must be a contiguous {dtype} CUDA tensor of {x.numel()} elements on the input's device")
    with torch.cuda.device(x.device):
        st = _lib.tcr_irregular_scan_ex(x.data_ptr(), offsets.data_ptr(), out.data_ptr(), x.numel(), nseg, flags,
                                        _stream_handle(stream))
    if st != OK:
        raise TcrError(st, "tcr_irregular_scan_ex")
    return out


def reduce(x: torch.Tensor, out: Optional[torch.Tensor] = None,
           stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """tcr_reduce: one-element tensor holding the sum of x."""
    _check_input(x)
    if out is None:
        out = torch.empty(1, dtype=torch.float32, device=x.device)
    _check_output(out, 1, x)
    with torch.cuda.device(x.device):
        st = _lib.tcr_reduce(x.data_ptr(), out.data_ptr(), x.numel(), _stream_handle(stream))
    if st != OK:
        raise TcrError(st, "tcr_reduce")
    return out


def scan(x: torch.Tensor, out: Optional[torch.Tensor] = None,
         stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """tcr_scan: inclusive running sums of x."""
    _check_input(x)
    if out is None:
        out = torch.empty(x.numel(), dtype=torch.float32, device=x.device)
    _check_output(out, x.numel(), x)
    with torch.cuda.device(x.device):
        st = _lib.tcr_scan(x.data_ptr(), out.data_ptr(), x.numel(), _stream_handle(stream))
    if st != OK:
        raise TcrError(st, "tcr_scan")
    return out


def autotune(op: int, x: torch.Tensor, out: torch.Tensor, seg_len: int,
             stream: Optional[torch.cuda.Stream] = None) -> None:
    """tcr_autotune: time the candidate launch shapes for (op, x.numel(), seg_len) and keep the fastest."""
    _check_input(x)
    if not (out.is_cuda and out.dtype == torch.float32 and out.is_contiguous() and out.device == x.device):
        raise TypeError("out must be a contiguous float32 CUDA tensor on the input's device")
    need = x.numel() if op in (OP_SEGMENTED_SCAN, OP_SCAN) else (1 if op == OP_REDUCE else x.numel() // max(seg_len, 1))
    if out.numel() < need:
        raise TypeError(f"out needs at least {need} elements")
    with torch.cuda.device(x.device):
        st = _lib.tcr_autotune(op, x.data_ptr(), out.data_ptr(), x.numel(), seg_len, _stream_handle(stream))
    if st != OK:
        raise TcrError(st, "tcr_autotune")


def autotune_irregular(op: int, x: torch.Tensor, offsets: torch.Tensor, out: torch.Tensor,
                       stream: Optional[torch.cuda.Stream] = None) -> None:
    """tcr_autotune_irregular: time the tile shapes of the irregular reduce (op 4) or scan (op 5) and keep the fastest."""
    _check_input(x)
    nseg = _check_offsets(x, offsets)
    need = x.numel() if op == OP_IRREGULAR_SCAN else nseg
    if not (out.is_cuda and out.dtype == torch.float32 and out.is_contiguous() and out.device == x.device and out.numel() >= need):
        raise TypeError(f"out must be a contiguous float32 CUDA tensor of at least {need} elements on the input's device")
    with torch.cuda.device(x.device):
        st = _lib.tcr_autotune_irregular(op, x.data_ptr(), offsets.data_ptr(), out.data_ptr(), x.numel(), nseg, _stream_handle(stream))
    if st != OK:
        raise TcrError(st, "tcr_autotune_irregular")


def tuning_export() -> str:
    size = _lib.tcr_tuning_export(None, 0)
    buf = ctypes.create_string_buffer(int(size))
    _lib.tcr_tuning_export(buf, size)
    return buf.value.decode()


def tuning_import(text: str) -> None:
    st = _lib.tcr_tuning_import(text.encode())
    if st != OK:
        raise TcrError(st, "tcr_tuning_import")


def segmented_moments(x: torch.Tensor, seg_len: int, stream: Optional[torch.cuda.Stream] = None):
    """tcr_segmented_moments: (sum, sum of squares) of every segment, two float32 tensors."""
    _check_input(x)
    n = x.numel()
    count = n // seg_len if seg_len > 0 else 0
    a = torch.empty(count, dtype=torch.float32, device=x.device)
    q = torch.empty(count, dtype=torch.float32, device=x.device)
    with torch.cuda.device(x.device):
        st = _lib.tcr_segmented_moments(x.data_ptr(), a.data_ptr(), q.data_ptr(), n, seg_len, _stream_handle(stream))
    if st != OK:
        raise TcrError(st, "tcr_segmented_moments")
    return a, q


def workspace_bytes(op: int, n: int, seg_len: int) -> int:
    return int(_lib.tcr_workspace_bytes(op, n, seg_len))


def set_workspace(buffer: Optional[torch.Tensor]) -> None:
    """tcr_set_workspace: use `buffer` (any contiguous CUDA tensor; the caller keeps it alive) on its device, or
    return the current device to library-owned workspaces with None."""
    if buffer is None:
        st = _lib.tcr_set_workspace(None, 0)
    else:
        if not (buffer.is_cuda and buffer.is_contiguous()):
            raise TypeError("workspace must be a contiguous CUDA tensor")
        with torch.cuda.device(buffer.device):
            st = _lib.tcr_set_workspace(buffer.data_ptr(), buffer.numel() * buffer.element_size())
    if st != OK:
        raise TcrError(st, "tcr_set_workspace")


def set_variant(key: str, value: str = "") -> None:
    st = _lib.tcr_set_variant(key.encode(), value.encode())
    if st != OK:
        raise TcrError(st, f"tcr_set_variant({key!r}, {value!r})")


def kernel_name(op: int, n: int, seg_len: int) -> str:
    return _lib.tcr_kernel_name(op, n, seg_len).decode()


def check_device_flags(stream: Optional[torch.cuda.Stream] = None) -> None:
    st = _lib.tcr_check_device_flags(_stream_handle(stream))
    if st != OK:
        raise TcrError(st, "tcr_check_device_flags")


def release() -> None:
    _lib.tcr_release()


def release_stream(stream: Optional[torch.cuda.Stream] = None) -> None:
    st = _lib.tcr_release_stream(_stream_handle(stream))
    if st != OK:
        raise TcrError(st, "tcr_release_stream")


def raw() -> ctypes.CDLL:
    """The loaded library, for tests that exercise the C ABI's own error paths."""
    return _lib
