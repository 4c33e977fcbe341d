"""Binding of libminhash_probe.so: device-side measurements that the roofline
figures are set against (instruction issue rates of the hash kernels' inner
steps, streaming-read and row-gather bandwidth).  Argument marshalling only.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libminhash_probe.so")
EXPORTS = ("mh_probe_n_kinds", "mh_probe_kind_name", "mh_probe_issue", "mh_probe_stream_read", "mh_probe_copy",
           "mh_probe_gather_rows")
N_SIMPLE = (0, 1, 2, 3, 5)

_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError("%s is missing: build it with `python -m paper_1205_2958_amd.build`" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz, dbl = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t, ctypes.c_double
        fp, dp = ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double)
        L.mh_probe_n_kinds.restype = i32
        L.mh_probe_kind_name.argtypes = [i32]
        L.mh_probe_kind_name.restype = ctypes.c_char_p
        L.mh_probe_issue.argtypes = [i32, i32, i32, i32, dbl, vp, vp, i32, fp, dp]
        L.mh_probe_issue.restype = i32
        L.mh_probe_stream_read.argtypes = [vp, sz, i32, vp, i32, fp]
        L.mh_probe_stream_read.restype = i32
        L.mh_probe_copy.argtypes = [vp, vp, sz, vp, i32, fp]
        L.mh_probe_copy.restype = i32
        L.mh_probe_gather_rows.argtypes = [vp, sz, sz, i32, vp, sz, i32, i32, vp, i32, fp]
        L.mh_probe_gather_rows.restype = i32
        _lib = L
    return _lib


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise RuntimeError("%s failed with code %d" % (what, rc))


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def kinds():
    return [lib().mh_probe_kind_name(i).decode() for i in range(lib().mh_probe_n_kinds())]


def issue(kind: int, n_simple: int, prio: bool, waves_per_simd: int, scratch: torch.Tensor, clock_ghz: float = 2.4,
          reps: int = 3):
    """(ms, issue slots per 1 probed + n_simple simple instructions per SIMD at clock_ghz)."""
    ms, slots = ctypes.c_float(0.0), ctypes.c_double(0.0)
    _check(lib().mh_probe_issue(kind, n_simple, int(prio), waves_per_simd, clock_ghz, scratch.data_ptr(), _stream(), reps,
                                ctypes.byref(ms), ctypes.byref(slots)), "mh_probe_issue")
    return float(ms.value), float(slots.value)


def stream_read(buf: torch.Tensor, blocks_per_cu: int = 8, reps: int = 5) -> float:
    """GB/s of a plain coalesced read of the whole tensor."""
    ms = ctypes.c_float(0.0)
    nbytes = buf.numel() * buf.element_size()
    _check(lib().mh_probe_stream_read(buf.data_ptr(), nbytes, blocks_per_cu, _stream(), reps, ctypes.byref(ms)),
           "mh_probe_stream_read")
    return nbytes / (ms.value * 1e-3) / 1e9


def copy(src: torch.Tensor, dst: torch.Tensor, reps: int = 1) -> float:
    """Launches the copy kernel of known size (reads and writes src's bytes); returns ms."""
    ms = ctypes.c_float(0.0)
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() >= nbytes
    _check(lib().mh_probe_copy(src.data_ptr(), dst.data_ptr(), nbytes, _stream(), reps, ctypes.byref(ms)), "mh_probe_copy")
    return float(ms.value)


def gather_rows(table: torch.Tensor, row_bytes: int, rows: torch.Tensor, in_flight: int = 8, blocks_per_cu: int = 8,
                reps: int = 3) -> float:
    """GB/s (row_bytes per listed row) of reading whole table rows at the given int32 row numbers."""
    assert table.dim() == 2 and table.is_contiguous() and rows.dtype == torch.int32 and rows.is_contiguous()
    pitch = table.shape[1] * table.element_size()
    assert int(rows.max().item()) < table.shape[0] and int(rows.min().item()) >= 0
    ms = ctypes.c_float(0.0)
    _check(lib().mh_probe_gather_rows(table.data_ptr(), table.shape[0], pitch, row_bytes, rows.data_ptr(), rows.numel(),
                                      in_flight, blocks_per_cu, _stream(), reps, ctypes.byref(ms)), "mh_probe_gather_rows")
    n_used = rows.numel() // in_flight * in_flight     # whole groups only; the remainder is below one group per wave
    return float(n_used) * row_bytes / (ms.value * 1e-3) / 1e9
