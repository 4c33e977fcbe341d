"""Thin Python binding of the C-ABI library declared in ``include/minhash.h``.

Argument marshalling only: every step of the path (row binning, hashing,
minima, truncation, packing) runs in the HIP kernels of ``libminhash.so``.
PyTorch is used for device memory and streams, nothing else.  There is no CPU
fallback: if the shared library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

FAMILY_2U_M31 = 0
FAMILY_4U_M31 = 1
FAMILY_2U_M61 = 2
FAMILY_4U_M61 = 3
FAMILY_PERM = 4
FAMILY_2U_MS32 = 5
FAMILY_2U_MS32_HIGH = 6
FLAG_VALIDATE = 1
FLAG_GENERIC_MOD = 2
FLAG_EXACT_FOLD = 4
WORKSPACE_ALIGN = 256
STATIC_SCRATCH_BYTES = 64 << 20
ERR_TOO_LARGE = -10

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libminhash.so")

EXPORTS = (
    "minhash_signatures",
    "minhash_signatures_profiled",
    "minhash_signatures_static",
    "minhash_workspace_bytes",
    "minhash_check_coeffs",
    "minhash_status",
    "minhash_status_async",
    "minhash_pack_indices",
    "minhash_unpack_indices",
    "minhash_signatures_packed",
    "minhash_expand_indices",
    "minhash_match_counts",
    "minhash_resemblance_estimates",
    "minhash_libsvm_count",
    "minhash_libsvm_parse",
    "minhash_error_string",
    "minhash_last_hip_error",
    "minhash_version",
)


class MinhashError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__("minhash error %d: %s" % (code, text))
        self.code = code


_lib = None


def lib() -> ctypes.CDLL:
    """Loads libminhash.so; raises if it has not been built (python -m paper_1205_2958_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                "%s is missing: build it with `python -m paper_1205_2958_amd.build`; "
                "there is no fallback implementation" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, i32, u64, u32, sz = (ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64,
                                      ctypes.c_uint32, ctypes.c_size_t)
        sig = [vp, vp, i64, u64, i32, i32, i32, vp, i64, vp, i64, vp, sz, vp, u32]
        L.minhash_signatures.argtypes = sig
        L.minhash_signatures.restype = ctypes.c_int
        L.minhash_signatures_profiled.argtypes = sig + [ctypes.POINTER(ctypes.c_float)]
        L.minhash_signatures_profiled.restype = ctypes.c_int
        L.minhash_signatures_static.argtypes = [vp, vp, i64, i64, u64, i32, i32, i32, vp, i64, vp, i64, vp, vp, u32]
        L.minhash_signatures_static.restype = ctypes.c_int
        L.minhash_workspace_bytes.argtypes = [i64, i64, i32, i32]
        L.minhash_workspace_bytes.restype = sz
        L.minhash_check_coeffs.argtypes = [vp, i32, i32]
        L.minhash_check_coeffs.restype = ctypes.c_int
        L.minhash_status.argtypes = [vp, vp]
        L.minhash_status.restype = ctypes.c_int
        L.minhash_status_async.argtypes = [vp, vp, vp]
        L.minhash_status_async.restype = ctypes.c_int
        L.minhash_pack_indices.argtypes = [vp, vp, i64, vp, vp, vp, i64, vp, vp]
        L.minhash_pack_indices.restype = ctypes.c_int
        L.minhash_unpack_indices.argtypes = [vp, vp, vp, vp, i64, i64, vp, vp, vp]
        L.minhash_unpack_indices.restype = ctypes.c_int
        L.minhash_signatures_packed.argtypes = [vp, vp, vp, vp, i64, i64, u64, i32, i32, i32, vp, vp, i64, vp, sz, vp, u32]
        L.minhash_signatures_packed.restype = ctypes.c_int
        L.minhash_expand_indices.argtypes = [vp, i64, i64, i32, i32, vp, vp]
        L.minhash_expand_indices.restype = ctypes.c_int
        L.minhash_match_counts.argtypes = [vp, i64, i64, i32, i32, vp, i64, vp, vp]
        L.minhash_match_counts.restype = ctypes.c_int
        L.minhash_resemblance_estimates.argtypes = [vp, vp, vp, i64, u64, i32, i32, vp, vp]
        L.minhash_resemblance_estimates.restype = ctypes.c_int
        L.minhash_libsvm_count.argtypes = [vp, sz, i32, i32, ctypes.POINTER(i64), ctypes.POINTER(i64),
                                           ctypes.POINTER(ctypes.c_uint32), vp]
        L.minhash_libsvm_count.restype = ctypes.c_int
        L.minhash_libsvm_parse.argtypes = [vp, sz, i32, i32, i64, i64, vp, vp, vp, vp]
        L.minhash_libsvm_parse.restype = ctypes.c_int
        L.minhash_error_string.argtypes = [ctypes.c_int]
        L.minhash_error_string.restype = ctypes.c_char_p
        L.minhash_last_hip_error.argtypes = []
        L.minhash_last_hip_error.restype = ctypes.c_char_p
        L.minhash_version.argtypes = []
        L.minhash_version.restype = ctypes.c_int
        _lib = L
    return _lib


def error_string(code: int) -> str:
    return lib().minhash_error_string(code).decode()


def _raise(code: int):
    text = error_string(code)
    if code == -7:
        text += " (" + lib().minhash_last_hip_error().decode() + ")"
    raise MinhashError(code, text)


def version() -> int:
    return lib().minhash_version()


def workspace_bytes(n_rows: int, nnz_upper_bound: int, k: int, family: int) -> int:
    return int(lib().minhash_workspace_bytes(n_rows, nnz_upper_bound, k, family))


def check_coeffs(host_coeffs, family: int) -> None:
    """host_coeffs: NumPy uint64 [k, degree] on the host."""
    import numpy as np

    c = np.ascontiguousarray(host_coeffs, dtype=np.uint64)
    rc = lib().minhash_check_coeffs(c.ctypes.data_as(ctypes.c_void_p), c.shape[0], family)
    if rc != 0:
        _raise(rc)


def alloc_workspace(n_rows: int, nnz_upper_bound: int, k: int, family: int, device) -> torch.Tensor:
    nbytes = workspace_bytes(n_rows, nnz_upper_bound, k, family)
    if nbytes == 0:
        raise MinhashError(-1, "workspace size query rejected the arguments")
    ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
    assert ws.data_ptr() % WORKSPACE_ALIGN == 0
    return ws


def _ptr(t: Optional[torch.Tensor]) -> int:
    return 0 if t is None else t.data_ptr()


def _stream_handle(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream


def _check_common(row_ptr, col_idx, params, family):
    if row_ptr.dtype != torch.int64 or not row_ptr.is_contiguous():
        raise TypeError("row_ptr must be a contiguous int64 tensor")
    if col_idx.element_size() != 4 or not col_idx.is_contiguous():
        raise TypeError("col_idx must be a contiguous tensor of 4-byte unsigned indices (int32/uint32 storage)")
    if not params.is_contiguous():
        raise TypeError("params must be contiguous")
    want = 4 if family == FAMILY_PERM else 8
    if params.element_size() != want:
        raise TypeError("params must hold %d-byte elements for this family (uint64 coefficients, uint32 table entries)"
                        % want)
    for name, t in (("col_idx", col_idx), ("params", params)):
        if t.device != row_ptr.device:
            raise TypeError("%s must be on the device of row_ptr" % name)


def _check_out(out, row_ptr):
    """The library writes every byte of a row's pitch (signature, then zeros), so the
    tensor must own all of them: 2-d uint8, contiguous, one row per data row."""
    if out.dtype != torch.uint8 or out.dim() != 2 or out.device != row_ptr.device:
        raise TypeError("out must be a 2-d uint8 tensor on the device of row_ptr")
    if out.shape[0] != row_ptr.numel() - 1:
        raise TypeError("out must have one row per data row")
    if not out.is_contiguous():
        raise TypeError("out must be contiguous (the row pitch is its second dimension)")


def _marshal(row_ptr, col_idx, D, k, b, family, params, out, out_stride, perm_ld, workspace, stream):
    _check_common(row_ptr, col_idx, params, family)
    n_rows = row_ptr.numel() - 1
    sig_bytes = (k * b + 7) // 8
    if out is None:
        out_stride = sig_bytes if out_stride is None else out_stride
        out = torch.empty((n_rows, out_stride), dtype=torch.uint8, device=row_ptr.device)
    else:
        _check_out(out, row_ptr)
        if out_stride is not None and out_stride != out.shape[1]:
            raise TypeError("out_stride %d does not match the row pitch %d of out" % (out_stride, out.shape[1]))
        out_stride = out.shape[1]
    if workspace is not None and (workspace.device != row_ptr.device or not workspace.is_contiguous()):
        raise TypeError("workspace must be a contiguous tensor on the device of row_ptr")
    if family == FAMILY_PERM:
        if perm_ld is None:
            perm_ld = params.shape[1]
    else:
        perm_ld = 0
    if workspace is None:
        workspace = alloc_workspace(n_rows, col_idx.numel(), k, family, row_ptr.device)
    args = [_ptr(row_ptr), _ptr(col_idx), n_rows, D, k, b, family, _ptr(params), perm_ld, _ptr(out), out_stride,
            _ptr(workspace), workspace.numel() * workspace.element_size(), _stream_handle(stream)]
    return args, out, workspace


def minhash_signatures(row_ptr: torch.Tensor, col_idx: torch.Tensor, D: int, k: int, b: int, family: int,
                       params: torch.Tensor, out: Optional[torch.Tensor] = None, out_stride: Optional[int] = None,
                       perm_ld: Optional[int] = None, workspace: Optional[torch.Tensor] = None, stream=None,
                       flags: int = 0) -> torch.Tensor:
    """Enqueues the signature computation on ``stream`` (default: torch's current
    stream) and returns the uint8 [n_rows, out_stride] output tensor.  Does not
    synchronise.  All tensors live on the GPU; see include/minhash.h for layouts."""
    args, out, workspace = _marshal(row_ptr, col_idx, D, k, b, family, params, out, out_stride, perm_ld, workspace,
                                    stream)
    rc = lib().minhash_signatures(*args, flags)
    if rc != 0:
        _raise(rc)
    return out


def minhash_signatures_profiled(row_ptr, col_idx, D, k, b, family, params, out=None, out_stride=None, perm_ld=None,
                                workspace=None, stream=None, flags: int = 0) -> Tuple[torch.Tensor, float]:
    """Same, but waits for the stream and also returns the duration (ms) of the
    hash / gather kernel measured with HIP events on that stream."""
    args, out, workspace = _marshal(row_ptr, col_idx, D, k, b, family, params, out, out_stride, perm_ld, workspace,
                                    stream)
    ms = ctypes.c_float(0.0)
    rc = lib().minhash_signatures_profiled(*args, flags, ctypes.byref(ms))
    if rc != 0:
        _raise(rc)
    return out, float(ms.value)


def minhash_signatures_static(row_ptr: torch.Tensor, col_idx: torch.Tensor, nnz_upper_bound: int, D: int, k: int, b: int,
                              family: int, params: torch.Tensor, out: torch.Tensor, status: Optional[torch.Tensor] = None,
                              perm_ld: Optional[int] = None, stream=None, flags: int = 0) -> torch.Tensor:
    """The same computation in the library's built-in work space, for callers that
    may not allocate: ``out`` (uint8 [n_rows, out_stride]) and the optional
    ``status`` (one int32 on the device) are the caller's, nothing is allocated
    here or in the library.  Raises MinhashError(ERR_TOO_LARGE) for a batch the
    built-in buffer cannot serve."""
    _check_common(row_ptr, col_idx, params, family)
    _check_out(out, row_ptr)
    if status is not None and (status.dtype != torch.int32 or status.numel() < 1 or status.device != row_ptr.device):
        raise TypeError("status must be an int32 tensor on the device of the inputs")
    if family == FAMILY_PERM:
        perm_ld = params.shape[1] if perm_ld is None else perm_ld
    else:
        perm_ld = 0
    rc = lib().minhash_signatures_static(_ptr(row_ptr), _ptr(col_idx), row_ptr.numel() - 1, nnz_upper_bound, D, k, b,
                                         family, _ptr(params), perm_ld, _ptr(out), out.shape[1], _ptr(status),
                                         _stream_handle(stream), flags)
    if rc != 0:
        _raise(rc)
    return out


def status(workspace: torch.Tensor, stream=None) -> int:
    """Waits for the stream; 0, or the negative code of what VALIDATE found."""
    return int(lib().minhash_status(_ptr(workspace), _stream_handle(stream)))


def status_async(workspace: torch.Tensor, status_out: torch.Tensor, stream=None) -> None:
    """Enqueues the store of what ``status`` would report into ``status_out`` (one int32 on the device)."""
    if status_out.dtype != torch.int32 or status_out.numel() < 1 or status_out.device != workspace.device:
        raise TypeError("status_out must be an int32 tensor on the device of the workspace")
    rc = lib().minhash_status_async(_ptr(workspace), _ptr(status_out), _stream_handle(stream))
    if rc != 0:
        _raise(rc)


def pack_indices(row_ptr: torch.Tensor, col_idx: torch.Tensor, stream=None):
    """Sorted rows as tiles of differences (see include/minhash.h).  Returns device tensors
    (width int32-storage [n], word_ptr int64 [n+1], words int32-storage [word_ptr[n]]); waits
    for the stream to learn the size and raises if a row was not sorted."""
    if row_ptr.dtype != torch.int64 or not row_ptr.is_contiguous() or col_idx.element_size() != 4 or not col_idx.is_contiguous():
        raise TypeError("row_ptr must be contiguous int64, col_idx contiguous with 4-byte elements")
    n = row_ptr.numel() - 1
    dev = row_ptr.device
    width = torch.empty(max(n, 1), dtype=torch.int32, device=dev)
    word_ptr = torch.empty(n + 1, dtype=torch.int64, device=dev)
    words = torch.empty(max(col_idx.numel(), 1), dtype=torch.int32, device=dev)
    st = torch.empty(1, dtype=torch.int32, device=dev)
    rc = lib().minhash_pack_indices(_ptr(row_ptr), _ptr(col_idx), n, _ptr(width), _ptr(word_ptr), _ptr(words),
                                    col_idx.numel(), _ptr(st), _stream_handle(stream))
    if rc != 0:
        _raise(rc)
    code = int(st.item())
    if code != 0:
        _raise(code)
    return width[:n], word_ptr, words[: int(word_ptr[-1].item())]


def unpack_indices(row_ptr: torch.Tensor, width: torch.Tensor, word_ptr: torch.Tensor, words: torch.Tensor,
                   out: torch.Tensor, status: torch.Tensor, stream=None) -> torch.Tensor:
    """Enqueues the decoding of packed rows into ``out`` (4-byte elements, at least
    row_ptr[-1] of them); ``status`` (one int32 on the device) receives the result code.
    Does not synchronise."""
    for t in (width, word_ptr, words, out):
        if not t.is_contiguous() or t.device != row_ptr.device:
            raise TypeError("packed arrays must be contiguous tensors on the device of row_ptr")
    if width.element_size() != 4 or words.element_size() != 4 or out.element_size() != 4 or word_ptr.dtype != torch.int64:
        raise TypeError("width, words and out hold 4-byte elements, word_ptr int64")
    n = row_ptr.numel() - 1
    rc = lib().minhash_unpack_indices(_ptr(row_ptr), _ptr(width), _ptr(word_ptr), _ptr(words), words.numel(), n, _ptr(out),
                                      _ptr(status), _stream_handle(stream))
    if rc != 0:
        _raise(rc)
    return out


def minhash_signatures_packed(row_ptr: torch.Tensor, width: torch.Tensor, word_ptr: torch.Tensor, words: torch.Tensor, D: int,
                              k: int, b: int, family: int, params: torch.Tensor, out: Optional[torch.Tensor] = None,
                              workspace: Optional[torch.Tensor] = None, nnz_upper_bound: Optional[int] = None, stream=None,
                              flags: int = 0) -> torch.Tensor:
    """Signatures of rows given as tiles of differences (``pack_indices``), decoded inside the hash
    kernels.  ``nnz_upper_bound`` sizes the workspace when none is passed (a tile never takes more
    words than it has indices, but it may take fewer, so the word count is no bound); without it the
    last entry of row_ptr is read from the device.  Does not synchronise otherwise."""
    for t in (width, word_ptr, words, params):
        if not t.is_contiguous() or t.device != row_ptr.device:
            raise TypeError("arrays must be contiguous tensors on the device of row_ptr")
    if row_ptr.dtype != torch.int64 or word_ptr.dtype != torch.int64 or width.element_size() != 4 or words.element_size() != 4:
        raise TypeError("row_ptr and word_ptr are int64, width and words hold 4-byte elements")
    if params.element_size() != 8:
        raise TypeError("params must hold uint64 coefficients")
    n = row_ptr.numel() - 1
    sig = (k * b + 7) // 8
    if out is None:
        out = torch.empty((n, sig), dtype=torch.uint8, device=row_ptr.device)
    else:
        _check_out(out, row_ptr)
    if workspace is None:
        if nnz_upper_bound is None:
            nnz_upper_bound = int((row_ptr[-1] - row_ptr[0]).item()) if n > 0 else 0
        workspace = alloc_workspace(n, nnz_upper_bound, k, family, row_ptr.device)
    rc = lib().minhash_signatures_packed(_ptr(row_ptr), _ptr(width), _ptr(word_ptr), _ptr(words), words.numel(), n, D, k, b,
                                         family, _ptr(params), _ptr(out), out.shape[1], _ptr(workspace),
                                         workspace.numel() * workspace.element_size(), _stream_handle(stream), flags)
    if rc != 0:
        _raise(rc)
    return out


def expand_indices(sig: torch.Tensor, k: int, b: int, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """int32-storage [n_rows, k] tensor of uint32 positions j*2^b + s_ij (see include/minhash.h)."""
    n = sig.shape[0]
    if out is None:
        out = torch.empty((n, k), dtype=torch.int32, device=sig.device)
    rc = lib().minhash_expand_indices(_ptr(sig), n, sig.stride(0), k, b, _ptr(out), _stream_handle(stream))
    if rc != 0:
        _raise(rc)
    return out


def match_counts(sig: torch.Tensor, k: int, b: int, pairs: torch.Tensor, out: Optional[torch.Tensor] = None,
                 stream=None) -> torch.Tensor:
    """int32-storage [n_pairs] tensor of uint32 counts of equal b-bit values; pairs is int64 [n_pairs, 2]."""
    n_pairs = pairs.shape[0]
    if pairs.dtype != torch.int64 or not pairs.is_contiguous():
        raise TypeError("pairs must be a contiguous int64 tensor [n_pairs, 2]")
    if out is None:
        out = torch.empty(n_pairs, dtype=torch.int32, device=sig.device)
    rc = lib().minhash_match_counts(_ptr(sig), sig.shape[0], sig.stride(0), k, b, _ptr(pairs), n_pairs, _ptr(out),
                                    _stream_handle(stream))
    if rc != 0:
        _raise(rc)
    return out


def resemblance_estimates(counts: torch.Tensor, f1: torch.Tensor, f2: torch.Tensor, D: int, k: int, b: int,
                          out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """float64 [n_pairs] tensor of R_b-hat; f1, f2 are int64 set sizes."""
    n_pairs = counts.shape[0]
    if out is None:
        out = torch.empty(n_pairs, dtype=torch.float64, device=counts.device)
    rc = lib().minhash_resemblance_estimates(_ptr(counts), _ptr(f1), _ptr(f2), n_pairs, D, k, b, _ptr(out),
                                             _stream_handle(stream))
    if rc != 0:
        _raise(rc)
    return out


def parse_libsvm(buf, index_base: int = 1, n_threads: int = 16, pin_memory: bool = False, labels: bool = True):
    """Parses LibSVM text held in ``buf`` (bytes, bytearray, mmap or anything with the
    buffer protocol) into host tensors (row_ptr int64 [n+1], col_idx int32-storage
    uint32 [nnz], labels float32 [n] or None) and returns them with the largest index.
    The arrays can be pinned so that they feed ``stream_batches`` directly."""
    import numpy as np

    view = np.frombuffer(buf, dtype=np.uint8)
    ptr = view.ctypes.data if view.size else 0
    n_rows, nnz, mx = ctypes.c_int64(0), ctypes.c_int64(0), ctypes.c_uint32(0)
    n_threads = max(1, int(n_threads))
    shares = np.zeros(2 * n_threads, dtype=np.int64)                   # per-thread counts, handed from pass 1 to pass 2
    rc = lib().minhash_libsvm_count(ptr, view.size, index_base, n_threads, ctypes.byref(n_rows), ctypes.byref(nnz),
                                    ctypes.byref(mx), shares.ctypes.data)
    if rc != 0:
        _raise(rc)
    row_ptr = torch.empty(n_rows.value + 1, dtype=torch.int64, pin_memory=pin_memory)
    col_idx = torch.empty(nnz.value, dtype=torch.int32, pin_memory=pin_memory)
    lab = torch.empty(n_rows.value, dtype=torch.float32) if labels else None
    rc = lib().minhash_libsvm_parse(ptr, view.size, index_base, n_threads, n_rows.value, nnz.value, shares.ctypes.data,
                                    row_ptr.data_ptr(), col_idx.data_ptr(), lab.data_ptr() if labels else 0)
    if rc != 0:
        _raise(rc)
    return row_ptr, col_idx, lab, int(mx.value)


def _slice_cuts(offsets_h: torch.Tensor, n: int, total: int, n_slices: int):
    """Rows at which a batch is cut into about n_slices slices of equal payload (offsets_h: the pinned
    int64 prefix array of the payload, row_ptr or word_ptr, starting at 0)."""
    if n_slices <= 1 or n < n_slices or total <= 0:
        return [0, n]
    marks = torch.searchsorted(offsets_h, torch.arange(1, n_slices, dtype=torch.int64) * (total // n_slices))
    return sorted(set([0, n] + [int(min(max(int(m), 1), n)) for m in marks]))


def _copy_in_slices(dst: torch.Tensor, pieces, offsets_h: torch.Tensor, cuts, total: int, events, stream) -> None:
    """Copies the pieces of a payload array into dst on `stream`, cutting them again where a slice of rows
    ends, and records events[c] when the payload of slice c (rows cuts[c] .. cuts[c+1]) is complete; the
    last slice is complete when the caller's own event after this call is."""
    at, next_cut = 0, 1
    for p in pieces:
        done = 0
        while done < p.numel():
            upto = int(offsets_h[cuts[next_cut]]) if next_cut < len(cuts) - 1 else total
            take = min(p.numel() - done, max(upto - at, 0))
            if take > 0:
                dst[at: at + take].copy_(p[done: done + take].view(torch.int32), non_blocking=True)
                at += take
                done += take
            if at >= upto and next_cut < len(cuts) - 1:
                events[next_cut - 1].record(stream)
                next_cut += 1
    while next_cut < len(cuts) - 1:               # slices whose rows are empty at the end of the payload
        events[next_cut - 1].record(stream)
        next_cut += 1


def stream_batches(batches, D: int, k: int, b: int, family: int, params: torch.Tensor, max_rows: int, max_nnz: int,
                   perm_ld: Optional[int] = None, flags: int = 0, edge_slices: int = 4):
    """Streams host-resident batches through the GPU with copies and kernels
    overlapped (the three-phase batch loop of Section 3.2: copy a chunk of sets to
    the GPU, hash it there, copy the results back, repeat).

    ``batches`` is a sequence of ``(row_ptr, col_idx)`` pairs of pinned host
    tensors, row_ptr rebased to start at 0; col_idx may also be a list of pinned
    tensors holding consecutive pieces of the index array (torch's pinned
    allocator rounds every request up to a power of two, so large arrays are
    cheaper to pin in 1 GiB pieces).  Batch i+1 is copied host-to-device on
    a side stream while batch i is hashed on the compute stream and the
    signatures of batch i-1 travel back on a third stream; two sets of device
    buffers alternate.  The first and the last batch go in ``edge_slices`` slices
    of rows with about equal numbers of indices, each hashed as soon as its indices
    have arrived: nothing hides the first copy or the last kernel, so both are made
    short.  Returns the list of pinned uint8 host tensors
    [n_rows_i, ceil(k*b/8)], complete when the function returns.
    """
    dev = params.device
    sig = (k * b + 7) // 8
    n_buf = 2
    rp_d = [torch.empty(max_rows + 1, dtype=torch.int64, device=dev) for _ in range(n_buf)]
    col_d = [torch.empty(max_nnz, dtype=torch.int32, device=dev) for _ in range(n_buf)]
    out_d = [torch.empty((max_rows, sig), dtype=torch.uint8, device=dev) for _ in range(n_buf)]
    ws = alloc_workspace(max_rows, max_nnz, k, family, dev)
    n_slices = max(1, edge_slices)
    codes = torch.zeros(len(batches) + 2 * n_slices, dtype=torch.int32, device=dev)     # what each call reported: the next one clears it
    n_calls = 0
    slice_done = [torch.cuda.Event() for _ in range(n_slices)]
    s_in, s_run, s_out = torch.cuda.Stream(dev), torch.cuda.Stream(dev), torch.cuda.Stream(dev)
    now = torch.cuda.current_stream(dev)
    for s in (s_in, s_run, s_out):
        s.wait_stream(now)
    in_done = [torch.cuda.Event() for _ in range(n_buf)]
    run_done = [torch.cuda.Event() for _ in range(n_buf)]
    out_done = [torch.cuda.Event() for _ in range(n_buf)]
    results = []
    for i, (rp_h, col_h) in enumerate(batches):
        n = rp_h.numel() - 1
        pieces = list(col_h) if isinstance(col_h, (list, tuple)) else [col_h]
        nnz = sum(p.numel() for p in pieces)
        if n > max_rows or nnz > max_nnz:
            raise ValueError("batch %d exceeds max_rows / max_nnz" % i)
        u = i % n_buf
        out_h = torch.empty((n, sig), dtype=torch.uint8, pin_memory=True)
        results.append(out_h)
        if i >= n_buf:
            s_in.wait_event(run_done[u])          # the kernel that read this input buffer has finished
        edge = i == 0 or i == len(batches) - 1
        cuts = _slice_cuts(rp_h, n, nnz, n_slices) if edge and int(rp_h[0]) == 0 else [0, n]
        with torch.cuda.stream(s_in):
            rp_d[u][: n + 1].copy_(rp_h, non_blocking=True)
            _copy_in_slices(col_d[u], pieces, rp_h, cuts, nnz, slice_done, s_in)
            in_done[u].record(s_in)
        if i >= n_buf:
            s_run.wait_event(out_done[u])         # the previous signatures left this output buffer
        for c in range(len(cuts) - 1):            # (offsets in row_ptr are absolute: a slice is the same arrays from another row on)
            r0, r1 = cuts[c], cuts[c + 1]
            s_run.wait_event(slice_done[c] if c < len(cuts) - 2 else in_done[u])
            minhash_signatures(rp_d[u][r0: r1 + 1], col_d[u][:nnz], D, k, b, family, params, out=out_d[u][r0:r1],
                               out_stride=sig, perm_ld=perm_ld, workspace=ws, stream=s_run, flags=flags)
            if r1 > r0:
                status_async(ws, codes[n_calls: n_calls + 1], stream=s_run)
                n_calls += 1
        run_done[u].record(s_run)
        s_out.wait_event(run_done[u])
        with torch.cuda.stream(s_out):
            out_h.copy_(out_d[u][:n], non_blocking=True)
            out_done[u].record(s_out)
    for s in (s_in, s_run, s_out):
        s.synchronize()
    now.wait_stream(s_out)
    # the deferred checks of every batch (work-list overflow, MINHASH_FLAG_VALIDATE findings); every batch was
    # bounded by max_rows / max_nnz above, so an overflow can only come from offsets that contradict the sizes
    bad = [int(c) for c in codes[:n_calls].cpu().tolist() if c != 0]
    if bad:
        _raise(bad[0])
    return results


def stream_batches_packed(batches, D: int, k: int, b: int, family: int, params: torch.Tensor, max_rows: int, max_nnz: int,
                          max_words: int, flags: int = 0, decode_in_kernel: bool = True, edge_slices: int = 4):
    """``stream_batches`` for rows that cross the host link as tiles of differences
    (``pack_indices``): about half the bytes for sorted heavy-tailed rows, so that
    the copies hide under the kernels again.

    ``batches`` is a sequence of ``(row_ptr, width, word_ptr, words)`` of pinned host
    tensors (``words`` may be a list of pinned pieces).  Per batch: copy on one
    stream, decode into a col_idx buffer and hash on a second (the decoder runs right
    before the hash kernels of its batch: launched on a stream of its own it would
    wait for the persistent hash kernel of the batch before anyway, and start late),
    signatures back on a third; two sets of packed buffers alternate.  Returns the
    pinned uint8 host tensors [n_rows_i, ceil(k*b/8)], complete on return.

    With ``decode_in_kernel`` (the default) there is no decoder pass at all: the
    hash kernels fetch the words and decode each tile while they stage it
    (``minhash_signatures_packed``).  The first and the last batch then go in
    ``edge_slices`` slices of rows with about equal numbers of words, each
    hashed as soon as its words have arrived (the offsets in word_ptr are absolute,
    so a slice is the same arrays from another row on): nothing hides the first
    copy or the last kernel, so both are made short.
    """
    dev = params.device
    sig = (k * b + 7) // 8
    n_buf = 2
    rp_d = [torch.empty(max_rows + 1, dtype=torch.int64, device=dev) for _ in range(n_buf)]
    wp_d = [torch.empty(max_rows + 1, dtype=torch.int64, device=dev) for _ in range(n_buf)]
    wd_d = [torch.empty(max(max_rows, 1), dtype=torch.int32, device=dev) for _ in range(n_buf)]
    words_d = [torch.empty(max(max_words, 1), dtype=torch.int32, device=dev) for _ in range(n_buf)]
    col_d = None if decode_in_kernel else torch.empty(max(max_nnz, 1), dtype=torch.int32, device=dev)    # one stream: one buffer
    out_d = [torch.empty((max_rows, sig), dtype=torch.uint8, device=dev) for _ in range(n_buf)]
    codes = torch.zeros(max(len(batches), 1), dtype=torch.int32, device=dev)            # the decoder's reports
    n_slices = max(1, edge_slices) if decode_in_kernel else 1
    hash_codes = torch.zeros(len(batches) + 2 * n_slices, dtype=torch.int32, device=dev)    # the hash calls', one per call
    n_calls = 0
    slice_done = [torch.cuda.Event() for _ in range(n_slices)]
    ws = alloc_workspace(max_rows, max_nnz, k, family, dev)
    s_in, s_run, s_out = (torch.cuda.Stream(dev) for _ in range(3))
    now = torch.cuda.current_stream(dev)
    for s in (s_in, s_run, s_out):
        s.wait_stream(now)
    in_done = [torch.cuda.Event() for _ in range(n_buf)]
    run_done = [torch.cuda.Event() for _ in range(n_buf)]
    out_done = [torch.cuda.Event() for _ in range(n_buf)]
    results = []
    for i, (rp_h, width_h, wp_h, words_h) in enumerate(batches):
        n = rp_h.numel() - 1
        pieces = list(words_h) if isinstance(words_h, (list, tuple)) else [words_h]
        n_words = sum(p.numel() for p in pieces)
        nnz = int(rp_h[-1]) - int(rp_h[0])
        if n > max_rows or nnz > max_nnz or n_words > max_words or int(rp_h[0]) != 0:
            raise ValueError("batch %d exceeds max_rows / max_nnz / max_words, or its row_ptr does not start at 0" % i)
        u = i % n_buf
        out_h = torch.empty((n, sig), dtype=torch.uint8, pin_memory=True)
        results.append(out_h)
        if i >= n_buf:
            s_in.wait_event(run_done[u])          # decoder and kernels that read this set of buffers (row_ptr too) have finished
        # rows at which the batch is cut (the first and the last batch only)
        edge = i == 0 or i == len(batches) - 1
        cuts = _slice_cuts(wp_h, n, n_words, n_slices) if edge else [0, n]
        with torch.cuda.stream(s_in):
            rp_d[u][: n + 1].copy_(rp_h, non_blocking=True)
            wp_d[u][: n + 1].copy_(wp_h, non_blocking=True)
            wd_d[u][:n].copy_(width_h.view(torch.int32), non_blocking=True)
            _copy_in_slices(words_d[u], pieces, wp_h, cuts, n_words, slice_done, s_in)
            in_done[u].record(s_in)
        if i >= n_buf:
            s_run.wait_event(out_done[u])         # the previous signatures left this output buffer
        if decode_in_kernel:
            for c in range(len(cuts) - 1):
                r0, r1 = cuts[c], cuts[c + 1]
                s_run.wait_event(slice_done[c] if c < len(cuts) - 2 else in_done[u])
                minhash_signatures_packed(rp_d[u][r0: r1 + 1], wd_d[u][r0:r1], wp_d[u][r0: r1 + 1], words_d[u][:n_words], D, k, b,
                                          family, params, out=out_d[u][r0:r1], workspace=ws,
                                          nnz_upper_bound=max_nnz, stream=s_run, flags=flags)
                if r1 > r0:
                    status_async(ws, hash_codes[n_calls: n_calls + 1], stream=s_run)
                    n_calls += 1
        else:
            s_run.wait_event(in_done[u])
            unpack_indices(rp_d[u][: n + 1], wd_d[u][:n], wp_d[u][: n + 1], words_d[u][:n_words], col_d, codes[i: i + 1],
                           stream=s_run)
            minhash_signatures(rp_d[u][: n + 1], col_d[:nnz], D, k, b, family, params, out=out_d[u][:n],
                               out_stride=sig, workspace=ws, stream=s_run, flags=flags)
            if n > 0:
                status_async(ws, hash_codes[n_calls: n_calls + 1], stream=s_run)
                n_calls += 1
        run_done[u].record(s_run)
        s_out.wait_event(run_done[u])
        with torch.cuda.stream(s_out):
            out_h.copy_(out_d[u][:n], non_blocking=True)
            out_done[u].record(s_out)
    for s in (s_in, s_run, s_out):
        s.synchronize()
    now.wait_stream(s_out)
    bad = [int(c) for c in codes[: len(batches)].cpu().tolist() + hash_codes[:n_calls].cpu().tolist() if c != 0]
    if bad:
        _raise(bad[0])
    return results

