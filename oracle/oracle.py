"""ctypes loader for the plain-C CPU oracle (test infrastructure only).

Nothing here computes anything: it builds ``minhash_oracle.c`` with gcc when
the shared object is missing or stale, and marshals NumPy arrays into the three
C functions.  The arithmetic lives in the C file, which cites the paper.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "minhash_oracle.c")
_LIB = os.path.join(_HERE, "libminhash_oracle.so")

FAMILY_2U_M31, FAMILY_4U_M31, FAMILY_2U_M61, FAMILY_4U_M61, FAMILY_PERM, FAMILY_2U_MS32, FAMILY_2U_MS32_HIGH = range(7)
EMPTY_MIN = 0xFFFFFFFF


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no arch-specific flags)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fPIC", "-shared", _SRC, "-o", tmp, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _bind(path: str):
    lib = ctypes.CDLL(path)
    vp, i64, i32, u64 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64
    lib.minhash_minima_oracle.argtypes = [vp, vp, i64, u64, i32, i32, vp, i64, vp]
    lib.minhash_minima_oracle.restype = ctypes.c_int
    lib.minhash_pack_oracle.argtypes = [vp, i64, i32, i32, vp, i64]
    lib.minhash_pack_oracle.restype = ctypes.c_int
    lib.minhash_signatures_oracle.argtypes = [vp, vp, i64, u64, i32, i32, i32, vp, i64, vp, i64, vp]
    lib.minhash_signatures_oracle.restype = ctypes.c_int
    lib.minhash_expand_oracle.argtypes = [vp, i64, i64, i32, i32, vp]
    lib.minhash_expand_oracle.restype = ctypes.c_int
    lib.minhash_match_counts_oracle.argtypes = [vp, i64, i64, i32, i32, vp, i64, vp]
    lib.minhash_match_counts_oracle.restype = ctypes.c_int
    lib.minhash_resemblance_oracle.argtypes = [vp, vp, vp, i64, u64, i32, i32, vp]
    lib.minhash_resemblance_oracle.restype = ctypes.c_int
    lib.minhash_pack_indices_oracle.argtypes = [vp, vp, i64, vp, vp, vp, i64]
    lib.minhash_pack_indices_oracle.restype = ctypes.c_int
    lib.minhash_unpack_indices_oracle.argtypes = [vp, vp, vp, vp, i64, i64, vp]
    lib.minhash_unpack_indices_oracle.restype = ctypes.c_int
    return lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _prep(row_ptr, col_idx, params, family):
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int64)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.uint32)
    if family == FAMILY_PERM:
        params = np.ascontiguousarray(params, dtype=np.uint32)
        perm_ld = params.shape[1]
    else:
        params = np.ascontiguousarray(params, dtype=np.uint64)
        perm_ld = 0
    return row_ptr, col_idx, params, perm_ld


class Oracle:
    """The three C entry points of one compiled oracle object.

    ``lib_path`` defaults to the in-tree build of ``minhash_oracle.c``; the
    mutation tests pass the path of a deliberately broken build instead.
    """

    def __init__(self, lib_path: str | None = None):
        self._lib = _bind(lib_path if lib_path is not None else build())

    def minima(self, row_ptr, col_idx, D, k, family, params) -> np.ndarray:
        """uint32 [n_rows, k] full minima (0xFFFFFFFF for an empty row)."""
        row_ptr, col_idx, params, perm_ld = _prep(row_ptr, col_idx, params, family)
        n = row_ptr.shape[0] - 1
        out = np.empty((n, k), dtype=np.uint32)
        rc = self._lib.minhash_minima_oracle(_ptr(row_ptr), _ptr(col_idx), n, D, k, family, _ptr(params), perm_ld,
                                             _ptr(out))
        if rc != 0:
            raise ValueError("oracle rejected the arguments: %d" % rc)
        return out

    def pack(self, minima_arr, b, out_stride=None) -> np.ndarray:
        """uint8 [n_rows, out_stride] packed signatures of the lowest b bits."""
        m = np.ascontiguousarray(minima_arr, dtype=np.uint32)
        n, k = m.shape
        sig = (k * b + 7) // 8
        out_stride = sig if out_stride is None else out_stride
        out = np.full((n, out_stride), 0xAA, dtype=np.uint8)
        rc = self._lib.minhash_pack_oracle(_ptr(m), n, k, b, _ptr(out), out_stride)
        if rc != 0:
            raise ValueError("oracle rejected the arguments: %d" % rc)
        return out

    def signatures(self, row_ptr, col_idx, D, k, b, family, params, out_stride=None) -> np.ndarray:
        """uint8 [n_rows, out_stride] packed signatures."""
        row_ptr, col_idx, params, perm_ld = _prep(row_ptr, col_idx, params, family)
        n = row_ptr.shape[0] - 1
        sig = (k * b + 7) // 8
        out_stride = sig if out_stride is None else out_stride
        out = np.full((n, out_stride), 0xAA, dtype=np.uint8)
        scratch = np.empty((max(n, 1), k), dtype=np.uint32)
        rc = self._lib.minhash_signatures_oracle(_ptr(row_ptr), _ptr(col_idx), n, D, k, b, family, _ptr(params),
                                                 perm_ld, _ptr(out), out_stride, _ptr(scratch))
        if rc != 0:
            raise ValueError("oracle rejected the arguments: %d" % rc)
        return out


    def expand(self, sig, k, b) -> np.ndarray:
        """uint32 [n_rows, k]: positions of the ones of the 2^b x k expansion."""
        sig = np.ascontiguousarray(sig, dtype=np.uint8)
        n = sig.shape[0]
        out = np.empty((n, k), dtype=np.uint32)
        rc = self._lib.minhash_expand_oracle(_ptr(sig), n, sig.shape[1], k, b, _ptr(out))
        if rc != 0:
            raise ValueError("oracle rejected the arguments: %d" % rc)
        return out

    def match_counts(self, sig, k, b, pairs) -> np.ndarray:
        """uint32 [n_pairs]: number of equal b-bit values for each pair of rows."""
        sig = np.ascontiguousarray(sig, dtype=np.uint8)
        pairs = np.ascontiguousarray(pairs, dtype=np.int64).reshape(-1, 2)
        out = np.empty(pairs.shape[0], dtype=np.uint32)
        rc = self._lib.minhash_match_counts_oracle(_ptr(sig), sig.shape[0], sig.shape[1], k, b, _ptr(pairs),
                                                   pairs.shape[0], _ptr(out))
        if rc != 0:
            raise ValueError("oracle rejected the arguments: %d" % rc)
        return out

    def resemblance(self, counts, f1, f2, D, k, b) -> np.ndarray:
        """float64 [n_pairs]: the estimator R_b-hat of eq. eqn_R_b."""
        counts = np.ascontiguousarray(counts, dtype=np.uint32)
        f1 = np.ascontiguousarray(f1, dtype=np.int64)
        f2 = np.ascontiguousarray(f2, dtype=np.int64)
        out = np.empty(counts.shape[0], dtype=np.float64)
        rc = self._lib.minhash_resemblance_oracle(_ptr(counts), _ptr(f1), _ptr(f2), counts.shape[0], D, k, b, _ptr(out))
        if rc != 0:
            raise ValueError("oracle rejected the arguments: %d" % rc)
        return out


    def pack_indices(self, row_ptr, col_idx):
        """(width uint32 [n], word_ptr int64 [n+1], words uint32 [word_ptr[n]]): rows as tiles of differences."""
        row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int64)
        col_idx = np.ascontiguousarray(col_idx, dtype=np.uint32)
        n = row_ptr.shape[0] - 1
        width = np.zeros(max(n, 1), dtype=np.uint32)
        word_ptr = np.zeros(n + 1, dtype=np.int64)
        cap = int(row_ptr[-1] - row_ptr[0]) + 1
        words = np.full(cap, 0xAAAAAAAA, dtype=np.uint32)
        rc = self._lib.minhash_pack_indices_oracle(_ptr(row_ptr), _ptr(col_idx), n, _ptr(width), _ptr(word_ptr),
                                                   _ptr(words), cap)
        if rc != 0:
            raise ValueError("oracle rejected the arguments: %d" % rc)
        return width[:n], word_ptr, words[: int(word_ptr[-1])].copy()

    def unpack_indices(self, row_ptr, width, word_ptr, words) -> np.ndarray:
        """uint32 [nnz]: the index array the tiles stand for."""
        row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int64)
        width = np.ascontiguousarray(width, dtype=np.uint32)
        word_ptr = np.ascontiguousarray(word_ptr, dtype=np.int64)
        words = np.ascontiguousarray(words, dtype=np.uint32)
        n = row_ptr.shape[0] - 1
        out = np.full(max(int(row_ptr[-1]), 1), 0xAAAAAAAA, dtype=np.uint32)
        rc = self._lib.minhash_unpack_indices_oracle(_ptr(row_ptr), _ptr(width), _ptr(word_ptr), _ptr(words),
                                                     words.shape[0], n, _ptr(out))
        if rc != 0:
            raise ValueError("oracle rejected the arguments: %d" % rc)
        return out[: int(row_ptr[-1])]


_default = None


def default() -> Oracle:
    global _default
    if _default is None:
        _default = Oracle()
    return _default


def minima(row_ptr, col_idx, D, k, family, params) -> np.ndarray:
    return default().minima(row_ptr, col_idx, D, k, family, params)


def pack(minima_arr, b, out_stride=None) -> np.ndarray:
    return default().pack(minima_arr, b, out_stride)


def signatures(row_ptr, col_idx, D, k, b, family, params, out_stride=None) -> np.ndarray:
    return default().signatures(row_ptr, col_idx, D, k, b, family, params, out_stride)


def expand(sig, k, b) -> np.ndarray:
    return default().expand(sig, k, b)


def match_counts(sig, k, b, pairs) -> np.ndarray:
    return default().match_counts(sig, k, b, pairs)


def resemblance(counts, f1, f2, D, k, b) -> np.ndarray:
    return default().resemblance(counts, f1, f2, D, k, b)


def pack_indices(row_ptr, col_idx):
    return default().pack_indices(row_ptr, col_idx)


def unpack_indices(row_ptr, width, word_ptr, words) -> np.ndarray:
    return default().unpack_indices(row_ptr, width, word_ptr, words)


def unpack(packed: np.ndarray, k: int, b: int) -> np.ndarray:
    """Read the bit layout back, for tests: uint32 [n_rows, k] of b-bit values.
    Written with numpy.unpackbits so that it shares nothing with the C packer."""
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    n = packed.shape[0]
    bits = np.unpackbits(packed, axis=1, bitorder="little")[:, : k * b].reshape(n, k, b)
    weights = (np.uint64(1) << np.arange(b, dtype=np.uint64))
    return (bits.astype(np.uint64) * weights).sum(axis=2).astype(np.uint32)
