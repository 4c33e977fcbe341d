"""The C-ABI library without a GPU: it loads, exports what the header declares,
and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_1205_2958_amd import minhash as mh
from paper_1205_2958_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "minhash.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(mh.LIB_PATH):
        from paper_1205_2958_amd import build
        build.build()
    return mh.lib()


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(minhash_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert len(names) >= 8
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(mh.EXPORTS) == names


def test_version_and_error_strings(lib):
    assert mh.version() == 100
    for code in range(0, -10, -1):
        assert mh.error_string(code) and mh.error_string(code) != "unknown error code"
    assert mh.error_string(-99) == "unknown error code"


def test_status_calls_reject_null_pointers(lib):
    import ctypes
    assert lib.minhash_status(None, None) == -1
    assert lib.minhash_status_async(None, None, None) == -1
    assert lib.minhash_status_async(ctypes.c_void_p(256), None, None) == -1


def test_workspace_size_query():
    small = mh.workspace_bytes(1000, 650_000, 64, mh.FAMILY_2U_M31)
    big = mh.workspace_bytes(350_000, 1_300_000_000, 500, mh.FAMILY_2U_M31)
    assert 0 < small < big
    assert small % mh.WORKSPACE_ALIGN == 0 and big % mh.WORKSPACE_ALIGN == 0
    assert mh.workspace_bytes(-1, 10, 64, 0) == 0
    assert mh.workspace_bytes(10, -1, 64, 0) == 0
    assert mh.workspace_bytes(10, 10, 0, 0) == 0
    assert mh.workspace_bytes(10, 10, 64, 9) == 0
    assert mh.workspace_bytes(10, 10, 64, mh.FAMILY_4U_M61) > 0
    assert mh.workspace_bytes(1 << 31, 10, 64, 0) == 0


def test_coefficient_range_check():
    for fam in (mh.FAMILY_2U_M31, mh.FAMILY_4U_M31, mh.FAMILY_2U_M61, mh.FAMILY_4U_M61):
        c = W.coefficients(16, fam, seed=1)
        mh.check_coeffs(c, fam)
        c[3, 1] = W.family_prime(fam)
        with pytest.raises(mh.MinhashError) as e:
            mh.check_coeffs(c, fam)
        assert e.value.code == -8
    with pytest.raises(mh.MinhashError):
        mh.check_coeffs(np.zeros((4, 2), dtype=np.uint64), mh.FAMILY_PERM)
    for fam in (mh.FAMILY_2U_MS32, mh.FAMILY_2U_MS32_HIGH):
        c = W.coefficients(16, fam, seed=2)
        mh.check_coeffs(c, fam)
        bad = c.copy()
        bad[5, 1] &= np.uint64(0xFFFFFFFE)                         # even multiplier
        with pytest.raises(mh.MinhashError) as e:
            mh.check_coeffs(bad, fam)
        assert e.value.code == -8
        bad = c.copy()
        bad[2, 0] = 1 << 32                                        # constant term too wide
        with pytest.raises(mh.MinhashError):
            mh.check_coeffs(bad, fam)


def _call(lib, n_rows=4, D=1 << 24, k=64, b=8, family=0, perm_ld=0, out_stride=64, ws=0x1000, ws_bytes=1 << 20,
          row_ptr=0x1000, col_idx=0x1000, params=0x1000, out=0x1000, flags=0):
    return lib.minhash_signatures(row_ptr, col_idx, n_rows, D, k, b, family, params, perm_ld, out, out_stride, ws,
                                  ws_bytes, 0, flags)


def test_bad_arguments_are_rejected_before_any_launch(lib):
    # (no GPU in this process: had any of these reached a HIP call it would fail differently)
    assert _call(lib, n_rows=0) == 0                                  # empty batch is a no-op
    assert _call(lib, n_rows=-1) == -1
    assert _call(lib, n_rows=1 << 31) == -1
    assert _call(lib, family=7) == -2
    assert _call(lib, family=-1) == -2
    assert _call(lib, family=mh.FAMILY_4U_M61, D=1 << 32, n_rows=0) == 0
    assert _call(lib, family=mh.FAMILY_4U_M61, flags=2) == -1           # no % ablation for p = 2^61 - 1
    assert _call(lib, D=0) == -3
    assert _call(lib, D=(1 << 32) + 1) == -3
    assert _call(lib, D=(1 << 31) - 1) == -3                          # D must be below p = 2^31 - 1
    assert _call(lib, D=(1 << 31), family=mh.FAMILY_2U_M31) == -3
    assert _call(lib, family=mh.FAMILY_2U_MS32, D=1000) == -3         # multiply-shift needs D = 2^s
    assert _call(lib, family=mh.FAMILY_2U_MS32_HIGH, D=1) == -3
    assert _call(lib, family=mh.FAMILY_2U_MS32, D=1 << 32, n_rows=0) == 0
    assert _call(lib, k=0) == -4
    assert _call(lib, k=65537, out_stride=1 << 20) == -4
    assert _call(lib, b=0) == -4
    assert _call(lib, b=33, out_stride=1 << 20) == -4
    assert _call(lib, out_stride=63) == -5
    assert _call(lib, family=mh.FAMILY_PERM, perm_ld=63) == -5
    assert _call(lib, perm_ld=64) == -5                               # perm_ld must be 0 for hash families
    assert _call(lib, flags=8) == -1
    assert _call(lib, flags=4, family=mh.FAMILY_4U_M61, D=1 << 30) == -1   # the exact-fold switch: not for 4U p = 2^61-1,
    assert _call(lib, flags=4, family=mh.FAMILY_2U_MS32) == -1             # multiply-shift
    assert _call(lib, flags=4, family=mh.FAMILY_PERM, perm_ld=64) == -1    # or the permutation table
    assert _call(lib, flags=2, family=mh.FAMILY_2U_M61, D=1 << 30) == -1   # the % ablation exists for p = 2^31-1 only
    assert _call(lib, row_ptr=0) == -1
    assert _call(lib, params=0) == -1
    assert _call(lib, out=0) == -1
    assert _call(lib, ws=0) == -6
    assert _call(lib, ws=0x1001) == -6                                # misaligned
    assert _call(lib, ws_bytes=128) == -6                             # too small for the work list


def _call_static(lib, n_rows=4, nnz_ub=1000, D=1 << 24, k=64, b=8, family=0, perm_ld=0, out_stride=64, row_ptr=0x1000,
                 col_idx=0x1000, params=0x1000, out=0x1000, status=0, flags=0):
    return lib.minhash_signatures_static(row_ptr, col_idx, n_rows, nnz_ub, D, k, b, family, params, perm_ld, out,
                                         out_stride, status, 0, flags)


def test_static_entry_point_rejects_bad_arguments_and_oversized_batches_before_any_hip_call(lib):
    assert _call_static(lib, n_rows=-1) == -1
    assert _call_static(lib, nnz_ub=-1) == -1
    assert _call_static(lib, family=9) == -2
    assert _call_static(lib, D=0) == -3
    assert _call_static(lib, k=0) == -4
    assert _call_static(lib, out_stride=63) == -5
    assert _call_static(lib, flags=8) == -1
    assert _call_static(lib, out=0) == -1
    # the built-in buffer holds 64 MiB: a webspam-sized batch does not fit, nor does a bound beyond 2^46
    assert _call_static(lib, n_rows=350_000, nnz_ub=1_300_000_000, k=500, out_stride=500) == mh.ERR_TOO_LARGE
    assert _call_static(lib, nnz_ub=(1 << 46) + 1) == mh.ERR_TOO_LARGE
    assert _call_static(lib, n_rows=3_000_000, nnz_ub=0) == mh.ERR_TOO_LARGE      # the work list alone is too long
    assert b"built-in" in lib.minhash_error_string(mh.ERR_TOO_LARGE)
    # the header's sufficient condition, on shapes on both sides of it
    def bound(n, nnz, k):
        P = nnz // 8192 + min(n, nnz // 8192)
        return 32 * (n + P + nnz // 2048) + 16 * min(n, nnz // 512) + 4 * k * P + 2048
    for n, nnz, k in [(200_000, 100_000_000, 500), (1_000, 650_000, 64), (1_000_000, 30_000_000, 200)]:
        assert bound(n, nnz, k) <= mh.STATIC_SCRATCH_BYTES
        # accepted as far as the host-side checks go: without a GPU the call then fails in the HIP runtime
        # (with one, the made-up pointers must not reach a kernel)
        import torch
        if not torch.cuda.is_available():
            assert _call_static(lib, n_rows=n, nnz_ub=nnz, k=k, out_stride=k) == -7


def test_packed_row_entry_points_validate_before_any_launch(lib):
    P = 0x1000
    lib.minhash_pack_indices.argtypes = [ctypes.c_void_p] * 2 + [ctypes.c_int64] + [ctypes.c_void_p] * 3 + [ctypes.c_int64] + [ctypes.c_void_p] * 2
    lib.minhash_unpack_indices.argtypes = [ctypes.c_void_p] * 4 + [ctypes.c_int64] * 2 + [ctypes.c_void_p] * 3
    assert lib.minhash_pack_indices(P, P, -1, P, P, P, 10, P, 0) == -1
    assert lib.minhash_pack_indices(P, P, 4, P, P, P, -1, P, 0) == -1
    assert lib.minhash_pack_indices(0, P, 4, P, P, P, 10, P, 0) == -1
    assert lib.minhash_pack_indices(P, P, 4, P, P, P, 10, 0, 0) == -1          # the status word is required
    assert lib.minhash_pack_indices(P, 0, 4, P, P, P, 10, P, 0) == -1
    assert lib.minhash_unpack_indices(P, P, P, P, 10, -1, P, P, 0) == -1
    assert lib.minhash_unpack_indices(P, P, P, P, -1, 4, P, P, 0) == -1
    assert lib.minhash_unpack_indices(P, P, P, P, 10, 4, 0, P, 0) == -1
    assert lib.minhash_unpack_indices(P, P, P, P, 10, 4, P, 0, 0) == -1
    u64, i32, sz, u32 = ctypes.c_uint64, ctypes.c_int32, ctypes.c_size_t, ctypes.c_uint32
    lib.minhash_signatures_packed.argtypes = [ctypes.c_void_p] * 4 + [ctypes.c_int64] * 2 + [u64, i32, i32, i32, ctypes.c_void_p,
                                                                                         ctypes.c_void_p, ctypes.c_int64,
                                                                                         ctypes.c_void_p, sz, ctypes.c_void_p, u32]
    call = lambda **kw: lib.minhash_signatures_packed(*[kw.get(n, d) for n, d in (
        ("row_ptr", P), ("width", P), ("word_ptr", P), ("words", P), ("words_len", 100), ("n_rows", 4), ("D", 1 << 24), ("k", 64),
        ("b", 8), ("family", 0), ("params", P), ("out", P), ("out_stride", 64), ("ws", P), ("ws_bytes", 1 << 20), ("stream", 0),
        ("flags", 0))])
    assert call(family=mh.FAMILY_PERM) == -2                      # the table kernel takes col_idx
    assert call(words_len=-1) == -1
    assert call(width=0) == -1
    assert call(words=0) == -1
    assert call(n_rows=0) == 0
    assert call(D=0) == -3
    assert call(out_stride=63) == -5
    assert call(ws=0) == -6


def test_profiled_entry_point_validates_the_same_way(lib):
    ms = ctypes.c_float(-1.0)
    rc = lib.minhash_signatures_profiled(0x1000, 0x1000, 4, 0, 64, 8, 0, 0x1000, 0, 0x1000, 64, 0x1000, 1 << 20, 0, 0,
                                         ctypes.byref(ms))
    assert rc == -3 and ms.value == 0.0


def test_binding_refuses_to_run_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(mh, "_lib", None)
    monkeypatch.setattr(mh, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(FileNotFoundError):
        mh.lib()


def test_consumer_entry_points_validate_before_any_launch(lib):
    P = 0x1000
    assert lib.minhash_expand_indices(P, 0, 500, 500, 8, P, 0) == 0              # no rows: no-op
    assert lib.minhash_expand_indices(P, 4, 499, 500, 8, P, 0) == -5             # pitch below the signature size
    assert lib.minhash_expand_indices(P, 4, 500, 500, 0, P, 0) == -4
    assert lib.minhash_expand_indices(P, 4, 2000, 500, 32, P, 0) == -4           # k * 2^b must fit 32 bits
    assert lib.minhash_expand_indices(0, 4, 500, 500, 8, P, 0) == -1
    assert lib.minhash_match_counts(P, 4, 500, 500, 8, P, 0, P, 0) == 0
    assert lib.minhash_match_counts(P, 4, 500, 500, 8, 0, 3, P, 0) == -1
    assert lib.minhash_match_counts(P, 4, 500, 500, 8, P, -1, P, 0) == -1
    assert lib.minhash_match_counts(P, 4, 10, 500, 8, P, 3, P, 0) == -5
    assert lib.minhash_resemblance_estimates(P, P, P, 0, 1 << 24, 500, 8, P, 0) == 0
    assert lib.minhash_resemblance_estimates(P, P, P, 5, 0, 500, 8, P, 0) == -3
    assert lib.minhash_resemblance_estimates(P, P, P, 5, 1 << 24, 500, 33, P, 0) == -4
    assert lib.minhash_resemblance_estimates(0, P, P, 5, 1 << 24, 500, 8, P, 0) == -1


def test_probe_library_loads_and_exports_its_entry_points():
    """The measurement library behind bench.py --probe: loads without a GPU, exports what its binding
    declares, names its instruction kinds, and refuses bad arguments before any launch."""
    from paper_1205_2958_amd import probe
    L = probe.lib()
    for name in probe.EXPORTS:
        assert hasattr(L, name), name
    kinds = probe.kinds()
    assert "v_mad_u64_u32" in kinds and "v_min3_u32" in kinds and "v_add_u32" in kinds
    P = 0x1000
    ms, slots = ctypes.c_float(0), ctypes.c_double(0)
    assert L.mh_probe_issue(len(kinds), 0, 0, 4, 2.4, P, 0, 1, ctypes.byref(ms), ctypes.byref(slots)) == -1     # no such kind
    assert L.mh_probe_issue(0, 4, 0, 4, 2.4, P, 0, 1, ctypes.byref(ms), ctypes.byref(slots)) == -1              # n_simple not offered
    assert L.mh_probe_issue(0, 1, 0, 9, 2.4, P, 0, 1, ctypes.byref(ms), ctypes.byref(slots)) == -1              # waves per SIMD
    assert L.mh_probe_stream_read(P, 100, 8, 0, 1, ctypes.byref(ms)) == -1                                       # too small
    assert L.mh_probe_stream_read(P + 4, 1 << 20, 8, 0, 1, ctypes.byref(ms)) == -1                               # misaligned
    assert L.mh_probe_copy(0, P, 1 << 20, 0, 1, ctypes.byref(ms)) == -1
    assert L.mh_probe_gather_rows(P, 100, 800, 808, P, 1000, 8, 8, 0, 1, ctypes.byref(ms)) == -1                 # row longer than the pitch
    assert L.mh_probe_gather_rows(P, 100, 800, 800, P, 1000, 12, 8, 0, 1, ctypes.byref(ms)) == -1                # rows in flight

