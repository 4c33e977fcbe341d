"""bench.py's command line and roofline model, without a GPU: more than one GPU
is refused with a message, a machine without a GPU is refused (no CPU path
stands in), and the issue-slot figures the roofline is priced with follow from
the instruction mixes by the stated rule."""
import importlib.util
import os
import subprocess
import sys

import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench_module():
    spec = importlib.util.spec_from_file_location("bench_under_test", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    sys.modules["bench_under_test"] = mod          # forked workers find the module's functions by this name
    spec.loader.exec_module(mod)
    return mod


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=300)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


@pytest.mark.skipif(torch.cuda.is_available(), reason="this machine has a GPU")
def test_no_gpu_means_no_number():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "1", "--warmup", "0"],
                       capture_output=True, text=True, timeout=300)
    assert r.returncode != 0
    assert "needs a GPU" in r.stderr
    assert '"metric"' not in r.stdout


def test_issue_slots_follow_from_the_mixes():
    b = _bench_module()
    W = b.W
    assert b.ALU_PEAK_SLOTS == 256 * 4 * 16 * 2.4e9
    # multiply + max(full, (full + simple) / 2)
    assert b.issue_slots((1.0, 1.0, 1.0)) == 2.0
    assert b.issue_slots((2.0, 0.5, 3.5)) == 4.0          # simple instructions fill the other half-slots
    assert b.issue_slots((0.0, 3.0, 1.0)) == 3.0          # full-issue instructions bound it
    want = {W.FAMILY_2U_M31: 2.0, W.FAMILY_4U_M31: 5.5, W.FAMILY_2U_M61: 3.75, W.FAMILY_2U_MS32: 1.5}
    for fam, slots in want.items():
        assert b.issue_slots(b.ISSUE_MIX[fam]) == slots
    assert b.issue_slots(b.ISSUE_MIX_OTHER_D_FRAC[W.FAMILY_2U_M31]) == 4.75
    assert b.issue_slots(b.ISSUE_MIX_OTHER_D_FRAC[W.FAMILY_4U_M31]) == 8.25
    assert b.issue_slots(b.ISSUE_MIX_OTHER_D_BIG[W.FAMILY_2U_M31]) == 4.75
    assert b.issue_slots(b.ISSUE_MIX_OTHER_D_BIG[W.FAMILY_4U_M31]) == 8.25
    assert b.issue_slots(b.ISSUE_MIX_OTHER_D[W.FAMILY_2U_M31]) == 5.75
    assert b.issue_slots(b.ISSUE_MIX_OTHER_D[W.FAMILY_4U_M31]) == 9.25


def test_oracle_pool_deals_rows_to_shards_and_puts_them_back_in_order():
    """The worker pool of bench.py and the GPU tests only deals rows out and collects them: its result must be what
    one call of the oracle on the whole sample gives, for a hash family and for the permutation
    family (where every shard gets the table rows of its own nonzeros, renumbered)."""
    import numpy as np
    from oracle import oracle

    from oracle.pool import OraclePool
    from paper_1205_2958_amd import workloads as W

    pool = OraclePool(3)
    try:
        nnz = np.array([5, 0, 900, 17, 1, 300, 64, 0, 2], dtype=np.int64)
        D, k = 1 << 12, 24
        rp, col = W.row_ptr_from_nnz(nnz), W.csr_indices_np(nnz, D, seed=3)
        c = W.coefficients(k, W.FAMILY_4U_M31, seed=4)
        got, dt, used = pool.signatures(rp, col, D, k, 6, W.FAMILY_4U_M31, c)
        assert used == 3 and dt > 0
        assert np.array_equal(got, oracle.signatures(rp, col, D, k, 6, W.FAMILY_4U_M31, c))
        got1, _, used1 = pool.signatures(rp, col, D, k, 6, W.FAMILY_4U_M31, c, procs=1)
        assert used1 == 1 and np.array_equal(got1, got)
        table = W.perm_table_np(D, k, seed=5)
        got, _, _ = pool.signatures(rp, col, D, k, 4, W.FAMILY_PERM, None, table_rows=table[col])
        assert np.array_equal(got, oracle.signatures(rp, col, D, k, 4, W.FAMILY_PERM, table))
    finally:
        pool.close()
