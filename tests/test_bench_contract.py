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
