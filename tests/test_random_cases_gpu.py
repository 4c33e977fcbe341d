"""Differential test on seeded random cases (tests/random_cases.py): every byte of the GPU's output,
pad bytes included, against the CPU oracle, through each entry point that computes signatures.
The oracle's calls run in the worker processes while the GPU works on the same block of cases."""
import numpy as np
import pytest
import torch

import random_cases as R
from paper_1205_2958_amd import minhash as mh

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
BLOCK = 32          # cases per block: one oracle call each, in parallel


def _gpu_output(c):
    n = c["rp"].shape[0] - 1
    base = c["base"]
    rp_d = torch.from_numpy(c["rp"] + base).to(DEV)
    col_h = np.concatenate([np.full(base, 0xFFFFFFFF, np.uint32), c["col"]]) if base else c["col"]
    col_d = torch.from_numpy(col_h.view(np.int32)).to(DEV) if col_h.size else torch.zeros(0, dtype=torch.int32, device=DEV)
    par_d = torch.from_numpy(c["params"].view(np.int32 if c["family"] == mh.FAMILY_PERM else np.int64)).to(DEV)
    out = torch.full((n, c["stride"]), 0xAB, dtype=torch.uint8, device=DEV)
    args = (c["D"], c["k"], c["b"], c["family"], par_d)
    entry = c["entry"]
    if entry == "static":
        st = torch.zeros(1, dtype=torch.int32, device=DEV)
        try:
            mh.minhash_signatures_static(rp_d, col_d, int(c["rp"][-1]), *args, out, status=st, flags=c["flags"])
            assert int(st.item()) == 0
        except mh.MinhashError as e:
            assert e.code == mh.ERR_TOO_LARGE
            entry = "plain"
    if entry == "plain":
        mh.minhash_signatures(rp_d, col_d, *args, out=out, flags=c["flags"])
    elif entry == "packed":
        width, word_ptr, words = mh.pack_indices(rp_d, col_d)
        mh.minhash_signatures_packed(rp_d, width, word_ptr, words, *args, out=out, flags=c["flags"])
    torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("first_seed", [7000 + BLOCK * i for i in range(40)])
def test_random_cases_equal_the_oracle(first_seed, oracle_pool):
    cases = [R.make_case(first_seed + i) for i in range(BLOCK)]
    pending = oracle_pool.cases_async([(c["rp"], c["col"], c["D"], c["k"], c["b"], c["family"], c["params"], c["stride"])
                                       for c in cases])
    got = []
    for c in cases:
        print("case", R.describe(c), flush=True)
        got.append(_gpu_output(c))
    want = pending.get()
    bad = [R.describe(c) for c, g, w in zip(cases, got, want) if g.shape != w.shape or not np.array_equal(g, w)]
    assert not bad, "GPU and oracle differ on:\n" + "\n".join(bad)
