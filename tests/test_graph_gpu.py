"""The signature calls under HIP graph capture: they only launch kernels on the caller's stream (the
header of the work list is cleared by a kernel, nothing is allocated, nothing waits), so a captured
call can be replayed on new data of the same shape.  Each replay is checked against the oracle,
with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_1205_2958_amd import minhash as mh
from paper_1205_2958_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _batch(n_rows, max_nnz, D, seed, long_row=0):
    """n_rows rows whose lengths change with the seed (some empty), at most max_nnz indices in all."""
    rng = np.random.Generator(np.random.PCG64(seed))
    nnz = rng.integers(0, 160, size=n_rows).astype(np.int64)
    nnz[rng.integers(0, n_rows, size=n_rows // 10)] = 0
    if long_row:
        nnz[int(rng.integers(0, n_rows))] = long_row          # one row that is split into chunks
    assert nnz.sum() <= max_nnz
    col = W.csr_indices_np(nnz, D if D & (D - 1) == 0 else 1 << 30, seed)
    return W.row_ptr_from_nnz(nnz), (col % np.uint32(D)).astype(np.uint32) if D & (D - 1) else col


@pytest.mark.parametrize("entry", ["workspace", "static"])
@pytest.mark.parametrize("family,D,k,b", [(mh.FAMILY_2U_M31, 1 << 24, 64, 8), (mh.FAMILY_2U_M61, 1 << 30, 500, 1),
                                          (mh.FAMILY_4U_M31, 16609143, 200, 4)])
def test_captured_call_replayed_on_new_rows_equals_the_oracle(entry, family, D, k, b):
    n_rows, max_nnz = 600, 600 * 160 + 40000
    c = W.coefficients(k, family, seed=3 + k)
    par_d = torch.from_numpy(c.view(np.int64)).to(DEV)
    rp_d = torch.zeros(n_rows + 1, dtype=torch.int64, device=DEV)
    col_d = torch.zeros(max_nnz, dtype=torch.int32, device=DEV)
    out = torch.zeros((n_rows, (k * b + 7) // 8), dtype=torch.uint8, device=DEV)
    ws = mh.alloc_workspace(n_rows, max_nnz, k, family, DEV)
    st = torch.zeros(1, dtype=torch.int32, device=DEV)

    def call():
        if entry == "static":
            mh.minhash_signatures_static(rp_d, col_d, max_nnz, D, k, b, family, par_d, out, status=st)
        else:
            mh.minhash_signatures(rp_d, col_d, D, k, b, family, par_d, out=out, workspace=ws)

    def load(seed, long_row):
        rp, col = _batch(n_rows, max_nnz, D, seed, long_row)
        rp_d.copy_(torch.from_numpy(rp))
        col_d[: col.shape[0]].copy_(torch.from_numpy(col.view(np.int32)))
        return rp, col

    load(1, 0)
    call()                                  # eager first: launch constants of this device are looked up once, outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.graph(graph, stream=side):
        call()
    for seed, long_row in ((11, 0), (12, 30000), (13, 0), (14, 9000)):
        rp, col = load(seed, long_row)
        out.fill_(0xEE)                     # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        if entry == "static":
            assert int(st.item()) == 0
        else:
            assert mh.status(ws) == 0
        want = oracle.signatures(rp, col, D, k, b, family, c)
        assert np.array_equal(out.cpu().numpy(), want), "replay with seed %d differs" % seed
