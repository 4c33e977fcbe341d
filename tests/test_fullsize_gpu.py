"""Full-size workloads, in the launch configuration bench.py times: the GPU
library's output on sampled rows (longest, shortest, around the split point,
random) against the CPU oracle, row by row and bit for bit.  The rows are
generated on the GPU with the torch generator; each sampled row is also
re-generated with the NumPy generator, which must give the same indices."""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_1205_2958_amd import minhash as mh
from paper_1205_2958_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
SPLIT = 8192          # rows longer than this are processed in chunks and merged


def _sample_rows(nnz, seed, eval_budget, k, heavy_from=None):
    """The rows the oracle looks at: W.stratified_rows (first, last, shortest, longest row, the
    rows next to 1, 2, 4, ... times the split point, optionally the heaviest rows, then rows
    drawn in turn from the ten deciles of the length distribution until the budget is spent)."""
    rows, cover = W.stratified_rows(nnz, k, eval_budget, seed=seed, split=SPLIT, heavy_from=heavy_from)
    return rows, cover


def _run_workload(name, batch=0):
    w = W.WORKLOADS[name]
    nnz = w.nnz(batch)
    rp_np = W.row_ptr_from_nnz(nnz)
    seed = w.data_seed + batch
    col = W.csr_indices_torch(nnz, w.D, seed, DEV)
    rp = torch.from_numpy(rp_np).to(DEV)
    if w.family == W.FAMILY_PERM:
        params = W.perm_table_torch(w.D, w.k, w.param_seed, DEV)
        params_np = None
    else:
        params_np = W.coefficients(w.k, w.family, w.param_seed)
        params = torch.from_numpy(params_np.view(np.int64)).to(DEV)
    out = torch.full((len(nnz), w.sig_bytes()), 0xAA, dtype=torch.uint8, device=DEV)
    ws = mh.alloc_workspace(len(nnz), int(rp_np[-1]), w.k, w.family, DEV)
    mh.minhash_signatures(rp, col, w.D, w.k, w.b, w.family, params, out=out, workspace=ws)
    assert mh.status(ws) == 0
    return w, nnz, rp_np, seed, col, params, params_np, out


def _check_rows(pool, w, nnz, rp_np, seed, col, params, params_np, out, rows, D=None):
    """Signatures of `rows` from the device output against the oracle (rows dealt to the worker
    processes).  The rows' indices come from the device buffer; each is also generated again with
    the NumPy generator, which must give the same indices (unless D folds them)."""
    rows = np.asarray(rows, dtype=np.int64)
    take = torch.from_numpy(np.concatenate([np.arange(rp_np[r], rp_np[r + 1]) for r in rows])).to(DEV)
    idx = col[take].cpu().numpy().view(np.uint32)
    s_rp = W.row_ptr_from_nnz(nnz[rows])
    if D is None:
        D = w.D
        assert np.array_equal(idx, W.csr_indices_np(nnz[rows], w.D, seed, rows=rows)), "generators disagree"
    if w.family == W.FAMILY_PERM:
        # only the table rows these sets touch travel to the host: table[t] for every nonzero, in CSR order
        table_rows = params[col[take].long()].cpu().numpy().view(np.uint32)
        want, _, _ = pool.signatures(s_rp, idx, D, w.k, w.b, w.family, None, table_rows=table_rows)
    else:
        want, _, _ = pool.signatures(s_rp, idx, D, w.k, w.b, w.family, params_np)
    got = out[torch.from_numpy(rows).to(DEV)].cpu().numpy()
    if not np.array_equal(got, want):
        bad = np.flatnonzero((got != want).any(axis=1))
        raise AssertionError("%d of %d sampled rows differ from the oracle, first: row %d (nnz %d)"
                             % (len(bad), len(rows), rows[bad[0]], nnz[rows[bad[0]]]))


@pytest.mark.parametrize("name,budget", [
    ("large_2u", 1.5e10),
    ("large_4u", 6.0e9),
    ("perm_table", 1.2e8),          # every sampled nonzero brings an 800-byte table row to the host
    ("large_2u_ms32", 6.0e9),
    ("short_rows_2u", 3.0e9),
    ("large_4u_m61", 1.5e9),
])
def test_large_workloads_sampled_rows(name, budget, oracle_pool):
    w, nnz, rp_np, seed, col, params, params_np, out = _run_workload(name)
    rows, cover = _sample_rows(nnz, seed=17, eval_budget=budget, k=w.k)
    assert cover["rows"] >= 100 and cover["longest_row"] == nnz.max()
    _check_rows(oracle_pool, w, nnz, rp_np, seed, col, params, params_np, out, rows)
    # every row was written: none still holds the poison pattern the buffer was filled with
    assert out.shape == (w.n_rows, w.sig_bytes())
    assert bool((out != 0xAA).any(dim=1).all().item())


@pytest.mark.parametrize("name", ["large_2u", "large_4u", "huge_2u_m61", "large_4u_m61"])
@pytest.mark.parametrize("D", [16_609_143, 500_000_003, 1_010_017_424])
def test_universe_sizes_of_the_papers_datasets_sampled_rows(name, D, oracle_pool):
    """The headline rows hashed into a universe that is not a power of two (Table tab_data: webspam's
    16 609 143 and the expanded rcv1's 1 010 017 424, and one size in between), each of which takes
    a kernel form of its own (with p = 2^61-1: the residue modulo D in 32-bit steps, in one stage above
    2^29 and in two below); indices are folded into [0, D) as bench.py --universe does."""
    w = W.WORKLOADS[name]
    nnz = w.nnz(0)
    rp_np = W.row_ptr_from_nnz(nnz)
    col = W.csr_indices_torch(nnz, w.D, w.data_seed, DEV)
    col.remainder_(D)
    rp = torch.from_numpy(rp_np).to(DEV)
    params_np = W.coefficients(w.k, w.family, w.param_seed)
    params = torch.from_numpy(params_np.view(np.int64)).to(DEV)
    out = torch.full((len(nnz), w.sig_bytes()), 0xAA, dtype=torch.uint8, device=DEV)
    ws = mh.alloc_workspace(len(nnz), int(rp_np[-1]), w.k, w.family, DEV)
    mh.minhash_signatures(rp, col, D, w.k, w.b, w.family, params, out=out, workspace=ws)
    assert mh.status(ws) == 0
    rows, cover = _sample_rows(nnz, seed=23, eval_budget={"huge_2u_m61": 4e9, "large_4u_m61": 7e8}.get(name, 1.5e9), k=w.k)
    assert cover["rows"] >= 100
    _check_rows(oracle_pool, w, nnz, rp_np, w.data_seed, col, params, params_np, out, rows, D=D)
    assert bool((out != 0xAA).any(dim=1).all().item())


def test_many_short_rows_do_not_depend_on_how_units_are_handed_out():
    """A batch of 2x10^6 short rows is handed to the wavefronts in runs of 32 rows that halve
    towards the end of the launch; slices of 3 000 rows (fewer than there are resident wavefronts:
    no run, hardly a ticket) are handed out row by row.  Every row of a slice must get the
    signature it has in the whole batch, wherever the slice lies: in the long runs, across the
    levels of shorter runs and among the last single rows.  Two larger slices get runs of their own
    sizes."""
    w, nnz, rp_np, seed, col, params, params_np, out = _run_workload("short_rows_2u")
    n = len(nnz)
    slices = [(lo, 3_000) for lo in (0, 1_000_003, n - 700_000, n - 200_000, n - 60_000, n - 12_000, n - 3_000)]
    slices += [(500_000, 150_000), (1_200_000, 520_000)]      # batches that get runs of 2 and of 8 rows
    for lo, size in slices:
        hi = min(n, lo + size)
        rp_part = torch.from_numpy(rp_np[lo:hi + 1] - rp_np[lo]).to(DEV)
        col_part = col[int(rp_np[lo]):int(rp_np[hi])]
        part = mh.minhash_signatures(rp_part, col_part, w.D, w.k, w.b, w.family, params)
        assert torch.equal(part, out[lo:hi]), "rows %d..%d differ between the whole batch and a slice of it" % (lo, hi)


@pytest.mark.parametrize("batch", [0, 9])
def test_heavy_tailed_m61_batch_sampled_rows(batch, oracle_pool):
    """First and last batch of the heavy-tailed workload: the longest row (10^6 nonzeros: 123 chunks,
    each with a vector of partial minima, merged by the finalize kernel), rows of at least 10^5
    nonzeros in seeded random order while they fit three fifths of the budget, and rows from every
    decile of the length distribution."""
    w, nnz, rp_np, seed, col, params, params_np, out = _run_workload("huge_2u_m61", batch)
    assert nnz.max() == 1_000_000                     # the batch contains rows at the cap
    rows, cover = _sample_rows(nnz, seed=18 + batch, eval_budget=2.0e10, k=w.k, heavy_from=100_000)
    assert cover["longest_row"] == 1_000_000 and cover["rows"] >= 300
    assert int((nnz[rows] >= 100_000).sum()) >= 40
    _check_rows(oracle_pool, w, nnz, rp_np, seed, col, params, params_np, out, rows)
    # b = 1, k = 500: 63 bytes per row, the last 4 bits of the last byte are pad and must be 0
    assert int((out[:, 62] & 0xF0).max().item()) == 0


def test_guarded_m61_path_equals_the_exact_fold_on_a_whole_batch():
    """10^12 evaluations hit the guard of the carry-free 2U-M61 form about 2 000 times, so this
    batch exercises the exact re-evaluation on ordinary data.  Its full 32-bit minima must equal,
    row for row, those of the carry-propagating form (which the sampled rows above and the
    engineered cases pin to the oracle)."""
    w = W.WORKLOADS["huge_2u_m61"]
    nnz = w.nnz(0)
    rp_np = W.row_ptr_from_nnz(nnz)
    col = W.csr_indices_torch(nnz, w.D, w.data_seed, DEV)
    rp = torch.from_numpy(rp_np).to(DEV)
    params_np = W.coefficients(w.k, w.family, w.param_seed)
    params = torch.from_numpy(params_np.view(np.int64)).to(DEV)
    ws = mh.alloc_workspace(len(nnz), int(rp_np[-1]), w.k, w.family, DEV)
    outs = []
    for flags in (0, mh.FLAG_EXACT_FOLD):
        out = torch.full((len(nnz), 4 * w.k), 0xAA, dtype=torch.uint8, device=DEV)
        mh.minhash_signatures(rp, col, w.D, w.k, 32, w.family, params, out=out, workspace=ws, flags=flags)
        assert mh.status(ws) == 0
        outs.append(out)
    assert torch.equal(outs[0], outs[1])
    # and one short row of it against the oracle at full width
    r = int(np.argsort(nnz, kind="stable")[len(nnz) // 2])
    lo, hi = int(rp_np[r]), int(rp_np[r + 1])
    idx = col[lo:hi].cpu().numpy().view(np.uint32)
    want = oracle.signatures(np.array([0, hi - lo], dtype=np.int64), idx, w.D, w.k, 32, w.family, params_np)
    assert np.array_equal(outs[0][r].cpu().numpy(), want[0])


def test_2u_doubled_key_equals_the_two_maxima_form_on_a_whole_batch():
    """The headline kernel (`large_2u`: one running maximum of the doubled key, doubtful values
    computed again) against the same batch under MINHASH_FLAG_EXACT_FOLD, which keeps a signed
    and an unsigned maximum of the key and never looks twice: full 32-bit minima of all
    350 000 rows.  (GPU against GPU; the sampled rows above pin both forms to the oracle.)"""
    w = W.WORKLOADS["large_2u"]
    nnz = w.nnz(0)
    rp_np = W.row_ptr_from_nnz(nnz)
    col = W.csr_indices_torch(nnz, w.D, w.data_seed, DEV)
    rp = torch.from_numpy(rp_np).to(DEV)
    params_np = W.coefficients(w.k, w.family, w.param_seed)
    params = torch.from_numpy(params_np.view(np.int64)).to(DEV)
    ws = mh.alloc_workspace(len(nnz), int(rp_np[-1]), w.k, w.family, DEV)
    outs = []
    for flags in (0, mh.FLAG_EXACT_FOLD):
        out = torch.full((len(nnz), 4 * w.k), 0xAA, dtype=torch.uint8, device=DEV)
        mh.minhash_signatures(rp, col, w.D, w.k, 32, w.family, params, out=out, workspace=ws, flags=flags)
        assert mh.status(ws) == 0
        outs.append(out)
    assert torch.equal(outs[0], outs[1])
    # the two-maxima form itself against the oracle on a few rows at full width
    order = np.argsort(nnz, kind="stable")
    for r in (int(order[0]), int(order[len(nnz) // 2]), int(order[-1])):
        lo, hi = int(rp_np[r]), int(rp_np[r + 1])
        idx = col[lo:hi].cpu().numpy().view(np.uint32)
        want = oracle.signatures(np.array([0, hi - lo], dtype=np.int64), idx, w.D, w.k, 32, w.family, params_np)
        assert np.array_equal(outs[1][r].cpu().numpy(), want[0])


def test_4u_full_keys_equal_the_shifted_ones_on_a_whole_batch():
    """`large_4u` with the folded values kept in a signed and an unsigned running maximum (the
    default for power-of-two D) against the same batch with the shifted keys that are formed
    evaluation by evaluation: full 32-bit minima, row for row."""
    w = W.WORKLOADS["large_4u"]
    nnz = w.nnz(0)
    rp_np = W.row_ptr_from_nnz(nnz)
    col = W.csr_indices_torch(nnz, w.D, w.data_seed, DEV)
    rp = torch.from_numpy(rp_np).to(DEV)
    params = torch.from_numpy(W.coefficients(w.k, w.family, w.param_seed).view(np.int64)).to(DEV)
    ws = mh.alloc_workspace(len(nnz), int(rp_np[-1]), w.k, w.family, DEV)
    outs = []
    for flags in (0, mh.FLAG_EXACT_FOLD):
        out = torch.full((len(nnz), 4 * w.k), 0xAA, dtype=torch.uint8, device=DEV)
        mh.minhash_signatures(rp, col, w.D, w.k, 32, w.family, params, out=out, workspace=ws, flags=flags)
        assert mh.status(ws) == 0
        outs.append(out)
    assert torch.equal(outs[0], outs[1])
