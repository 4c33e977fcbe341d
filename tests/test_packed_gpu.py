"""Packed index rows on the GPU (minhash_pack_indices / minhash_unpack_indices) against the
CPU checker's plain definition of the same form, word for word, and signatures computed from
unpacked rows against the oracle."""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_1205_2958_amd import minhash as mh
from paper_1205_2958_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _dev(a):
    if a.dtype == np.uint32:
        return torch.from_numpy(a.view(np.int32)).to(DEV)
    return torch.from_numpy(a).to(DEV)


def _host_u32(t):
    return t.cpu().numpy().view(np.uint32)


def _round_trip(rp, col):
    rp_d, col_d = _dev(rp), _dev(col)
    width, word_ptr, words = mh.pack_indices(rp_d, col_d)
    w_o, wp_o, words_o = oracle.pack_indices(rp, col)
    assert np.array_equal(_host_u32(width), w_o)
    assert np.array_equal(word_ptr.cpu().numpy(), wp_o)
    assert np.array_equal(_host_u32(words), words_o)
    out = torch.full((max(col.shape[0], 1),), 0x5A5A5A5A, dtype=torch.int32, device=DEV)
    st = torch.full((1,), 99, dtype=torch.int32, device=DEV)
    mh.unpack_indices(rp_d, width, word_ptr, words, out, st)
    torch.cuda.synchronize()
    assert int(st.item()) == 0
    assert np.array_equal(_host_u32(out)[: col.shape[0]], col)
    return width, word_ptr, words


def test_rows_around_the_tile_size_and_gaps_of_every_magnitude():
    rng = np.random.Generator(np.random.PCG64(717))
    lens = [0, 1, 2, 3, 4, 5, 63, 64, 65, 255, 256, 257, 511, 512, 513, 1000, 0, 4095, 4096, 4097, 8192, 20000, 1, 0]
    rows = []
    for n in lens:
        top = int(rng.choice([4, 1 << 8, 1 << 16, 1 << 24, (1 << 32) - 1]))
        gaps = rng.integers(0, max(top // max(n, 1), 1) + 1, size=n, dtype=np.uint64)
        rows.append(np.minimum(np.cumsum(gaps), (1 << 32) - 1).astype(np.uint32))
    rp = W.row_ptr_from_nnz(np.array(lens, dtype=np.int64))
    _round_trip(rp, np.concatenate(rows))


def test_widths_from_0_to_32_bits():
    rows = []
    for w in range(0, 33):
        d = (1 << w) - 1 if w else 0
        n = 300
        steps = np.zeros(n, dtype=np.uint64)
        steps[5] = d                                   # the widest difference decides the width of the whole row
        steps[299] = d >> 1
        if w == 32:
            steps[299] = 0
        rows.append(np.cumsum(steps).astype(np.uint32))
    rp = W.row_ptr_from_nnz(np.full(33, 300, dtype=np.int64))
    width, _, _ = _round_trip(rp, np.concatenate(rows))
    assert _host_u32(width).tolist() == list(range(33))


def test_many_short_rows_and_one_long_row_share_spans():
    """Spans of 4 096 positions cut across rows: thousands of rows of one to three indices, empty
    rows, and one row of 100 000 indices whose tiles are decoded by many wavefronts."""
    rng = np.random.Generator(np.random.PCG64(81))
    lens = np.concatenate([rng.integers(0, 4, size=6000), [100_000], rng.integers(0, 4, size=3000), [700, 0, 0, 1]]).astype(np.int64)
    rp = W.row_ptr_from_nnz(lens)
    col = W.csr_indices_np(lens, 1 << 30, seed=5)
    _round_trip(rp, col)


def test_row_ptr_need_not_start_at_zero():
    lens = np.array([10, 600, 0, 3], dtype=np.int64)
    col_all = np.concatenate([np.arange(7, dtype=np.uint32), W.csr_indices_np(lens, 1 << 20, seed=9)])
    rp = W.row_ptr_from_nnz(lens) + 7
    rp_d, col_d = _dev(rp), _dev(col_all)
    width, word_ptr, words = mh.pack_indices(rp_d, col_d)
    w_o, wp_o, words_o = oracle.pack_indices(rp, col_all)
    assert np.array_equal(_host_u32(words), words_o) and np.array_equal(word_ptr.cpu().numpy(), wp_o)
    out = torch.zeros(col_all.shape[0], dtype=torch.int32, device=DEV)
    st = torch.zeros(1, dtype=torch.int32, device=DEV)
    mh.unpack_indices(rp_d, width, word_ptr, words, out, st)
    torch.cuda.synchronize()
    assert int(st.item()) == 0 and np.array_equal(_host_u32(out)[7:], col_all[7:]) and not _host_u32(out)[:7].any()


def test_bad_input_is_reported_and_nothing_is_written_outside_the_buffers():
    rp = np.array([0, 3], dtype=np.int64)
    with pytest.raises(mh.MinhashError) as e:
        mh.pack_indices(_dev(rp), _dev(np.array([5, 4, 6], dtype=np.uint32)))        # not sorted
    assert e.value.code == -9
    # unpacking with a word buffer that is shorter than the offsets say
    lens = np.array([600, 300], dtype=np.int64)
    rp = W.row_ptr_from_nnz(lens)
    col = W.csr_indices_np(lens, 1 << 24, seed=3)
    width, word_ptr, words = mh.pack_indices(_dev(rp), _dev(col))
    out = torch.full((900,), -1, dtype=torch.int32, device=DEV)
    st = torch.zeros(1, dtype=torch.int32, device=DEV)
    mh.unpack_indices(_dev(rp), width, word_ptr, words[: words.numel() - 5].contiguous(), out, st)
    torch.cuda.synchronize()
    assert int(st.item()) == -6
    # an empty batch
    st.fill_(5)
    mh.unpack_indices(torch.zeros(1, dtype=torch.int64, device=DEV), width[:0], word_ptr[:1], words[:0], out, st)
    torch.cuda.synchronize()
    assert int(st.item()) == 0


def test_signatures_from_unpacked_rows_equal_the_oracle(oracle_pool):
    """The path the streamed workload takes: packed rows -> col_idx on the device -> signatures."""
    w = W.WORKLOADS["huge_2u_m61"]
    nnz = w.nnz(3)[:3000]
    rp = W.row_ptr_from_nnz(nnz)
    col = W.csr_indices_np(nnz, w.D, w.data_seed + 3)
    c = W.coefficients(w.k, w.family, w.param_seed)
    rp_d = _dev(rp)
    width, word_ptr, words = mh.pack_indices(rp_d, _dev(col))
    assert words.numel() < 0.75 * col.shape[0]                # the form is denser than 32 bits per index
    out = torch.empty(col.shape[0], dtype=torch.int32, device=DEV)
    st = torch.zeros(1, dtype=torch.int32, device=DEV)
    mh.unpack_indices(rp_d, width, word_ptr, words, out, st)
    sig = mh.minhash_signatures(rp_d, out, w.D, w.k, w.b, w.family, torch.from_numpy(c.view(np.int64)).to(DEV))
    torch.cuda.synchronize()
    assert int(st.item()) == 0
    want, _, _ = oracle_pool.signatures(rp, col, w.D, w.k, w.b, w.family, c)
    assert np.array_equal(sig.cpu().numpy(), want)


def test_streamed_packed_batches_equal_the_oracle():
    """Five batches of unequal size, packed on the device, parked in pinned host memory and
    streamed back through copy / decode / hash / copy-back on four streams."""
    D, k, b, family = 1 << 30, 500, 1, mh.FAMILY_2U_M61
    nnz = W.lomax_nnz(900, scale=580.4, tail=0.8, lo=1, hi=40_000, seed=77)
    nnz[13] = 0
    rp, col = W.row_ptr_from_nnz(nnz), W.csr_indices_np(nnz, D, seed=78)
    c = W.coefficients(k, family, seed=79)
    want = oracle.signatures(rp, col, D, k, b, family, c)
    bounds = [0, 200, 201, 450, 700, 900]
    batches, max_words = [], 0
    for lo, hi in zip(bounds[:-1], bounds[1:]):
        rp_b = (rp[lo:hi + 1] - rp[lo]).copy()
        width, word_ptr, words = mh.pack_indices(_dev(rp_b), _dev(col[rp[lo]:rp[hi]].copy()))
        words_h = words.cpu().pin_memory()
        if lo in (0, 450):                                      # words handed over in pieces
            cut = words_h.numel() // 3
            words_h = [words_h[:cut].clone().pin_memory(), words_h[cut:].clone().pin_memory()]
        batches.append((torch.from_numpy(rp_b).pin_memory(), width.cpu().pin_memory(), word_ptr.cpu().pin_memory(), words_h))
        max_words = max(max_words, words.numel())
    max_rows = max(h - l for l, h in zip(bounds[:-1], bounds[1:]))
    max_nnz = max(int(rp[h] - rp[l]) for l, h in zip(bounds[:-1], bounds[1:]))
    for decode_in_kernel, slices in ((True, 4), (True, 1), (True, 7), (True, 500), (False, 4)):    # the first batch goes in slices of rows
        outs = mh.stream_batches_packed(batches, D, k, b, family, torch.from_numpy(c.view(np.int64)).to(DEV), max_rows, max_nnz,
                                        max_words, decode_in_kernel=decode_in_kernel, edge_slices=slices)
        got = np.concatenate([o.numpy() for o in outs], axis=0)
        assert np.array_equal(got, want), (decode_in_kernel, slices)


# ------------------------------------------------------------------ decoded inside the hash kernels
EDGE_NNZ = [0, 1, 2, 3, 4, 5, 7, 8, 9, 63, 64, 65, 255, 256, 257, 511, 512, 513, 1000, 0, 4095, 8191, 8192, 8193, 16384,
            16385, 20000, 1, 0, 50000]


def _packed_signatures(rp, col, D, k, b, family, c, flags=0):
    rp_d = _dev(rp)
    width, word_ptr, words = mh.pack_indices(rp_d, _dev(col))
    n = rp.shape[0] - 1
    out = torch.full((n, (k * b + 7) // 8), 0xAA, dtype=torch.uint8, device=DEV)
    ws = mh.alloc_workspace(n, int(col.shape[0]), k, family, DEV)
    ws.fill_(0xCD)
    mh.minhash_signatures_packed(rp_d, width, word_ptr, words, D, k, b, family, torch.from_numpy(c.view(np.int64)).to(DEV),
                                 out=out, workspace=ws, flags=flags)
    st = mh.status(ws)
    return out.cpu().numpy(), st


@pytest.mark.parametrize("family,D,k,b", [
    (mh.FAMILY_2U_M31, 1 << 24, 500, 8),          # one maximum of a doubled key: second looks read the tiles again
    (mh.FAMILY_2U_M31, 1 << 30, 500, 8),          # two maxima
    (mh.FAMILY_4U_M31, 1 << 24, 500, 8),
    (mh.FAMILY_2U_M61, 1 << 30, 500, 1),
    (mh.FAMILY_4U_M61, 1 << 30, 100, 2),
    (mh.FAMILY_2U_MS32, 1 << 24, 500, 8),
    (mh.FAMILY_2U_M31, 16609143, 500, 8),
    (mh.FAMILY_4U_M31, 1010017424, 500, 8),
    (mh.FAMILY_2U_M31, 1 << 24, 64, 8),           # eight slices of the nonzeros per tile
    (mh.FAMILY_2U_M31, 1 << 24, 200, 12),         # seven functions per lane, fields that straddle bytes
    (mh.FAMILY_2U_M61, 1 << 30, 1030, 1),         # three function tiles per row
])
def test_signatures_decoded_in_the_kernel_equal_the_oracle(family, D, k, b):
    nnz = np.minimum(np.array(EDGE_NNZ, dtype=np.int64), D)
    rp = W.row_ptr_from_nnz(nnz)
    gen_D = D if D & (D - 1) == 0 else 1 << 30
    col = W.csr_indices_np(nnz, gen_D, seed=400 + family + k)
    if gen_D != D:                                   # fold into [0, D) and sort again: the packed form needs sorted rows
        col = (col % np.uint32(D)).astype(np.uint32)
        col = np.concatenate([np.sort(col[rp[r]:rp[r + 1]]) for r in range(len(nnz))])
    c = W.coefficients(k, family, seed=500 + k)
    got, st = _packed_signatures(rp, col, D, k, b, family, c)
    assert st == 0
    want = oracle.signatures(rp, col, D, k, b, family, c)
    if not np.array_equal(got, want):
        bad = np.flatnonzero((got != want).any(axis=1))
        raise AssertionError("rows %s differ (nnz %s)" % (bad[:8].tolist(), nnz[bad[:8]].tolist()))


def test_very_short_packed_rows_whose_values_are_mostly_doubtful():
    """Rows of 0 to 40 nonzeros at D = 2^24: most running maxima of the doubled key are doubtful, so
    nearly every value takes the second look, which reads the packed tile again."""
    D, k = 1 << 24, 500
    nnz = np.array(list(range(0, 41)) * 3, dtype=np.int64)
    rp, col = W.row_ptr_from_nnz(nnz), W.csr_indices_np(nnz, D, seed=909)
    for family, b in ((mh.FAMILY_2U_M31, 8), (mh.FAMILY_2U_M61, 1)):
        c = W.coefficients(k, family, seed=910)
        got, st = _packed_signatures(rp, col, D, k, b, family, c)
        assert st == 0 and np.array_equal(got, oracle.signatures(rp, col, D, k, b, family, c))


def test_packed_batch_of_empty_rows_has_no_words_and_is_still_served():
    """Every row empty: the word array has length 0 (a null pointer from the binding); the rows get
    the signature of the empty set, and unpacking writes nothing."""
    D, k, b, family = 71, 257, 3, mh.FAMILY_2U_M31
    nnz = np.zeros(3, dtype=np.int64)
    rp, col = W.row_ptr_from_nnz(nnz), np.zeros(0, dtype=np.uint32)
    c = W.coefficients(k, family, seed=12)
    rp_d = _dev(rp)
    width, word_ptr, words = mh.pack_indices(rp_d, torch.zeros(1, dtype=torch.int32, device=DEV)[:0])
    assert words.numel() == 0 and int(word_ptr[-1].item()) == 0
    n = 3
    out = torch.full((n, (k * b + 7) // 8), 0xAA, dtype=torch.uint8, device=DEV)
    ws = mh.alloc_workspace(n, 0, k, family, DEV)
    mh.minhash_signatures_packed(rp_d, width, word_ptr, words, D, k, b, family, torch.from_numpy(c.view(np.int64)).to(DEV),
                                 out=out, workspace=ws)
    assert mh.status(ws) == 0
    assert np.array_equal(out.cpu().numpy(), oracle.signatures(rp, col, D, k, b, family, c))
    st = torch.full((1,), 99, dtype=torch.int32, device=DEV)
    sink = torch.full((4,), 0x5A5A5A5A, dtype=torch.int32, device=DEV)
    mh.unpack_indices(rp_d, width, word_ptr, words, sink, st)
    torch.cuda.synchronize()
    assert int(st.item()) == 0 and bool((sink == 0x5A5A5A5A).all())


def test_packed_input_that_does_not_fit_its_word_array_is_reported_not_followed():
    D, k, family = 1 << 24, 64, mh.FAMILY_2U_M31
    nnz = np.array([600, 300, 5], dtype=np.int64)
    rp, col = W.row_ptr_from_nnz(nnz), W.csr_indices_np(nnz, D, seed=3)
    c = torch.from_numpy(W.coefficients(k, family, seed=4).view(np.int64)).to(DEV)
    rp_d = _dev(rp)
    width, word_ptr, words = mh.pack_indices(rp_d, _dev(col))
    ws = mh.alloc_workspace(3, 905, k, family, DEV)
    # the word array handed over is shorter than the offsets say
    mh.minhash_signatures_packed(rp_d, width, word_ptr, words[: words.numel() - 5].contiguous(), D, k, 8, family, c, workspace=ws)
    assert mh.status(ws) == -9
    # a width that is no width
    bad = width.clone()
    bad[1] = 40
    mh.minhash_signatures_packed(rp_d, bad, word_ptr, words, D, k, 8, family, c, workspace=ws)
    assert mh.status(ws) == -9
    # and the permutation table is not served this way
    with pytest.raises(mh.MinhashError) as e:
        mh.minhash_signatures_packed(rp_d, width, word_ptr, words, D, k, 8, mh.FAMILY_PERM, c, workspace=ws)
    assert e.value.code == -2
