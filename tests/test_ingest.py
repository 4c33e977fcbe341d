"""LibSVM ingest (host only): the threaded parser against a line-by-line Python reading of the same text."""
import numpy as np
import pytest

from paper_1205_2958_amd import minhash as mh
from paper_1205_2958_amd import workloads as W


def reference_parse(text: str, base: int):
    rows, labels = [], []
    for line in text.split("\n"):
        line = line.split("#", 1)[0].strip(" \t\r")
        if not line:
            continue
        parts = line.split()
        labels.append(float(parts[0].split("e")[0].split("E")[0]))
        rows.append([int(tok.split(":")[0]) - base for tok in parts[1:]])
    nnz = np.array([len(r) for r in rows], dtype=np.int64)
    col = np.array([t for r in rows for t in r], dtype=np.uint32)
    return W.row_ptr_from_nnz(nnz), col, np.array(labels, dtype=np.float32)


def make_text(rp, col, base, rng, crlf=False):
    lines = []
    for i in range(len(rp) - 1):
        label = rng.choice(["+1", "-1", "1", "0", "3.5", "-0.25"])
        feats = " ".join("%d:%s" % (int(t) + base, rng.choice(["1", "1.0", "0.5", "2e-3"])) for t in col[rp[i]:rp[i + 1]])
        lines.append(label + (" " + feats if feats else ""))
    return ("\r\n" if crlf else "\n").join(lines) + "\n"


@pytest.mark.parametrize("threads", [1, 3, 16])
@pytest.mark.parametrize("base", [0, 1])
def test_parser_matches_reference(threads, base):
    rng = np.random.default_rng(threads * 10 + base)
    nnz = W.lognormal_nnz(3000, 60.0, 1.0, 0, 3000, seed=7)
    nnz[[0, 17, 2999]] = 0
    rp, col = W.row_ptr_from_nnz(nnz), W.csr_indices_np(nnz, 1 << 24, seed=8)
    text = make_text(rp, col, base, rng)
    want_rp, want_col, want_lab = reference_parse(text, base)
    got_rp, got_col, got_lab, mx = mh.parse_libsvm(text.encode(), index_base=base, n_threads=threads)
    assert np.array_equal(got_rp.numpy(), want_rp) and np.array_equal(want_rp, rp)
    assert np.array_equal(got_col.numpy().view(np.uint32), want_col) and np.array_equal(want_col, col)
    assert np.array_equal(got_lab.numpy(), want_lab)
    assert mx == int(col.max())


def test_formatting_corner_cases():
    text = ("# a comment line\n"
            "+1 3:1 7:0.5   12:1e-3  \r\n"
            "\n"
            "   \t \n"
            "-1\n"
            "0.5 1:1 # trailing comment 9:9\n"
            "2 4294967296:1")                       # largest index, no final newline
    rp, col, lab, mx = mh.parse_libsvm(text.encode(), index_base=1, n_threads=4)
    assert rp.tolist() == [0, 3, 3, 4, 5]
    assert col.numpy().view(np.uint32).tolist() == [2, 6, 11, 0, 4294967295]
    assert lab.tolist() == [1.0, -1.0, 0.5, 2.0]
    assert mx == 4294967295
    rp, col, lab, mx = mh.parse_libsvm(b"", n_threads=4)
    assert rp.tolist() == [0] and col.numel() == 0 and lab.numel() == 0


@pytest.mark.parametrize("bad", [b"1 0:1\n", b"1 5\n", b"1 x:1\n", b"abc 1:1\n", b"1 4294967297:1\n", b"1 3:1\n1 :1\n"])
def test_malformed_lines_are_reported(bad):
    with pytest.raises(mh.MinhashError) as e:
        mh.parse_libsvm(bad, index_base=1, n_threads=2)
    assert e.value.code == -9


def test_large_text_many_threads_equals_one_thread():
    rng = np.random.default_rng(5)
    nnz = W.lognormal_nnz(20000, 200.0, 1.0, 1, 5000, seed=9)
    rp, col = W.row_ptr_from_nnz(nnz), W.csr_indices_np(nnz, 1 << 24, seed=10)
    lines = []
    for i in range(len(nnz)):
        lines.append("1 " + " ".join("%d:1" % (int(t) + 1) for t in col[rp[i]:rp[i + 1]]))
    blob = ("\n".join(lines) + "\n").encode()
    a = mh.parse_libsvm(blob, n_threads=1)
    b = mh.parse_libsvm(blob, n_threads=16)
    assert np.array_equal(a[0].numpy(), rp) and np.array_equal(b[0].numpy(), rp)
    assert np.array_equal(a[1].numpy().view(np.uint32), col) and np.array_equal(b[1].numpy().view(np.uint32), col)


@pytest.mark.parametrize("final_newline", [True, False])
def test_every_index_width_and_long_values(final_newline):
    """Indices of 1 to 10 digits (the word-at-a-time conversion covers eight), leading zeros,
    values longer than the scanner's windows, tabs and double blanks between entries."""
    rng = np.random.default_rng(11)
    lines, rows = [], []
    for i in range(400):
        row, toks = [], []
        for _ in range(int(rng.integers(0, 40))):
            digits = int(rng.integers(1, 11))
            t = int(rng.integers(10 ** (digits - 1), min(10 ** digits, 2 ** 32 + 1)))
            row.append(t - 1)
            written = ("0" * int(rng.integers(0, 12)) if rng.random() < 0.1 else "") + str(t)
            toks.append(written + ":" + str(rng.choice(["1", "", "0.123456789012345678901234", "1e-30", "x" * 40])))
        rows.append(row)
        seps = [str(rng.choice([" ", " ", " ", "  ", "\t", " \t"])) for _ in toks]
        lines.append("-1" + "".join(s + t for s, t in zip(seps, toks)) + ("  " if rng.random() < 0.2 else ""))
    text = "\n".join(lines) + ("\n" if final_newline else "")
    rp, col, lab, mx = mh.parse_libsvm(text.encode(), index_base=1, n_threads=3)
    assert rp.tolist() == np.concatenate([[0], np.cumsum([len(r) for r in rows])]).tolist()
    assert col.numpy().view(np.uint32).tolist() == [t for r in rows for t in r]
    assert mx == max(t for r in rows for t in r)
    assert lab.tolist() == [-1.0] * len(rows)


def test_short_texts_near_the_buffer_end():
    """Texts shorter than the scanner's windows, and entries that end at the last byte."""
    for text, want in [(b"1 2:1", [1]), (b"1 2:1\n", [1]), (b"1 12345678:1", [12345677]), (b"1 1:1 2:1 3:1 4:1", [0, 1, 2, 3]),
                       (b"1 123456789:1 5:", [123456788, 4]), (b"1\n", []), (b"7", [])]:
        rp, col, lab, mx = mh.parse_libsvm(text, index_base=1, n_threads=2)
        assert col.numpy().view(np.uint32).tolist() == want and rp.tolist() == [0, len(want)]


def test_share_counts_of_another_text_are_refused():
    """Pass 2 trusts the per-thread counts of pass 1 only as far as they fit: counts taken
    from a different text of the same length give an error, not a write out of bounds."""
    import ctypes

    def text_with(n_first):                     # two lines, the entries split n_first / 40 - n_first, same length
        a = " ".join("%07d:1" % (i + 1) for i in range(n_first))
        b = " ".join("%07d:1" % (i + 1) for i in range(40 - n_first))
        return ("1 " + a + "\n1 " + b + "\n").encode() * 2000
    t1, t2 = text_with(10), text_with(30)
    assert len(t1) == len(t2)
    L = mh.lib()
    th = 4
    n, z, m = ctypes.c_int64(0), ctypes.c_int64(0), ctypes.c_uint32(0)
    shares = np.zeros(2 * th, dtype=np.int64)
    b1 = np.frombuffer(t1, dtype=np.uint8)
    assert L.minhash_libsvm_count(b1.ctypes.data, b1.size, 1, th, ctypes.byref(n), ctypes.byref(z), ctypes.byref(m),
                                  shares.ctypes.data) == 0
    assert shares[0::2].sum() == n.value == 4000 and shares[1::2].sum() == z.value == 80000
    guard = 1000
    rp = np.full(n.value + 1 + 2 * guard, -7, dtype=np.int64)
    col = np.full(z.value + 2 * guard, 0xABCDEF01, dtype=np.uint32)
    lab = np.full(n.value + 2 * guard, -7.0, dtype=np.float32)

    def parse(buf, sh):
        return L.minhash_libsvm_parse(buf.ctypes.data, buf.size, 1, th, n.value, z.value, sh.ctypes.data,
                                      rp[guard:].ctypes.data, col[guard:].ctypes.data, lab[guard:].ctypes.data)
    assert parse(b1, shares) == 0
    assert col[guard:guard + 10].tolist() == list(range(10))
    wrong = shares.copy()
    wrong[1] -= 5
    wrong[3] += 5                                # totals still match, the split does not
    assert parse(b1, wrong) == -1
    # a text whose rows hold other counts: the totals agree, the position of every row does not
    shifted = np.frombuffer(t2[len(t2) // 2:] + t1[:len(t1) // 2], dtype=np.uint8)
    assert shifted.size == b1.size
    assert parse(shifted, shares) == -1
    for arr, fill in ((rp, -7), (col, 0xABCDEF01), (lab, -7.0)):
        assert (arr[:guard] == fill).all() and (arr[-guard:] == fill).all()
