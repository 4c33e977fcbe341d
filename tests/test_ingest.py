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
