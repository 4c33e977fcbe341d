"""The binary CSR copy that the preprocessing command writes and reads back."""
import numpy as np
import pytest

from paper_1205_2958_amd import preprocess


def test_round_trip(tmp_path):
    rp = np.array([0, 3, 3, 7], dtype=np.int64)
    col = np.array([5, 9, 4000000000, 0, 1, 2, 3], dtype=np.uint32)
    labels = np.array([1.0, -1.0, 0.5], dtype=np.float32)
    path = str(tmp_path / "d.csr")
    preprocess.save_csr(path, rp, col, labels, 4000000000)
    rp2, col2, lab2, mx = preprocess.load_csr(path)
    assert mx == 4000000000
    assert np.array_equal(rp2, rp) and np.array_equal(col2, col) and np.array_equal(lab2, labels)


def test_empty_data_set(tmp_path):
    path = str(tmp_path / "e.csr")
    preprocess.save_csr(path, np.zeros(1, np.int64), np.zeros(0, np.uint32), np.zeros(0, np.float32), -1)
    rp, col, lab, mx = preprocess.load_csr(path)
    assert rp.tolist() == [0] and col.size == 0 and lab.size == 0 and mx == -1


def test_text_is_not_taken_for_binary(tmp_path):
    path = tmp_path / "t.svm"
    path.write_text("+1 1:1 2:1\n")
    assert preprocess.load_csr(str(path)) is None


def test_truncated_file_is_refused(tmp_path):
    path = str(tmp_path / "d.csr")
    preprocess.save_csr(path, np.array([0, 2], np.int64), np.array([1, 2], np.uint32), np.ones(1, np.float32), 2)
    data = open(path, "rb").read()
    open(path, "wb").write(data[:-3])
    with pytest.raises(ValueError):
        preprocess.load_csr(path)
