"""The file-to-signature command end to end on the GPU (parse, batch loop of
Section 3.2, hash, expand) against the oracle run on the same rows."""
import json

import numpy as np
import pytest

from oracle import oracle
from paper_1205_2958_amd import workloads as W

pytestmark = pytest.mark.gpu


def _write_libsvm(path, rp, col, labels):
    with open(path, "w") as f:
        for i in range(len(rp) - 1):
            feats = " ".join("%d:1" % (int(t) + 1) for t in col[rp[i]:rp[i + 1]])
            f.write(("%+d" % labels[i]) + (" " + feats if feats else "") + "\n")


@pytest.mark.parametrize("family_name,universe", [("2u", 0), ("4u", 16609143), ("2u61", 1 << 30), ("ms32", 0)])
def test_file_to_signatures(tmp_path, family_name, universe):
    from paper_1205_2958_amd import preprocess

    rng = np.random.Generator(np.random.PCG64(71))
    nnz = np.concatenate([rng.integers(0, 400, size=700), [0, 9000, 1, 20000]]).astype(np.int64)
    rp = W.row_ptr_from_nnz(nnz)
    col = W.csr_indices_np(nnz, 1 << 22, seed=72)
    labels = rng.choice([-1, 1], size=len(nnz))
    src = tmp_path / "data.svm"
    _write_libsvm(src, rp, col, labels)
    k, b = 130, 4
    prefix = str(tmp_path / "out")
    meta = preprocess.run(str(src), prefix, k, b, family_name, seed=5, universe=universe, batch_rows=256,
                          index_base=1, threads=4, expand=True, log=lambda *_: None)
    assert meta["rows"] == len(nnz) and meta["nonzeros"] == int(rp[-1])
    assert json.load(open(prefix + ".json"))["D"] == meta["D"]
    family = preprocess.FAMILIES[family_name]
    D = meta["D"]
    expect_D = universe or int(col.max()) + 1
    if family_name == "ms32":
        expect_D = 1 << (expect_D - 1).bit_length()        # multiply-shift hashes into a power of two
    assert D == expect_D
    want = oracle.signatures(rp, col, D, k, b, family, W.coefficients(k, family, 5))
    sig = np.load(prefix + ".sig.npy")
    assert np.array_equal(sig, want)
    assert np.array_equal(np.load(prefix + ".labels.npy"), labels.astype(np.float32))
    assert np.array_equal(np.load(prefix + ".expanded.npy").view(np.uint32), oracle.expand(want, k, b))


def test_binary_copy_gives_the_same_signatures(tmp_path):
    from paper_1205_2958_amd import preprocess

    nnz = np.array([5, 0, 300, 2500, 1, 77], dtype=np.int64)
    rp = W.row_ptr_from_nnz(nnz)
    col = W.csr_indices_np(nnz, 1 << 20, seed=9)
    labels = np.array([1, -1, 1, 1, -1, 1])
    src = tmp_path / "data.svm"
    _write_libsvm(src, rp, col, labels)
    quiet = dict(log=lambda *_: None)
    m1 = preprocess.run(str(src), str(tmp_path / "a"), 64, 8, "2u", 3, 0, 4, 1, 2, False,
                        save_csr_path=str(tmp_path / "data.csr"), **quiet)
    m2 = preprocess.run(str(tmp_path / "data.csr"), str(tmp_path / "b"), 64, 8, "2u", 3, 0, 4, 1, 2, False, **quiet)
    assert m1["D"] == m2["D"] and m1["nonzeros"] == m2["nonzeros"] == int(rp[-1])
    assert np.array_equal(np.load(str(tmp_path / "a.sig.npy")), np.load(str(tmp_path / "b.sig.npy")))
    assert np.array_equal(np.load(str(tmp_path / "b.labels.npy")), labels.astype(np.float32))
    want = oracle.signatures(rp, col, m2["D"], 64, 8, preprocess.FAMILIES["2u"], W.coefficients(64, preprocess.FAMILIES["2u"], 3))
    assert np.array_equal(np.load(str(tmp_path / "b.sig.npy")), want)


def test_round_universe_hashes_into_the_next_power_of_two(tmp_path):
    from paper_1205_2958_amd import preprocess

    nnz = np.array([40, 3, 900], dtype=np.int64)
    rp = W.row_ptr_from_nnz(nnz)
    col = (W.csr_indices_np(nnz, 1 << 20, seed=19) % np.uint32(1000003)).astype(np.uint32)
    src = tmp_path / "data.svm"
    _write_libsvm(src, rp, col, np.array([1, 1, -1]))
    meta = preprocess.run(str(src), str(tmp_path / "r"), 64, 8, "4u", 4, 1000003, 8, 1, 2, False, log=lambda *_: None,
                          round_universe=True)
    assert meta["D"] == 1 << 20
    want = oracle.signatures(rp, col, 1 << 20, 64, 8, preprocess.FAMILIES["4u"], W.coefficients(64, preprocess.FAMILIES["4u"], 4))
    assert np.array_equal(np.load(str(tmp_path / "r.sig.npy")), want)
