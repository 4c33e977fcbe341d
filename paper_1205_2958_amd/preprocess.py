"""LibSVM text in, b-bit minwise signatures out: the preprocessing pipeline of
Section 3.2 (load the data, hash it on the GPU in batches, store k*b bits per
example) as one command.

    python -m paper_1205_2958_amd.preprocess data.svm out_prefix --k 200 --b 8 --family 2u

writes ``out_prefix.sig.npy`` (uint8 [n, ceil(k*b/8)], value j of a row in bits
[j*b, (j+1)*b) of its little-endian bit string), ``out_prefix.labels.npy``
(float32 [n]) and ``out_prefix.json`` (k, b, family, D, seed, so that the hash
functions can be drawn again).  ``--expand`` also writes
``out_prefix.expanded.npy`` (int32 [n, k]): the positions of the k ones of each
example in the 2^b * k dimensional binary vector that Section 1.1 feeds to a
linear learner.  ``--save-csr file`` keeps a binary copy of the parsed data,
which is accepted as input in place of the text, so that trying other k, b or
hash families (the experiments of Section 4) parses the text once.

This module only moves buffers: parsing is the library's threaded parser,
hashing and expansion are its kernels.
"""
from __future__ import annotations

import argparse
import json
import mmap
import os
import sys
import time

import numpy as np
import torch

from . import minhash as mh
from . import workloads as W

CSR_MAGIC = b"MHCSR1\0\0"


def save_csr(path: str, row_ptr: np.ndarray, col_idx: np.ndarray, labels: np.ndarray, max_index: int) -> None:
    """Binary copy of a parsed data set: magic, n_rows, nnz, largest index (three
    little-endian int64), then row_ptr int64[n+1], col_idx uint32[nnz], labels
    float32[n].  Parsing text runs at a few GB/s; reading this back runs at the
    speed of the file system, so a data set is parsed once."""
    n, nnz = int(row_ptr.shape[0]) - 1, int(col_idx.shape[0])
    with open(path, "wb") as f:
        f.write(CSR_MAGIC)
        f.write(np.array([n, nnz, max_index], dtype="<i8").tobytes())
        f.write(np.ascontiguousarray(row_ptr, dtype="<i8").tobytes())
        f.write(np.ascontiguousarray(col_idx).view(np.uint32).astype("<u4", copy=False).tobytes())
        f.write(np.ascontiguousarray(labels, dtype="<f4").tobytes())


def load_csr(path: str):
    """Memory-maps a file written by save_csr; returns (row_ptr, col_idx, labels, max_index)
    as NumPy views of the file, or None when the file does not start with the magic."""
    with open(path, "rb") as f:
        head = f.read(len(CSR_MAGIC) + 24)
    if len(head) < len(CSR_MAGIC) + 24 or head[:len(CSR_MAGIC)] != CSR_MAGIC:
        return None
    n, nnz, max_index = (int(v) for v in np.frombuffer(head[len(CSR_MAGIC):], dtype="<i8"))
    if n < 0 or nnz < 0:
        raise ValueError("corrupt CSR file header")
    off = len(CSR_MAGIC) + 24
    need = off + 8 * (n + 1) + 4 * nnz + 4 * n
    if os.path.getsize(path) != need:
        raise ValueError("CSR file has %d bytes, its header announces %d" % (os.path.getsize(path), need))
    row_ptr = np.memmap(path, dtype="<i8", mode="r", offset=off, shape=(n + 1,))
    col_idx = np.memmap(path, dtype="<u4", mode="r", offset=off + 8 * (n + 1), shape=(nnz,)) if nnz else np.zeros(0, "<u4")
    labels = np.memmap(path, dtype="<f4", mode="r", offset=off + 8 * (n + 1) + 4 * nnz, shape=(n,)) if n else np.zeros(0, "<f4")
    if n and (int(row_ptr[0]) != 0 or int(row_ptr[-1]) != nnz):
        raise ValueError("corrupt CSR file: row_ptr does not span the index array")
    return row_ptr, col_idx, labels, max_index


FAMILIES = {
    "2u": mh.FAMILY_2U_M31, "4u": mh.FAMILY_4U_M31, "2u61": mh.FAMILY_2U_M61, "4u61": mh.FAMILY_4U_M61,
    "ms32": mh.FAMILY_2U_MS32, "ms32high": mh.FAMILY_2U_MS32_HIGH,
}


def _pinned_copy(a: np.ndarray) -> torch.Tensor:
    t = torch.empty(a.shape, dtype=torch.from_numpy(np.empty(0, dtype=a.dtype)).dtype, pin_memory=True)
    t.numpy()[...] = a
    return t


def run(path: str, prefix: str, k: int, b: int, family_name: str, seed: int, universe: int, batch_rows: int,
        index_base: int, threads: int, expand: bool, log=print, save_csr_path: str = "",
        round_universe: bool = False) -> dict:
    family = FAMILIES[family_name]
    dev = torch.device("cuda:0")
    t0 = time.perf_counter()
    binary = load_csr(path)
    if binary is not None:
        rp, col, lab_np, max_index = binary
        size = 0
    else:
        with open(path, "rb") as f:
            size = f.seek(0, 2)
            if size == 0:
                raise SystemExit("empty input file")
            mm = mmap.mmap(f.fileno(), 0, access=mmap.ACCESS_READ)
            try:
                row_ptr, col_idx, labels, max_index = mh.parse_libsvm(mm, index_base=index_base, n_threads=threads)
            finally:
                mm.close()
        rp, col, lab_np = row_ptr.numpy(), col_idx.numpy().view(np.uint32), labels.numpy()
        if save_csr_path:
            save_csr(save_csr_path, rp, col, lab_np, max_index)
    n = int(rp.shape[0]) - 1
    nnz = int(col.shape[0])
    t_parse = time.perf_counter() - t0
    if binary is not None:
        log("mapped %d rows, %d nonzeros, largest index %d from the binary copy" % (n, nnz, max_index))
    else:
        log("parsed %d rows, %d nonzeros, largest index %d in %.2f s (%.2f GB/s)"
            % (n, nnz, max_index, t_parse, size / t_parse / 1e9))

    D = universe or (max_index + 1)
    if round_universe and D & (D - 1) and (1 << (D - 1).bit_length()) < W.family_prime(family):
        D = 1 << (D - 1).bit_length()
    if max_index >= D:
        raise SystemExit("the data holds index %d, beyond the universe size %d" % (max_index, D))
    if family in (mh.FAMILY_2U_MS32, mh.FAMILY_2U_MS32_HIGH):
        if D & (D - 1):                                  # multiply-shift hashes into a power of two
            D = 1 << (D - 1).bit_length()
    elif D >= W.family_prime(family):
        raise SystemExit("universe size %d needs the larger prime: use --family 2u61 or 4u61" % D)

    coeffs = W.coefficients(k, family, seed)
    mh.check_coeffs(coeffs, family)
    params = torch.from_numpy(coeffs.view(np.int64)).to(dev)

    batches, max_rows, max_nnz = [], 1, 1
    for lo in range(0, n, batch_rows):
        hi = min(n, lo + batch_rows)
        a, z = int(rp[lo]), int(rp[hi])
        batches.append((_pinned_copy(np.asarray(rp[lo:hi + 1]) - a), _pinned_copy(np.asarray(col[a:z]).view(np.int32))))
        max_rows, max_nnz = max(max_rows, hi - lo), max(max_nnz, z - a)
    t1 = time.perf_counter()
    outs = mh.stream_batches(batches, D, k, b, family, params, max_rows, max_nnz) if batches else []
    t_hash = time.perf_counter() - t1
    sig_bytes = (k * b + 7) // 8
    sig = np.concatenate([o.numpy() for o in outs], axis=0) if outs else np.zeros((0, sig_bytes), np.uint8)
    log("hashed in %.3f s (%.3g evaluations/s, copies included)" % (t_hash, nnz * k / max(t_hash, 1e-9)))

    np.save(prefix + ".sig.npy", sig)
    np.save(prefix + ".labels.npy", np.asarray(lab_np, dtype=np.float32))
    meta = {"rows": n, "nonzeros": nnz, "k": k, "b": b, "family": family_name, "D": D, "seed": seed,
            "sig_bytes": sig_bytes, "parse_s": round(t_parse, 3), "hash_s": round(t_hash, 3)}
    if expand:
        if b > 16:
            raise SystemExit("--expand needs b <= 16 (positions are int32)")
        rows = []
        for lo in range(0, n, batch_rows):
            s_d = torch.from_numpy(sig[lo:lo + batch_rows]).to(dev)
            rows.append(mh.expand_indices(s_d, k, b).cpu().numpy())
        np.save(prefix + ".expanded.npy", np.concatenate(rows, axis=0) if rows else np.zeros((0, k), np.int32))
        meta["expanded_dim"] = (1 << b) * k
    with open(prefix + ".json", "w") as f:
        json.dump(meta, f, indent=1)
    return meta


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("input", help="LibSVM text file: label index:value ... per line (values are ignored: binary data)")
    ap.add_argument("prefix", help="output prefix")
    ap.add_argument("--k", type=int, default=200, help="hash functions (signature fields)")
    ap.add_argument("--b", type=int, default=8, help="bits kept of each minimum")
    ap.add_argument("--family", choices=sorted(FAMILIES), default="2u")
    ap.add_argument("--seed", type=int, default=1, help="seed of the hash-function coefficients")
    ap.add_argument("--universe", type=int, default=0, help="D (default: largest index + 1)")
    ap.add_argument("--batch-rows", type=int, default=200_000)
    ap.add_argument("--index-base", type=int, default=1, choices=[0, 1])
    ap.add_argument("--threads", type=int, default=16)
    ap.add_argument("--expand", action="store_true", help="also write the positions of the ones of the 2^b*k expansion")
    ap.add_argument("--round-universe", action="store_true",
                    help="hash into the next power of two above D (the functions then map the indices into a "
                         "superset of the universe, Section 3.3 assumes D = 2^s anyway): the kernels for "
                         "power-of-two D are up to twice as fast")
    ap.add_argument("--save-csr", default="", help="also write the parsed data as a binary CSR file; such a file is "
                                                   "accepted as input in place of the text")
    a = ap.parse_args(argv)
    if not torch.cuda.is_available():
        print("preprocess needs a GPU", file=sys.stderr)
        return 2
    meta = run(a.input, a.prefix, a.k, a.b, a.family, a.seed, a.universe, a.batch_rows, a.index_base, a.threads,
               a.expand, save_csr_path=a.save_csr, round_universe=a.round_universe)
    print(json.dumps(meta))
    return 0


if __name__ == "__main__":
    sys.exit(main())
