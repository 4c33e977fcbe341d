"""LibSVM text in, b-bit minwise signatures out: the preprocessing pipeline of
Section 3.2 (load the data, hash it on the GPU in batches, store k*b bits per
example) as one command.

    python -m paper_1205_2958_amd.preprocess data.svm out_prefix --k 200 --b 8 --family 2u

writes ``out_prefix.sig.npy`` (uint8 [n, ceil(k*b/8)], value j of a row in bits
[j*b, (j+1)*b) of its little-endian bit string), ``out_prefix.labels.npy``
(float32 [n]) and ``out_prefix.json`` (k, b, family, D, seed, so that the hash
functions can be drawn again).  ``--expand`` also writes ``out_prefix.expanded.npy``
(int32 [n, k]): the positions of the k ones of each example in the 2^b * k
dimensional binary vector that Section 1.1 feeds to a linear learner.

This module only moves buffers: parsing is the library's threaded parser,
hashing and expansion are its kernels.
"""
from __future__ import annotations

import argparse
import json
import mmap
import sys
import time

import numpy as np
import torch

from . import minhash as mh
from . import workloads as W

FAMILIES = {
    "2u": mh.FAMILY_2U_M31, "4u": mh.FAMILY_4U_M31, "2u61": mh.FAMILY_2U_M61, "4u61": mh.FAMILY_4U_M61,
    "ms32": mh.FAMILY_2U_MS32, "ms32high": mh.FAMILY_2U_MS32_HIGH,
}


def _pinned_copy(a: np.ndarray) -> torch.Tensor:
    t = torch.empty(a.shape, dtype=torch.from_numpy(a[:0]).dtype, pin_memory=True)
    t.numpy()[...] = a
    return t


def run(path: str, prefix: str, k: int, b: int, family_name: str, seed: int, universe: int, batch_rows: int,
        index_base: int, threads: int, expand: bool, log=print) -> dict:
    family = FAMILIES[family_name]
    dev = torch.device("cuda:0")
    t0 = time.perf_counter()
    with open(path, "rb") as f:
        size = f.seek(0, 2)
        if size == 0:
            raise SystemExit("empty input file")
        mm = mmap.mmap(f.fileno(), 0, access=mmap.ACCESS_READ)
        try:
            row_ptr, col_idx, labels, max_index = mh.parse_libsvm(mm, index_base=index_base, n_threads=threads)
        finally:
            mm.close()
    n = row_ptr.numel() - 1
    nnz = col_idx.numel()
    t_parse = time.perf_counter() - t0
    log("parsed %d rows, %d nonzeros, largest index %d in %.2f s (%.2f GB/s)"
        % (n, nnz, max_index, t_parse, size / t_parse / 1e9))

    D = universe or (max_index + 1)
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

    rp = row_ptr.numpy()
    col = col_idx.numpy()
    batches, max_rows, max_nnz = [], 1, 1
    for lo in range(0, n, batch_rows):
        hi = min(n, lo + batch_rows)
        a, z = int(rp[lo]), int(rp[hi])
        batches.append((_pinned_copy(rp[lo:hi + 1] - a), _pinned_copy(col[a:z])))
        max_rows, max_nnz = max(max_rows, hi - lo), max(max_nnz, z - a)
    t1 = time.perf_counter()
    outs = mh.stream_batches(batches, D, k, b, family, params, max_rows, max_nnz) if batches else []
    t_hash = time.perf_counter() - t1
    sig_bytes = (k * b + 7) // 8
    sig = np.concatenate([o.numpy() for o in outs], axis=0) if outs else np.zeros((0, sig_bytes), np.uint8)
    log("hashed in %.3f s (%.3g evaluations/s, copies included)" % (t_hash, nnz * k / max(t_hash, 1e-9)))

    np.save(prefix + ".sig.npy", sig)
    np.save(prefix + ".labels.npy", labels.numpy())
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
    a = ap.parse_args(argv)
    if not torch.cuda.is_available():
        print("preprocess needs a GPU", file=sys.stderr)
        return 2
    meta = run(a.input, a.prefix, a.k, a.b, a.family, a.seed, a.universe, a.batch_rows, a.index_base, a.threads,
               a.expand)
    print(json.dumps(meta))
    return 0


if __name__ == "__main__":
    sys.exit(main())
