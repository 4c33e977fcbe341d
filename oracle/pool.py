"""Worker processes that run the CPU oracle on shards of rows (test infrastructure
only, like everything under oracle/: used by the GPU tests and by the
cpu_baseline leg of bench.py).

The pool only deals rows out and puts the signatures back in order; every
shard is one call of the unchanged single-threaded C oracle.  It must be
created before the process touches the GPU: the workers are forked.
"""
from __future__ import annotations

import time

import numpy as np

FAMILY_PERM = 4


def _row_ptr(lens: np.ndarray) -> np.ndarray:
    rp = np.zeros(lens.shape[0] + 1, dtype=np.int64)
    np.cumsum(lens, out=rp[1:])
    return rp


def _oracle_worker(args):
    from oracle import oracle
    rp, col, D, k, b, family, params = args
    return oracle.signatures(rp, col, D, k, b, family, params)


def _oracle_case_worker(args):
    from oracle import oracle
    rp, col, D, k, b, family, params, out_stride = args
    return oracle.signatures(rp, col, D, k, b, family, params, out_stride)


class OraclePool:
    """Worker processes that run the unchanged single-threaded C oracle, one shard of
    rows each.  Forked before this process touches the GPU; jobs are sent later."""

    def __init__(self, procs: int):
        import multiprocessing as mp
        from oracle import oracle

        oracle.build()
        self.procs = procs
        self.pool = mp.get_context("fork").Pool(procs)
        empty = (np.zeros(2, np.int64), np.zeros(0, np.uint32), 1 << 24, 8, 8, 0, np.zeros((8, 2), np.uint64))
        self.pool.map(_oracle_worker, [empty] * procs)          # every worker has the library loaded

    def close(self):
        self.pool.close()
        self.pool.join()

    def cases_async(self, cases):
        """Starts one oracle call per case (rp, col, D, k, b, family, params, out_stride), each whole in one
        worker; returns the pending result, whose get() gives the signature arrays in order."""
        return self.pool.map_async(_oracle_case_worker, cases, chunksize=1)

    def signatures(self, rp, col, D, k, b, family, params, procs=None, table_rows=None):
        """Signatures of all rows of the CSR (rp, col), rows dealt to `procs` shards of
        about equal nonzeros (longest rows first, each to the least loaded shard).
        For the permutation family `table_rows` holds table[t] for the nonzeros in
        CSR order; every shard gets its own rows of it, renumbered from 0.
        Returns (uint8 [n, sig_bytes], seconds, shards used)."""
        procs = procs or self.procs
        n = rp.shape[0] - 1
        lens = np.diff(rp)
        shard_of = np.zeros(n, dtype=np.int64)
        load = np.zeros(procs, dtype=np.int64)
        for r in np.argsort(-lens, kind="stable"):
            s = int(np.argmin(load))
            shard_of[r] = s
            load[s] += lens[r] + 1
        jobs, members = [], []
        for s in range(procs):
            rows = np.flatnonzero(shard_of == s)
            if rows.size == 0:
                continue
            pieces = [np.arange(rp[r], rp[r + 1]) for r in rows]
            take = np.concatenate(pieces) if pieces else np.zeros(0, np.int64)
            sub_rp = _row_ptr(lens[rows])
            if family == FAMILY_PERM:
                sub_col = np.arange(take.shape[0], dtype=np.uint32)      # the oracle reads table[t][j]: row t of the shard's slice
                jobs.append((sub_rp, sub_col, max(int(take.shape[0]), 1), k, b, family, table_rows[take]))
            else:
                jobs.append((sub_rp, col[take], D, k, b, family, params))
            members.append(rows)
        t0 = time.perf_counter()
        parts = self.pool.map(_oracle_worker, jobs, chunksize=1)
        dt = time.perf_counter() - t0
        sig = np.zeros((n, (k * b + 7) // 8), dtype=np.uint8)
        for rows, part in zip(members, parts):
            sig[rows] = part
        return sig, dt, len(jobs)
