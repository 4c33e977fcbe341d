"""Seeded synthetic inputs for the minwise-hashing preprocessing path.

This module only *draws inputs*: row lengths, feature indices, hash
coefficients, permutation tables and planted-resemblance set pairs.  It holds
none of the method's arithmetic (no hashing, no minima, no packing), so both
the GPU path and the CPU checker can be fed from it without sharing code.

The shapes follow the two datasets of the paper's Table "tab_data" (webspam:
350 000 sets, D about 2^24, about 3 700 nonzeros per set; expanded rcv1:
D about 2^30, about 10^4 nonzeros per set), which are not available here; the
inputs below stand in for them.

Feature indices of one row are produced by a keyed bijection of [0, 2^s)
(an unbalanced Feistel network whose round keys depend on the seed and the
row number) applied to the positions 0..nnz-1, then sorted.  A bijection makes
the indices of a row distinct by construction, every index is (close to)
uniform in [0, D), and each element depends only on (seed, row, position), so
the same recipe runs element-wise in NumPy on the host or in torch on a GPU
and yields identical bits.  All intermediate values stay below 2^63 so that
signed 64-bit arithmetic never wraps.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

M31 = (1 << 31) - 1
M61 = (1 << 61) - 1

FAMILY_2U_M31 = 0
FAMILY_4U_M31 = 1
FAMILY_2U_M61 = 2
FAMILY_4U_M61 = 3
FAMILY_PERM = 4
FAMILY_2U_MS32 = 5        # multiply-shift 2U of Section 3.3, lowest s bits
FAMILY_2U_MS32_HIGH = 6   # the same, highest s bits

_FEISTEL_ROUNDS = 6
_MASK31 = 0x7FFFFFFF


# --------------------------------------------------------------------------
# element-wise integer mixing that behaves identically in numpy and torch
# --------------------------------------------------------------------------
def _mix31(v):
    """Scramble values in [0, 2^31) to values in [0, 2^31).

    Works on int64 numpy arrays and int64 torch tensors alike; every product
    is of two numbers below 2^31, so nothing exceeds 2^62.
    """
    v = v * 0x2C1B3C6D
    v = (v ^ (v >> 15) ^ (v >> 31)) & _MASK31
    v = v * 0x297A2D39
    v = (v ^ (v >> 14) ^ (v >> 30)) & _MASK31
    return v


def _round_keys_np(seed: int, rows: np.ndarray) -> np.ndarray:
    """int64 [len(rows), rounds] round keys, each in [0, 2^31)."""
    rows = rows.astype(np.int64)
    lo = rows & _MASK31
    hi = (rows >> 31) & _MASK31
    base = _mix31(lo ^ _mix31(hi ^ np.int64(seed & _MASK31)))
    keys = np.empty((rows.shape[0], _FEISTEL_ROUNDS), dtype=np.int64)
    for r in range(_FEISTEL_ROUNDS):
        keys[:, r] = _mix31(base ^ np.int64((0x3C6EF372 * (r + 1)) & _MASK31))
    return keys


def _feistel(pos, keys_of, s: int):
    """Keyed bijection of [0, 2^s) applied element-wise to ``pos``.

    ``keys_of(r)`` returns the per-element key array of round ``r``.
    """
    rb = s // 2
    lb = s - rb
    mask_r = (1 << rb) - 1
    mask_l = (1 << lb) - 1
    right = pos & mask_r
    left = (pos >> rb) & mask_l
    for r in range(_FEISTEL_ROUNDS):
        k = keys_of(r)
        if r % 2 == 0:
            left = left ^ (_mix31((right + k) & _MASK31) & mask_l)
        else:
            right = right ^ (_mix31((left + k) & _MASK31) & mask_r)
    return (left << rb) | right


def _check_pow2(D: int) -> int:
    s = int(D).bit_length() - 1
    if D < 4 or (1 << s) != D or s > 32:
        raise ValueError("the bijective index generator needs D = 2^s, 2 <= s <= 32")
    return s


# --------------------------------------------------------------------------
# row lengths
# --------------------------------------------------------------------------
def lognormal_nnz(n_rows: int, median: float, sigma: float, lo: int, hi: int, seed: int) -> np.ndarray:
    """nnz_i = clip(rint(exp(ln(median) + sigma * Z_i)), lo, hi)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    z = rng.standard_normal(n_rows)
    nnz = np.rint(np.exp(math.log(median) + sigma * z))
    return np.clip(nnz, lo, hi).astype(np.int64)


def lomax_nnz(n_rows: int, scale: float, tail: float, lo: int, hi: int, seed: int) -> np.ndarray:
    """Shifted power law: nnz_i = clip(floor(scale * (U^(-1/tail) - 1)) + 1, lo, hi).

    The density falls off as x^-(1 + tail); tail = 0.8 gives the x^-1.8 tail of
    the heavy-tailed workload.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    u = 1.0 - rng.random(n_rows)  # (0, 1]
    nnz = np.floor(scale * (np.power(u, -1.0 / tail) - 1.0)) + 1.0
    return np.clip(nnz, lo, hi).astype(np.int64)


def row_ptr_from_nnz(nnz: np.ndarray) -> np.ndarray:
    row_ptr = np.zeros(nnz.shape[0] + 1, dtype=np.int64)
    np.cumsum(nnz, out=row_ptr[1:])
    return row_ptr


# --------------------------------------------------------------------------
# feature indices
# --------------------------------------------------------------------------
def csr_indices_np(nnz: np.ndarray, D: int, seed: int, row_offset: int = 0, rows: Optional[np.ndarray] = None) -> np.ndarray:
    """Sorted, distinct uint32 indices in [0, D) for every row, concatenated.

    ``row_offset`` is added to the row number in the key derivation so that a
    slice of rows of a large workload can be generated on its own; ``rows``
    gives the row numbers one by one instead (``nnz[i]`` is then the length of
    row ``rows[i]``), for a sample of rows that are not neighbours.
    """
    s = _check_pow2(D)
    nnz = np.asarray(nnz, dtype=np.int64)
    if nnz.size and int(nnz.max()) > D:
        raise ValueError("a row cannot hold more than D distinct indices")
    n = nnz.shape[0]
    row_ptr = row_ptr_from_nnz(nnz)
    total = int(row_ptr[-1])
    if total == 0:
        return np.zeros(0, dtype=np.uint32)
    row_of = np.repeat(np.arange(n, dtype=np.int64), nnz)
    pos = np.arange(total, dtype=np.int64) - row_ptr[row_of]
    numbers = np.arange(n, dtype=np.int64) + row_offset if rows is None else np.asarray(rows, dtype=np.int64)
    if numbers.shape[0] != n:
        raise ValueError("one row number per row length")
    keys = _round_keys_np(seed, numbers)
    idx = _feistel(pos, lambda r: keys[row_of, r], s)
    order_key = (row_of << 32) | idx
    order_key.sort()
    return (order_key & 0xFFFFFFFF).astype(np.uint32)


def csr_indices_torch(nnz: np.ndarray, D: int, seed: int, device, row_offset: int = 0,
                      rows_per_block: int = 32768):
    """Same bits as :func:`csr_indices_np`, produced with torch ops on ``device``.

    Returns an int32 tensor holding the uint32 bit patterns (torch has no
    native uint32 arithmetic; the caller hands the pointer to the library).
    Rows are processed in blocks to bound temporary memory.
    """
    import torch

    s = _check_pow2(D)
    nnz = np.asarray(nnz, dtype=np.int64)
    if nnz.size and int(nnz.max()) > D:
        raise ValueError("a row cannot hold more than D distinct indices")
    n = nnz.shape[0]
    row_ptr = row_ptr_from_nnz(nnz)
    total = int(row_ptr[-1])
    out = torch.empty(total, dtype=torch.int32, device=device)
    keys_all = _round_keys_np(seed, np.arange(n, dtype=np.int64) + row_offset)
    for r0 in range(0, n, rows_per_block):
        r1 = min(n, r0 + rows_per_block)
        e0, e1 = int(row_ptr[r0]), int(row_ptr[r1])
        if e1 == e0:
            continue
        nnz_b = torch.from_numpy(nnz[r0:r1]).to(device)
        rp_b = torch.from_numpy(row_ptr[r0:r1] - e0).to(device)
        keys = torch.from_numpy(keys_all[r0:r1]).to(device)
        row_of = torch.repeat_interleave(torch.arange(r1 - r0, dtype=torch.int64, device=device), nnz_b)
        pos = torch.arange(e1 - e0, dtype=torch.int64, device=device) - rp_b[row_of]
        idx = _feistel(pos, lambda r: keys[:, r][row_of], s)
        order_key = (row_of << 32) | idx
        order_key = torch.sort(order_key).values
        out[e0:e1] = (order_key & 0xFFFFFFFF).to(torch.int32)  # wraps to the uint32 bit pattern
        del row_of, pos, idx, order_key
    return out


# --------------------------------------------------------------------------
# which rows of a batch a checker looks at
# --------------------------------------------------------------------------
def stratified_rows(nnz: np.ndarray, k: int, eval_budget: float, seed: int, split: int = 8192,
                    max_row_evals: Optional[float] = None, heavy_from: Optional[int] = None):
    """A seeded sample of row numbers for comparing a batch's signatures with a
    slow checker, chosen by row length alone (no hashing here):

      * the first and the last row, the shortest row and the longest row
        (the longest that ``max_row_evals`` allows, if given);
      * for m = 1, 2, 4, 8, ... times ``split``, the length at which rows are
        cut into chunks, the row whose length is closest to m * split from below
        and the one closest from above;
      * if ``heavy_from`` is given, rows of at least that many nonzeros, in
        seeded random order;
      * then rows drawn in turn from the ten deciles of the length distribution
        (seeded, without replacement), decile 0 first, until the budget of
        ``eval_budget`` evaluations (nonzeros * k) is spent.

    The named rows and the heavy ones are taken while they fit three fifths of
    the budget (the first row always is); the deciles get the rest.  Returns (sorted row numbers, dict with the achieved coverage).
    """
    nnz = np.asarray(nnz, dtype=np.int64)
    n = nnz.shape[0]
    rng = np.random.Generator(np.random.PCG64(seed))
    order = np.argsort(nnz, kind="stable")
    lens = nnz[order]
    cap = np.inf if max_row_evals is None else max_row_evals
    ok = lambda r: float(nnz[r]) * k <= cap
    must = [0, n - 1, int(order[0])]
    at_cap = n if max_row_evals is None else int(np.searchsorted(lens, max_row_evals / k, side="right"))
    if at_cap > 0:
        must.append(int(order[at_cap - 1]))                           # the longest row the cap allows
    top = int(lens[-1])
    m = 1
    while m * split <= top:                                           # m = 1, 2, 4, 8, ...
        at = int(np.searchsorted(lens, m * split, side="right"))      # lens[at-1] <= m*split < lens[at]
        if at > 0:
            must.append(int(order[at - 1]))
        if at < n:
            must.append(int(order[at]))
        m *= 2
    picked, spent = [], 0.0
    seen = set()

    def take(r: int, limit: float) -> bool:
        nonlocal spent
        if r in seen:
            return True
        cost = float(nnz[r]) * k
        if not ok(r) or (picked and spent + cost > limit):
            return False
        seen.add(r)
        picked.append(r)
        spent += cost
        return True

    # the named rows and the heavy ones may spend three fifths of the budget; the deciles get the rest
    for r in must:
        take(r, 0.6 * eval_budget)
    if heavy_from is not None:
        heavy = np.flatnonzero(nnz >= heavy_from)
        for r in rng.permutation(heavy):
            if spent >= 0.6 * eval_budget:
                break
            take(int(r), 0.6 * eval_budget)
    deciles = [rng.permutation(part) for part in np.array_split(order, 10)]
    at = [0] * 10
    live = True
    while live and spent < eval_budget:
        live = False
        for d in range(10):
            while at[d] < len(deciles[d]):
                r = int(deciles[d][at[d]])
                at[d] += 1
                if r in seen:
                    continue
                if take(r, eval_budget):
                    live = True
                break
    rows = np.array(sorted(picked), dtype=np.int64)
    total_evals = float(nnz.sum()) * k
    cover = {
        "rows": int(rows.shape[0]),
        "nonzeros": int(nnz[rows].sum()),
        "pct_of_evaluations": 100.0 * spent / total_evals if total_evals else 100.0,
        "longest_row": int(nnz[rows].max()) if rows.size else 0,
        "rule": "first, last, shortest, longest row; rows next to 1, 2, 4, ... times %d nonzeros; %srows drawn in turn "
                "from the ten length deciles, seed %d" % (split, "rows of at least %d nonzeros in random order; " % heavy_from
                                                          if heavy_from is not None else "", seed),
    }
    return rows, cover


# --------------------------------------------------------------------------
# hash parameters
# --------------------------------------------------------------------------
def family_prime(family: int) -> int:
    if family in (FAMILY_2U_M31, FAMILY_4U_M31):
        return M31
    if family in (FAMILY_2U_M61, FAMILY_4U_M61):
        return M61
    raise ValueError("family has no prime")


def family_degree(family: int) -> int:
    """Number of coefficients per function (2 for 2U, 4 for 4U)."""
    if family in (FAMILY_2U_M31, FAMILY_2U_M61, FAMILY_2U_MS32, FAMILY_2U_MS32_HIGH):
        return 2
    if family in (FAMILY_4U_M31, FAMILY_4U_M61):
        return 4
    raise ValueError("family has no coefficients")


def coefficients(k: int, family: int, seed: int) -> np.ndarray:
    """uint64 [k, degree]; every coefficient uniform in {0, ..., p-1}.  For the
    multiply-shift families: c0 uniform in [0, 2^32), c1 uniform over the odd
    numbers below 2^32 (Section 3.3)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    if family in (FAMILY_2U_MS32, FAMILY_2U_MS32_HIGH):
        c = rng.integers(0, 1 << 32, size=(k, 2), dtype=np.uint64)
        c[:, 1] |= np.uint64(1)
        return c
    p = family_prime(family)
    return rng.integers(0, p, size=(k, family_degree(family)), dtype=np.uint64)


def perm_table_np(D: int, k: int, seed: int, perm_ld: Optional[int] = None) -> np.ndarray:
    """uint32 [D, perm_ld]; column j < k is an independent uniformly random
    permutation of [0, D) (NumPy's shuffle is Fisher-Yates); pad columns are 0."""
    perm_ld = k if perm_ld is None else perm_ld
    if perm_ld < k:
        raise ValueError("perm_ld < k")
    rng = np.random.Generator(np.random.PCG64(seed))
    table = np.zeros((D, perm_ld), dtype=np.uint32)
    for j in range(k):
        table[:, j] = rng.permutation(D).astype(np.uint32)
    return table


def perm_table_torch(D: int, k: int, seed: int, device, perm_ld: Optional[int] = None):
    """int32 tensor [D, perm_ld] of uint32 bit patterns on ``device``; column j
    is a uniformly random permutation of [0, D) from torch's seeded generator.
    Used for the full-size permutation workload, where drawing 200 permutations
    of 2^24 elements on the host would take minutes."""
    import torch

    perm_ld = k if perm_ld is None else perm_ld
    if perm_ld < k:
        raise ValueError("perm_ld < k")
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    table = torch.zeros((D, perm_ld), dtype=torch.int32, device=device)
    for j in range(k):
        table[:, j] = torch.randperm(D, generator=gen, device=device, dtype=torch.int64).to(torch.int32)
    return table


# --------------------------------------------------------------------------
# planted-resemblance pairs for the statistical checks
# --------------------------------------------------------------------------
def planted_pairs(n_pairs: int, D: int, union: int, shared: int, seed: int, only1: Optional[int] = None):
    """CSR of 2*n_pairs rows: rows 2i and 2i+1 are sets with
    |S1 ∩ S2| = shared and |S1 ∪ S2| = union (resemblance shared/union); the
    non-shared elements are split evenly unless ``only1`` gives the number that
    belong to S1 alone.  Returns (row_ptr, col_idx, f1, f2).
    """
    if not 0 <= shared <= union:
        raise ValueError("need 0 <= shared <= union")
    rest = union - shared
    if only1 is None:
        only1 = rest // 2
    if not 0 <= only1 <= rest:
        raise ValueError("need 0 <= only1 <= union - shared")
    only2 = rest - only1
    f1, f2 = shared + only1, shared + only2
    pool = csr_indices_np(np.full(n_pairs, union, dtype=np.int64), D, seed).reshape(n_pairs, union)
    rng = np.random.Generator(np.random.PCG64(seed + 7919))
    cols = []
    for i in range(n_pairs):
        members = pool[i][rng.permutation(union)]
        s1 = np.sort(np.concatenate([members[:shared], members[shared:shared + only1]]))
        s2 = np.sort(np.concatenate([members[:shared], members[shared + only1:]]))
        cols.append(s1)
        cols.append(s2)
    nnz = np.tile(np.array([f1, f2], dtype=np.int64), n_pairs)
    return row_ptr_from_nnz(nnz), np.concatenate(cols).astype(np.uint32), f1, f2


# --------------------------------------------------------------------------
# the five workloads
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    name: str
    n_rows: int
    D: int
    family: int
    k: int
    b: int
    data_seed: int
    param_seed: int
    nnz_kind: str                      # "lognormal" | "lomax"
    nnz_args: dict = field(default_factory=dict)
    batch_rows: Optional[int] = None   # rows per streamed batch (None: one batch)

    def nnz(self, batch: int = 0) -> np.ndarray:
        n = self.n_rows if self.batch_rows is None else self.batch_rows
        seed = self.data_seed + batch
        if self.nnz_kind == "lognormal":
            return lognormal_nnz(n, seed=seed, **self.nnz_args)
        if self.nnz_kind == "lomax":
            return lomax_nnz(n, seed=seed, **self.nnz_args)
        raise ValueError(self.nnz_kind)

    def n_batches(self) -> int:
        return 1 if self.batch_rows is None else self.n_rows // self.batch_rows

    def sig_bytes(self) -> int:
        return (self.k * self.b + 7) // 8


WORKLOADS = {
    "tiny_2u": Workload("tiny_2u", 1_000, 1 << 24, FAMILY_2U_M31, 64, 8, 1001, 2001, "lognormal",
                        dict(median=400.0, sigma=1.0, lo=1, hi=5_000)),
    "large_2u": Workload("large_2u", 350_000, 1 << 24, FAMILY_2U_M31, 500, 8, 1002, 2002, "lognormal",
                         dict(median=math.exp(7.721), sigma=1.0, lo=1, hi=50_000)),
    "large_4u": Workload("large_4u", 350_000, 1 << 24, FAMILY_4U_M31, 500, 8, 1002, 2003, "lognormal",
                         dict(median=math.exp(7.721), sigma=1.0, lo=1, hi=50_000)),
    "perm_table": Workload("perm_table", 350_000, 1 << 24, FAMILY_PERM, 200, 4, 1002, 3004, "lognormal",
                           dict(median=math.exp(7.721), sigma=1.0, lo=1, hi=50_000)),
    # the hash the paper itself times as "GPU 2U" (Section 3.3), on the webspam-shaped rows
    "large_2u_ms32": Workload("large_2u_ms32", 350_000, 1 << 24, FAMILY_2U_MS32, 500, 8, 1002, 2006, "lognormal",
                              dict(median=math.exp(7.721), sigma=1.0, lo=1, hi=50_000)),
    # 4U with the larger prime on the webspam-shaped rows (no configuration of the paper; times the Horner-form kernels)
    "large_4u_m61": Workload("large_4u_m61", 350_000, 1 << 24, FAMILY_4U_M61, 500, 8, 1002, 2008, "lognormal",
                             dict(median=math.exp(7.721), sigma=1.0, lo=1, hi=50_000)),
    # many short rows (the unexpanded rcv1 has about 73 nonzeros per document): per-row costs, not arithmetic
    "short_rows_2u": Workload("short_rows_2u", 2_000_000, 1 << 24, FAMILY_2U_M31, 500, 8, 1007, 2007, "lognormal",
                              dict(median=60.0, sigma=0.6, lo=1, hi=5_000)),
    "huge_2u_m61": Workload("huge_2u_m61", 2_000_000, 1 << 30, FAMILY_2U_M61, 500, 1, 1005, 2005, "lomax",
                            dict(scale=580.4, tail=0.8, lo=1, hi=1_000_000), batch_rows=200_000),
}
