"""Pins for the CPU oracle: facts fixed by the paper and by mathematics, none of
them computed by the oracle itself.

Every function takes an ``oracle.Oracle``-like object ``o`` (methods ``minima``,
``pack``, ``signatures``) and raises AssertionError on a mismatch, so the same
pins run against the real oracle (must pass) and against deliberately broken
builds of it (at least one must fail; see test_oracle_mutants.py).

Expected values come from: explicit application of permutations in pure
Python, NumPy reductions (``min``), Python's big-integer ``pow`` (modular
powers and inverses), closed forms, the collision identity of Section 1.1
eq. (1), Theorem 1 (Section 1.1) with the C/A formulas given there, the
"lowest b bits" example of Section 1.1, and algebraic invariants of ``min``.
"""
from __future__ import annotations

import itertools
import math
import os

import numpy as np

from paper_1205_2958_amd import workloads as W

M31, M61 = W.M31, W.M61
F2_31, F4_31, F2_61, F4_61, FPERM = (W.FAMILY_2U_M31, W.FAMILY_4U_M31, W.FAMILY_2U_M61, W.FAMILY_4U_M61,
                                      W.FAMILY_PERM)
HASH_FAMILIES = (F2_31, F4_31, F2_61, F4_61)
EMPTY = 0xFFFFFFFF
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _csr(rows):
    nnz = np.array([len(r) for r in rows], dtype=np.int64)
    col = np.array([t for r in rows for t in r], dtype=np.uint32)
    return W.row_ptr_from_nnz(nnz), col


def _coeffs(family, rows_of_coeffs):
    deg = W.family_degree(family)
    c = np.zeros((len(rows_of_coeffs), deg), dtype=np.uint64)
    for j, r in enumerate(rows_of_coeffs):
        for i, v in enumerate(r):
            c[j, i] = v
    return c


def _random_rows(rng, n, D, max_nnz):
    rows = []
    for _ in range(n):
        m = int(rng.integers(1, max_nnz + 1))
        rows.append(sorted(set(int(x) for x in rng.integers(0, D, size=m))))
    return rows


# ---------------------------------------------------------------- permutations
def pin_explicit_permutations_all_subsets(o):
    """Section 1.1: z_j = min(pi_j(S)).  Every non-empty subset of a 10-element
    universe under 5 permutations, applied element by element in Python."""
    D, k = 10, 5
    rng = np.random.Generator(np.random.PCG64(11))
    perms = [rng.permutation(D).tolist() for _ in range(k)]
    table = np.array(perms, dtype=np.uint32).T.copy()          # [D][k]
    subsets = [s for r in range(1, D + 1) for s in itertools.combinations(range(D), r)]
    rp, col = _csr(subsets)
    got = o.minima(rp, col, D, k, FPERM, table)
    for i, s in enumerate(subsets):
        for j in range(k):
            assert got[i, j] == min(perms[j][t] for t in s), (s, j)


def pin_explicit_permutations_random_sets(o):
    """Same definition on D = 64, k = 16, random subsets, with a padded table
    (leading dimension larger than k) whose pad columns hold junk."""
    D, k, ld = 64, 16, 19
    rng = np.random.Generator(np.random.PCG64(12))
    perms = [rng.permutation(D).tolist() for _ in range(k)]
    table = np.full((D, ld), 0, dtype=np.uint32)
    table[:, :k] = np.array(perms, dtype=np.uint32).T
    table[:, k:] = 0                                            # junk smaller than any real entry
    rows = _random_rows(rng, 200, D, 20)
    rp, col = _csr(rows)
    got = o.minima(rp, col, D, k, FPERM, table)
    for i, s in enumerate(rows):
        for j in range(k):
            assert got[i, j] == min(perms[j][t] for t in s)


def pin_identity_permutation_gives_set_minimum(o):
    D, k = 4096, 3
    table = np.repeat(np.arange(D, dtype=np.uint32)[:, None], k, axis=1).copy()
    rng = np.random.Generator(np.random.PCG64(13))
    rows = _random_rows(rng, 100, D, 50)
    rp, col = _csr(rows)
    got = o.minima(rp, col, D, k, FPERM, table)
    want = np.array([min(r) for r in rows], dtype=np.uint32)
    assert np.array_equal(got, np.repeat(want[:, None], k, axis=1))


# ---------------------------------------------------------------- closed forms
def pin_constant_hash(o):
    """All higher coefficients zero: h(t) = (c mod p) mod D for every t, so every
    non-empty row's minimum is c mod D.  Function j gets its own constant, which
    also pins the [k][degree] coefficient layout."""
    rng = np.random.Generator(np.random.PCG64(21))
    for family in HASH_FAMILIES:
        p = W.family_prime(family)
        for D in (1 << 24, 1000003, 1, 2, p - 1):
            if D > (1 << 32):
                continue
            consts = [0, 1, D - 1, D, D + 1, p - 1, p - 2, (p - 1) // 2] + [int(x) for x in rng.integers(0, p, size=8)]
            consts = [c % p for c in consts]
            co = _coeffs(family, [[c] for c in consts])
            rows = _random_rows(rng, 6, min(D, 1 << 20), 9)
            rp, col = _csr(rows)
            got = o.minima(rp, col, D, len(consts), family, co)
            want = np.array([c % D for c in consts], dtype=np.uint64).astype(np.uint32)
            assert np.array_equal(got, np.repeat(want[None, :], len(rows), axis=0)), (family, D)


def pin_identity_hash_gives_set_minimum(o):
    """c = (0, 1[, 0, 0]): h(t) = t because t < D < p, so the minimum is min(S)."""
    rng = np.random.Generator(np.random.PCG64(22))
    for family in HASH_FAMILIES:
        for D in (1 << 24, 1 << 30, 999983):
            rows = _random_rows(rng, 50, D, 40)
            rp, col = _csr(rows)
            got = o.minima(rp, col, D, 1, family, _coeffs(family, [[0, 1]]))
            want = np.array([min(r) for r in rows], dtype=np.uint32)
            assert np.array_equal(got[:, 0], want), (family, D)


def pin_monomials_via_python_pow(o):
    """Exactly one coefficient set to 1: h(t) = (t^i mod p) mod D, with the power
    taken by Python's big-integer pow().  Separates every coefficient slot."""
    rng = np.random.Generator(np.random.PCG64(23))
    for family in HASH_FAMILIES:
        p, deg = W.family_prime(family), W.family_degree(family)
        for D in (1 << 24, 1 << 30, 16609143):
            rows = _random_rows(rng, 40, D, 12) + [[0], [1], [D - 1], [0, D - 1]]
            rp, col = _csr(rows)
            co = _coeffs(family, [[1 if i == e else 0 for i in range(deg)] for e in range(deg)])
            got = o.minima(rp, col, D, deg, family, co)
            for r, s in enumerate(rows):
                for e in range(deg):
                    assert got[r, e] == min(pow(t, e, p) % D for t in s), (family, D, e)


def pin_modular_inverse_identities(o):
    """Single-element rows {t}.  With c1 = t^-1 mod p (Python pow(t, -1, p)),
    c0 + c1 t is congruent to c0 + 1, so h(t) = ((c0 + 1) mod p) mod D exactly.
    c0 = p - 1 forces the wrap to residue 0, c0 = p - 2 the largest residue p - 1.
    For 4U the same with c3 = (t^3)^-1 and with c2 = (t^2)^-1."""
    rng = np.random.Generator(np.random.PCG64(24))
    for family in HASH_FAMILIES:
        p, deg = W.family_prime(family), W.family_degree(family)
        for D in (1 << 24, 1 << 30, p - 1, 1000003):
            if D > (1 << 32):
                continue
            ts = [1, 2, 3, min(D, 1 << 20) - 1] + [int(x) for x in rng.integers(1, min(D, 1 << 30), size=12)]
            c0s = [p - 1, p - 2, 0, 12345 % p, int(rng.integers(0, p))]
            for t in ts:
                rp, col = _csr([[t]])
                rows_c, want = [], []
                for c0 in c0s:
                    for e in range(1, deg):
                        c = [0] * deg
                        c[0] = c0
                        c[e] = pow(pow(t, e, p), -1, p)
                        rows_c.append(c)
                        want.append(((c0 + 1) % p) % D)
                got = o.minima(rp, col, D, len(rows_c), family, _coeffs(family, rows_c))
                assert got[0].tolist() == want, (family, D, t)


def pin_fermat_and_negation(o):
    """c = (c0, p - 1): h(t) = ((c0 - t) mod p) mod D, a sign-sensitive closed form
    (p - 1 is -1 mod p).  With c0 = t it gives 0; with c0 = t - 1 it wraps to p - 1."""
    rng = np.random.Generator(np.random.PCG64(25))
    for family in (F2_31, F2_61):
        p = W.family_prime(family)
        D = 1 << 24
        for t in [1, 5, D - 1] + [int(x) for x in rng.integers(1, D, size=10)]:
            c0s = [t, t - 1, 0, p - 1, int(rng.integers(0, p))]
            rp, col = _csr([[t]])
            got = o.minima(rp, col, D, len(c0s), family, _coeffs(family, [[c0, p - 1] for c0 in c0s]))
            assert got[0].tolist() == [((c0 - t) % p) % D for c0 in c0s]


def pin_small_coefficients_no_wrap(o):
    """If c0 + c1 (D - 1) < 2^31 - 1 the reduction mod p does nothing for either
    prime, so both 2U families equal (c0 + c1 t) mod D computed by NumPy in
    64-bit integers, and a row's minimum is NumPy's min over that."""
    rng = np.random.Generator(np.random.PCG64(26))
    D, k = 1 << 16, 24
    c = rng.integers(0, 1 << 14, size=(k, 2), dtype=np.uint64)
    rows = _random_rows(rng, 60, D, 80)
    rp, col = _csr(rows)
    g31 = o.minima(rp, col, D, k, F2_31, c)
    g61 = o.minima(rp, col, D, k, F2_61, c)
    for i, s in enumerate(rows):
        t = np.array(s, dtype=np.uint64)
        want = ((c[:, 0:1] + c[:, 1:2] * t[None, :]) % np.uint64(D)).min(axis=1).astype(np.uint32)
        assert np.array_equal(g31[i], want)
        assert np.array_equal(g61[i], want)


def pin_4u_with_zero_high_terms_is_2u(o):
    rng = np.random.Generator(np.random.PCG64(27))
    for f2, f4 in ((F2_31, F4_31), (F2_61, F4_61)):
        p = W.family_prime(f2)
        D, k = 1 << 24, 16
        c2 = rng.integers(0, p, size=(k, 2), dtype=np.uint64)
        c4 = np.zeros((k, 4), dtype=np.uint64)
        c4[:, :2] = c2
        rows = _random_rows(rng, 30, D, 60)
        rp, col = _csr(rows)
        assert np.array_equal(o.minima(rp, col, D, k, f2, c2), o.minima(rp, col, D, k, f4, c4))


def pin_big_integer_cross_check(o):
    """Random coefficients, single-element rows: the unreduced polynomial evaluated
    with Python's unbounded integers, then % p and % D.  (A cross-check of the
    128-bit C arithmetic against overflow, not an independent definition.)"""
    rng = np.random.Generator(np.random.PCG64(28))
    for family in HASH_FAMILIES:
        p, deg = W.family_prime(family), W.family_degree(family)
        for D in (1 << 24, 1 << 30, p - 1, 16609143, 1010017424):
            if D >= p or D > (1 << 32):
                continue
            k = 12
            c = rng.integers(0, p, size=(k, deg), dtype=np.uint64)
            c[0, :] = p - 1
            ts = [0, 1, D - 1] + [int(x) for x in rng.integers(0, D, size=20)]
            rp, col = _csr([[t] for t in ts])
            got = o.minima(rp, col, D, k, family, c)
            for r, t in enumerate(ts):
                for j in range(k):
                    poly = sum(int(c[j, i]) * t ** i for i in range(deg))
                    assert got[r, j] == (poly % p) % D, (family, D, t, j)


# ---------------------------------------------------------------- multiply-shift 2U (Section 3.3)
FMS, FMS_HIGH = W.FAMILY_2U_MS32, W.FAMILY_2U_MS32_HIGH


def pin_multiply_shift_against_numpy_uint32(o):
    """Section 3.3, eq. eqn_h_s: ((a1 + a2 t) mod 2^32) mod 2^s.  NumPy's uint32
    arithmetic wraps modulo 2^32 by itself, which is the overflow the paper relies
    on; the lowest s bits are a mask, the highest s bits a shift."""
    rng = np.random.Generator(np.random.PCG64(51))
    for D in (2, 1 << 8, 1 << 24, 1 << 30, 1 << 32):
        s_bits = D.bit_length() - 1
        k = 20
        c = W.coefficients(k, FMS, seed=52 + s_bits)
        c[0] = (0xFFFFFFFF, 0xFFFFFFFF)
        c[1] = (0, 1)
        rows = _random_rows(rng, 40, D, 30) + [[0], [D - 1], [0, D - 1]]
        rp, col = _csr(rows)
        low = o.minima(rp, col, D, k, FMS, c)
        high = o.minima(rp, col, D, k, FMS_HIGH, c)
        c0 = c[:, 0].astype(np.uint32)[:, None]
        c1 = c[:, 1].astype(np.uint32)[:, None]
        for i, srow in enumerate(rows):
            t = np.array(srow, dtype=np.uint32)[None, :]
            with np.errstate(over="ignore"):
                v = c0 + c1 * t                                   # uint32, wraps
            assert np.array_equal(low[i], (v & np.uint32(D - 1)).min(axis=1)), (D, i)
            assert np.array_equal(high[i], (v >> np.uint32(32 - s_bits)).min(axis=1) if s_bits else None), (D, i)


def pin_multiply_shift_is_a_bijection_of_the_universe(o):
    """With an odd multiplier the lowest-s-bits map t -> h(t) permutes [0, 2^s): over
    single-element rows every location appears exactly once, and a row holding the
    whole universe has minimum 0.  The identity multiplier gives h(t) = (c0 + t) mod D."""
    D, k = 256, 6
    c = W.coefficients(k, FMS, seed=53)
    c[0] = (5, 1)
    rp, col = _csr([[t] for t in range(D)] + [list(range(D))])
    m = o.minima(rp, col, D, k, FMS, c)
    for j in range(k):
        assert sorted(m[:D, j].tolist()) == list(range(D))
        assert m[D, j] == 0
    assert m[:D, 0].tolist() == [(5 + t) % D for t in range(D)]
    hi = o.minima(rp, col, D, 1, FMS_HIGH, np.array([[0, 1 << 24]], dtype=np.uint64) | np.uint64(0))
    # multiplier 2^24 is even, hence not a legal draw, but the arithmetic is defined: (t * 2^24 mod 2^32) >> 24 = t
    assert hi[:D, 0].tolist() == list(range(D))


# ---------------------------------------------------------------- ranges, sentinel
def pin_ranges_and_empty_rows(o):
    """Minima of non-empty rows lie in [0, D); an empty row gives 0xFFFFFFFF in every
    slot, hence all-ones b-bit fields; packed fields are < 2^b; pad bits/bytes are 0."""
    rng = np.random.Generator(np.random.PCG64(31))
    for family in HASH_FAMILIES:
        p = W.family_prime(family)
        D, k = 1 << 20, 37
        c = rng.integers(0, p, size=(k, W.family_degree(family)), dtype=np.uint64)
        rows = [[], [5]] + _random_rows(rng, 20, D, 30) + [[]]
        rp, col = _csr(rows)
        m = o.minima(rp, col, D, k, family, c)
        assert np.all(m[0] == EMPTY) and np.all(m[-1] == EMPTY)
        assert np.all(m[1:-1] < D)
        for b in (1, 3, 8, 13):
            sig = (k * b + 7) // 8
            s = o.signatures(rp, col, D, k, b, family, c, out_stride=sig + 3)
            assert np.all(s[:, sig:] == 0)
            bits = np.unpackbits(s[:, :sig], axis=1, bitorder="little")
            assert np.all(bits[:, k * b:] == 0)
            assert np.all(bits[0, :k * b] == 1) and np.all(bits[-1, :k * b] == 1)


# ---------------------------------------------------------------- truncation / layout
def pin_lowest_bits_example(o):
    """Section 1.1 example (golden file): z = 7 keeps 1 for b = 1 and 3 for b = 2."""
    with open(os.path.join(GOLDEN, "lowest_bits_example.txt")) as f:
        cases = [tuple(int(x) for x in line.split()) for line in f if line.strip() and not line.startswith("#")]
    assert cases
    for z, b, want in cases:
        packed = o.pack(np.array([[z]], dtype=np.uint32), b)
        assert packed.shape == (1, 1) and int(packed[0, 0]) == want


def pin_bit_layout_by_hand(o):
    """Value j sits in bits [j b, (j+1) b) of the row's little-endian bit string."""
    m = np.array([[0x1A5, 0x2F3, 0xFFFFFFFF, 0x80000001, 0x6]], dtype=np.uint32)
    assert o.pack(m, 8).tolist() == [[0xA5, 0xF3, 0xFF, 0x01, 0x06]]
    assert o.pack(m, 4).tolist() == [[0x35, 0x1F, 0x06]]                 # low nibble = even j
    assert o.pack(m, 1).tolist() == [[0b01111]]                          # bits 1,1,1,1,0
    assert o.pack(m, 2).tolist() == [[0b01111101, 0b10]]                 # 01,11,11,01 | 10
    # b = 12: 0x1A5, 0x2F3, 0xFFF, 0x001, 0x006 -> bytes A5 31 2F FF 1F 00 06 00
    assert o.pack(m, 12).tolist() == [[0xA5, 0x31, 0x2F, 0xFF, 0x1F, 0x00, 0x06, 0x00]]
    assert o.pack(m, 32).tobytes() == m.astype("<u4").tobytes()
    # b = 6: 0x25, 0x33, 0x3F, 0x01, 0x06 -> bit string by hand
    want_bits = []
    for v in (0x25, 0x33, 0x3F, 0x01, 0x06):
        want_bits += [(v >> i) & 1 for i in range(6)]
    want_bits += [0] * 2
    want = np.packbits(np.array(want_bits, dtype=np.uint8), bitorder="little").tolist()
    assert o.pack(m, 6).tolist() == [want]


def pin_pack_roundtrip_all_b(o):
    from oracle import oracle as loader
    rng = np.random.Generator(np.random.PCG64(32))
    for k in (1, 7, 8, 13, 64, 500):
        m = rng.integers(0, 1 << 32, size=(5, k), dtype=np.uint64).astype(np.uint32)
        for b in range(1, 33):
            packed = o.pack(m, b)
            assert packed.shape[1] == (k * b + 7) // 8
            back = loader.unpack(packed, k, b)
            assert np.array_equal(back, m & np.uint32((1 << b) - 1 if b < 32 else 0xFFFFFFFF)), (k, b)


def pin_signatures_equal_pack_of_minima(o):
    rng = np.random.Generator(np.random.PCG64(33))
    D, k = 1 << 24, 21
    c = rng.integers(0, M31, size=(k, 2), dtype=np.uint64)
    rows = _random_rows(rng, 15, D, 50)
    rp, col = _csr(rows)
    m = o.minima(rp, col, D, k, F2_31, c)
    for b in (1, 4, 8, 10, 32):
        assert np.array_equal(o.signatures(rp, col, D, k, b, F2_31, c), o.pack(m, b))


# ---------------------------------------------------------------- invariants of min
def pin_min_invariants(o):
    """Order and duplicates do not matter; S subset of T gives m(T) <= m(S);
    m(S union T) = min(m(S), m(T)); a row's result does not depend on other rows."""
    rng = np.random.Generator(np.random.PCG64(41))
    D, k = 1 << 24, 32
    for family in (F2_31, F4_31, F2_61):
        c = rng.integers(0, W.family_prime(family), size=(k, W.family_degree(family)), dtype=np.uint64)
        S = sorted(set(int(x) for x in rng.integers(0, D, size=300)))
        T = sorted(set(int(x) for x in rng.integers(0, D, size=200)))
        U = sorted(set(S) | set(T))
        shuffled = [S[i] for i in rng.permutation(len(S))]
        dup = shuffled + shuffled[:50]
        rp, col = _csr([S, T, U, shuffled, dup, S[:100]])
        m = o.minima(rp, col, D, k, family, c)
        assert np.array_equal(m[3], m[0]) and np.array_equal(m[4], m[0])
        assert np.array_equal(m[2], np.minimum(m[0], m[1]))
        assert np.all(m[0] <= m[5])
        alone = o.minima(*_csr([T]), D, k, family, c)
        assert np.array_equal(alone[0], m[1])


# ---------------------------------------------------------------- statistics
def _theorem1_pb(D, f1, f2, R, b):
    """P_b = C1 + (1 - C2) R with the C and A expressions given with Theorem 1."""
    r1, r2 = f1 / D, f2 / D
    A1 = r1 * (1 - r1) ** (2 ** b - 1) / (1 - (1 - r1) ** (2 ** b))
    A2 = r2 * (1 - r2) ** (2 ** b - 1) / (1 - (1 - r2) ** (2 ** b))
    C1 = A1 * r2 / (r1 + r2) + A2 * r1 / (r1 + r2)
    C2 = A1 * r1 / (r1 + r2) + A2 * r2 / (r1 + r2)
    return C1 + (1 - C2) * R


def pin_collision_probability_permutations(o, n_pairs=60, k=300):
    """Section 1.1 eq. (1): with independent uniformly random permutations the
    fraction of equal minima estimates R = |S1 n S2| / |S1 u S2|; Theorem 1 gives
    the fraction of equal b-bit values.  D = 2^14 keeps the tables small and makes
    r = |S|/D large enough (about 0.06) that the C terms of Theorem 1 matter."""
    from oracle import oracle as loader
    D, union = 1 << 14, 1500
    table = W.perm_table_np(D, k, seed=5151)
    for shared in (150, 750, 1350):
        R = shared / union
        rp, col, f1, f2 = W.planted_pairs(n_pairs, D, union, shared, seed=6000 + shared)
        m = o.minima(rp, col, D, k, FPERM, table)
        n = n_pairs * k
        got = float(np.mean(m[0::2] == m[1::2]))
        tol = 4.5 * math.sqrt(R * (1 - R) / n)
        assert abs(got - R) <= tol, (shared, got, R, tol)
        for b in (1, 2, 4):
            u = loader.unpack(o.signatures(rp, col, D, k, b, FPERM, table), k, b)
            gb = float(np.mean(u[0::2] == u[1::2]))
            pb = _theorem1_pb(D, f1, f2, R, b)
            tolb = 4.5 * math.sqrt(pb * (1 - pb) / n) + 2e-3      # Theorem 1 assumes large D
            assert abs(gb - pb) <= tolb, (shared, b, gb, pb, tolb)


def pin_collision_probability_hashes(o, n_pairs=40, k=200):
    """Same identity for the 2U / 4U families at D = 2^24 on sparse sets, where the
    paper's appendix finds 2U indistinguishable from true permutations; an absolute
    slack of 0.01 allows for the families being only approximately min-wise
    independent.  For sparse sets P_b is close to 2^-b + (1 - 2^-b) R."""
    from oracle import oracle as loader
    D, union = 1 << 24, 1000
    for family in (F2_31, F4_31, F2_61):
        c = W.coefficients(k, family, seed=7000 + family)
        for shared in (100, 500, 900):
            R = shared / union
            rp, col, f1, f2 = W.planted_pairs(n_pairs, D, union, shared, seed=8000 + shared)
            m = o.minima(rp, col, D, k, family, c)
            n = n_pairs * k
            got = float(np.mean(m[0::2] == m[1::2]))
            tol = 4.5 * math.sqrt(R * (1 - R) / n) + 0.01
            assert abs(got - R) <= tol, (family, shared, got, R)
            for b in (1, 4):
                u = loader.unpack(o.signatures(rp, col, D, k, b, family, c), k, b)
                gb = float(np.mean(u[0::2] == u[1::2]))
                pb = _theorem1_pb(D, f1, f2, R, b)
                assert abs(pb - (2.0 ** -b + (1 - 2.0 ** -b) * R)) < 1e-3
                tolb = 4.5 * math.sqrt(pb * (1 - pb) / n) + 0.01
                assert abs(gb - pb) <= tolb, (family, shared, b, gb, pb)


# ---------------------------------------------------------------- consumers of the signature
def pin_expansion_has_k_ones_and_inner_product_counts_matches(o):
    """Section 1.1: a signature expands into a 2^b x k vector with exactly k ones,
    and P_b-hat is the inner product of two such vectors divided by k.  The j-th
    one lies in block j; the inner product of two expansions (size of the
    intersection of the index sets) is the number of equal b-bit values, which is
    also counted here with NumPy on the unpacked fields."""
    from oracle import oracle as loader
    rng = np.random.Generator(np.random.PCG64(61))
    for k, b in ((500, 8), (77, 3), (13, 1), (64, 16), (9, 12), (4, 30)):
        m = rng.integers(0, 1 << 32, size=(12, k), dtype=np.uint64).astype(np.uint32)
        m[1] = m[0]
        m[2, : k // 2] = m[0, : k // 2]
        sig = o.pack(m, b, out_stride=(k * b + 7) // 8 + 2)
        fields = loader.unpack(sig, k, b)
        idx = o.expand(sig, k, b)
        assert idx.shape == (12, k)
        block = (np.arange(k, dtype=np.uint64) << np.uint64(b))
        assert np.array_equal(idx.astype(np.uint64), block[None, :] + fields.astype(np.uint64))
        pairs = np.array([[0, 1], [0, 2], [3, 4], [5, 5], [11, 0]], dtype=np.int64)
        counts = o.match_counts(sig, k, b, pairs)
        for q, (r1, r2) in enumerate(pairs):
            assert counts[q] == len(set(idx[r1].tolist()) & set(idx[r2].tolist()))
            assert counts[q] == int((fields[r1] == fields[r2]).sum())
        assert counts[0] == k and counts[3] == k and counts[1] >= k // 2


def pin_estimator_closed_forms(o):
    """eq. eqn_R_b with Theorem 1's terms.  Equal densities r1 = r2 = r give C1 = C2 = A,
    so R-hat = (P - A)/(1 - A); for b = 1, A = (1-r)/(2-r): with r = 1/2, A = 1/3, and
    P = 2/3 gives exactly 1/2.  P = 1 gives 1 for any equal densities.  For very sparse
    sets A tends to 2^-b, and for b = 32 the estimator is P-hat itself."""
    r = o.resemblance(np.array([2], dtype=np.uint32), [8], [8], 16, 3, 1)
    assert abs(r[0] - 0.5) < 1e-15
    for b in (1, 2, 4, 8, 16):
        r = o.resemblance(np.array([500, 250], dtype=np.uint32), [3000, 3000], [3000, 3000], 1 << 24, 500, b)
        assert abs(r[0] - 1.0) < 1e-12
        a = 2.0 ** -b
        assert abs(r[1] - (0.5 - a) / (1 - a)) < 1e-3
    r = o.resemblance(np.array([123], dtype=np.uint32), [4000], [900], 1 << 30, 500, 32)
    assert abs(r[0] - 123 / 500) < 1e-9


def pin_estimator_is_unbiased_for_unequal_set_sizes(o, n_pairs=150, k=400):
    """Nested sets of very different density (r1 = 0.05, r2 = 0.49, R = 0.1) under true
    random permutations: the mean of R_b-hat must sit on R.  With densities this
    unequal C1 and C2 differ by more than 0.1, so exchanging them, or the roles of
    r1 and r2, shifts the mean far outside the tolerance."""
    D, f1, f2 = 1 << 12, 200, 2000
    table = W.perm_table_np(D, k, seed=6262)
    rp, col, g1, g2 = W.planted_pairs(n_pairs, D, union=f2, shared=f1, seed=6363, only1=0)
    assert (g1, g2) == (f1, f2)
    pairs = np.arange(2 * n_pairs, dtype=np.int64).reshape(-1, 2)
    for b in (1, 2, 4):
        sig = o.signatures(rp, col, D, k, b, FPERM, table)
        counts = o.match_counts(sig, k, b, pairs)
        est = o.resemblance(counts, np.full(n_pairs, f1), np.full(n_pairs, f2), D, k, b)
        mean, sd = float(est.mean()), float(est.std(ddof=1))
        tol = 4.5 * sd / math.sqrt(n_pairs) + 3e-3            # Theorem 1 assumes large D
        assert abs(mean - f1 / f2) <= tol, (b, mean, tol)


# ---------------------------------------------------------------- packed index rows
def _bits_of_words(words):
    """The little-endian bit string of a word array, as a Python int (bit q of word j is bit 32 j + q)."""
    v = 0
    for j, x in enumerate(words):
        v |= int(x) << (32 * j)
    return v


def pin_packed_rows_by_hand(o):
    """The tile form of a row, written out by hand: first index as it is, then the differences
    inside the tile at the bit length of the widest one, LSB-first."""
    # differences 2, 0, 13: widest 13 -> 4 bits; fields 0x2, 0x0, 0xD from bit 0 of the second word
    width, word_ptr, words = o.pack_indices(np.array([0, 4]), np.array([5, 7, 7, 20], dtype=np.uint32))
    assert width.tolist() == [4] and word_ptr.tolist() == [0, 2] and words.tolist() == [5, 0xD02]
    # two rows; the second has one index (no differences: width 0, one word)
    width, word_ptr, words = o.pack_indices(np.array([0, 3, 4]), np.array([1, 2, 4, 9], dtype=np.uint32))
    assert width.tolist() == [2, 0] and word_ptr.tolist() == [0, 2, 3] and words.tolist() == [1, 0b1001, 9]
    # an empty row takes no words; equal indices give width 0
    width, word_ptr, words = o.pack_indices(np.array([0, 0, 3]), np.array([6, 6, 6], dtype=np.uint32))
    assert width.tolist() == [0, 0] and word_ptr.tolist() == [0, 0, 1] and words.tolist() == [6]
    # full width: difference 2^32 - 1
    width, word_ptr, words = o.pack_indices(np.array([0, 2]), np.array([0, 0xFFFFFFFF], dtype=np.uint32))
    assert width.tolist() == [32] and words.tolist() == [0, 0xFFFFFFFF]
    # 11 fields of 3 bits straddle the first word boundary: 33 bits -> two words after the first index
    idx = np.cumsum(np.array([10, 7, 1, 2, 3, 4, 5, 6, 7, 0, 1, 5], dtype=np.uint32)).astype(np.uint32)
    width, word_ptr, words = o.pack_indices(np.array([0, 12]), idx)
    assert width.tolist() == [3] and word_ptr.tolist() == [0, 3] and int(words[0]) == 10
    want = 0
    for i, d in enumerate([7, 1, 2, 3, 4, 5, 6, 7, 0, 1, 5]):
        want |= d << (3 * i)
    assert _bits_of_words(words[1:]) == want
    assert o.unpack_indices(np.array([0, 12]), width, word_ptr, words).tolist() == idx.tolist()


def pin_packed_rows_tiles_are_independent(o):
    """A row of 600 indices is three tiles (256, 256, 88).  The jump between two tiles is stored
    nowhere (each tile starts with its first index as it is) and does not widen the fields; every
    tile can be read without the others."""
    steps = np.ones(600, dtype=np.int64)
    steps[0] = 1000
    steps[256] = 5_000_000          # between tile 0 and tile 1: not a difference inside a tile
    steps[300] = 9                  # the widest difference inside a tile: 4 bits
    idx = np.cumsum(steps).astype(np.uint32)
    rp = np.array([0, 600])
    width, word_ptr, words = o.pack_indices(rp, idx)
    assert width.tolist() == [4]
    per_full = 1 + (255 * 4 + 31) // 32
    assert word_ptr.tolist() == [0, 2 * per_full + 1 + (87 * 4 + 31) // 32]
    for t, first in enumerate((0, 256, 512)):
        assert int(words[t * per_full]) == int(idx[first])
    # reading tile 1 alone, by the definition: first index plus running sum of 4-bit fields
    bits = _bits_of_words(words[per_full + 1: 2 * per_full])
    got = [int(words[per_full])]
    for i in range(255):
        got.append(got[-1] + ((bits >> (4 * i)) & 15))
    assert got == idx[256:512].tolist()
    assert o.unpack_indices(rp, width, word_ptr, words).tolist() == idx.tolist()


def pin_packed_rows_round_trip(o):
    """Unpacking what was packed gives the rows back, for rows of every length around the tile size
    and gaps of every magnitude; a tile never takes more words than it has indices."""
    rng = np.random.Generator(np.random.PCG64(515))
    lens = [0, 1, 2, 3, 255, 256, 257, 511, 512, 513, 1000, 0, 5, 2049]
    rows = []
    for n in lens:
        top = int(rng.choice([4, 1 << 8, 1 << 16, 1 << 24, (1 << 32) - 1]))
        gaps = rng.integers(0, max(top // max(n, 1), 1) + 1, size=n, dtype=np.uint64)
        rows.append(np.minimum(np.cumsum(gaps), (1 << 32) - 1).astype(np.uint32))
    rp = W.row_ptr_from_nnz(np.array(lens, dtype=np.int64))
    col = np.concatenate(rows) if rows else np.zeros(0, np.uint32)
    width, word_ptr, words = o.pack_indices(rp, col)
    assert int(word_ptr[-1]) == words.shape[0] <= col.shape[0]
    assert np.all(np.diff(word_ptr) >= 0) and np.all(width <= 32)
    for r, n in enumerate(lens):
        assert (word_ptr[r + 1] - word_ptr[r] == 0) == (n == 0)
    assert np.array_equal(o.unpack_indices(rp, width, word_ptr, words), col)
    # a row that is not sorted is refused
    try:
        o.pack_indices(np.array([0, 3]), np.array([5, 4, 6], dtype=np.uint32))
    except ValueError:
        pass
    else:
        raise AssertionError("an unsorted row was packed")


FAST_PINS = [
    pin_explicit_permutations_all_subsets,
    pin_explicit_permutations_random_sets,
    pin_identity_permutation_gives_set_minimum,
    pin_constant_hash,
    pin_identity_hash_gives_set_minimum,
    pin_monomials_via_python_pow,
    pin_modular_inverse_identities,
    pin_fermat_and_negation,
    pin_small_coefficients_no_wrap,
    pin_4u_with_zero_high_terms_is_2u,
    pin_big_integer_cross_check,
    pin_multiply_shift_against_numpy_uint32,
    pin_multiply_shift_is_a_bijection_of_the_universe,
    pin_ranges_and_empty_rows,
    pin_lowest_bits_example,
    pin_bit_layout_by_hand,
    pin_pack_roundtrip_all_b,
    pin_signatures_equal_pack_of_minima,
    pin_min_invariants,
    pin_expansion_has_k_ones_and_inner_product_counts_matches,
    pin_estimator_closed_forms,
    pin_estimator_is_unbiased_for_unequal_set_sizes,
    pin_packed_rows_by_hand,
    pin_packed_rows_tiles_are_independent,
    pin_packed_rows_round_trip,
]
STAT_PINS = [pin_collision_probability_permutations, pin_collision_probability_hashes]
ALL_PINS = FAST_PINS + STAT_PINS
