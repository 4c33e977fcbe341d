/*
 * CPU oracle for b-bit minwise-hash signatures.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the checker that the GPU library is compared against.  It is
 * deliberately plain, single-threaded and slow, shares no code, header, table
 * or trick with the GPU path, and must never be called from the product path.
 *
 * What it computes is the definition itself, written out:
 *
 *   - a data vector is a set S of nonzero feature indices in {0..D-1}
 *     (Section 1.1);
 *   - the j-th hashed value of S is the minimum, over the nonzero locations t
 *     of S, of the mapped location h_j(t) (Section 2, last paragraph);
 *   - h_j is the 2-universal hash  ((a1 + a2 t) mod p) mod D  (Section 2,
 *     eq. "eqn_h_2U"), the 4-universal hash
 *     ((a1 + a2 t + a3 t^2 + a4 t^3) mod p) mod D  (eq. "eqn_h_4U"), or the j-th
 *     column of an explicit "fully random permutation matrix" of size D x k
 *     (Section 1.5);
 *   - or h_j is the multiply-shift form  ((a1 + a2 t) mod 2^32) mod 2^s  with
 *     D = 2^s and a2 odd (Section 3.3, eq. "eqn_h_s"), which is what the paper
 *     times as "2U".  The paper prints "mod 2^s" (the lowest s bits) while citing
 *     a scheme that keeps the highest s bits of the 32-bit value; both are here,
 *     as two families;
 *   - only the lowest b bits of every minimum are kept (Section 1.1), and a
 *     data vector becomes k b-bit integers (Section 1.1, after eq. "eqn_R_b").
 *
 * The file also holds the three consumers of a signature that Section 1.1
 * defines: the 2^b x k expansion, the count of equal b-bit values of two rows
 * (k times P_b-hat), and the estimator R_b-hat of eq. "eqn_R_b" with Theorem 1's
 * C terms.
 *
 * Readings where the paper is silent (all stated in the repository's design
 * notes): coefficients are 0-based here, c[j][i] multiplies t^i; the whole
 * polynomial is reduced mod p before mod D; the minimum of an empty set is
 * 0xFFFFFFFF; value j occupies bits [j*b, (j+1)*b) of the row's bit string,
 * bit q of the string being bit (q mod 8) of byte (q div 8); pad bits are 0.
 *
 * Arithmetic: unsigned __int128 and the % operator.  No Mersenne folding, no
 * power-of-two shortcut for mod D.  The cubic is reduced term by term only to
 * stay inside 128 bits, which is legal because reduction mod p is a ring
 * homomorphism.
 *
 * Pins: tests/test_oracle_pins.py (closed forms, explicit permutations on tiny
 * D, modular-inverse and power identities through Python's big integers, the
 * collision identity of Section 1.1 eq. (1) and Theorem 1 on planted pairs,
 * the truncation example, union/subset/order invariants).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

typedef unsigned __int128 u128;

enum {
    ORACLE_2U_M31 = 0,
    ORACLE_4U_M31 = 1,
    ORACLE_2U_M61 = 2,
    ORACLE_4U_M61 = 3,
    ORACLE_PERM = 4,
    ORACLE_2U_MS32 = 5,        /* multiply-shift 2U, lowest s bits  */
    ORACLE_2U_MS32_HIGH = 6    /* multiply-shift 2U, highest s bits */
};

#define ORACLE_EMPTY_MIN 0xFFFFFFFFu

static int family_prime_degree(int family, uint64_t *p, int *deg)
{
    switch (family) {
    case ORACLE_2U_M31: *p = 2147483647ull; *deg = 2; return 0;
    case ORACLE_4U_M31: *p = 2147483647ull; *deg = 4; return 0;
    case ORACLE_2U_M61: *p = 2305843009213693951ull; *deg = 2; return 0;
    case ORACLE_4U_M61: *p = 2305843009213693951ull; *deg = 4; return 0;
    default: return -1;
    }
}

/* (c[0] + c[1] t + ... + c[deg-1] t^(deg-1)) mod p, then mod D.
 * Section 2, eqs. "eqn_h_2U" and "eqn_h_4U". */
static uint64_t hash_location(const uint64_t *c, int deg, uint64_t p, uint64_t D, uint64_t t)
{
    u128 acc = 0;
    u128 power = 1;              /* t^i mod p */
    for (int i = 0; i < deg; ++i) {
        u128 term = ((u128)(c[i] % p) * power) % p;
        acc = (acc + term) % p;
        if (i + 1 < deg) power = (power * (u128)(t % p)) % p;
    }
    return (uint64_t)(acc % (u128)D);
}

/* Section 3.3, eq. "eqn_h_s": ((c[0] + c[1] t) mod 2^32) mod 2^s with D = 2^s.
 * high != 0 keeps the s highest bits of the 32-bit value instead of the s lowest. */
static uint64_t hash_multiply_shift(const uint64_t *c, uint64_t D, uint64_t t, int high)
{
    u128 two32 = (u128)1 << 32;
    u128 v = ((u128)c[0] + (u128)c[1] * (u128)t) % two32;
    if (!high) return (uint64_t)(v % (u128)D);
    return (uint64_t)(v / (two32 / (u128)D));
}

/*
 * Full (untruncated) minima: minima[i*k + j] = min over t in row i of h_j(t),
 * or 0xFFFFFFFF for an empty row.  Host pointers throughout.
 * Returns 0, or a negative code for arguments it cannot interpret.
 */
int minhash_minima_oracle(const int64_t *row_ptr, const uint32_t *col_idx, int64_t n_rows,
                          uint64_t D, int32_t k, int32_t family, const void *params,
                          int64_t perm_ld, uint32_t *minima)
{
    if (n_rows < 0 || k < 1 || D < 1 || D > (1ull << 32)) return -1;
    if (n_rows == 0) return 0;
    if (!row_ptr || !params || !minima) return -1;

    uint64_t p = 0;
    int deg = 0;
    int multiply_shift = (family == ORACLE_2U_MS32 || family == ORACLE_2U_MS32_HIGH);
    if (family == ORACLE_PERM) {
        if (perm_ld < k) return -5;
    } else if (multiply_shift) {
        if ((D & (D - 1)) != 0) return -3;                 /* D = 2^s */
        if (family == ORACLE_2U_MS32_HIGH && D < 2) return -3;
    } else {
        if (family_prime_degree(family, &p, &deg) != 0) return -2;
        if (D >= p) return -3;
    }

    for (int64_t i = 0; i < n_rows; ++i) {
        int64_t lo = row_ptr[i], hi = row_ptr[i + 1];
        for (int32_t j = 0; j < k; ++j) {
            uint64_t m = ORACLE_EMPTY_MIN;
            for (int64_t e = lo; e < hi; ++e) {
                uint64_t t = col_idx[e];
                uint64_t v;
                if (family == ORACLE_PERM) {
                    const uint32_t *table = (const uint32_t *)params;
                    v = table[(size_t)t * (size_t)perm_ld + (size_t)j];
                } else if (multiply_shift) {
                    const uint64_t *coeffs = (const uint64_t *)params;
                    v = hash_multiply_shift(coeffs + (size_t)j * 2, D, t, family == ORACLE_2U_MS32_HIGH);
                } else {
                    const uint64_t *coeffs = (const uint64_t *)params;
                    v = hash_location(coeffs + (size_t)j * (size_t)deg, deg, p, D, t);
                }
                if (v < m) m = v;
            }
            minima[(size_t)i * (size_t)k + (size_t)j] = (uint32_t)m;
        }
    }
    return 0;
}

/*
 * Keep the lowest b bits of each of the k values and lay them out as one bit
 * string per row, one bit at a time.  out rows are out_stride bytes apart and
 * are cleared first, so pad bits and pad bytes are 0.
 */
int minhash_pack_oracle(const uint32_t *minima, int64_t n_rows, int32_t k, int32_t b,
                        uint8_t *out, int64_t out_stride)
{
    if (n_rows < 0 || k < 1 || b < 1 || b > 32) return -4;
    int64_t sig_bytes = ((int64_t)k * b + 7) / 8;
    if (out_stride < sig_bytes) return -5;
    if (n_rows == 0) return 0;
    if (!minima || !out) return -1;
    for (int64_t i = 0; i < n_rows; ++i) {
        uint8_t *row = out + (size_t)i * (size_t)out_stride;
        memset(row, 0, (size_t)out_stride);
        for (int32_t j = 0; j < k; ++j) {
            uint32_t z = minima[(size_t)i * (size_t)k + (size_t)j];
            for (int32_t bit = 0; bit < b; ++bit) {
                if ((z >> bit) & 1u) {
                    int64_t q = (int64_t)j * b + bit;
                    row[q / 8] |= (uint8_t)(1u << (q % 8));
                }
            }
        }
    }
    return 0;
}

/*
 * Same argument list as the GPU library's entry point, minus workspace,
 * stream and flags, with host pointers.  scratch holds n_rows*k uint32.
 */
int minhash_signatures_oracle(const int64_t *row_ptr, const uint32_t *col_idx, int64_t n_rows,
                              uint64_t D, int32_t k, int32_t b, int32_t family,
                              const void *params, int64_t perm_ld,
                              uint8_t *out, int64_t out_stride, uint32_t *scratch)
{
    if (b < 1 || b > 32 || k < 1) return -4;
    int rc = minhash_minima_oracle(row_ptr, col_idx, n_rows, D, k, family, params, perm_ld, scratch);
    if (rc != 0) return rc;
    return minhash_pack_oracle(scratch, n_rows, k, b, out, out_stride);
}

/* ======================================================================
 * Consumers of the signature (Section 1.1, Theorem 1 and eq. "eqn_R_b").
 * ====================================================================== */

/* value j of a packed row: bits [j*b, (j+1)*b) of the little-endian bit string, read one bit at a time */
static uint32_t packed_field(const uint8_t *row, int32_t j, int32_t b)
{
    uint32_t v = 0;
    for (int32_t bit = 0; bit < b; ++bit) {
        int64_t q = (int64_t)j * b + bit;
        if ((row[q / 8] >> (q % 8)) & 1u) v |= (1u << bit);
    }
    return v;
}

/*
 * Expansion into the 2^b x k-length binary vector with exactly k ones (Section
 * 1.1, paragraph after eq. "eqn_R_b"): the j-th one of row i sits at position
 * j*2^b + s_ij.  out[i*k + j] is that position.  Needs k*2^b <= 2^32.
 */
int minhash_expand_oracle(const uint8_t *sig, int64_t n_rows, int64_t sig_stride, int32_t k, int32_t b,
                          uint32_t *out)
{
    if (n_rows < 0 || k < 1 || b < 1 || b > 32) return -4;
    if (((unsigned __int128)k << b) > ((unsigned __int128)1 << 32)) return -4;
    if (sig_stride < ((int64_t)k * b + 7) / 8) return -5;
    if (n_rows == 0) return 0;
    if (!sig || !out) return -1;
    for (int64_t i = 0; i < n_rows; ++i)
        for (int32_t j = 0; j < k; ++j)
            out[(size_t)i * (size_t)k + (size_t)j] =
                (uint32_t)(((uint64_t)j << b) + packed_field(sig + (size_t)i * (size_t)sig_stride, j, b));
    return 0;
}

/*
 * k * P_b-hat of eq. "eqn_R_b": for every listed pair of rows the number of j
 * with equal b-bit values.  pairs holds 2*n_pairs row numbers.
 */
int minhash_match_counts_oracle(const uint8_t *sig, int64_t n_rows, int64_t sig_stride, int32_t k, int32_t b,
                                const int64_t *pairs, int64_t n_pairs, uint32_t *counts)
{
    if (n_rows < 0 || n_pairs < 0 || k < 1 || b < 1 || b > 32) return -4;
    if (sig_stride < ((int64_t)k * b + 7) / 8) return -5;
    if (n_pairs == 0) return 0;
    if (!sig || !pairs || !counts) return -1;
    for (int64_t q = 0; q < n_pairs; ++q) {
        int64_t r1 = pairs[2 * q], r2 = pairs[2 * q + 1];
        if (r1 < 0 || r1 >= n_rows || r2 < 0 || r2 >= n_rows) return -1;
        uint32_t c = 0;
        for (int32_t j = 0; j < k; ++j)
            if (packed_field(sig + (size_t)r1 * (size_t)sig_stride, j, b) ==
                packed_field(sig + (size_t)r2 * (size_t)sig_stride, j, b)) ++c;
        counts[q] = c;
    }
    return 0;
}

/*
 * R_b-hat = (P_b-hat - C_{1,b}) / (1 - C_{2,b})  (eq. "eqn_R_b"), with the C and A
 * terms given with Theorem 1:  r = f/D,  A = r (1-r)^(2^b - 1) / (1 - (1-r)^(2^b)),
 * C1 = A1 r2/(r1+r2) + A2 r1/(r1+r2),  C2 = A1 r1/(r1+r2) + A2 r2/(r1+r2).
 * f1, f2 are the sizes of the two sets (both >= 1).  Double precision.
 */
static double theorem1_A(double r, int32_t b)
{
    double n = ldexp(1.0, b);                     /* 2^b */
    return r * pow(1.0 - r, n - 1.0) / (1.0 - pow(1.0 - r, n));
}
int minhash_resemblance_oracle(const uint32_t *counts, const int64_t *f1, const int64_t *f2, int64_t n_pairs,
                               uint64_t D, int32_t k, int32_t b, double *r_hat)
{
    if (n_pairs < 0 || k < 1 || b < 1 || b > 32 || D < 1) return -4;
    if (n_pairs == 0) return 0;
    if (!counts || !f1 || !f2 || !r_hat) return -1;
    for (int64_t q = 0; q < n_pairs; ++q) {
        double r1 = (double)f1[q] / (double)D, r2 = (double)f2[q] / (double)D;
        double A1 = theorem1_A(r1, b), A2 = theorem1_A(r2, b);
        double C1 = A1 * r2 / (r1 + r2) + A2 * r1 / (r1 + r2);
        double C2 = A1 * r1 / (r1 + r2) + A2 * r2 / (r1 + r2);
        double P = (double)counts[q] / (double)k;
        r_hat[q] = (P - C1) / (1.0 - C2);
    }
    return 0;
}

/* ------------------------------------------------------------------ packed index rows
 * Not from the paper: the GPU library can take sorted rows over the host link as
 * tiles of differences (its answer to Section 3.6's finding that moving the data
 * dominates once hashing is fast).  The checker holds the plain definition of
 * that form, one bit at a time:
 *
 *   a row of n non-decreasing indices is cut into tiles of 256 (the last one
 *   shorter); a tile is one 32-bit word holding its first index, then the
 *   differences between neighbours inside the tile, w bits each, written
 *   LSB-first into 32-bit words, the last word padded with zeros; w is the bit
 *   length of the largest such difference of the row; word_ptr[r] is where row
 *   r's words start.
 *
 * Returns 0, -1 for bad arguments, -9 for a row that is not sorted, -6 when
 * `capacity` words do not suffice.
 */
int minhash_pack_indices_oracle(const int64_t *row_ptr, const uint32_t *col_idx, int64_t n_rows, uint32_t *width,
                                int64_t *word_ptr, uint32_t *words, int64_t capacity)
{
    if (!row_ptr || !word_ptr || n_rows < 0) return -1;
    int64_t at = 0;
    for (int64_t r = 0; r < n_rows; ++r) {
        const uint32_t *row = col_idx + row_ptr[r];
        const int64_t n = row_ptr[r + 1] - row_ptr[r];
        if (n < 0) return -1;
        /* the widest difference between neighbours that share a tile */
        uint32_t widest = 0;
        for (int64_t i = 1; i < n; ++i) {
            if (row[i] < row[i - 1]) return -9;
            if (i % 256 != 0 && row[i] - row[i - 1] > widest) widest = row[i] - row[i - 1];
        }
        uint32_t w = 0;
        while (w < 32 && (widest >> w) != 0) ++w;
        width[r] = w;
        word_ptr[r] = at;
        for (int64_t first = 0; first < n; first += 256) {
            const int64_t m = n - first < 256 ? n - first : 256;
            const int64_t n_words = 1 + ((m - 1) * (int64_t)w + 31) / 32;
            if (at + n_words > capacity) return -6;
            for (int64_t j = 0; j < n_words; ++j) words[at + j] = 0;
            words[at] = row[first];
            int64_t bit = 0;                         /* position in the bit string that starts at word 1 */
            for (int64_t i = 1; i < m; ++i) {
                const uint32_t d = row[first + i] - row[first + i - 1];
                for (uint32_t q = 0; q < w; ++q, ++bit)
                    if ((d >> q) & 1u) words[at + 1 + bit / 32] |= 1u << (bit % 32);
            }
            at += n_words;
        }
    }
    word_ptr[n_rows] = at;
    return 0;
}

/* The inverse: col_idx from the tiles.  Returns -6 if an offset leaves the `n_words` words given. */
int minhash_unpack_indices_oracle(const int64_t *row_ptr, const uint32_t *width, const int64_t *word_ptr,
                                  const uint32_t *words, int64_t n_words, int64_t n_rows, uint32_t *col_idx)
{
    if (!row_ptr || !word_ptr || n_rows < 0) return -1;
    for (int64_t r = 0; r < n_rows; ++r) {
        uint32_t *row = col_idx + row_ptr[r];
        const int64_t n = row_ptr[r + 1] - row_ptr[r];
        const uint32_t w = width[r];
        if (n < 0 || w > 32) return -1;
        int64_t at = word_ptr[r];
        for (int64_t first = 0; first < n; first += 256) {
            const int64_t m = n - first < 256 ? n - first : 256;
            const int64_t tile_words = 1 + ((m - 1) * (int64_t)w + 31) / 32;
            if (at < 0 || at + tile_words > n_words) return -6;
            uint32_t value = words[at];
            row[first] = value;
            int64_t bit = 0;
            for (int64_t i = 1; i < m; ++i) {
                uint32_t d = 0;
                for (uint32_t q = 0; q < w; ++q, ++bit)
                    if ((words[at + 1 + bit / 32] >> (bit % 32)) & 1u) d |= 1u << q;
                value += d;
                row[first + i] = value;
            }
            at += tile_words;
        }
    }
    return 0;
}
