// Exact integer arithmetic of the hash families, written for the gfx950 VALU.
//
// Everything here is unsigned integer work; results are bit-exact values of
//     h(t) = ((c0 + c1 t [+ c2 t^2 + c3 t^3]) mod p) mod D      (Section 2, eqs. eqn_h_2U, eqn_h_4U)
// for the Mersenne primes p = 2^31-1 and p = 2^61-1.  Section 3.4 replaces the
// modulo by shifts and masks because 2^31 = 1 (mod p): a value v = 2^31 S + y
// is congruent to S + y.  The same fact is used here, arranged so that one
// evaluation costs one 32x32->64 multiply-add plus a handful of half-cost
// integer instructions:
//
//   * The multiplicand is doubled when the nonzero is staged (2t instead of t),
//     so the 64-bit product is 2W and its two 32-bit halves are S = W >> 31 and
//     2 (W mod 2^31): the fold is one shift and one add, no funnel shift.
//   * The polynomial carries an offset of +1 (W = X + 1).  S + y then lies in
//     [1, 2^32) and X mod p is  S + y - 1  when S + y <= p  and  S + y - 2^31
//     otherwise, i.e.  (x + (x >> 31) - 1) & p  with x = S + y: the canonical
//     residue without a compare.  (Section 3.4's routine ends with the same
//     "subtract p if the folded value reached p" step; a non-canonical residue
//     p would give p mod D instead of 0.)
//   * For the cubic, t, t^2 mod p, t^3 mod p are computed once per nonzero while
//     staging, so the k functions need three multiply-adds each and a single
//     fold.  Coefficients and powers are re-centred to (-p/2, p/2) so that the
//     doubled sum of three products still fits 64 bits; a multiple of p added
//     to the constant term keeps it positive.
//
// The functions compile for the host as well, so that a CPU test can compare
// them with the % operator on edge values and random inputs.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define MH_HD __host__ __device__ __forceinline__
#else
#define MH_HD inline
#endif

namespace mh {

constexpr uint32_t P31 = 0x7FFFFFFFu;
constexpr uint64_t P61 = (1ull << 61) - 1;
constexpr uint32_t EMPTY_MIN = 0xFFFFFFFFu;   // minimum of an empty set

// ---------------------------------------------------------------- mod D
// D a power of two: and with D-1.  Otherwise r mod D for r < 2^31 through the
// exact quotient by an invariant divisor: with l = ceil(log2 D) and
// M = ceil(2^(31+l) / D) < 2^32, floor(r / D) = floor(r M / 2^(31+l)) for every
// r < 2^31 (M D = 2^(31+l) + e with 0 <= e < D <= 2^l, so r M / 2^(31+l) exceeds
// r / D by less than 1 / D).  One multiply-high, one shift by l - 1, one
// multiply-subtract; no correction step.
struct ModD {
    uint32_t D;      // low 32 bits of D (D = 2^32 only occurs with power-of-two paths)
    uint32_t mask;   // D - 1 when D is a power of two
    uint32_t M;      // ceil(2^(31+l) / D) for D >= 3 not a power of two
    uint32_t sh;     // l - 1
    uint32_t pow2;
    uint32_t M61q;   // floor(2^61 / D'), D' = D 2^j in (2^29, 2^32 / 3]: 61-bit residues mod D in 32-bit steps (0: not served)
    uint64_t M64;    // floor((2^64 - 1) / D): 61-bit residues mod D, see reduce61_mod_d
};
static_assert(sizeof(ModD) == 32, "the new word takes the place of padding: kernel arguments keep their offsets");

// D 2^j, the multiple of D in (2^29, 2^30) for D below 2^29 (not a power of two), D itself above that
MH_HD uint32_t scaled_up_d(uint64_t D)                   // 3 <= D < 2^32
{
    const uint32_t d = (uint32_t)D;
    const int lz = __builtin_clz(d);
    return lz > 2 ? d << (lz - 2) : d;
}

MH_HD ModD make_mod_d(uint64_t D)
{
    ModD m;
    m.D = (uint32_t)D;
    m.pow2 = (D & (D - 1)) == 0 ? 1u : 0u;
    m.mask = (uint32_t)(D - 1);
    m.M = 0;
    m.sh = 0;
    m.M64 = ~0ull / D;
    m.M61q = 0;
    if (!m.pow2 && D >= 3 && 3 * D <= (1ull << 32)) m.M61q = (uint32_t)((1ull << 61) / scaled_up_d(D));
    if (!m.pow2 && D < (1ull << 31)) {       // the exact-quotient path serves p = 2^31-1 only (D < p)
        uint32_t l = 0;
        while ((1ull << l) < D) ++l;         // l >= 2
        m.M = (uint32_t)(((1ull << (31 + l)) + D - 1) / D);
        m.sh = l - 1;
    }
    return m;
}

MH_HD uint32_t mulhi_u32(uint32_t a, uint32_t b) { return (uint32_t)(((uint64_t)a * b) >> 32); }

template <bool POW2>
MH_HD uint32_t reduce_mod_d(uint32_t r, const ModD& md)   // r < 2^31
{
    if (POW2) return r & md.mask;
    uint32_t q = mulhi_u32(r, md.M) >> md.sh;
    return r - q * md.D;
}

// Any D below 2^28 that is not a power of two: a key that orders residues r < 2^31 by
// r mod D without computing r mod D.  With l = ceil(log2 D), N = 32 + l and
// M = floor(2^N / D) = 2^32 + m_low (33 bits), P = r M + bias = r m_low + (r 2^32 + bias)
// is one multiply-add whose 64-bit addend carries r in its high word.  Then
// P / 2^N = r / D + b - e with b = bias / 2^N = 2^-(l+1) + 2^-30 and the shortfall
// e = r (2^N / D - M) / 2^N in [0, 2^-(l+1)), so the fraction of P / 2^N lies in
// (v / D + 2^-30, v / D + 2^-(l+1) + 2^-30] for v = r mod D, which is inside
// (v / D, (v + 1) / D) for l <= 28.  Its top 32 bits, bits [l, 32 + l) of P, are the
// key: keys of different v differ by more than 2^-(l+1) - 2^-32 in the same direction,
// and floor(key D / 2^32), one multiply-high per row, gives v back.
struct FracD {
    uint32_t m_low;   // floor(2^(32+l) / D) - 2^32
    uint32_t bias;    // 2^31 + 2^(l+2) < 2^32
    uint32_t l;       // ceil(log2 D), 2..28
};
MH_HD bool frac_key_serves(uint64_t D) { return D >= 3 && D < (1ull << 28) && (D & (D - 1)) != 0; }
MH_HD FracD make_frac_d(uint64_t D)
{
    FracD f;
    f.l = 0;
    while ((1ull << f.l) < D) ++f.l;
    f.m_low = (uint32_t)((1ull << (32 + f.l)) / D);      // the quotient lies in (2^32, 2^33): its low word
    f.bias = (1u << 31) + (1u << (f.l + 2));
    return f;
}
MH_HD uint32_t frac_key(uint32_t r, const FracD& f)      // r < 2^31
{
    const uint64_t P = (uint64_t)r * f.m_low + (((uint64_t)r << 32) | f.bias);
    return (uint32_t)(P >> f.l);
}
MH_HD uint32_t finish_frac_key(uint32_t key, uint32_t D) { return mulhi_u32(key, D); }

// D of at least p / 3 (and below p = 2^31-1): the quotient of a residue r < p by D is 0, 1
// or 2, so r mod D is the smallest of r, r - D and r - 2D as unsigned words: a difference
// that would be negative wraps to the true difference plus 2^32 - D or 2^32 - 2D, both
// positive, and so exceeds the one that is right.
MH_HD bool small_quotient_serves(uint64_t D) { return 3 * D >= (uint64_t)P31 && D < (uint64_t)P31 && (D & (D - 1)) != 0; }
MH_HD uint32_t reduce_small_quotient(uint32_t r, uint32_t D)      // r < p
{
    const uint32_t a = r - D, b = a - D;
    const uint32_t m = a < b ? a : b;
    return r < m ? r : m;
}

// r mod D for r < 2^61 and any D in [1, 2^32] (the p = 2^61-1 families with a D that
// the mask path cannot serve): q = floor(r M64 / 2^64) falls short of the true
// quotient by at most one, because r (2^64 / D - M64) < 2 r < 2^64 / 4; one
// conditional subtraction finishes it.
//
// D of at most 2^32 / 3 (not a power of two) needs no 64-bit quotient.  With D' = D 2^j in (2^29, 2^32 / 3]
// and M = floor(2^61 / D') < 2^32, q = floor(floor(r / 2^29) M / 2^32) is one multiply-high of 32-bit
// words.  Both factors are rounded down, so q <= floor(r / D'); and with a = r / 2^29, m = 2^61 / D' the
// rounded factors multiply to more than (a - 1)(m - 1) > a m - a - m, where (a + m) / 2^32 < r / 2^61 +
// 2^29 / D' < 2, and the floor loses less than one more: q >= floor(r / D') - 2.  So r - q D' lies in
// [0, 3 D'), fits 32 bits, and is computed in 32-bit words (the low word of r less the low word of q D');
// the smallest of it, it less D' and it less 2 D' as unsigned words is r mod D' (reduce_small_quotient).
// For j > 0 that value, below 2^30, is then taken modulo D by the exact quotient that serves p = 2^31-1.
MH_HD uint64_t mulhi_u64(uint64_t a, uint64_t b) { return (uint64_t)(((unsigned __int128)a * b) >> 64); }
MH_HD uint32_t reduce61_mod_d(uint64_t r, const ModD& md, uint64_t D)
{
    if (md.M61q) {
        const uint32_t dp = scaled_up_d(D);
        const uint32_t q = mulhi_u32((uint32_t)(r >> 29), md.M61q);
        uint32_t v = reduce_small_quotient((uint32_t)r - q * dp, dp);
        if (dp != (uint32_t)D) v = reduce_mod_d<false>(v, md);
        return v;
    }
    uint64_t q = mulhi_u64(r, md.M64);
    uint64_t v = r - q * D;
    return (uint32_t)(v >= D ? v - D : v);
}

// ---------------------------------------------------------------- p = 2^31 - 1, helpers for staging
MH_HD uint32_t m31_reduce64(uint64_t v)     // v < 2^64 -> canonical residue
{
    v = (v & P31) + (v >> 31);              // < 2^31 + 2^33
    v = (v & P31) + (v >> 31);              // < 2^31 + 8
    uint32_t r = (uint32_t)v;
    return r >= P31 ? r - P31 : r;
}
MH_HD uint32_t m31_mul(uint32_t a, uint32_t b) { return m31_reduce64((uint64_t)a * b); }

// centre a canonical residue into [-(p-1)/2, (p-1)/2]
MH_HD int32_t m31_centre(uint32_t r) { return r > (P31 >> 1) ? (int32_t)(r - P31) : (int32_t)r; }

// x = S + y in [1, 2^32) congruent to X + 1  ->  canonical X mod p
MH_HD uint32_t m31_finish(uint32_t x) { return (x + (x >> 31) - 1u) & P31; }

// ---------------------------------------------------------------- 2U, p = 2^31 - 1
struct Fn2U31 {
    uint32_t c1;     // linear coefficient
    uint64_t add;    // 2 (c0 + 1)
};
MH_HD Fn2U31 prep_2u31(uint64_t c0, uint64_t c1)
{
    Fn2U31 f;
    f.c1 = (uint32_t)c1;
    f.add = 2 * c0 + 2;
    return f;
}
MH_HD uint32_t stage_2u31(uint32_t t) { return t << 1; }      // t < D < 2^31

// x = S + y for the 2U polynomial
MH_HD uint32_t fold_2u31(const Fn2U31& f, uint32_t t2)
{
    // 2W = c1 (2t) + 2 (c0 + 1) < 2^63;  hi = W >> 31 < 2^31,  lo = 2 (W mod 2^31)
    uint64_t w2 = (uint64_t)f.c1 * t2 + f.add;
    return (uint32_t)(w2 >> 32) + ((uint32_t)w2 >> 1);
}

template <bool POW2>
MH_HD uint32_t hash_2u31(const Fn2U31& f, uint32_t t2, const ModD& md)
{
    return reduce_mod_d<POW2>(m31_finish(fold_2u31(f, t2)), md);
}

// Other D: without the +1 offset the folded value x = S + y lies in [0, 2p)
// (S = X >> 31 < D - 1 < p and y <= p), so the canonical residue is the unsigned
// minimum of x and x - p, and the exact quotient finishes it: one instruction
// fewer than m31_finish.
MH_HD Fn2U31 prep_2u31_raw(uint64_t c0, uint64_t c1)
{
    Fn2U31 f;
    f.c1 = (uint32_t)c1;
    f.add = 2 * c0;
    return f;
}
MH_HD uint32_t hash_2u31_raw(const Fn2U31& f, uint32_t t2, const ModD& md)
{
    uint32_t x = fold_2u31(f, t2);
    uint32_t y = x - P31;
    return reduce_mod_d<false>(y < x ? y : x, md);
}

// Power-of-two D = 2^s: the kernels evaluate the NEGATED polynomial.  With c1' = -c1
// mod p and the constant p - c0 in [1, p] the folded value x lies in [1, 2p] and is
// congruent to -X, so its representative in [1, p] is p - (X mod p), whose low s bits
// are the complement of the hashed location (2^31 - 1 - r = ~r modulo 2^s).  That
// representative is x for x <= p and x - p = x + 1 - 2^31 otherwise, i.e.
// x + (x >> 31) modulo 2^s.  Shifting left by 32 - s instead of masking keeps the
// order of the low s bits, and shift, add and shift fuse into a logical shift and one
// add-then-shift instruction.  The running MAXIMUM of these keys gives the minimum
// location: mask - (max >> (32 - s)).  For s = 0 the shift count is held at 31 and
// the final "& mask" clears the bit.  (4U uses this form when asked for keys that are
// formed evaluation by evaluation; otherwise see prep_2u31_full.)
MH_HD uint32_t neg_key_shift(uint32_t mask)          // 32 - s for mask = 2^s - 1, at most 31
{
    uint32_t s = 0;
    while (s < 32 && ((mask >> s) & 1u)) ++s;
    return s == 0 ? 31u : 32u - s;
}
MH_HD uint32_t m31_neg_key(uint32_t x, uint32_t shift) { return (x + (x >> 31)) << shift; }

// 2U, power-of-two D = 2^s, with the folded value as the key.  Multiplying by 2^j
// modulo p = 2^31-1 rotates a 31-bit residue left by j bits, so with both negated
// coefficients multiplied by 2^(31-s) the s wanted bits (the complement of the hashed
// location) are the top s bits of the representative in [1, p], and the 31-bit
// representative itself is an order-preserving key.  The folded x = hi + y is that
// representative whenever x <= p, i.e. whenever bit 31 of x is clear.  When it is set,
// the representative is x - p <= hi <= D - 1 (hi = V >> 31 with V < p D for t < D): a
// small value.
MH_HD uint32_t rotl31(uint32_t v, uint32_t j)        // v <= p, 0 <= j <= 31: v 2^j modulo p (p stays p)
{
    j %= 31u;
    return j ? ((v << j) | (v >> (31u - j))) & (uint32_t)P31 : v;
}
MH_HD uint32_t full_key_rotation(uint32_t mask)     // 31 - s for mask = 2^s - 1
{
    uint32_t s = 0;
    while (s < 32 && ((mask >> s) & 1u)) ++s;
    return 31u - s;
}
MH_HD Fn2U31 prep_2u31_full(uint64_t c0, uint64_t c1, uint32_t rotation)
{
    Fn2U31 f;
    f.c1 = rotl31(c1 ? (uint32_t)(P31 - c1) : 0u, rotation);
    f.add = 2 * (uint64_t)rotl31((uint32_t)((uint64_t)P31 - c0), rotation);
    return f;
}
// x itself, for callers that keep a signed and an unsigned running maximum of it
// (finish_full_keys, further down): nothing is ever doubtful then.
MH_HD int32_t key_full_2u31(const Fn2U31& f, uint32_t t2) { return (int32_t)fold_2u31(f, t2); }
// One running maximum is enough if x is doubled: 2x modulo 2^32 = 2 hi + lo (lo = 2y is
// even) is 2x exactly for x <= p, and for x > p it wraps to 2 (x - 2^31) =
// 2 (representative - 1) <= 2 (D - 2).  So an UNSIGNED running maximum of at least
// 2 (D - 1) ends on an evaluation with x <= p and is exact; a smaller one marks the
// value as doubtful, and it is then computed again exactly.  With n evaluations behind
// a value that happens with probability (D / 2^31)^n.  The doubled key can be formed
// with two simple instructions (hi + hi, + lo) or with one shift-then-add; the kernel
// uses one form for each nonzero of a pair, which balances its instruction classes.
MH_HD uint32_t key_full2_2u31(const Fn2U31& f, uint32_t t2)
{
    const uint64_t w2 = (uint64_t)f.c1 * t2 + f.add;
    return ((uint32_t)(w2 >> 32) << 1) + (uint32_t)w2;
}
MH_HD bool full2_key_doubtful(uint32_t key, uint32_t mask) { return key < 2u * mask; }                     // mask = D - 1 < 2^30
// one shift by rotation + 1 (rotation <= 31, and 31 only for D = 1, where the mask is 0 and the amount does not matter)
MH_HD uint32_t finish_full2_key(uint32_t key, uint32_t rotation, uint32_t mask) { return mask - ((key >> ((rotation + 1u) & 31u)) & mask); }
constexpr int32_t FULL_KEY_INIT = INT32_MIN;
MH_HD uint32_t finish_neg_key(uint32_t key, uint32_t shift, uint32_t mask) { return mask - ((key >> shift) & mask); }

// ---------------------------------------------------------------- 4U, p = 2^31 - 1
// K31 p is added to the constant term so that the centred sum stays positive:
// three products of magnitude at most ((p-1)/2)^2 need K31 p >= 3 ((p-1)/2)^2.
constexpr uint64_t H31 = (uint64_t)(P31 >> 1);                               // (p-1)/2 = 2^30 - 1
constexpr uint64_t K31 = (3 * H31 * H31 + (uint64_t)P31 - 1) / (uint64_t)P31;

struct Fn4U31 {
    int32_t c1, c2, c3;   // centred coefficients of t, t^2, t^3
    uint64_t add;         // 2 (c0 + 1 + K31 p)
};
MH_HD Fn4U31 prep_4u31(uint64_t c0, uint64_t c1, uint64_t c2, uint64_t c3)
{
    Fn4U31 f;
    f.c1 = m31_centre((uint32_t)c1);
    f.c2 = m31_centre((uint32_t)c2);
    f.c3 = m31_centre((uint32_t)c3);
    f.add = 2 * (c0 + 1 + K31 * (uint64_t)P31);
    return f;
}
struct Pow4U31 { int32_t t1, t2, t3; };   // 2 * centred (t, t^2 mod p, t^3 mod p)
MH_HD Pow4U31 stage_4u31(uint32_t t)      // t < D < p
{
    uint32_t s = m31_mul(t, t);
    uint32_t c = m31_mul(s, t);
    Pow4U31 w;
    w.t1 = 2 * m31_centre(t);
    w.t2 = 2 * m31_centre(s);
    w.t3 = 2 * m31_centre(c);
    return w;
}

MH_HD uint32_t fold_4u31(const Fn4U31& f, const Pow4U31& w)
{
    // 2W' = add + c1 t1 + c2 t2 + c3 t3, exact in two's complement, 0 < 2W' < 0.75 * 2^64
    // (each product fits int64; the running sum is kept unsigned so that wrapping is defined)
    uint64_t w2 = f.add;
    w2 += (uint64_t)((int64_t)f.c1 * w.t1);
    w2 += (uint64_t)((int64_t)f.c2 * w.t2);
    w2 += (uint64_t)((int64_t)f.c3 * w.t3);
    uint32_t hi = (uint32_t)(w2 >> 32), lo = (uint32_t)w2;
    // W' = 2^62 s1 + 2^31 s0 + y  ==  s1 + s0 + y  (mod p);  at most 2^32 - 2
    return (lo >> 1) + (hi & P31) + (hi >> 31);
}

template <bool POW2>
MH_HD uint32_t hash_4u31(const Fn4U31& f, const Pow4U31& w, const ModD& md)
{
    return reduce_mod_d<POW2>(m31_finish(fold_4u31(f, w)), md);
}
// Other D: x in [1, 2p] congruent to X + 1, so X mod p is the unsigned minimum of
// x - 1 and x - 1 - p = x - 2^31 (an xor with the sign bit).
MH_HD uint32_t hash_4u31_np2(const Fn4U31& f, const Pow4U31& w, const ModD& md)
{
    uint32_t x = fold_4u31(f, w);
    uint32_t a = x - 1u, b = x ^ 0x80000000u;
    return reduce_mod_d<false>(b < a ? b : a, md);
}
// Power-of-two D, negated cubic (see above neg_key_shift): the centred coefficients change
// sign (their range is symmetric) and the constant becomes p - c0 in [1, p], so the
// folded value is congruent to -X and lies in [1, 2^32 - 2] as before.
MH_HD Fn4U31 prep_4u31_neg(uint64_t c0, uint64_t c1, uint64_t c2, uint64_t c3)
{
    Fn4U31 f;
    f.c1 = -m31_centre((uint32_t)c1);
    f.c2 = -m31_centre((uint32_t)c2);
    f.c3 = -m31_centre((uint32_t)c3);
    f.add = 2 * (((uint64_t)P31 - c0) + K31 * (uint64_t)P31);
    return f;
}
MH_HD uint32_t key_neg_4u31(const Fn4U31& f, const Pow4U31& w, uint32_t shift) { return m31_neg_key(fold_4u31(f, w), shift); }

// 4U, power-of-two D, without any instruction after the fold and without a guard: the
// negated coefficients are multiplied by 2^(31-s) as in prep_2u31_full, so that the
// representative in [1, p] of the folded x is an order-preserving key.  Here x is
// spread over all of [1, 2p], so neither half can be dropped: the caller keeps two
// running maxima of x, one comparing signed words (it ends on the largest x <= p, if
// any) and one comparing unsigned words (it ends on the largest x > p, if any), and
// the largest representative is the larger of the first and the second minus p.
MH_HD Fn4U31 prep_4u31_full(uint64_t c0, uint64_t c1, uint64_t c2, uint64_t c3, uint32_t rotation)
{
    Fn4U31 f;
    f.c1 = -m31_centre(rotl31((uint32_t)c1, rotation));
    f.c2 = -m31_centre(rotl31((uint32_t)c2, rotation));
    f.c3 = -m31_centre(rotl31((uint32_t)c3, rotation));
    f.add = 2 * ((uint64_t)rotl31((uint32_t)((uint64_t)P31 - c0), rotation) + K31 * (uint64_t)P31);
    return f;
}
constexpr uint32_t FULL_KEY_INIT_UNSIGNED = 0u;
MH_HD uint32_t finish_full_keys(int32_t smax, uint32_t umax, uint32_t rotation, uint32_t mask)
{
    const uint32_t low = smax > 0 ? (uint32_t)smax : 0u;                          // largest x in [1, p]
    const uint32_t high = umax > (uint32_t)P31 ? umax - (uint32_t)P31 : 0u;       // largest x in (p, 2p], less p
    const uint32_t rep = low > high ? low : high;
    return mask - ((rep >> rotation) & mask);
}

// ---------------------------------------------------------------- 2U, p = 2^61 - 1
// W = c1 t + c0 + 1 with c1 = 2^32 e1 + e0, t < 2^31:
//   L = e0 t + (c0 + 1)            < 2^63 + 2^61
//   H = e1 t + (L >> 32)           < 2^62
//   W = 2^32 H + (L mod 2^32) = 2^61 (H >> 29) + [ (H mod 2^29) : L mod 2^32 ]
// and 2^61 = 1 (mod p), so x = y + (H >> 29) with y the 61-bit bracket; x lies in
// [1, 2^61 + 2^33) and X mod p is x - 1 if bit 61 of x is clear, x - 2^61 otherwise.
struct Fn2U61 {
    uint32_t e0, e1;   // c1 = 2^32 e1 + e0
    uint64_t add;      // c0 + 1
};
MH_HD Fn2U61 prep_2u61(uint64_t c0, uint64_t c1)
{
    Fn2U61 f;
    f.e0 = (uint32_t)c1;
    f.e1 = (uint32_t)(c1 >> 32);
    f.add = c0 + 1;
    return f;
}

// canonical residue (61 bits) for t < 2^31
MH_HD uint64_t residue_2u61(const Fn2U61& f, uint32_t t)
{
    uint64_t L = (uint64_t)f.e0 * t + f.add;
    uint64_t H = (uint64_t)f.e1 * t + (L >> 32);
    uint64_t y = ((H & 0x1FFFFFFFull) << 32) | (L & 0xFFFFFFFFull);
    uint64_t x = y + (H >> 29);
    uint64_t c = x >> 61;
    return (x + c - 1) & P61;
}

// low 32 bits of the canonical residue only (all that a power-of-two D needs), t < 2^31.
// Then H < 2^60 + 2^32, so H >> 29 fits 32 bits: x_lo = L_lo + (H >> 29) with carry c1,
// and bit 61 of x is set exactly when c1 = 1 and bits 32..60 of W are all ones.
MH_HD uint32_t residue_lo_2u61(const Fn2U61& f, uint32_t t)
{
    uint64_t L = (uint64_t)f.e0 * t + f.add;
    uint64_t H = (uint64_t)f.e1 * t + (L >> 32);
    uint32_t Hl = (uint32_t)H, Hh = (uint32_t)(H >> 32);
    uint32_t s_lo = (Hl >> 29) | (Hh << 3);          // H >> 29
    uint32_t x_lo = (uint32_t)L + s_lo;
    uint32_t c1 = x_lo < s_lo ? 1u : 0u;
    uint32_t c2 = ((Hl | 0xE0000000u) == 0xFFFFFFFFu) ? c1 : 0u;
    return x_lo + c2 - 1u;
}

// canonical residue for any t < 2^32 (D above 2^31 or not a power of two)
MH_HD uint64_t residue_wide_2u61(const Fn2U61& f, uint32_t t)
{
    uint64_t L0 = (uint64_t)f.e0 * t;
    uint64_t L = L0 + f.add;                               // may wrap once
    uint64_t carry = L < L0 ? 1ull : 0ull;
    uint64_t H = (uint64_t)f.e1 * t + (L >> 32) + (carry << 32);   // < 2^62
    uint64_t y = ((H & 0x1FFFFFFFull) << 32) | (L & 0xFFFFFFFFull);
    uint64_t x = y + (H >> 29);
    uint64_t c = x >> 61;
    return (x + c - 1) & P61;
}

// POW2 here also means D <= 2^31, so that t < 2^31
template <bool POW2>
MH_HD uint32_t hash_2u61(const Fn2U61& f, uint32_t t, const ModD& md, uint64_t D)
{
    if (POW2) return residue_lo_2u61(f, t) & md.mask;
    return reduce61_mod_d(residue_wide_2u61(f, t), md, D);
}

// Power-of-two D = 2^s <= 2^31, negated and rotated form with a guard (compare
// prep_2u31_full).  With c1' = -c1 mod p and the constant p - c0 in [1, p],
// V = c1' t + (p - c0) is congruent to -X, and its representative in [1, p] is
// p - (X mod p), whose low s bits are the complement of the hashed location.
// Multiplying by 2^j modulo p = 2^61-1 rotates a 61-bit residue left by j bits, so
// with both coefficients multiplied by 2^j, j = 32 - s, those s bits arrive at the top
// of the low 32-bit word of the representative: that word, with whatever lies below
// the s bits, is an order-preserving key as it stands.  The folded x = y + (H >> 29)
// lies in [1, 2^61 + 2^31 + 4), and as long as its bit 61 is clear it is that
// representative, so the key is L_lo + (H >> 29), one add, no carries, no shift.  When
// bit 61 is set, x = 2^61 + d with d < 2^31 + 4, the representative is x - p = d + 1,
// and the key comes out as d: one too small, and in any case below 2^31 + 5.  So an
// unsigned running maximum of at least GUARD61_FLOOR = 2^31 + 5 ends on an evaluation
// with bit 61 clear, is exact, and no evaluation with bit 61 set has a representative
// above it; a smaller maximum marks the value as doubtful, and it is then computed
// again with the exact path (hash_2u61).  With n evaluations behind a value that
// happens with probability about 2^-n.
MH_HD uint64_t rotl61(uint64_t v, uint32_t j)      // v <= p, 1 <= j <= 32: v 2^j modulo p (p stays p)
{
    return ((v << j) | (v >> (61u - j))) & P61;
}
MH_HD Fn2U61 prep_2u61_neg(uint64_t c0, uint64_t c1, uint32_t shift)   // shift = neg_key_shift(mask)
{
    const uint64_t n = rotl61(c1 ? P61 - c1 : 0, shift);
    Fn2U61 f;
    f.e0 = (uint32_t)n;
    f.e1 = (uint32_t)(n >> 32);
    f.add = rotl61(P61 - c0, shift);
    return f;
}
MH_HD uint32_t key_neg_2u61(const Fn2U61& f, uint32_t t)   // t < 2^31; the location is finish_neg_key(key, shift, mask)
{
    const uint64_t L = (uint64_t)f.e0 * t + f.add;
    const uint64_t H = (uint64_t)f.e1 * t + (L >> 32);
    return (uint32_t)L + (uint32_t)(H >> 29);
}
constexpr uint32_t GUARD61_FLOOR = 0x80000005u;

// ---------------------------------------------------------------- 4U, p = 2^61-1 (eq. eqn_4U with the prime of Section 3.4's last paragraph)
// Horner form: three steps acc <- acc t + c, each one 62-bit x 32-bit product
// built from two widening multiply-adds (the low word of the addend joins the low
// product, its high word the high product, so neither overflows 64 bits for any
// t < 2^32), followed by the 2^61 = 1 (mod p) fold of residue_2u61.  The fold is
// left partial between steps: acc stays below 2^61 + 2^34, which the next step
// accepts.  The last addend carries the +1 offset, so the final x lies in
// [1, 2^61 + 2^34) and the canonical residue is (x + (x >> 61) - 1) & p.
struct Fn4U61 {
    uint32_t c3lo, c3hi, c2lo, c2hi, c1lo, c1hi, a0lo, a0hi;   // a0 = c0 + 1 <= p
};
MH_HD Fn4U61 prep_4u61(uint64_t c0, uint64_t c1, uint64_t c2, uint64_t c3)
{
    Fn4U61 f;
    f.c3lo = (uint32_t)c3; f.c3hi = (uint32_t)(c3 >> 32);
    f.c2lo = (uint32_t)c2; f.c2hi = (uint32_t)(c2 >> 32);
    f.c1lo = (uint32_t)c1; f.c1hi = (uint32_t)(c1 >> 32);
    f.a0lo = (uint32_t)(c0 + 1); f.a0hi = (uint32_t)((c0 + 1) >> 32);
    return f;
}

// one Horner step on (lo, hi) words; hi < 2^30 on entry and on exit
MH_HD void horner_step_61(uint32_t& lo, uint32_t& hi, uint32_t t, uint32_t add_lo, uint32_t add_hi)
{
    uint64_t L = (uint64_t)lo * t + add_lo;                 // <= (2^32-1)^2 + 2^32 - 1 < 2^64
    uint64_t H = (uint64_t)hi * t + (L >> 32) + add_hi;     // < 2^62 + 2^33
    uint32_t Hl = (uint32_t)H, Hh = (uint32_t)(H >> 32);
    uint32_t s_lo = (Hl >> 29) | (Hh << 3);                 // (H >> 29) mod 2^32
    uint32_t s_hi = Hh >> 29;                               // (H >> 29) >> 32: 0..2
    uint32_t x_lo = (uint32_t)L + s_lo;
    uint32_t carry = x_lo < s_lo ? 1u : 0u;
    lo = x_lo;
    hi = (Hl & 0x1FFFFFFFu) + s_hi + carry;                 // < 2^29 + 4
}

// canonical residue (61 bits) for any t < 2^32
MH_HD uint64_t residue_4u61(const Fn4U61& f, uint32_t t)
{
    uint32_t lo = f.c3lo, hi = f.c3hi;
    horner_step_61(lo, hi, t, f.c2lo, f.c2hi);
    horner_step_61(lo, hi, t, f.c1lo, f.c1hi);
    horner_step_61(lo, hi, t, f.a0lo, f.a0hi);
    uint64_t x = ((uint64_t)hi << 32) | lo;
    return (x + (x >> 61) - 1) & P61;
}

// low 32 bits of the canonical residue (all that a power-of-two D <= 2^32 needs)
MH_HD uint32_t residue_lo_4u61(const Fn4U61& f, uint32_t t)
{
    uint32_t lo = f.c3lo, hi = f.c3hi;
    horner_step_61(lo, hi, t, f.c2lo, f.c2hi);
    horner_step_61(lo, hi, t, f.c1lo, f.c1hi);
    horner_step_61(lo, hi, t, f.a0lo, f.a0hi);
    return lo + (hi >> 29) - 1u;
}

template <bool POW2>
MH_HD uint32_t hash_4u61(const Fn4U61& f, uint32_t t, const ModD& md, uint64_t D)
{
    if (POW2) return residue_lo_4u61(f, t) & md.mask;
    return reduce61_mod_d(residue_4u61(f, t), md, D);
}

// ---------------------------------------------------------------- multiply-shift 2U (Section 3.3, eq. eqn_h_s)
// ((c0 + c1 t) mod 2^32) mod 2^s: the low word of one multiply-add, then a mask
// (lowest s bits, as the paper prints it) or a shift (highest s bits, the form of
// the scheme it cites).  The integer overflow does the "mod 2^32".
struct Fn2UMS32 {
    uint32_t c1;
    uint64_t add;    // c0, widened: the addend of the 64-bit multiply-add whose low word is used
};
MH_HD Fn2UMS32 prep_2ums32(uint64_t c0, uint64_t c1)
{
    Fn2UMS32 f;
    f.c1 = (uint32_t)c1;
    f.add = (uint64_t)(uint32_t)c0;
    return f;
}
template <bool HIGH>
MH_HD uint32_t hash_2ums32(const Fn2UMS32& f, uint32_t t, uint32_t mask, uint32_t shift)
{
    uint32_t v = (uint32_t)((uint64_t)f.c1 * t + f.add);
    return HIGH ? (v >> shift) : (v & mask);      // shift = 32 - s, 0 <= shift <= 31
}

// The running minimum needs neither the mask nor the shift per evaluation.
// Highest s bits: v -> v >> shift is monotone, so the minimum of the shifted
// values is the shifted minimum of the 32-bit values.  Lowest s bits: with both
// coefficients multiplied by 2^shift the 32-bit value is (v mod 2^s) 2^shift, an
// order-preserving image of the lowest s bits, and the same final shift brings
// the minimum back.  The hot loop is then one multiply-add and one minimum.
template <bool HIGH>
MH_HD Fn2UMS32 prep_2ums32_key(uint64_t c0, uint64_t c1, uint32_t shift)    // shift = 32 - s, 0 <= shift <= 32
{
    if (HIGH) return prep_2ums32(c0, c1);
    Fn2UMS32 f;
    f.c1 = shift >= 32 ? 0u : (uint32_t)c1 << shift;
    f.add = shift >= 32 ? 0ull : (uint64_t)((uint32_t)c0 << shift);
    return f;
}
MH_HD uint32_t key_2ums32(const Fn2UMS32& f, uint32_t t) { return (uint32_t)((uint64_t)f.c1 * t + f.add); }
MH_HD uint32_t finish_2ums32(uint32_t min_key, uint32_t shift) { return shift >= 32 ? 0u : min_key >> shift; }

// ------------------------------------------------------------------ tickets to work units
// Which units of the work list a ticket stands for.  Tickets map to units in
// regions: units of long items, one per ticket (they are listed first); then
// runs of `run` consecutive units (a power of two of at most 32, sized so that a
// wavefront still draws about 12 of them); then, level by level, runs of half
// that size, a quarter, ... down to one unit, LEVEL_DRAWS tickets per wavefront
// and level; then what is left, unit by unit.  A launch so ends on single short
// items without all wavefronts drawing tickets for single items at once: one
// address takes fewer than 10^8 atomics a second, and some thousand wavefronts
// that each finish a short row in a few microseconds ask for more.  The
// wavefronts still busy with the last tickets of one level are matched by two
// draws of half the size for the others.  Batches of long rows get runs of one
// and are handed out unit by unit.  A ticket beyond the last unit gets the empty
// range [n_units, n_units + 1).
struct TicketMap {
    static constexpr uint32_t LEVEL_DRAWS = 2;
    uint32_t n_units;       // fits 32 bits (the host refuses larger batches)
    uint32_t single;        // tickets below this are units of long items
    uint32_t n_runs;        // then n_runs tickets of 1 << lg_run units each
    uint32_t lg_run;
    uint32_t per_level;     // tickets of each level of shorter runs

    MH_HD void range(uint32_t tk, uint32_t* first, uint32_t* end) const
    {
        if (tk < single) {
            *first = tk;
            *end = tk + 1;
            return;
        }
        uint32_t t = tk - single;
        if (t < n_runs) {
            *first = single + (t << lg_run);
            *end = *first + (1u << lg_run);
            return;
        }
        t -= n_runs;
        const uint32_t run = 1u << lg_run;
        uint64_t base = (uint64_t)single + ((uint64_t)n_runs << lg_run);
        const uint32_t level = lg_run ? t / per_level : 0u;     // level 0: runs of run / 2, level 1: run / 4, ...
        if (level < lg_run) {
            const uint32_t r_lg = lg_run - 1u - level;
            base += (uint64_t)per_level * (run - (run >> level));   // the levels before took run/2 + ... + run/2^level units per ticket column
            *first = (uint32_t)(base + ((uint64_t)(t - level * per_level) << r_lg));
            *end = *first + (1u << r_lg);
            return;
        }
        const uint64_t u = base + (uint64_t)per_level * (run - 1u) + (t - lg_run * per_level);
        *first = u < n_units ? (uint32_t)u : n_units;
        *end = *first + 1;
    }
};
MH_HD TicketMap make_ticket_map(uint64_t units, uint64_t single_units, uint32_t waves)
{
    TicketMap m;
    m.n_units = (uint32_t)units;
    m.single = (uint32_t)(single_units < units ? single_units : units);
    const uint32_t rest = m.n_units - m.single;
    const uint32_t want = rest / (waves * 12u);
    m.lg_run = want < 2 ? 0u : (want >= 32 ? 5u : 31u - (uint32_t)__builtin_clz(want));
    m.per_level = waves * TicketMap::LEVEL_DRAWS;
    // the levels take per_level * (run - 1) units, fewer than rest / 6 by the choice of run
    m.n_runs = m.lg_run ? (rest - m.per_level * ((1u << m.lg_run) - 1u)) >> m.lg_run : 0u;
    return m;
}

// ---------------------------------------------------------------- packed index rows
// A tile of m indices (1..256) whose in-tile differences are w bits wide takes one word for
// its first index and ceil((m - 1) w / 32) words of differences.
constexpr uint32_t PACKED_TILE = 256;
MH_HD uint32_t packed_tile_words(uint32_t m, uint32_t w) { return 1u + ((m - 1u) * w + 31u) / 32u; }

// ---------------------------------------------------------------- row offsets
// What the row-binning kernel makes of one row's offsets.  A row is [begin, end) in
// col_idx; lo = row_ptr[0] and hi = row_ptr[n_rows] bound the part of col_idx the
// caller vouches for, nnz_cap is the number of nonzeros the workspace was sized
// for.  Returns 0 for a row that may be read, 1 for offsets that decrease or
// leave [lo, hi] (an offset that overshoots and comes back, as in [0, 1000, 5],
// gives its row a positive length that a test of neighbours alone accepts),
// 4 when [lo, hi) itself holds more than nnz_cap nonzeros.  Without `validate`
// only a negative length is caught (the row is then treated as empty, silently).
MH_HD uint32_t row_extent_status(int64_t begin, int64_t end, int64_t lo, int64_t hi, uint64_t nnz_cap, bool validate)
{
    if (end < begin) return 1u;
    if (!validate) return 0u;
    if (lo < 0 || hi < lo || begin < lo || begin > hi || end > hi) return 1u;
    if ((uint64_t)(hi - lo) > nnz_cap) return 4u;
    return 0u;
}

}  // namespace mh
