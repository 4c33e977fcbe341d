// Host build of the GPU library's integer arithmetic (csrc/mh_arith.h), compared
// with the plain definition  ((polynomial) mod p) mod D  evaluated with 128-bit
// integers and the % operator.  Prints "OK <count>" or the first mismatch.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "mh_arith.h"

typedef unsigned __int128 u128;

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint64_t rnd()
{
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return rng_state;
}

static uint64_t ref_poly(const uint64_t* c, int deg, uint64_t p, uint64_t D, uint64_t t)
{
    u128 acc = 0, pw = 1;
    for (int i = 0; i < deg; ++i) { acc = (acc + (u128)c[i] * pw) % p; pw = pw * t % p; }
    return (uint64_t)(acc % D);
}

static long checks = 0, guard_hits = 0, guard_saves = 0, full_bit31 = 0, full_doubtful = 0, full4_high = 0;
#define FAIL(...) do { printf("MISMATCH " __VA_ARGS__); printf("\n"); exit(1); } while (0)

static void check31(uint64_t D, const uint64_t* c, uint32_t t)
{
    using namespace mh;
    ModD md = make_mod_d(D);
    uint64_t want2 = ref_poly(c, 2, P31, D, t), want4 = ref_poly(c, 4, P31, D, t);
    Fn2U31 f2 = prep_2u31(c[0], c[1]);
    Fn4U31 f4 = prep_4u31(c[0], c[1], c[2], c[3]);
    uint32_t g2, g4;
    if (md.pow2) {
        g2 = hash_2u31<true>(f2, stage_2u31(t), md);
        g4 = hash_4u31<true>(f4, stage_4u31(t), md);
        const uint32_t ks = neg_key_shift(md.mask);
        // 2U full keys: a key that is not doubtful is exact; a doubtful one either has bit 31 set or lies below D - 1,
        // and an evaluation with bit 31 set never has a representative above D - 1
        {
            const uint32_t rot = full_key_rotation(md.mask);
            const int32_t fk = key_full_2u31(prep_2u31_full(c[0], c[1], rot), stage_2u31(t));
            if (fk >= 0 && md.mask - (((uint32_t)fk >> rot) & md.mask) != want2) FAIL("2U31 full key D=%llu t=%u c=(%llu,%llu)", (unsigned long long)D, t,
                                                                                      (unsigned long long)c[0], (unsigned long long)c[1]);
            if (fk < 0) {
                const uint32_t rep = (uint32_t)fk - (uint32_t)P31;             // x - p, the representative in [1, p]
                if (rep > md.mask) FAIL("2U31 full key: representative %u above D - 1 with bit 31 set, D=%llu t=%u", rep, (unsigned long long)D, t);
                if (md.mask - ((rep >> rot) & md.mask) != want2) FAIL("2U31 full key: x - p is not the representative D=%llu t=%u", (unsigned long long)D, t);
                ++full_bit31;
            }
            // the doubled key: twice the signed key when bit 31 is clear, at most 2 (D - 2) otherwise
            {
                const uint32_t k2x = key_full2_2u31(prep_2u31_full(c[0], c[1], rot), stage_2u31(t));
                if (fk >= 0 && (k2x != 2u * (uint32_t)fk || finish_full2_key(k2x, rot, md.mask) != want2)) FAIL("2U31 doubled key D=%llu t=%u", (unsigned long long)D, t);
                if (fk < 0 && (D < 2 || k2x > 2u * (md.mask - 1u)) && D > 1) FAIL("2U31 doubled key: wrapped value %u above 2 (D - 2), D=%llu", k2x, (unsigned long long)D);
                if (fk < 0 && !full2_key_doubtful(k2x, md.mask) && D > 1) FAIL("2U31 doubled key: wrapped value not doubtful");
            }
            // the same value through the two-maxima finish, which D > 2^26 uses
            const uint32_t two = fk > 0 ? finish_full_keys(fk, FULL_KEY_INIT_UNSIGNED, rot, md.mask)
                                        : finish_full_keys(FULL_KEY_INIT, (uint32_t)fk, rot, md.mask);
            if (two != want2) FAIL("2U31 two-maxima finish D=%llu t=%u", (unsigned long long)D, t);
            full_doubtful += full2_key_doubtful(key_full2_2u31(prep_2u31_full(c[0], c[1], rot), stage_2u31(t)), md.mask);
            checks += 2;
        }
        // 4U full keys: either half of [1, 2p] gives the location once reduced to [1, p]
        {
            const uint32_t rot = full_key_rotation(md.mask);
            const uint32_t x = fold_4u31(prep_4u31_full(c[0], c[1], c[2], c[3], rot), stage_4u31(t));
            if (x == 0 || x > 2u * (uint32_t)P31) FAIL("4U31 full key out of range");
            const uint32_t got = (int32_t)x > 0 ? finish_full_keys((int32_t)x, FULL_KEY_INIT_UNSIGNED, rot, md.mask)
                                                : finish_full_keys(FULL_KEY_INIT, x, rot, md.mask);
            if (got != want4) FAIL("4U31 full key D=%llu t=%u", (unsigned long long)D, t);
            full4_high += (int32_t)x < 0;
            ++checks;
        }
        uint32_t n4 = finish_neg_key(key_neg_4u31(prep_4u31_neg(c[0], c[1], c[2], c[3]), stage_4u31(t), ks), ks, md.mask);
        if (n4 != want4) FAIL("4U31 negated key D=%llu t=%u c=(%llu,%llu,%llu,%llu) got %u want %llu", (unsigned long long)D, t,
                              (unsigned long long)c[0], (unsigned long long)c[1], (unsigned long long)c[2],
                              (unsigned long long)c[3], n4, (unsigned long long)want4);
    } else {
        g2 = hash_2u31<false>(f2, stage_2u31(t), md);
        g4 = hash_4u31<false>(f4, stage_4u31(t), md);
    }
    if (g2 != want2) FAIL("2U31 D=%llu t=%u c=(%llu,%llu) got %u want %llu", (unsigned long long)D, t,
                          (unsigned long long)c[0], (unsigned long long)c[1], g2, (unsigned long long)want2);
    if (g4 != want4) FAIL("4U31 D=%llu t=%u c=(%llu,%llu,%llu,%llu) got %u want %llu", (unsigned long long)D, t,
                          (unsigned long long)c[0], (unsigned long long)c[1], (unsigned long long)c[2],
                          (unsigned long long)c[3], g4, (unsigned long long)want4);
    checks += 2;
}

static void check61(uint64_t D, const uint64_t* c, uint32_t t)
{
    using namespace mh;
    ModD md = make_mod_d(D);
    uint64_t want = ref_poly(c, 2, P61, D, t);
    Fn2U61 f = prep_2u61(c[0], c[1]);
    u128 full = ((u128)c[1] * t + c[0]) % P61;
    if (t < (1u << 31)) {
        uint64_t r = residue_2u61(f, t);
        if (r != (uint64_t)full) FAIL("2U61 residue t=%u got %llu want %llu", t, (unsigned long long)r,
                                      (unsigned long long)(uint64_t)full);
    }
    if (residue_wide_2u61(f, t) != (uint64_t)full) FAIL("2U61 wide residue t=%u", t);
    uint32_t g = (md.pow2 && D <= (1ull << 31)) ? hash_2u61<true>(f, t, md, D) : hash_2u61<false>(f, t, md, D);
    if (g != want) FAIL("2U61 D=%llu t=%u c=(%llu,%llu) got %u want %llu", (unsigned long long)D, t,
                        (unsigned long long)c[0], (unsigned long long)c[1], g, (unsigned long long)want);
    ++checks;
    if (md.pow2 && D <= (1ull << 31)) {
        // the carry-free key of the negated, rotated form: exact whenever bit 61 of the folded value is clear;
        // otherwise one too small and below GUARD61_FLOOR
        const uint32_t ks61 = neg_key_shift(md.mask);
        const Fn2U61 fn = prep_2u61_neg(c[0], c[1], ks61);
        const uint32_t key = key_neg_2u61(fn, t);
        const u128 V = (u128)(((uint64_t)fn.e1 << 32) | fn.e0) * t + fn.add;
        const uint64_t x = (uint64_t)(V & P61) + (uint64_t)(V >> 61);
        const uint32_t loc = finish_neg_key(key, ks61, md.mask);
        if ((x >> 61) == 0) {
            if (loc != want) FAIL("2U61 carry-free key D=%llu t=%u c=(%llu,%llu) got %u want %llu", (unsigned long long)D, t,
                                  (unsigned long long)c[0], (unsigned long long)c[1], loc, (unsigned long long)want);
        } else {
            if (key >= GUARD61_FLOOR) FAIL("2U61 carry-free key: bit 61 set and key %u not below the floor", key);
            if (key + 1u != (uint32_t)(x - P61)) FAIL("2U61 carry-free key: not one below the representative");
            if (finish_neg_key(key + 1u, ks61, md.mask) != want) FAIL("2U61: representative of a folded value with bit 61 set");
            ++guard_hits;
            if (loc != want) ++guard_saves;
        }
        ++checks;
    }
    // 4U with the same prime: Horner form against the power-sum definition
    uint64_t want4 = ref_poly(c, 4, P61, D, t);
    Fn4U61 f4 = prep_4u61(c[0], c[1], c[2], c[3]);
    u128 full4 = 0, pw = 1;
    for (int i = 0; i < 4; ++i) { full4 = (full4 + (u128)c[i] * pw) % P61; pw = pw * t % P61; }
    if (residue_4u61(f4, t) != (uint64_t)full4) FAIL("4U61 residue t=%u c=(%llu,%llu,%llu,%llu)", t, (unsigned long long)c[0],
                                                     (unsigned long long)c[1], (unsigned long long)c[2], (unsigned long long)c[3]);
    uint32_t g4 = md.pow2 ? hash_4u61<true>(f4, t, md, D) : hash_4u61<false>(f4, t, md, D);
    if (g4 != want4) FAIL("4U61 D=%llu t=%u got %u want %llu", (unsigned long long)D, t, g4, (unsigned long long)want4);
    ++checks;
}

int main()
{
    using namespace mh;
    const uint64_t p31 = P31, p61 = P61;
    // m31_reduce64 against % on edge and random 64-bit values (Section 3.4's reduction)
    {
        std::vector<uint64_t> vs = {0, 1, p31 - 1, p31, p31 + 1, 2 * p31 - 1, 2 * p31, 2 * p31 + 1, 1ull << 31, (1ull << 32) - 1,
                                    (p31 - 1) * (p31 - 1), (p31 - 1) * (p31 - 1) + (p31 - 1), (1ull << 62) - 1,
                                    1ull << 62, ~0ull, ~0ull - 1, (1ull << 63), p31 << 31, (p31 << 31) + p31};
        for (int i = 0; i < 2000000; ++i) vs.push_back(rnd() >> (rnd() % 40));
        for (uint64_t v : vs) {
            if (m31_reduce64(v) != v % p31) FAIL("m31_reduce64(%llu)", (unsigned long long)v);
            ++checks;
        }
    }
    // mod-D by multiply-high
    {
        std::vector<uint64_t> Ds = {3, 5, 6, 7, 10, 1000003, 16609143, 1010017424, 2147483646, 2147483645, (1u << 30) + 1, (1u << 30) - 1};
        for (uint64_t D : Ds) {
            ModD md = make_mod_d(D);
            std::vector<uint32_t> rs = {0, 1, (uint32_t)D - 1, (uint32_t)D, (uint32_t)D + 1, P31 - 1, P31 - 2, (uint32_t)(2 * D % P31)};
            for (int i = 0; i < 200000; ++i) rs.push_back((uint32_t)(rnd() % P31));
            for (uint32_t r : rs) {
                if (r >= P31) continue;
                if (reduce_mod_d<false>(r, md) != r % D) FAIL("mod D=%llu r=%u", (unsigned long long)D, r);
                ++checks;
            }
        }
    }
    std::vector<uint64_t> D31 = {1, 2, 1 << 10, 1 << 24, 1u << 30, 3, 1000003, 16609143, 1010017424, p31 - 1};
    std::vector<uint64_t> D61 = {1, 2, 1 << 24, 1u << 30, 1ull << 31, 1ull << 32, 3, 1010017424, (1ull << 32) - 1, (1ull << 31) + 7,
                                 16609143, (1ull << 29) + 1, 1431655765, 1431655766};
    std::vector<uint64_t> edge31 = {0, 1, 2, p31 - 1, p31 - 2, (p31 - 1) / 2, (p31 - 1) / 2 + 1, (p31 + 1) / 2 + 1, 1 << 16, 12345};
    std::vector<uint64_t> edge61 = {0, 1, 2, p61 - 1, p61 - 2, (p61 - 1) / 2, (p61 + 1) / 2, 1ull << 32, (1ull << 32) - 1, 1ull << 60};
    for (uint64_t D : D31) {
        std::vector<uint32_t> ts = {0, 1, (uint32_t)(D - 1), (uint32_t)(D / 2), (uint32_t)((D - 1) / 3)};
        // all edge combinations for (c0, c1), with edge c2, c3
        for (uint64_t c0 : edge31) for (uint64_t c1 : edge31) for (uint32_t t : ts) {
            uint64_t c[4] = {c0, c1, edge31[(c0 + t) % edge31.size()], edge31[(c1 + 3) % edge31.size()]};
            check31(D, c, t);
        }
        for (int i = 0; i < 300000; ++i) {
            uint64_t c[4] = {rnd() % p31, rnd() % p31, rnd() % p31, rnd() % p31};
            if (i % 7 == 0) c[rnd() % 4] = edge31[rnd() % edge31.size()];
            uint32_t t = (uint32_t)(rnd() % D);
            check31(D, c, t);
        }
    }
    for (uint64_t D : D61) {
        std::vector<uint32_t> ts = {0, 1, (uint32_t)(D - 1), (uint32_t)(D / 2), (uint32_t)((D - 1) / 3)};
        ts.push_back(0xFFFFFFFFu % (uint32_t)(D > 0xFFFFFFFFull ? 0xFFFFFFFFull : D));
        for (uint64_t c0 : edge61) for (uint64_t c1 : edge61) for (uint32_t t : ts) {
            uint64_t c[4] = {c0, c1, edge61[(c0 + t) % edge61.size()], edge61[(c1 + 3) % edge61.size()]};
            check61(D, c, t);
            uint64_t e[4] = {c[2], c[3], c0, c1};          // every edge pair also as (c2, c3)
            check61(D, e, t);
        }
        for (int i = 0; i < 300000; ++i) {
            uint64_t c[4] = {rnd() % p61, rnd() % p61, rnd() % p61, rnd() % p61};
            if (i % 7 == 0) c[rnd() % 4] = edge61[rnd() % edge61.size()];
            uint32_t t = (uint32_t)(rnd() % D);
            check61(D, c, t);
        }
    }
    // Carry-free 2U-M61 key: coefficients built so that the negated form's H has its low 29 bits all
    // ones (the only case in which bit 61 of the folded value can be set), with the low-word sum on
    // either side of a carry.  Many of them must have bit 61 set, and some must be cases in which the
    // key as it stands gives the wrong location.
    {
        const long hits_before = guard_hits, saves_before = guard_saves;
        int built = 0;
        for (uint64_t D : {1ull << 30, 1ull << 31, 1ull << 24, 1ull << 1}) {
            for (int i = 0; i < 20000; ++i) {
                const uint32_t t = (uint32_t)(rnd() % D);
                if (t == 0) continue;
                const uint64_t n = 1 + rnd() % (p61 - 1);                    // the negated linear coefficient, in [1, p)
                const uint32_t e0 = (uint32_t)n, e1 = (uint32_t)(n >> 32);
                uint64_t add = 1 + rnd() % p61;                                 // p - c0, in [1, p]
                if (i % 3 == 0) add = (add & ~0xFFFFFFFFull) | (0xFFFFFFFFull - (rnd() % 5));   // low word near the top
                uint64_t L = (uint64_t)e0 * t + add;
                uint64_t H = (uint64_t)e1 * t + (L >> 32);
                const uint64_t d = ((1ull << 29) - 1 - H) & ((1ull << 29) - 1);  // raise H by d: add d 2^32 to L
                uint64_t add2 = add + (d << 32);
                if (add2 > p61) { if (add < (((1ull << 29) - d) << 32) + 1) continue; add2 = add - (((1ull << 29) - d) << 32); }
                if (add2 < 1 || add2 > p61) continue;
                // n and add2 are what the kernel multiplies and adds: the caller's coefficients, negated and
                // rotated left by the key shift; rotate back and negate to get those
                const uint32_t ks = neg_key_shift((uint32_t)(D - 1));
                auto rotr61 = [&](uint64_t v) { return ((v >> ks) | (v << (61u - ks))) & p61; };
                uint64_t c[4] = {p61 - rotr61(add2), p61 - rotr61(n), rnd() % p61, rnd() % p61};
                Fn2U61 f = prep_2u61_neg(c[0], c[1], ks);
                if (((uint64_t)f.e1 << 32 | f.e0) != n || f.add != add2) FAIL("engineered coefficients do not rotate back");
                if ((((uint64_t)f.e1 * t + (((uint64_t)f.e0 * t + f.add) >> 32)) & 0x1FFFFFFFull) != 0x1FFFFFFFull) FAIL("engineered case not built");
                check61(D, c, t);
                ++built;
            }
        }
        if (built < 10000 || guard_hits - hits_before < 1000) FAIL("carry-free key: %d built, %ld with bit 61 set", built, guard_hits - hits_before);
        if (guard_saves - saves_before < 100) FAIL("carry-free key: only %ld engineered cases came out wrong", guard_saves - saves_before);
    }
    // Fractional keys for D < 2^28 that is not a power of two: the location comes back exactly, and
    // keys are ordered like the locations, on edge residues and random ones
    {
        long n = 0;
        for (uint64_t D : {3ull, 5ull, 6ull, 7ull, 1000003ull, 16609143ull, (1ull << 28) - 1, (1ull << 27) + 1, (1ull << 24) - 1,
                           (1ull << 24) + 1, 65537ull, 100ull}) {
            if (!frac_key_serves(D)) FAIL("fractional key refuses D=%llu", (unsigned long long)D);
            const FracD fd = make_frac_d(D);
            std::vector<uint32_t> rs = {0, 1, (uint32_t)(D - 1), (uint32_t)D, (uint32_t)(D + 1), (uint32_t)(2 * D - 1), (uint32_t)(2 * D),
                                        (uint32_t)(p31 - 1), (uint32_t)(p31 - 2), (uint32_t)((p31 - 1) / D * D), (uint32_t)((p31 - 1) / D * D - 1),
                                        (uint32_t)((p31 - 1) / D * D + 1 < p31 ? (p31 - 1) / D * D + 1 : 0)};
            for (int i = 0; i < 200000; ++i) rs.push_back((uint32_t)(rnd() % p31));
            for (int i = 0; i < 2000; ++i) { uint64_t q = rnd() % ((p31 - 1) / D + 1); uint64_t r = q * D + (rnd() % 3) - 1 + (i & 1 ? D - 1 : 0); if (r < p31) rs.push_back((uint32_t)r); }
            uint32_t prev_key = 0; uint64_t prev_v = 0; bool have = false;
            for (uint32_t r : rs) {
                const uint32_t key = frac_key(r, fd);
                const uint64_t v = r % D;
                if (finish_frac_key(key, (uint32_t)D) != v) FAIL("fractional key D=%llu r=%u gives %u want %llu", (unsigned long long)D, r,
                                                                 finish_frac_key(key, (uint32_t)D), (unsigned long long)v);
                if (have && ((v < prev_v && !(key < prev_key)) || (v > prev_v && !(key > prev_key)))) FAIL("fractional key order D=%llu", (unsigned long long)D);
                prev_key = key; prev_v = v; have = true;
                ++n;
            }
        }
        if (frac_key_serves(1ull << 20) || frac_key_serves(1ull << 28) || frac_key_serves(1010017424ull) || frac_key_serves(2)) FAIL("fractional key accepts a D it cannot serve");
        checks += n;
    }
    // 61-bit residues modulo D in 32-bit steps (D <= 2^32 / 3, not a power of two) against the 64-bit %
    {
        long n = 0;
        const unsigned long long third = (1ull << 32) / 3;
        for (uint64_t D : {3ull, 5ull, 6ull, 7ull, 100ull, 65537ull, 1000003ull, 16609143ull, (1ull << 28) - 1, (1ull << 28) + 1, (1ull << 29) - 1,
                           (1ull << 29) + 1, (1ull << 29) + 12345, (1ull << 30) - 1, (1ull << 30) + 1, 1010017424ull, third - 1, third}) {
            const ModD md = make_mod_d(D);
            if (!md.M61q) FAIL("32-bit steps refuse D=%llu", (unsigned long long)D);
            const uint64_t dp = scaled_up_d(D);
            if (dp % D != 0 || dp <= (1ull << 29) || 3 * dp > (1ull << 32) || (dp / D & (dp / D - 1)) != 0)
                FAIL("scaled D=%llu gives %llu", (unsigned long long)D, (unsigned long long)dp);
            std::vector<uint64_t> rs = {0, 1, D - 1, D, D + 1, dp - 1, dp, dp + 1, 2 * dp - 1, 2 * dp, 3 * dp - 1, 3 * dp, p61 - 1, p61 - 2,
                                        (p61 - 1) / dp * dp, (p61 - 1) / dp * dp - 1, (1ull << 32) - 1, 1ull << 32, (1ull << 29) - 1, 1ull << 29,
                                        (1ull << 60) - 1, 1ull << 60};
            for (int i = 0; i < 300000; ++i) rs.push_back(rnd() % p61);
            for (int i = 0; i < 100000; ++i) rs.push_back((rnd() % p61) >> (rnd() % 61));
            for (int i = 0; i < 20000; ++i) {           // next to multiples of D', where a quotient that is off shows
                const uint64_t q = rnd() % ((p61 - 1) / dp + 1), r = q * dp + (rnd() % 5) - 2;
                if (r < p61) rs.push_back(r);
            }
            for (uint64_t r : rs) {
                const uint32_t got = reduce61_mod_d(r, md, D);
                if (got != r % D) FAIL("32-bit steps D=%llu r=%llu give %u want %llu", (unsigned long long)D, (unsigned long long)r, got,
                                       (unsigned long long)(r % D));
                ++n;
            }
        }
        for (uint64_t D : {1ull, 2ull, 1ull << 20, 1ull << 31, third + 1, (1ull << 31) + 7, (1ull << 32) - 1, 1ull << 32})
            if (make_mod_d(D).M61q) FAIL("32-bit steps accept D=%llu", (unsigned long long)D);
        checks += n;
    }
    // Small quotients for D >= p / 3: the smallest of r, r - D, r - 2D
    {
        for (uint64_t D : {715827883ull, 715827884ull, 1010017424ull, 1073741823ull, 1073741825ull, 2000000011ull, (unsigned long long)(p31 - 1), (unsigned long long)(p31 - 2)}) {
            if (!small_quotient_serves(D)) FAIL("small quotient refuses D=%llu", (unsigned long long)D);
            std::vector<uint32_t> rs = {0, 1, (uint32_t)(D - 1), (uint32_t)D, (uint32_t)(D + 1), (uint32_t)(p31 - 1), (uint32_t)(p31 - 2)};
            if (2 * D < p31) { rs.push_back((uint32_t)(2 * D - 1)); rs.push_back((uint32_t)(2 * D)); rs.push_back((uint32_t)(2 * D + 1)); }
            for (int i = 0; i < 200000; ++i) rs.push_back((uint32_t)(rnd() % p31));
            for (uint32_t r : rs) {
                if (reduce_small_quotient(r, (uint32_t)D) != r % D) FAIL("small quotient D=%llu r=%u", (unsigned long long)D, r);
                ++checks;
            }
        }
        if (small_quotient_serves(715827882ull) || small_quotient_serves(1ull << 30) || small_quotient_serves(p31)) FAIL("small quotient accepts a D it cannot serve");
    }
    // multiply-shift 2U (Section 3.3): ((c0 + c1 t) mod 2^32) mod 2^s, lowest or highest s bits
    for (int sbits = 0; sbits <= 32; ++sbits) {
        uint64_t D = 1ull << sbits;
        uint32_t mask = (uint32_t)(D - 1), shift = (uint32_t)(32 - sbits);
        for (int i = 0; i < 20000; ++i) {
            uint64_t c0 = rnd() & 0xFFFFFFFFull, c1 = (rnd() & 0xFFFFFFFFull) | 1ull;
            if (i % 5 == 0) c0 = 0xFFFFFFFFull;
            if (i % 7 == 0) c1 = 0xFFFFFFFFull;
            uint32_t t = (uint32_t)(rnd() % D);
            if (i % 11 == 0) t = (uint32_t)(D - 1);
            u128 v = ((u128)c0 + (u128)c1 * t) % ((u128)1 << 32);
            Fn2UMS32 f = prep_2ums32(c0, c1);
            if (hash_2ums32<false>(f, t, mask, shift) != (uint64_t)(v % D)) FAIL("multiply-shift low s=%d", sbits);
            if (sbits >= 1 && hash_2ums32<true>(f, t, mask, shift) != (uint64_t)(v / (((u128)1 << 32) / D)))
                FAIL("multiply-shift high s=%d", sbits);
            checks += 2;
            // the keys the kernel takes the minimum of: same value after the final shift, and
            // ordered like the hashed locations (checked on a second index under the same function)
            Fn2UMS32 fl = prep_2ums32_key<false>(c0, c1, shift), fh = prep_2ums32_key<true>(c0, c1, shift);
            uint32_t t2 = (uint32_t)(rnd() % D);
            uint32_t h1 = hash_2ums32<false>(f, t, mask, shift), h2 = hash_2ums32<false>(f, t2, mask, shift);
            uint32_t k1 = key_2ums32(fl, t), k2 = key_2ums32(fl, t2);
            if (finish_2ums32(k1, shift) != h1 || finish_2ums32(k2, shift) != h2 || (h1 < h2) != (k1 < k2))
                FAIL("multiply-shift low key s=%d", sbits);
            if (sbits >= 1) {
                uint32_t g1 = hash_2ums32<true>(f, t, mask, shift), g2 = hash_2ums32<true>(f, t2, mask, shift);
                uint32_t q1 = key_2ums32(fh, t), q2 = key_2ums32(fh, t2);
                uint32_t lo = q1 < q2 ? q1 : q2;
                if (finish_2ums32(q1, shift) != g1 || finish_2ums32(lo, shift) != (g1 < g2 ? g1 : g2))
                    FAIL("multiply-shift high key s=%d", sbits);
            }
            checks += 2;
        }
    }
    // TicketMap: the ranges of tickets 0, 1, 2, ... tile [0, units) in order, one unit per ticket among the
    // long items, runs of at most 32 elsewhere that never grow again once they shrank; later tickets are empty
    {
        const uint32_t wave_counts[] = {1, 4, 7, 64, 5120, 8192};
        const uint64_t unit_counts[] = {0, 1, 2, 63, 64, 65, 1000, 4095, 61440, 61441, 122880, 200000, 262144, 983040, 2000000, 2236962, 5000001};
        for (uint32_t waves : wave_counts)
            for (uint64_t units : unit_counts)
                for (int sv = 0; sv < 4; ++sv) {
                    const uint64_t single = sv == 0 ? 0 : sv == 1 ? units / 3 : sv == 2 ? units : units + 5;
                    const TicketMap tm = make_ticket_map(units, single, waves);
                    uint64_t covered = 0;
                    uint32_t tk = 0, prev_len = 32, n_tickets_past_long = 0;
                    for (; covered < units; ++tk) {
                        uint32_t a, b;
                        tm.range(tk, &a, &b);
                        if (a != covered || b <= a || b - a > 32 || b > units)
                            FAIL("ticket map: waves %u units %llu single %llu ticket %u covers [%u, %u), expected a range from %llu",
                                 waves, (unsigned long long)units, (unsigned long long)single, tk, a, b, (unsigned long long)covered);
                        if (a < (single < units ? single : units)) {
                            if (b - a != 1) FAIL("ticket map: long item in a run of %u", b - a);
                        } else {
                            if (b - a > prev_len) FAIL("ticket map: run grows from %u to %u at ticket %u", prev_len, b - a, tk);
                            prev_len = b - a;
                            ++n_tickets_past_long;
                        }
                        covered = b;
                        ++checks;
                    }
                    for (uint32_t extra = 0; extra < 3 * waves + 3; extra += waves / 2 + 1) {
                        uint32_t a, b;
                        tm.range(tk + extra, &a, &b);
                        if (a < units) FAIL("ticket map: ticket %u past the end covers unit %u", tk + extra, a);
                        ++checks;
                    }
                    // many short units: far fewer tickets than units, and only a few single ones at the end
                    const uint64_t rest = units - (single < units ? single : units);
                    if (rest >= (uint64_t)waves * 12 * 32 && n_tickets_past_long > rest / 32 + (uint64_t)waves * 2 * 5 + 32)
                        FAIL("ticket map: %u tickets for %llu short units on %u waves", n_tickets_past_long, (unsigned long long)rest, waves);
                }
    }
    // Row offsets as the row-binning kernel reads them: which rows of a row_ptr array may be read.
    // Each case is {row_ptr, nonzeros the workspace was sized for, status bits expected with
    // validation on, rows that must come out empty}.
    {
        struct Case { std::vector<int64_t> rp; uint64_t cap; uint32_t want; std::vector<int> emptied; };
        const std::vector<Case> cases = {
            {{0, 3, 3, 10}, 10, 0u, {}},                       // well-formed
            {{7, 9, 20}, 13, 0u, {}},                          // row_ptr[0] need not be 0
            {{0, 1000, 5}, 5, 1u, {0, 1}},                     // overshoots and comes back: row 0 would read 1000 indices
            {{0, 4, 3, 8}, 8, 1u, {1}},                        // an adjacent decrease inside the buffer
            {{-2, 1, 4}, 6, 1u, {0, 1}},                       // negative first offset
            {{5, 2, 9}, 9, 1u, {0, 1}},                        // second offset below the first: row 0 decreases, row 1 starts below lo
            {{0, 6, 12}, 11, 4u, {0, 1}},                      // more nonzeros than the workspace serves
            {{0, 0, 0}, 0, 0u, {}},                            // empty rows only
        };
        for (const Case& c : cases) {
            const int n = (int)c.rp.size() - 1;
            uint32_t status = 0;
            std::vector<int> emptied;
            for (int r = 0; r < n; ++r) {
                const uint32_t st = row_extent_status(c.rp[r], c.rp[r + 1], c.rp[0], c.rp[n], c.cap, true);
                status |= st;
                if (st) emptied.push_back(r);
                // without validation only a negative length is caught
                const uint32_t plain = row_extent_status(c.rp[r], c.rp[r + 1], 0, 0, c.cap, false);
                if (plain != (c.rp[r + 1] < c.rp[r] ? 1u : 0u)) FAIL("row extent without validation, row %d", r);
                // a row that passes is read inside [lo, hi) only and is no longer than the workspace's bound
                if (!st && (c.rp[r] < c.rp[0] || c.rp[r + 1] > c.rp[n] || (uint64_t)(c.rp[r + 1] - c.rp[r]) > c.cap))
                    FAIL("row extent: row %d accepted outside the vouched range", r);
                ++checks;
            }
            if (status != c.want || emptied != c.emptied) FAIL("row extent: status %u, expected %u (first offset %lld)", status, c.want, (long long)c.rp[0]);
        }
    }
    if (full_bit31 < 1000 || full_doubtful < full_bit31) FAIL("full keys: %ld with bit 31 set, %ld doubtful", full_bit31, full_doubtful);
    if (full4_high < 100000) FAIL("4U full keys: only %ld evaluations above p", full4_high);
    printf("OK %ld\n", checks);
    return 0;
}
