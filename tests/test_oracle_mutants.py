"""Plant one plausible mistake at a time in a copy of the oracle's C source
(on the CPU only) and check that at least one pin notices.  This is a test of
the pins, not of the oracle: a pin set that lets a dropped term, a wrong index
or a flipped bit order through would not be pinning anything."""
import os
import subprocess

import pytest

import pins
from oracle import oracle as loader

SRC = os.path.join(os.path.dirname(loader.__file__), "minhash_oracle.c")

# (name, text in the oracle source, replacement)
MUTANTS = [
    ("no_reduction_after_add", "acc = (acc + term) % p;", "acc = (acc + term);"),
    ("coefficients_reversed", "(u128)(c[i] % p) * power", "(u128)(c[deg - 1 - i] % p) * power"),
    ("linear_term_subtracted", "acc = (acc + term) % p;", "acc = (i == 1 ? acc + p - term : acc + term) % p;"),
    ("max_instead_of_min", "if (v < m) m = v;", "if (v > m || m == ORACLE_EMPTY_MIN) m = v;"),
    ("no_mod_D", "return (uint64_t)(acc % (u128)D);", "return (uint64_t)(acc);"),
    ("mod_D_plus_one", "return (uint64_t)(acc % (u128)D);", "return (uint64_t)(acc % (u128)(D + 1));"),
    ("mod_D_before_mod_p", "acc = (acc + term) % p;", "acc = ((acc + term) % (u128)D) % p;"),
    ("table_leading_dim_ignored", "table[(size_t)t * (size_t)perm_ld + (size_t)j]",
     "table[(size_t)t * (size_t)k + (size_t)j]"),
    ("powers_not_accumulated", "power = (power * (u128)(t % p)) % p;", "power = (u128)(t % p);"),
    ("power_of_wrong_base", "power = (power * (u128)(t % p)) % p;", "power = (power * (u128)((t + 1) % p)) % p;"),
    ("sentinel_changed", "#define ORACLE_EMPTY_MIN 0xFFFFFFFFu", "#define ORACLE_EMPTY_MIN 0x7FFFFFFFu"),
    ("first_nonzero_skipped", "for (int64_t e = lo; e < hi; ++e)", "for (int64_t e = lo + (hi - lo > 1); e < hi; ++e)"),
    ("last_nonzero_skipped", "for (int64_t e = lo; e < hi; ++e)", "for (int64_t e = lo; e < hi - (hi - lo > 1); ++e)"),
    ("arithmetic_in_64_bits", "typedef unsigned __int128 u128;", "typedef uint64_t u128;"),
    ("minima_transposed", "minima[(size_t)i * (size_t)k + (size_t)j] = (uint32_t)m;",
     "minima[(size_t)j * (size_t)n_rows + (size_t)i] = (uint32_t)m;"),
    ("bits_reversed_in_field", "int64_t q = (int64_t)j * b + bit;", "int64_t q = (int64_t)j * b + (b - 1 - bit);"),
    ("msb_first_bytes", "(uint8_t)(1u << (q % 8))", "(uint8_t)(0x80u >> (q % 8))"),
    ("highest_bits_kept", "if ((z >> bit) & 1u)", "if ((z >> (32 - b + bit)) & 1u)"),
    ("field_stride_off", "int64_t q = (int64_t)j * b + bit;", "int64_t q = (int64_t)j * (b < 32 ? b + 0 : b) + bit + (j > 0 && b == 3);"),
    ("multiply_shift_mod_2_31", "u128 two32 = (u128)1 << 32;", "u128 two32 = (u128)1 << 31;"),
    ("multiply_shift_high_is_low", "if (!high) return (uint64_t)(v % (u128)D);", "if (1) return (uint64_t)(v % (u128)D);"),
    ("multiply_shift_coefficients_swapped", "u128 v = ((u128)c[0] + (u128)c[1] * (u128)t) % two32;",
     "u128 v = ((u128)c[1] + (u128)c[0] * (u128)t) % two32;"),
    ("estimator_c1_c2_exchanged", "r_hat[q] = (P - C1) / (1.0 - C2);", "r_hat[q] = (P - C2) / (1.0 - C1);"),
    ("estimator_densities_exchanged", "double C1 = A1 * r2 / (r1 + r2) + A2 * r1 / (r1 + r2);",
     "double C1 = A1 * r1 / (r1 + r2) + A2 * r2 / (r1 + r2);"),
    ("estimator_exponent_off_by_one", "return r * pow(1.0 - r, n - 1.0) / (1.0 - pow(1.0 - r, n));",
     "return r * pow(1.0 - r, n) / (1.0 - pow(1.0 - r, n));"),
    ("expansion_block_stride", "(uint32_t)(((uint64_t)j << b) + packed_field(", "(uint32_t)(((uint64_t)j * b) + packed_field("),
    ("match_counts_compare_wrong_field", "packed_field(sig + (size_t)r2 * (size_t)sig_stride, j, b)) ++c;",
     "packed_field(sig + (size_t)r2 * (size_t)sig_stride, (j + 1) % k, b)) ++c;"),
    ("wrong_prime_31", "case ORACLE_2U_M31: *p = 2147483647ull;", "case ORACLE_2U_M31: *p = 2147483648ull;"),
    ("packed_fields_msb_first", "if ((d >> q) & 1u) words[at + 1 + bit / 32] |= 1u << (bit % 32);",
     "if ((d >> (w - 1 - q)) & 1u) words[at + 1 + bit / 32] |= 1u << (bit % 32);"),
    ("packed_width_counts_tile_boundaries", "if (i % 256 != 0 && row[i] - row[i - 1] > widest)", "if (row[i] - row[i - 1] > widest)"),
    ("packed_tile_of_255", "for (int64_t first = 0; first < n; first += 256) {\n            const int64_t m = n - first < 256 ? n - first : 256;\n            const int64_t n_words",
     "for (int64_t first = 0; first < n; first += 255) {\n            const int64_t m = n - first < 255 ? n - first : 255;\n            const int64_t n_words"),
    ("packed_first_index_as_difference", "words[at] = row[first];", "words[at] = first ? row[first] - row[first - 1] : row[first];"),
    ("unpack_forgets_to_accumulate", "value += d;", "value = d;"),
    ("wrong_prime_61", "case ORACLE_2U_M61: *p = 2305843009213693951ull;", "case ORACLE_2U_M61: *p = 2305843009213693953ull;"),
]


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_some_pin_catches(name, old, new, tmp_path):
    text = open(SRC).read()
    assert text.count(old) >= 1, "mutation site vanished from the oracle source: %r" % old
    mutated = text.replace(old, new)
    src = tmp_path / ("mutant_%s.c" % name)
    lib = tmp_path / ("libmutant_%s.so" % name)
    src.write_text(mutated)
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-w", "-fPIC", "-shared", str(src), "-o", str(lib), "-lm"])
    mutant = loader.Oracle(str(lib))
    caught = None
    for pin in pins.FAST_PINS:
        try:
            pin(mutant)
        except (AssertionError, ValueError):
            caught = pin.__name__
            break
    assert caught is not None, "no pin noticed the planted mistake %r" % name
