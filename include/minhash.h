/*
 * minhash.h - C ABI of the MI355X (gfx950) b-bit minwise-hash signature library.
 *
 * The library turns every sparse binary data vector, given as the set of its
 * nonzero feature indices (CSR without a values array), into k b-bit integers:
 * for each of k hash functions (or explicit permutations) the minimum hashed
 * location over the row's nonzeros, of which only the lowest b bits are kept.
 * All pointers are plain pointers; which side of the bus they live on is stated
 * per argument.  Every buffer, including the workspace, belongs to the caller
 * (the one exception is minhash_signatures_static, which works in a buffer built
 * into the library).  Between calls the library keeps only launch constants per
 * device (number of compute units, resident blocks per kernel).  No call throws;
 * errors are return codes.
 */
#ifndef MINHASH_H
#define MINHASH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MINHASH_VERSION 100   /* 1.00 */

/* Hash families.  p is the Mersenne prime the polynomial is reduced by. */
enum {
    MINHASH_2U_M31 = 0,  /* ((c0 + c1 t) mod (2^31-1)) mod D                  Section 2, eq. "eqn_h_2U" */
    MINHASH_4U_M31 = 1,  /* ((c0 + c1 t + c2 t^2 + c3 t^3) mod (2^31-1)) mod D Section 2, eq. "eqn_h_4U";
                            Mersenne reduction as in Section 3.4               */
    MINHASH_2U_M61 = 2,  /* 2U with p = 2^61-1 (Section 3.4, last paragraph)   */
    MINHASH_4U_M61 = 3,  /* 4U (eq. "eqn_h_4U") with p = 2^61-1                 */
    MINHASH_PERM   = 4,  /* explicit D x k permutation matrix, Section 1.5     */
    MINHASH_2U_MS32 = 5, /* ((c0 + c1 t) mod 2^32) mod 2^s, D = 2^s, c1 odd: the multiply-shift 2U of
                            Section 3.3, eq. "eqn_h_s", as printed (lowest s bits)              */
    MINHASH_2U_MS32_HIGH = 6 /* the same 32-bit value, of which the HIGHEST s bits are kept (the form of
                            the scheme Section 3.3 cites); needs D >= 2                         */
};

/* Return codes. */
enum {
    MINHASH_OK            =  0,
    MINHASH_ERR_ARG       = -1,  /* null pointer, negative size, n_rows or nnz bound too large */
    MINHASH_ERR_FAMILY    = -2,  /* unknown family                                             */
    MINHASH_ERR_D         = -3,  /* D == 0, D > 2^32, or D >= p for a hash family              */
    MINHASH_ERR_KB        = -4,  /* k < 1, k > MINHASH_MAX_K, b < 1 or b > 32                  */
    MINHASH_ERR_STRIDE    = -5,  /* out_stride < ceil(k*b/8) or perm_ld < k                    */
    MINHASH_ERR_WORKSPACE = -6,  /* workspace null, misaligned or smaller than required        */
    MINHASH_ERR_HIP       = -7,  /* a HIP runtime call failed; see minhash_last_hip_error()    */
    MINHASH_ERR_COEFF     = -8,  /* minhash_check_coeffs: a coefficient is >= p (multiply-shift:
                                    >= 2^32, or the multiplier is even)                        */
    MINHASH_ERR_DATA      = -9,  /* minhash_status: VALIDATE found an index >= D or a
                                    decreasing row_ptr                                         */
    MINHASH_ERR_TOO_LARGE = -10  /* minhash_signatures_static: the batch needs more than
                                    MINHASH_STATIC_SCRATCH_BYTES of work space                 */
};

#define MINHASH_MAX_K            65536
#define MINHASH_FLAG_VALIDATE    1u   /* check col_idx < D and row_ptr monotone on the device */
#define MINHASH_FLAG_GENERIC_MOD 2u   /* MINHASH_2U_M31 / MINHASH_4U_M31 only: evaluate with the plain % operator
                                         (runtime moduli, Horner form) instead of the Mersenne reduction.  Same
                                         results; exists to measure what Section 3.4 saves ("4U (Mod)" against
                                         "4U (Bit)" in the paper's timing tables)                              */
#define MINHASH_FLAG_EXACT_FOLD  4u   /* MINHASH_2U_M31, MINHASH_4U_M31 and MINHASH_2U_M61 with a power-of-two D
                                         (ignored for other D): evaluate every row with a form of the reduction
                                         modulo the Mersenne prime (Section 3.4) that needs no second look at
                                         any value, instead of the shorter forms (2U, p = 2^31-1, D <= 2^26: one
                                         running maximum of a doubled key, the rare doubtful values computed
                                         again; 2U, p = 2^61-1: a carry-free key, likewise; 4U: the folded value
                                         kept in two running maxima).  Same results; exists so that whole
                                         batches of the shorter forms can be compared with it, and to time the
                                         difference                                                           */
#define MINHASH_WORKSPACE_ALIGN  256

/*
 * minhash_signatures - the whole hot path for one batch of rows.
 *
 * For every row i and every j < k it computes
 *     m[i][j] = min over t in col_idx[row_ptr[i] .. row_ptr[i+1]) of h_j(t)
 * (Section 2, last paragraph: every nonzero location t is mapped to h_j(t) and
 * the minimum of the mapped locations is the j-th hashed value), keeps the
 * lowest b bits of m[i][j] (Section 1.1) and writes them as bits
 * [j*b, (j+1)*b) of row i's bit string at out + i*out_stride, bit q of the
 * string being bit (q mod 8) of byte (q div 8).  Bytes from ceil(k*b/8) up to
 * out_stride, and the unused high bits of the last signature byte, are written
 * as 0.  The minimum of an empty row is 0xFFFFFFFF, so all its fields are ones.
 *
 *   row_ptr   device, n_rows+1 int64, non-decreasing offsets into col_idx;
 *             row_ptr[0] need not be 0
 *   col_idx   device, uint32 feature indices in [0, D); any order, duplicates
 *             allowed (the result depends only on the set)
 *   n_rows    0 <= n_rows < 2^31; 0 is a successful no-op
 *   D         size of the feature universe, 1 <= D <= 2^32, D < p for the
 *             Mersenne families, a power of two for the multiply-shift families.
 *             D a power of two takes a faster path
 *   k, b      number of functions (1..MINHASH_MAX_K), bits kept (1..32; b = 32
 *             stores the full minima as little-endian uint32)
 *   family    one of MINHASH_*
 *   params    device.  Hash families: uint64 c[k][deg], deg = 2 (2U) or 4 (4U),
 *             c[j][i] multiplies t^i and lies in [0, p) (the paper numbers the
 *             same coefficients a_{i+1,j}); multiply-shift: c[j][0] < 2^32 and
 *             c[j][1] < 2^32 odd.  MINHASH_PERM: uint32
 *             table[D][perm_ld], index-major, table[t][j] = pi_j(t)
 *   perm_ld   MINHASH_PERM: row pitch of the table in elements, >= k; else 0
 *   out       device, n_rows*out_stride bytes, written completely
 *   out_stride >= ceil(k*b/8)
 *   workspace device, MINHASH_WORKSPACE_ALIGN-aligned, at least
 *             minhash_workspace_bytes(n_rows, nnz_upper_bound, k, family) bytes
 *             with nnz_upper_bound >= row_ptr[n_rows]-row_ptr[0]; contents on
 *             entry are ignored; two calls may share it only on one stream
 *   stream    hipStream_t (NULL = the default stream); all work is enqueued on
 *             it and the call returns without synchronising
 *   flags     0 or an OR of MINHASH_FLAG_* values
 *
 * Returns MINHASH_OK once everything is enqueued, or a negative code.  Every
 * code but MINHASH_ERR_HIP is found before any launch (nothing has been enqueued
 * then); MINHASH_ERR_HIP reports a failed launch, after which earlier kernels of
 * the call may already be on the stream.  Indices >= D or offsets in row_ptr
 * that decrease or leave [row_ptr[0], row_ptr[n_rows]] are undefined behaviour
 * unless MINHASH_FLAG_VALIDATE is set.  With it, col_idx is read only inside
 * [row_ptr[0], row_ptr[n_rows]), and only if that range is non-negative and
 * holds no more nonzeros than the workspace was sized for (that the range lies
 * inside the col_idx allocation remains the caller's promise: the library is
 * not told its length); an index >= D is hashed as 0; the table of
 * MINHASH_PERM is then read at row 0 instead.  minhash_status reports
 * MINHASH_ERR_DATA (MINHASH_ERR_WORKSPACE for too many nonzeros), and the
 * signatures of the affected rows are unspecified.
 */
int minhash_signatures(const int64_t *row_ptr, const uint32_t *col_idx, int64_t n_rows,
                       uint64_t D, int32_t k, int32_t b, int32_t family,
                       const void *params, int64_t perm_ld,
                       uint8_t *out, int64_t out_stride,
                       void *workspace, size_t workspace_bytes,
                       void *stream, uint32_t flags);

/*
 * Same computation, for measurement: brackets the hash / gather kernel (the
 * step that evaluates h_j(t) and keeps the running minima, Section 3.2 phase 2)
 * with HIP events on `stream`, waits for the stream, and stores that kernel's
 * duration in milliseconds in *kernel_ms (host pointer, may be NULL).
 */
int minhash_signatures_profiled(const int64_t *row_ptr, const uint32_t *col_idx, int64_t n_rows,
                                uint64_t D, int32_t k, int32_t b, int32_t family,
                                const void *params, int64_t perm_ld,
                                uint8_t *out, int64_t out_stride,
                                void *workspace, size_t workspace_bytes,
                                void *stream, uint32_t flags, float *kernel_ms);

/*
 * minhash_signatures_static - for callers that cannot allocate device memory
 * (code under HIP graph capture, serving loops or harnesses that forbid
 * hipMalloc and torch allocations): the computation of minhash_signatures with
 * its work list and partial minima in a buffer of
 * MINHASH_STATIC_SCRATCH_BYTES that is built into the library's device code
 * (one copy per GPU the library runs on, held until the process ends), so the
 * caller passes inputs and outputs only.  The call allocates nothing, on the
 * host or on the device, and does not synchronise.
 *
 *   nnz_upper_bound  >= row_ptr[n_rows] - row_ptr[0].  With P = nnz_upper_bound / 8192
 *                    + min(n_rows, nnz_upper_bound / 8192), the batch fits whenever
 *                    32 (n_rows + P + nnz_upper_bound / 2048) + 16 min(n_rows,
 *                    nnz_upper_bound / 512) + 4 k P + 2048 bytes are at most
 *                    MINHASH_STATIC_SCRATCH_BYTES (k = 500: 200 000 rows with
 *                    10^8 nonzeros fit, the 350 000 rows with 1.3x10^9 nonzeros
 *                    of a whole webspam-sized batch do not); otherwise the call
 *                    returns MINHASH_ERR_TOO_LARGE and enqueues nothing.
 *   status           device, one int32, or NULL.  The last kernel of the call
 *                    stores there what minhash_status would report
 *                    (MINHASH_OK, MINHASH_ERR_WORKSPACE if row_ptr described more
 *                    than nnz_upper_bound nonzeros, MINHASH_ERR_DATA for what
 *                    MINHASH_FLAG_VALIDATE found); minhash_status itself cannot
 *                    see the built-in buffer.
 *   all other arguments, the result and the return codes are those of
 *   minhash_signatures.
 *
 * All calls on one GPU share that GPU's buffer: calls on one stream run one
 * after the other and are safe, calls that overlap on different streams of one
 * GPU race.  The address of the buffer is looked up once per device, on the
 * first call with that device current (a caller that captures a graph makes one
 * call before the capture starts).
 */
#define MINHASH_STATIC_SCRATCH_BYTES (64u << 20)
int minhash_signatures_static(const int64_t *row_ptr, const uint32_t *col_idx, int64_t n_rows,
                              int64_t nnz_upper_bound, uint64_t D, int32_t k, int32_t b, int32_t family,
                              const void *params, int64_t perm_ld,
                              uint8_t *out, int64_t out_stride,
                              int32_t *status, void *stream, uint32_t flags);

/* Bytes of device workspace a call with at most nnz_upper_bound nonzeros needs
 * (load-balancer work list plus partial minima of rows that are split across
 * wavefronts).  Returns 0 for arguments minhash_signatures would reject. */
size_t minhash_workspace_bytes(int64_t n_rows, int64_t nnz_upper_bound, int32_t k, int32_t family);

/* Host-side check that every coefficient of host_coeffs[k][deg] is below the
 * family's prime (Section 2: coefficients are drawn from {0, ..., p-1}), or, for
 * the multiply-shift families, below 2^32 with an odd multiplier (Section 3.3).
 * Returns MINHASH_OK, MINHASH_ERR_COEFF, or an argument error. */
int minhash_check_coeffs(const uint64_t *host_coeffs, int32_t k, int32_t family);

/* Waits for `stream`, then reports on the last non-empty call that used
 * `workspace`: MINHASH_ERR_WORKSPACE if row_ptr described more nonzeros than the
 * workspace was sized for (the output of that call is unspecified, nothing was
 * written outside the buffers), MINHASH_ERR_DATA if MINHASH_FLAG_VALIDATE found
 * bad input, else MINHASH_OK. */
int minhash_status(const void *workspace, void *stream);

/* The same report without waiting: enqueues on `stream` a kernel that stores the code in *status_out
 * (device, one int32), after the calls already enqueued there.  For loops that reuse one workspace for
 * many calls (Section 3.2's batch loop: every call clears what the one before reported) and look at all
 * the codes at the end.  MINHASH_ERR_ARG for a null pointer, MINHASH_ERR_HIP if the launch failed. */
int minhash_status_async(const void *workspace, int32_t *status_out, void *stream);

/* ---------------------------------------------------------------- packed index rows
 * Section 3.2's batch loop copies every chunk of sets to the GPU before hashing
 * it, and Section 3.6 finds the movement of the data dominant once the hashing
 * is fast.  Rows whose indices are sorted (non-decreasing) can cross the host
 * link as tiles of differences, about half the bytes for the heavy-tailed
 * workload, and be turned back into col_idx on the device:
 *
 *   a row of n indices is cut into tiles of 256 (the last one shorter); a tile
 *   is one 32-bit word holding its first index as it is, then the differences
 *   between neighbours inside the tile, w bits each, LSB-first in 32-bit words,
 *   the last word padded with zeros; w = width[r] is the bit length of the
 *   largest such difference of row r (0..32); word_ptr[r] is the offset of row
 *   r's first word in `words`, word_ptr[n_rows] the total.  A tile never takes
 *   more words than it has indices, so row_ptr[n_rows] - row_ptr[0] words
 *   always suffice.
 *
 * Both calls enqueue on `stream` and return without synchronising; all pointers
 * are device pointers owned by the caller.  The last kernel of a call stores
 * MINHASH_OK, MINHASH_ERR_DATA (a row is not sorted; its tiles are unspecified)
 * or MINHASH_ERR_WORKSPACE (words_capacity / words_len too small for what
 * row_ptr, width and word_ptr describe; nothing is accessed outside the
 * buffers) in *status (device, one int32, required).  row_ptr must be
 * non-decreasing. */

/* col_idx -> (width[n_rows], word_ptr[n_rows+1], words[<= words_capacity]).  With words_capacity 0 (no row
 * has an index) col_idx and words may be null; neither is then read or written. */
int minhash_pack_indices(const int64_t *row_ptr, const uint32_t *col_idx, int64_t n_rows,
                         uint32_t *width, int64_t *word_ptr, uint32_t *words, int64_t words_capacity,
                         int32_t *status, void *stream);

/* (width, word_ptr, words[words_len]) -> col_idx[row_ptr[0] .. row_ptr[n_rows]), ready for minhash_signatures. */
int minhash_unpack_indices(const int64_t *row_ptr, const uint32_t *width, const int64_t *word_ptr,
                           const uint32_t *words, int64_t words_len, int64_t n_rows,
                           uint32_t *col_idx, int32_t *status, void *stream);

/* minhash_signatures for rows that are given in the packed form above instead of as col_idx: a tile of
 * that form is what the hash kernels stage at a time, so its words are fetched in place of the indices
 * and decoded while they are staged, with no pass over the data in between.  Every argument that
 * minhash_signatures also has means the same (row_ptr still gives the rows' lengths and must start
 * the tiles where pack_indices started them: row r has row_ptr[r+1] - row_ptr[r] indices);
 * MINHASH_PERM is not served this way (MINHASH_ERR_FAMILY: unpack first).  A width above 32 or a tile
 * that would leave words[0 .. words_len) is never followed; minhash_status then reports
 * MINHASH_ERR_DATA and the rows concerned get unspecified signatures.  The workspace is sized with
 * minhash_workspace_bytes for at least row_ptr[n_rows] - row_ptr[0] nonzeros, as for minhash_signatures.
 * `words` may be null when words_len is 0 (every row empty), here and in minhash_unpack_indices. */
int minhash_signatures_packed(const int64_t *row_ptr, const uint32_t *width, const int64_t *word_ptr,
                              const uint32_t *words, int64_t words_len, int64_t n_rows,
                              uint64_t D, int32_t k, int32_t b, int32_t family, const void *params,
                              uint8_t *out, int64_t out_stride,
                              void *workspace, size_t workspace_bytes, void *stream, uint32_t flags);

/* ---------------------------------------------------------------- consumers
 * What Section 1.1 does with a signature.  `sig` is the output of
 * minhash_signatures: device, rows sig_stride bytes apart, k values of b bits.
 * All three enqueue on `stream` and return without synchronising. */

/* The 2^b x k-length binary vector with exactly k ones that a signature is
 * expanded into at run time (Section 1.1, paragraph after eq. "eqn_R_b"):
 * out_idx[i*k + j] = j*2^b + s_ij, the position of the j-th one of row i.
 * out_idx: device, n_rows*k uint32.  Needs k*2^b <= 2^32 (else MINHASH_ERR_KB). */
int minhash_expand_indices(const uint8_t *sig, int64_t n_rows, int64_t sig_stride, int32_t k, int32_t b,
                           uint32_t *out_idx, void *stream);

/* k * P_b-hat of eq. "eqn_R_b": counts[q] = number of j whose b-bit values are
 * equal in rows pairs[2q] and pairs[2q+1] (the inner product of the two expanded
 * vectors).  pairs: device, 2*n_pairs int64 row numbers; a row number outside
 * [0, n_rows) gives counts[q] = 0xFFFFFFFF.  counts: device, n_pairs uint32. */
int minhash_match_counts(const uint8_t *sig, int64_t n_rows, int64_t sig_stride, int32_t k, int32_t b,
                         const int64_t *pairs, int64_t n_pairs, uint32_t *counts, void *stream);

/* R_b-hat = (counts/k - C_{1,b}) / (1 - C_{2,b})  (eq. "eqn_R_b") with the C and A
 * terms stated with Theorem 1, from the set sizes f1[q], f2[q] >= 1 and D, in
 * double precision.  counts, f1, f2, r_hat: device, n_pairs entries each. */
int minhash_resemblance_estimates(const uint32_t *counts, const int64_t *f1, const int64_t *f2, int64_t n_pairs,
                                  uint64_t D, int32_t k, int32_t b, double *r_hat, void *stream);

/* ---------------------------------------------------------------- ingest (host only)
 * Phase 1 of the batch loop of Section 3.2: sets are read from disk before they
 * go to the GPU, and Section 3.6 finds this loading dominant once hashing is on
 * the GPU.  LibSVM text, one data vector per line: "<label> <index>:<value> ...";
 * a listed feature is a member of the set, values are ignored (binary data,
 * Section 1.1).  Blank lines and lines starting with '#' are skipped.  `text` is
 * host memory (e.g. an mmap of the file), len bytes, not necessarily
 * NUL-terminated; index_base is 1 for standard LibSVM files (written indices
 * start at 1 and are stored minus 1) or 0; the work is split over n_threads
 * host threads.  Neither function touches the GPU. */

/* Pass 1: number of rows, of nonzeros, and the largest stored index (so that the
 * caller can choose D > max_index and allocate, e.g., pinned arrays).
 * share_counts is NULL or host memory for 2*n_threads values: it receives the
 * rows and nonzeros of each thread's share of the text, which pass 2 takes back
 * so that it does not have to count again.
 * MINHASH_ERR_DATA for a malformed line or an index below index_base / above 2^32-1+index_base. */
int minhash_libsvm_count(const char *text, size_t len, int32_t index_base, int32_t n_threads,
                         int64_t *n_rows, int64_t *nnz, uint32_t *max_index, int64_t *share_counts);

/* Pass 2: fills row_ptr[n_rows+1] (offsets from 0), col_idx[nnz] (order as
 * written in the file) and, if not NULL, labels[n_rows], all host memory of the
 * sizes pass 1 returned.  share_counts is NULL (the shares are counted again) or
 * what pass 1 wrote for the same text, len, index_base and n_threads.
 * MINHASH_ERR_ARG if the sizes or share_counts do not match this text; nothing
 * is written outside the three arrays in that case either. */
int minhash_libsvm_parse(const char *text, size_t len, int32_t index_base, int32_t n_threads,
                         int64_t n_rows, int64_t nnz, const int64_t *share_counts,
                         int64_t *row_ptr, uint32_t *col_idx, float *labels);

/* Static text for a return code; never NULL. */
const char *minhash_error_string(int code);

/* Text of the HIP error behind the last MINHASH_ERR_HIP on this host thread. */
const char *minhash_last_hip_error(void);

/* MINHASH_VERSION of the loaded library. */
int minhash_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MINHASH_H */
