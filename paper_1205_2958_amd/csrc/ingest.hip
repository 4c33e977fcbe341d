// Host-side ingest: LibSVM text -> CSR of nonzero feature indices (Section 3.2,
// phase 1: sets are read from disk in chunks before they go to the GPU; Section
// 3.6 reports that this loading dominates once hashing runs on the GPU).
//
// Two passes over a caller-provided text buffer (typically an mmap of the file),
// both split over threads at line boundaries: the first counts rows and
// nonzeros so that the caller can allocate (pinned) arrays of the exact size,
// the second writes row_ptr / col_idx / labels in place.  Feature values are
// skipped: the method works on binary data, a feature that is listed is a member
// of the set.  No GPU call anywhere in this file.
//
// The scanner works on lines that end in a newline inside the buffer (a last
// line without one is copied and terminated first), so none of its loops needs
// an end pointer: each stops at the newline at the latest.  Indices and values,
// which are nearly all of the text, are handled eight or sixteen bytes at a time.
#include <stdint.h>
#include <stddef.h>
#include <string.h>

#if defined(__SSE2__)
#include <emmintrin.h>
#endif

#include <string>
#include <thread>
#include <vector>

#include "minhash.h"

namespace {

struct Chunk {
    const char* begin;
    const char* end;
    int64_t rows = 0, nnz = 0;
    uint32_t max_index = 0;
    int error = 0;
};

enum { FILL_OK = 0, FILL_BAD_DATA = 1, FILL_COUNTS_DIFFER = 2 };

inline bool is_blank(char c) { return c == ' ' || c == '\t' || c == '\r'; }
inline bool is_digit(char c) { return c >= '0' && c <= '9'; }

// splits [text, text+len) into at most n pieces that end right after a newline
std::vector<Chunk> split_lines(const char* text, size_t len, int n)
{
    std::vector<Chunk> out;
    const char* end = text + len;
    const char* p = text;
    for (int i = 0; i < n && p < end; ++i) {
        const char* q = (i == n - 1) ? end : text + (len / n) * (size_t)(i + 1);
        if (q < p) q = p;
        if (q < end) {
            const void* nl = memchr(q, '\n', (size_t)(end - q));
            q = nl ? static_cast<const char*>(nl) + 1 : end;
        }
        Chunk c;
        c.begin = p;
        c.end = q;
        out.push_back(c);
        p = q;
    }
    return out;
}

// Where the scanner may read: [.., end) holds the text; an eight-byte load is allowed at
// every p <= wide8 and a sixteen-byte load at every p <= wide16 (null when the buffer is
// shorter than that).
struct Extent {
    const char* end;
    const char* wide8;
    const char* wide16;
};

inline Extent extent_of(const char* text, size_t len)
{
    return Extent{text + len, len >= 8 ? text + len - 8 : nullptr, len >= 16 ? text + len - 16 : nullptr};
}

inline uint64_t load8(const char* p)
{
    uint64_t w;
    memcpy(&w, p, 8);
    return w;
}

// Value of the first n (1..8) bytes of w read as decimal digits.  The first character is
// the lowest byte: the bytes minus '0' are moved to the top of the word, which pads with
// leading zeros, then neighbouring digits, pairs and quadruples are combined by three
// multiply-adds.
inline uint64_t digits_value(uint64_t w, int n)
{
    uint64_t d = (w ^ 0x3030303030303030ull) << ((8 - n) * 8);
    d = (d * 10 + (d >> 8)) & 0x00FF00FF00FF00FFull;
    d = (d * 100 + (d >> 16)) & 0x0000FFFF0000FFFFull;
    return (d * 10000 + (d >> 32)) & 0xFFFFFFFFull;
}

// Decimal digits at p (at least one, else false) -> *out; advances p past them.  Values
// above 2^32 are refused, any number of leading zeros is accepted.
inline bool parse_index(const char*& p, const Extent& x, uint64_t* out)
{
    uint64_t idx = 0;
    const char* q = p;
    if (x.wide8 && q <= x.wide8) {
        const uint64_t w = load8(q);
        const uint64_t d = w ^ 0x3030303030303030ull;
        // a byte that is not 0..9 has a high nibble, now or after adding 6
        const uint64_t other = ((d + 0x0606060606060606ull) | d) & 0xF0F0F0F0F0F0F0F0ull;
        const int n = other ? (__builtin_ctzll(other) >> 3) : 8;
        if (n == 0) return false;
        idx = digits_value(w, n);
        q += n;
    }
    const char* first = q;
    while (is_digit(*q)) {                                                 // beyond eight digits, or near the buffer's end
        idx = idx * 10 + (uint64_t)(*q - '0');
        if (idx > 0xFFFFFFFFull + 1) return false;
        ++q;
    }
    if (q == first && q == p) return false;
    p = q;
    *out = idx;
    return true;
}

#if defined(__SSE2__)
// The common entry "<1..8 digits>:<value><space>" inside one sixteen-byte window: returns
// the position after the space and the index, or nullptr when the window does not hold
// such an entry (the caller then takes the general path).  The next position depends only
// on the first byte below 0x21 in the window, so consecutive entries chain through one
// load, two vector operations and one bit scan; that this byte is a space, the digits and
// the colon are checked off that chain, by branches that are nearly always taken one way.
inline const char* entry_in_window(const char* p, const Extent& x, uint64_t* out)
{
    if (!x.wide16 || p > x.wide16) return nullptr;
    const __m128i v = _mm_loadu_si128(reinterpret_cast<const __m128i*>(p));
    const unsigned low = (unsigned)_mm_movemask_epi8(_mm_cmpeq_epi8(_mm_min_epu8(v, _mm_set1_epi8(0x20)), v));
    const unsigned space = (unsigned)_mm_movemask_epi8(_mm_cmpeq_epi8(v, _mm_set1_epi8(' ')));
    if (!low || ((low ^ (low - 1)) & space) == 0) return nullptr;          // lowest set bit of low is not a space
    const __m128i t = _mm_sub_epi8(v, _mm_set1_epi8('0'));
    const unsigned other = (unsigned)_mm_movemask_epi8(_mm_cmpeq_epi8(_mm_max_epu8(t, _mm_set1_epi8(10)), t));
    const int n = __builtin_ctz(other | 0x10000u);                         // leading digits in the window
    if (n == 0 || n > 8 || p[n] != ':') return nullptr;
    *out = digits_value(load8(p), n);
    return p + __builtin_ctz(low) + 1;
}
#else
inline const char* entry_in_window(const char*, const Extent&, uint64_t*) { return nullptr; }
#endif

// First blank or newline at or after p: the end of a value, which is not interpreted.
inline const char* skip_value(const char* p, const Extent& x)
{
    for (;;) {
        if (x.wide8 && p <= x.wide8) {
            const uint64_t w = load8(p);
            const uint64_t low = (w - 0x2121212121212121ull) & ~w & 0x8080808080808080ull;   // first hit: a byte below 0x21
            if (!low) { p += 8; continue; }
            p += __builtin_ctzll(low) >> 3;
        } else {
            while ((unsigned char)*p > ' ') ++p;
        }
        if (is_blank(*p) || *p == '\n') return p;
        ++p;                                                               // another control character: part of the value
    }
}

inline const char* after_newline(const char* p, const Extent& x)
{
    return static_cast<const char*>(memchr(p, '\n', (size_t)(x.end - p))) + 1;
}

// One line: "<label> <index>:<value> <index>:<value> ... [# comment]", ending in '\n' before x.end.
// Calls on_index for every index.  Returns a pointer past the newline, or nullptr on a malformed line.
template <class F>
inline const char* parse_line(const char* p, const Extent& x, bool* has_row, float* label, F on_index)
{
    while (is_blank(*p)) ++p;
    if (*p == '\n') { *has_row = false; return p + 1; }                    // blank line: not a row
    if (*p == '#') { *has_row = false; return after_newline(p, x); }       // comment line: not a row
    *has_row = true;
    // label: sign, digits, optional fraction (only the leading number is interpreted)
    {
        double sign = 1.0, v = 0.0;
        if (*p == '+' || *p == '-') { if (*p == '-') sign = -1.0; ++p; }
        bool any = false;
        while (is_digit(*p)) { v = v * 10.0 + (*p - '0'); ++p; any = true; }
        if (*p == '.') {
            ++p;
            double scale = 0.1;
            while (is_digit(*p)) { v += (*p - '0') * scale; scale *= 0.1; ++p; any = true; }
        }
        if (!any) return nullptr;
        while (!is_blank(*p) && *p != '\n') ++p;                           // exponent or anything else glued to the label
        if (label) *label = (float)(sign * v);
        if (*p == ' ') ++p;
    }
    for (;;) {
        uint64_t idx;
        while (const char* q = entry_in_window(p, x, &idx)) {              // runs of common entries
            p = q;
            if (!on_index(idx)) return nullptr;
        }
        while (is_blank(*p)) ++p;
        if (*p == '\n') return p + 1;
        if (*p == '#') return after_newline(p, x);
        if (!parse_index(p, x, &idx) || *p != ':') return nullptr;         // need "<digits>:"
        p = skip_value(p + 1, x);
        if (*p == ' ') ++p;                                                // so that the next entry can start a run
        if (!on_index(idx)) return nullptr;
    }
}

// Runs per_line(p, extent) -> next over every line of [begin, end); a last line without a
// newline is copied, terminated and padded so that the scanner's assumptions hold for it too.
template <class L>
inline bool for_each_line(const char* begin, const char* end, const Extent& x, L per_line)
{
    const char* last_nl = begin < end ? static_cast<const char*>(memrchr(begin, '\n', (size_t)(end - begin))) : nullptr;
    const char* closed = last_nl ? last_nl + 1 : begin;                    // lines before this end in a newline
    const char* p = begin;
    while (p < closed) {
        p = per_line(p, x);
        if (!p) return false;
    }
    if (closed < end) {
        std::string tail(closed, (size_t)(end - closed));
        tail.append("\n\0\0\0\0\0\0\0\0\0\0\0\0\0\0\0\0", 17);
        const Extent tx = extent_of(tail.data(), tail.size());
        if (!per_line(tail.data(), tx)) return false;
    }
    return true;
}

void count_chunk(Chunk* c, uint32_t base, Extent x)
{
    const bool ok = for_each_line(c->begin, c->end, x, [&](const char* p, const Extent& ex) {
        bool has_row = false;
        int64_t n = 0;
        uint32_t mx = c->max_index;
        const char* next = parse_line(p, ex, &has_row, nullptr, [&](uint64_t idx) {
            if (idx < base || idx - base > 0xFFFFFFFFull) return false;
            const uint32_t t = (uint32_t)(idx - base);
            if (t > mx) mx = t;
            ++n;
            return true;
        });
        if (next && has_row) { ++c->rows; c->nnz += n; c->max_index = mx; }
        return next;
    });
    if (!ok) c->error = 1;
}

// Writes the rows of one chunk at [row0, row1) and their indices at [nnz0, nnz1).  The limits
// come from a count that may have been taken earlier: a text that does not produce exactly
// these counts is reported, and nothing is written outside the two ranges.
void fill_chunk(const Chunk* c, uint32_t base, Extent x, int64_t row0, int64_t row1, int64_t nnz0, int64_t nnz1,
                int64_t* row_ptr, uint32_t* col_idx, float* labels, int* status)
{
    int64_t row = row0, at = nnz0;
    bool overrun = false;
    const bool ok = for_each_line(c->begin, c->end, x, [&](const char* p, const Extent& ex) {
        bool has_row = false;
        float label = 0.0f;
        const int64_t start = at;
        const char* next = parse_line(p, ex, &has_row, &label, [&](uint64_t idx) {
            if (at >= nnz1) { overrun = true; return false; }
            col_idx[at++] = (uint32_t)(idx - base);
            return true;
        });
        if (!next) return next;
        if (has_row) {
            if (row >= row1) { overrun = true; return (const char*)nullptr; }
            row_ptr[row] = start;
            if (labels) labels[row] = label;
            ++row;
        } else {
            at = start;
        }
        return next;
    });
    if (overrun) *status = FILL_COUNTS_DIFFER;
    else if (!ok) *status = FILL_BAD_DATA;
    else *status = (row == row1 && at == nnz1) ? FILL_OK : FILL_COUNTS_DIFFER;
}

int clamp_threads(int32_t n_threads, size_t len)
{
    int n = n_threads < 1 ? 1 : (n_threads > 256 ? 256 : n_threads);
    size_t by_size = len / (1u << 16) + 1;                                // at least 64 KiB of text per thread
    return (size_t)n > by_size ? (int)by_size : n;
}

void count_all(std::vector<Chunk>& chunks, uint32_t base, Extent x)
{
    std::vector<std::thread> pool;
    for (size_t i = 1; i < chunks.size(); ++i) pool.emplace_back(count_chunk, &chunks[i], base, x);
    if (!chunks.empty()) count_chunk(&chunks[0], base, x);
    for (auto& t : pool) t.join();
}

}  // namespace

extern "C" {

int minhash_libsvm_count(const char* text, size_t len, int32_t index_base, int32_t n_threads, int64_t* n_rows,
                         int64_t* nnz, uint32_t* max_index, int64_t* share_counts)
{
    if ((!text && len) || !n_rows || !nnz || index_base < 0 || index_base > 1) return MINHASH_ERR_ARG;
    if (share_counts && n_threads < 1) return MINHASH_ERR_ARG;
    std::vector<Chunk> chunks = split_lines(text, len, clamp_threads(n_threads, len));
    count_all(chunks, (uint32_t)index_base, extent_of(text, len));
    int64_t rows = 0, total = 0;
    uint32_t mx = 0;
    for (const Chunk& c : chunks) {
        if (c.error) return MINHASH_ERR_DATA;
        rows += c.rows;
        total += c.nnz;
        if (c.max_index > mx) mx = c.max_index;
    }
    if (share_counts) {
        for (int32_t i = 0; i < n_threads; ++i) {
            const bool used = (size_t)i < chunks.size();
            share_counts[2 * i] = used ? chunks[(size_t)i].rows : 0;
            share_counts[2 * i + 1] = used ? chunks[(size_t)i].nnz : 0;
        }
    }
    *n_rows = rows;
    *nnz = total;
    if (max_index) *max_index = mx;
    return MINHASH_OK;
}

int minhash_libsvm_parse(const char* text, size_t len, int32_t index_base, int32_t n_threads, int64_t n_rows,
                         int64_t nnz, const int64_t* share_counts, int64_t* row_ptr, uint32_t* col_idx, float* labels)
{
    if ((!text && len) || !row_ptr || (!col_idx && nnz) || n_rows < 0 || nnz < 0 || index_base < 0 || index_base > 1)
        return MINHASH_ERR_ARG;
    if (share_counts && n_threads < 1) return MINHASH_ERR_ARG;
    const Extent x = extent_of(text, len);
    std::vector<Chunk> chunks = split_lines(text, len, clamp_threads(n_threads, len));
    if (share_counts) {
        if (chunks.size() > (size_t)n_threads) return MINHASH_ERR_ARG;
        for (size_t i = 0; i < chunks.size(); ++i) {
            chunks[i].rows = share_counts[2 * i];
            chunks[i].nnz = share_counts[2 * i + 1];
            if (chunks[i].rows < 0 || chunks[i].nnz < 0) return MINHASH_ERR_ARG;
        }
    } else {
        count_all(chunks, (uint32_t)index_base, x);       // every share has to know where it writes
    }
    std::vector<int64_t> row0(chunks.size() + 1, 0), nnz0(chunks.size() + 1, 0);
    for (size_t i = 0; i < chunks.size(); ++i) {
        if (chunks[i].error) return MINHASH_ERR_DATA;
        if (chunks[i].rows > n_rows - row0[i] || chunks[i].nnz > nnz - nnz0[i]) return MINHASH_ERR_ARG;
        row0[i + 1] = row0[i] + chunks[i].rows;
        nnz0[i + 1] = nnz0[i] + chunks[i].nnz;
    }
    if (row0[chunks.size()] != n_rows || nnz0[chunks.size()] != nnz) return MINHASH_ERR_ARG;   // sizes from another buffer
    std::vector<int> status(chunks.size(), FILL_OK);
    std::vector<std::thread> pool;
    for (size_t i = 1; i < chunks.size(); ++i)
        pool.emplace_back(fill_chunk, &chunks[i], (uint32_t)index_base, x, row0[i], row0[i + 1], nnz0[i], nnz0[i + 1],
                          row_ptr, col_idx, labels, &status[i]);
    if (!chunks.empty())
        fill_chunk(&chunks[0], (uint32_t)index_base, x, row0[0], row0[1], nnz0[0], nnz0[1], row_ptr, col_idx, labels,
                   &status[0]);
    for (auto& t : pool) t.join();
    for (int e : status)
        if (e == FILL_BAD_DATA) return MINHASH_ERR_DATA;
    for (int e : status)
        if (e == FILL_COUNTS_DIFFER) return MINHASH_ERR_ARG;
    row_ptr[n_rows] = nnz;
    return MINHASH_OK;
}

}  // extern "C"
