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
#include <stdint.h>
#include <stddef.h>
#include <string.h>

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

inline bool is_space(char c) { return c == ' ' || c == '\t' || c == '\r'; }

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

// One line: "<label> <index>:<value> <index>:<value> ... [# comment]".  Calls on_index for every index.
// Returns a pointer past the line's newline (or end), or nullptr on a malformed line.
template <class F>
inline const char* parse_line(const char* p, const char* end, bool* has_row, float* label, F on_index)
{
    const char* eol = static_cast<const char*>(memchr(p, '\n', (size_t)(end - p)));
    const char* stop = eol ? eol : end;
    const char* next = eol ? eol + 1 : end;
    while (p < stop && is_space(*p)) ++p;
    if (p == stop || *p == '#') { *has_row = false; return next; }      // blank or comment line: not a row
    *has_row = true;
    // label: sign, digits, optional fraction / exponent (only the leading number is interpreted)
    {
        const char* q = p;
        double sign = 1.0, v = 0.0;
        if (q < stop && (*q == '+' || *q == '-')) { if (*q == '-') sign = -1.0; ++q; }
        bool any = false;
        while (q < stop && *q >= '0' && *q <= '9') { v = v * 10.0 + (*q - '0'); ++q; any = true; }
        if (q < stop && *q == '.') {
            ++q;
            double scale = 0.1;
            while (q < stop && *q >= '0' && *q <= '9') { v += (*q - '0') * scale; scale *= 0.1; ++q; any = true; }
        }
        if (!any) return nullptr;
        while (q < stop && !is_space(*q)) ++q;                            // exponent or anything else glued to the label
        if (label) *label = (float)(sign * v);
        p = q;
    }
    for (;;) {
        while (p < stop && is_space(*p)) ++p;
        if (p == stop || *p == '#') return next;
        uint64_t idx = 0;
        const char* q = p;
        while (q < stop && *q >= '0' && *q <= '9') { idx = idx * 10 + (uint64_t)(*q - '0'); if (idx > 0xFFFFFFFFull + 1) return nullptr; ++q; }
        if (q == p || q == stop || *q != ':') return nullptr;             // need "<digits>:"
        ++q;
        while (q < stop && !is_space(*q)) ++q;                            // the value is skipped
        if (!on_index(idx)) return nullptr;
        p = q;
    }
}

void count_chunk(Chunk* c, uint32_t base)
{
    const char* p = c->begin;
    while (p < c->end) {
        bool has_row = false;
        int64_t n = 0;
        uint32_t mx = c->max_index;
        const char* next = parse_line(p, c->end, &has_row, nullptr, [&](uint64_t idx) {
            if (idx < base || idx - base > 0xFFFFFFFFull) return false;
            uint32_t t = (uint32_t)(idx - base);
            if (t > mx) mx = t;
            ++n;
            return true;
        });
        if (!next) { c->error = 1; return; }
        if (has_row) { ++c->rows; c->nnz += n; c->max_index = mx; }
        p = next;
    }
}

void fill_chunk(const Chunk* c, uint32_t base, int64_t row0, int64_t nnz0, int64_t* row_ptr, uint32_t* col_idx,
                float* labels, int* error)
{
    const char* p = c->begin;
    int64_t row = row0, at = nnz0;
    while (p < c->end) {
        bool has_row = false;
        float label = 0.0f;
        const int64_t start = at;
        const char* next = parse_line(p, c->end, &has_row, &label, [&](uint64_t idx) {
            col_idx[at++] = (uint32_t)(idx - base);
            return true;
        });
        if (!next) { *error = 1; return; }
        if (has_row) {
            row_ptr[row] = start;
            if (labels) labels[row] = label;
            ++row;
        } else {
            at = start;
        }
        p = next;
    }
}

int clamp_threads(int32_t n_threads, size_t len)
{
    int n = n_threads < 1 ? 1 : (n_threads > 256 ? 256 : n_threads);
    size_t by_size = len / (1u << 16) + 1;                                // at least 64 KiB of text per thread
    return (size_t)n > by_size ? (int)by_size : n;
}

}  // namespace

extern "C" {

int minhash_libsvm_count(const char* text, size_t len, int32_t index_base, int32_t n_threads, int64_t* n_rows,
                         int64_t* nnz, uint32_t* max_index)
{
    if ((!text && len) || !n_rows || !nnz || index_base < 0 || index_base > 1) return MINHASH_ERR_ARG;
    std::vector<Chunk> chunks = split_lines(text, len, clamp_threads(n_threads, len));
    std::vector<std::thread> pool;
    for (size_t i = 1; i < chunks.size(); ++i) pool.emplace_back(count_chunk, &chunks[i], (uint32_t)index_base);
    if (!chunks.empty()) count_chunk(&chunks[0], (uint32_t)index_base);
    for (auto& t : pool) t.join();
    int64_t rows = 0, total = 0;
    uint32_t mx = 0;
    for (const Chunk& c : chunks) {
        if (c.error) return MINHASH_ERR_DATA;
        rows += c.rows;
        total += c.nnz;
        if (c.max_index > mx) mx = c.max_index;
    }
    *n_rows = rows;
    *nnz = total;
    if (max_index) *max_index = mx;
    return MINHASH_OK;
}

int minhash_libsvm_parse(const char* text, size_t len, int32_t index_base, int32_t n_threads, int64_t n_rows,
                         int64_t nnz, int64_t* row_ptr, uint32_t* col_idx, float* labels)
{
    if ((!text && len) || !row_ptr || (!col_idx && nnz) || n_rows < 0 || nnz < 0 || index_base < 0 || index_base > 1)
        return MINHASH_ERR_ARG;
    std::vector<Chunk> chunks = split_lines(text, len, clamp_threads(n_threads, len));
    {   // counts again per chunk (cheap next to the fill) so that every chunk knows where it writes
        std::vector<std::thread> pool;
        for (size_t i = 1; i < chunks.size(); ++i) pool.emplace_back(count_chunk, &chunks[i], (uint32_t)index_base);
        if (!chunks.empty()) count_chunk(&chunks[0], (uint32_t)index_base);
        for (auto& t : pool) t.join();
    }
    std::vector<int64_t> row0(chunks.size() + 1, 0), nnz0(chunks.size() + 1, 0);
    for (size_t i = 0; i < chunks.size(); ++i) {
        if (chunks[i].error) return MINHASH_ERR_DATA;
        row0[i + 1] = row0[i] + chunks[i].rows;
        nnz0[i + 1] = nnz0[i] + chunks[i].nnz;
    }
    if (row0[chunks.size()] != n_rows || nnz0[chunks.size()] != nnz) return MINHASH_ERR_ARG;   // sizes from another buffer
    std::vector<int> errors(chunks.size(), 0);
    std::vector<std::thread> pool;
    for (size_t i = 1; i < chunks.size(); ++i)
        pool.emplace_back(fill_chunk, &chunks[i], (uint32_t)index_base, row0[i], nnz0[i], row_ptr, col_idx, labels, &errors[i]);
    if (!chunks.empty()) fill_chunk(&chunks[0], (uint32_t)index_base, row0[0], nnz0[0], row_ptr, col_idx, labels, &errors[0]);
    for (auto& t : pool) t.join();
    for (int e : errors)
        if (e) return MINHASH_ERR_DATA;
    row_ptr[n_rows] = nnz;
    return MINHASH_OK;
}

}  // extern "C"
