// Packed index rows: a denser form of col_idx for the trip over PCIe.
//
// Section 3.2's batch loop copies a chunk of sets to the GPU, hashes it there and
// copies the results back; Section 3.6 finds that once the hashing is fast the
// movement of the data dominates.  On this GPU the 2U kernels consume indices
// faster than the host link delivers them as 32-bit words, so sorted rows can be
// sent as tiles of differences instead:
//
//   a row of n indices, non-decreasing, is cut into tiles of 256 (the last one
//   shorter).  A tile is one 32-bit word holding its first index as it is,
//   followed by the differences between neighbours inside the tile, each w bits
//   wide, packed LSB-first into 32-bit words, the last word padded with zeros.
//   w is one number per row: the bit length of the largest such difference in
//   the row (0 when all are 0 or the row has one index per tile; at most 32).
//   word_ptr[r] is the offset of row r's first word, word_ptr[n_rows] the total.
//
// A tile never needs more words than it has indices, so nnz words always suffice.
// Tiles are independent, which is what lets any number of wavefronts decode one
// long row.  minhash_pack_indices builds the form on the device (three kernels:
// widths, offsets, words); minhash_unpack_indices turns it back into the
// col_idx array that minhash_signatures takes.  Both walk the index array in
// spans of 4 096 positions, one wavefront per span: the tiles that start inside a
// span are that wavefront's, whichever rows they belong to.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "minhash.h"
#include "mh_arith.h"
#include "mh_host.h"

namespace {

constexpr int WAVE = 64;
constexpr int BLOCK = 256;
constexpr int WAVES_PER_BLOCK = BLOCK / WAVE;
constexpr uint32_t PK_TILE = mh::PACKED_TILE;
constexpr int64_t SPAN = 4096;

__host__ __device__ inline uint32_t tile_words(uint32_t m, uint32_t w) { return mh::packed_tile_words(m, w); }
__host__ __device__ inline uint64_t row_words(uint64_t n, uint32_t w)
{
    const uint64_t full = n / PK_TILE;
    const uint32_t rem = (uint32_t)(n % PK_TILE);
    return full * tile_words(PK_TILE, w) + (rem ? tile_words(rem, w) : 0u);
}

__device__ __forceinline__ void wave_sync_lds()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
__device__ __forceinline__ uint32_t uniform(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }

// Calls f(row, tile number in the row, position of the tile's first index, indices in the tile)
// for every tile that starts inside this wavefront's spans.  All arguments are wavefront-uniform.
template <class F>
__device__ __forceinline__ void for_each_tile(const int64_t* row_ptr, int64_t n_rows, F f)
{
    const int64_t first = row_ptr[0], last = row_ptr[n_rows];
    const int64_t n_waves = (int64_t)gridDim.x * WAVES_PER_BLOCK;
    const int64_t wave = (int64_t)blockIdx.x * WAVES_PER_BLOCK + (threadIdx.x >> 6);
    for (int64_t p0 = first + wave * SPAN; p0 < last; p0 += n_waves * SPAN) {
        const int64_t p1 = p0 + SPAN < last ? p0 + SPAN : last;
        // the row that holds position p0: the last r with row_ptr[r] <= p0 (rows before it that are empty do not matter)
        int64_t lo = 0, hi = n_rows;                 // row_ptr[lo] <= p0 < row_ptr[hi]
        while (hi - lo > 1) {
            const int64_t mid = lo + (hi - lo) / 2;
            if (row_ptr[mid] <= p0) lo = mid; else hi = mid;
        }
        int64_t r = lo;
        int64_t begin = row_ptr[r], end = row_ptr[r + 1];
        int64_t t = (p0 - begin + (int64_t)PK_TILE - 1) / (int64_t)PK_TILE;       // first tile of the row that starts at or after p0
        int64_t s = begin + t * (int64_t)PK_TILE;
        for (;;) {
            while (s >= end && r + 1 < n_rows) {     // on to the next row that has indices
                ++r;
                begin = end;
                end = row_ptr[r + 1];
                s = begin;
                t = 0;
            }
            if (s >= end || s >= p1) break;
            const uint32_t m = end - s < (int64_t)PK_TILE ? (uint32_t)(end - s) : PK_TILE;
            f(r, t, s, m);
            s += PK_TILE;
            ++t;
        }
    }
}

__device__ __forceinline__ uint32_t bit_length(uint32_t v) { return v ? 32u - (uint32_t)__builtin_clz(v) : 0u; }

// status bits: 1 = a row is not sorted, 2 = the word buffer is too small / an offset leaves it
__global__ __launch_bounds__(BLOCK) void pk_width_kernel(const int64_t* row_ptr, const uint32_t* col, int64_t n_rows, uint32_t* width,
                                                         uint32_t* status)
{
    const int lane = threadIdx.x & (WAVE - 1);
    for_each_tile(row_ptr, n_rows, [&](int64_t r, int64_t, int64_t s, uint32_t m) {
        uint32_t widest = 0, unsorted = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t i = (uint32_t)lane + (uint32_t)(WAVE * q);            // index in the tile
            if (i >= 1 && i < m) {
                const uint32_t a = col[s + i - 1], b = col[s + i];
                if (b < a) unsorted = 1;
                const uint32_t d = b - a;
                widest = d > widest ? d : widest;
            }
        }
        for (int d = 32; d >= 1; d >>= 1) {
            const uint32_t o = (uint32_t)__shfl_xor((int)widest, d, WAVE);
            widest = o > widest ? o : widest;
            unsorted |= (uint32_t)__shfl_xor((int)unsorted, d, WAVE);
        }
        if (lane == 0) {
            if (widest) atomicMax(&width[r], bit_length(widest));
            if (unsorted) atomicOr(status, 1u);
        }
    });
}

// word_ptr = exclusive prefix sums of the rows' word counts; one block
constexpr int SCAN_BLOCK = 1024;
__global__ __launch_bounds__(SCAN_BLOCK) void pk_offsets_kernel(const int64_t* row_ptr, const uint32_t* width, int64_t n_rows,
                                                                int64_t* word_ptr)
{
    __shared__ unsigned long long s_sum[SCAN_BLOCK];
    const int64_t per = (n_rows + SCAN_BLOCK - 1) / SCAN_BLOCK;
    const int64_t r0 = (int64_t)threadIdx.x * per, r1 = r0 + per < n_rows ? r0 + per : n_rows;
    unsigned long long mine = 0;
    for (int64_t r = r0; r < r1; ++r) mine += row_words((uint64_t)(row_ptr[r + 1] - row_ptr[r]), width[r]);
    s_sum[threadIdx.x] = mine;
    __syncthreads();
    for (int d = 1; d < SCAN_BLOCK; d <<= 1) {       // inclusive scan of the per-thread sums
        unsigned long long v = threadIdx.x >= (unsigned)d ? s_sum[threadIdx.x - d] : 0ull;
        __syncthreads();
        s_sum[threadIdx.x] += v;
        __syncthreads();
    }
    unsigned long long run = s_sum[threadIdx.x] - mine;
    for (int64_t r = r0; r < r1; ++r) {
        word_ptr[r] = (int64_t)run;
        run += row_words((uint64_t)(row_ptr[r + 1] - row_ptr[r]), width[r]);
    }
    if (threadIdx.x == SCAN_BLOCK - 1) word_ptr[n_rows] = (int64_t)s_sum[SCAN_BLOCK - 1];
}

__global__ __launch_bounds__(BLOCK) void pk_pack_kernel(const int64_t* row_ptr, const uint32_t* col, int64_t n_rows, const uint32_t* width,
                                                        const int64_t* word_ptr, uint32_t* words, int64_t capacity, uint32_t* status)
{
    __shared__ uint32_t s_words[WAVES_PER_BLOCK][PK_TILE + 1];
    const int lane = threadIdx.x & (WAVE - 1);
    uint32_t* buf = s_words[threadIdx.x >> 6];
    for_each_tile(row_ptr, n_rows, [&](int64_t r, int64_t t, int64_t s, uint32_t m) {
        const uint32_t w = uniform(width[r]);
        const uint32_t nw = tile_words(m, w);
        const int64_t at = word_ptr[r] + t * (int64_t)tile_words(PK_TILE, w);
        if (w > 32u || at < 0 || at + nw > capacity) {
            if (lane == 0) atomicOr(status, 2u);
            return;
        }
        for (uint32_t j = lane; j <= PK_TILE; j += WAVE) buf[j] = 0;
        wave_sync_lds();
        if (lane == 0) buf[0] = col[s];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t i = (uint32_t)lane + (uint32_t)(WAVE * q);
            if (i >= 1 && i < m && w > 0) {
                const uint32_t d = col[s + i] - col[s + i - 1];
                const uint32_t bit = (i - 1u) * w, j = 1u + (bit >> 5), sh = bit & 31u;
                atomicOr(&buf[j], d << sh);
                if (sh + w > 32u) atomicOr(&buf[j + 1], d >> (32u - sh));
            }
        }
        wave_sync_lds();
        for (uint32_t j = lane; j < nw; j += WAVE) words[at + j] = buf[j];
        wave_sync_lds();
    });
}

__global__ __launch_bounds__(BLOCK) void pk_unpack_kernel(const int64_t* row_ptr, const uint32_t* width, const int64_t* word_ptr,
                                                          const uint32_t* words, int64_t words_len, int64_t n_rows, uint32_t* col,
                                                          uint32_t* status)
{
    __shared__ uint32_t s_words[WAVES_PER_BLOCK][PK_TILE + 1];
    const int lane = threadIdx.x & (WAVE - 1);
    uint32_t* buf = s_words[threadIdx.x >> 6];
    for_each_tile(row_ptr, n_rows, [&](int64_t r, int64_t t, int64_t s, uint32_t m) {
        const uint32_t w = uniform(width[r]);
        const uint32_t nw = tile_words(m, w);
        const int64_t at = word_ptr[r] + t * (int64_t)tile_words(PK_TILE, w);
        if (w > 32u || at < 0 || at + nw > words_len) {       // an offset or width that does not fit the buffer: nothing is read
            if (lane == 0) atomicOr(status, 2u);
            return;
        }
        for (uint32_t j = lane; j < nw; j += WAVE) buf[j] = words[at + j];
        if (lane == 0) buf[nw] = 0;                            // the word a field at the very end may reach into
        wave_sync_lds();
        // lane l takes indices 4l .. 4l+3 of the tile: its own running sums first, then the sums of the lanes below
        const uint32_t mask = w >= 32u ? 0xFFFFFFFFu : (1u << w) - 1u;
        uint32_t v[4];
        uint32_t run = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t i = 4u * (uint32_t)lane + (uint32_t)q;
            uint32_t d = 0;
            if (i == 0) {
                d = buf[0];
            } else if (i < m && w > 0) {
                const uint32_t bit = (i - 1u) * w, j = 1u + (bit >> 5), sh = bit & 31u;
                const uint64_t two = ((uint64_t)buf[j + 1] << 32) | buf[j];
                d = (uint32_t)(two >> sh) & mask;
            }
            run += d;
            v[q] = run;
        }
        uint32_t below = run;                                  // inclusive scan of the lanes' totals
        for (int d = 1; d < WAVE; d <<= 1) {
            const uint32_t o = (uint32_t)__shfl_up((int)below, d, WAVE);
            if (lane >= d) below += o;
        }
        below -= run;
        // through the LDS once more, so that neighbouring lanes store neighbouring indices
        wave_sync_lds();
#pragma unroll
        for (int q = 0; q < 4; ++q) buf[4 * lane + q] = below + v[q];
        wave_sync_lds();
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t i = (uint32_t)lane + (uint32_t)(WAVE * q);
            if (i < m) __builtin_nontemporal_store(buf[i], col + s + i);
        }
        wave_sync_lds();
    });
}

__global__ void pk_fill_kernel(uint32_t* p, int64_t n, uint32_t value)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = value;
}
__global__ void pk_export_status_kernel(const uint32_t* flags, int32_t* status_out)
{
    const uint32_t f = *flags;
    *status_out = (f & 2u) ? MINHASH_ERR_WORKSPACE : (f & 1u) ? MINHASH_ERR_DATA : MINHASH_OK;
}

int grid_blocks()
{
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256 * 8;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
    return cus * 8;
}

}  // namespace

extern "C" {

int minhash_pack_indices(const int64_t* row_ptr, const uint32_t* col_idx, int64_t n_rows, uint32_t* width, int64_t* word_ptr,
                         uint32_t* words, int64_t words_capacity, int32_t* status, void* stream)
{
    if (n_rows < 0 || n_rows >= (1ll << 31) || words_capacity < 0) return MINHASH_ERR_ARG;
    // without capacity there are no indices to pack (anything else is reported by the kernels): col_idx and words may then be null
    if (!row_ptr || !word_ptr || !status || (n_rows > 0 && (!width || (words_capacity > 0 && (!col_idx || !words))))) return MINHASH_ERR_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    (void)hipGetLastError();
    uint32_t* flags = reinterpret_cast<uint32_t*>(status);     // the status word doubles as the flag word until the last kernel
    hipLaunchKernelGGL(pk_fill_kernel, dim3(1), dim3(64), 0, s, flags, (int64_t)1, 0u);
    if (n_rows > 0) {
        const int blocks = grid_blocks();
        hipLaunchKernelGGL(pk_fill_kernel, dim3(blocks), dim3(BLOCK), 0, s, width, n_rows, 0u);
        if (words_capacity > 0)       // (with no capacity every tile is reported by the packing kernel before it reads an index)
            hipLaunchKernelGGL(pk_width_kernel, dim3(blocks), dim3(BLOCK), 0, s, row_ptr, col_idx, n_rows, width, flags);
        hipLaunchKernelGGL(pk_offsets_kernel, dim3(1), dim3(SCAN_BLOCK), 0, s, row_ptr, width, n_rows, word_ptr);
        hipLaunchKernelGGL(pk_pack_kernel, dim3(blocks), dim3(BLOCK), 0, s, row_ptr, col_idx, n_rows, width, word_ptr, words,
                           words_capacity, flags);
    } else {
        hipLaunchKernelGGL(pk_fill_kernel, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(word_ptr), (int64_t)2, 0u);
    }
    hipLaunchKernelGGL(pk_export_status_kernel, dim3(1), dim3(1), 0, s, flags, status);
    return mh::launches_ok();
}

int minhash_unpack_indices(const int64_t* row_ptr, const uint32_t* width, const int64_t* word_ptr, const uint32_t* words,
                           int64_t words_len, int64_t n_rows, uint32_t* col_idx, int32_t* status, void* stream)
{
    if (n_rows < 0 || n_rows >= (1ll << 31) || words_len < 0) return MINHASH_ERR_ARG;
    if (!row_ptr || !status || (n_rows > 0 && (!width || !word_ptr || (!words && words_len > 0) || !col_idx))) return MINHASH_ERR_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    (void)hipGetLastError();
    uint32_t* flags = reinterpret_cast<uint32_t*>(status);
    hipLaunchKernelGGL(pk_fill_kernel, dim3(1), dim3(64), 0, s, flags, (int64_t)1, 0u);
    if (n_rows > 0)
        hipLaunchKernelGGL(pk_unpack_kernel, dim3(grid_blocks()), dim3(BLOCK), 0, s, row_ptr, width, word_ptr, words, words_len, n_rows,
                           col_idx, flags);
    hipLaunchKernelGGL(pk_export_status_kernel, dim3(1), dim3(1), 0, s, flags, status);
    return mh::launches_ok();
}

}  // extern "C"
