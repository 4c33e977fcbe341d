// b-bit minwise-hash signatures on MI355X (gfx950): kernels and the C ABI.
//
// One call of minhash_signatures enqueues, on the caller's stream:
//
//   mh_reset_kernel      clears the work-list header in the workspace and picks
//                        the chunk size of this call from the batch's size (a
//                        batch of up to 1 024 rows does this inside the next
//                        kernel, without atomics)
//   mh_bin_rows_kernel   load balancer: reads row_ptr, emits one work item per
//                        row, or one per chunk of nonzeros for long rows (each
//                        chunk gets a vector of k partial minima in the
//                        workspace); long items are listed first
//   mh_hash_kernel<..>   (hash families) or mh_perm_kernel<..> (permutation
//                        table): the hot loop.  Persistent wavefronts take
//                        (item, function-tile) units: their own grid index
//                        first, then tickets from an atomic counter.
//                        A wavefront stages 256 nonzeros at a time into LDS
//                        with coalesced loads (pre-computing what depends on t
//                        alone), then every lane evaluates its 8 hash functions
//                        on each staged nonzero, read back as LDS broadcasts,
//                        keeping 8 running minima in registers (Section 2, last
//                        paragraph: map every nonzero t to h_j(t), keep the
//                        minimum); for power-of-two D the running values are
//                        maxima of order-preserving keys for the complement of
//                        h_j(t), turned into the minimum once per row, and the
//                        rare values such a key cannot vouch for are computed
//                        again from the exact arithmetic before they are
//                        stored.  When k needs fewer than 64 lanes the spare
//                        lanes take slices of the nonzeros and are merged by
//                        cross-lane minima (lane swap, swizzle, row shifts).  Whole rows are
//                        truncated to b bits, packed and stored by the same
//                        wavefront; a chunk of a split row stores its k
//                        partial minima with plain coalesced stores.
//   mh_finalize_kernel   takes the minimum over the chunks of every split row
//                        (exact: the minimum over a union is the minimum of the
//                        minima of the parts), truncates, packs and stores.
//
// In the hash and table kernels wavefronts never synchronise with each other:
// each has its own LDS region and its own work units.  (The row-binning kernel's
// blocks and the blocks of the finalize kernel that share a row of many chunks
// do use block barriers.)
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include <atomic>
#include <mutex>
#include <type_traits>

#include "minhash.h"
#include "mh_arith.h"
#include "mh_host.h"

// Work space of minhash_signatures_static: one copy per GPU, held until the process
// ends.  Host code reaches it only through the address static_scratch() looks up.
static __device__ __align__(256) unsigned char scratch[MINHASH_STATIC_SCRATCH_BYTES];

namespace {

using namespace mh;


typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int WAVE = 64;
constexpr int WAVES_PER_BLOCK = 4;
constexpr int BLOCK = WAVE * WAVES_PER_BLOCK;
constexpr int TILE = 256;              // nonzeros staged per wavefront per step (4 per lane)
constexpr int HASH_FPL = 8;            // hash functions per lane
constexpr int FULL_KEY_MAX_LOG2_D = 26;     // largest power-of-two D for which 2U keeps a single maximum
constexpr uint32_t SHORT_ITEM = 16;         // nonzeros up to which a lane recomputes its doubtful values by itself
constexpr int HASH_ACC = 2 * HASH_FPL;      // the running extrema of a lane's functions and room for a second set of them
constexpr int HASH_FTILE = WAVE * HASH_FPL;   // 512 functions per wavefront pass
constexpr int PERM_FPL = 4;            // permutations per lane (one 16-byte load)
constexpr int PERM_FTILE = WAVE * PERM_FPL;   // 256
constexpr int MAX_FTILE = HASH_FTILE;
constexpr uint32_t MAX_CHUNK = 8192;   // rows longer than the chunk size are split into chunks of that many nonzeros;
constexpr uint32_t MIN_CHUNK = 64;     // the size is chosen per call on the device (see mh_reset_kernel), not below chunk_floor(k)
constexpr uint64_t SMALL_BATCH_PARTS = 32768;           // partial vectors reserved so that small batches can use
constexpr uint64_t SMALL_BATCH_BYTES = 64ull << 20;     // small chunks, capped to this many bytes
constexpr uint32_t LONG_ITEM = 2048;   // work items with more nonzeros than this are handed out first
constexpr uint32_t NO_SLOT = 0xFFFFFFFFu;

struct WorkHeader {                    // first 256 bytes of the workspace
    uint32_t n_long;                   // work items longer than LONG_ITEM: items[0 .. n_long)
    uint32_t n_short;                  // the others: items[cap_long .. cap_long + n_short)
    uint32_t n_split;
    uint32_t n_parts;
    uint32_t chunk;                    // chunk size of this call, a power of two in [chunk_floor(k), MAX_CHUNK]
    uint32_t ticket;
    uint32_t status;                   // bit 0: bad row_ptr, bit 1: index >= D, bit 2: work list overflow
    uint32_t pad[57];
};
static_assert(sizeof(WorkHeader) == 256, "header size");
static_assert(offsetof(WorkHeader, n_short) == 4 && offsetof(WorkHeader, n_split) == 8 && offsetof(WorkHeader, n_parts) == 12,
              "the row-binning kernel addresses the four counters as an array");

struct alignas(16) Item {              // one unit of row work
    int64_t begin;                     // offset of the first nonzero in col_idx
    uint32_t len;                      // number of nonzeros (at most the chunk size)
    uint32_t row;
    uint32_t slot;                     // NO_SLOT for a whole row, else index of this chunk's vector of partial minima
    uint32_t wlo, whi;                 // packed input only: offset of the item's first tile in the word array,
    uint32_t w;                        // and the bit width of the row's differences
};
static_assert(sizeof(Item) == 32, "item size: one 16-byte load takes begin, len and row");

struct SplitRow {                      // a row processed as several chunks
    uint32_t row;
    uint32_t first_part;               // its chunks own partial vectors first_part .. first_part + n_parts - 1
    uint32_t n_parts;
    uint32_t pad;
};

struct Layout {                        // host and device agree on the workspace layout through this
    size_t items_off, split_rows_off, partials_off, total;
    uint64_t cap_long, cap_short, cap_split, cap_parts;
};

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// The smallest chunk a call with k functions may use: a power of two with about 512 evaluations per lane
// behind every vector of partial minima (k >= 257: 64 nonzeros; 256: 128; 128: 256; up to 64: 512), so
// that a chunk is worth the k words its partial vector costs to write and to merge.
inline uint32_t chunk_floor(int32_t k)
{
    uint32_t slots = 64;
    while (slots < 512u && slots < (uint32_t)k) slots *= 2;
    const uint32_t c = 32768u / slots;
    return c < MIN_CHUNK ? MIN_CHUNK : c;
}

inline Layout make_layout(int64_t n_rows, int64_t nnz_ub, int32_t k, uint64_t reserve_bytes = SMALL_BATCH_BYTES)
{
    Layout L;
    const uint64_t n = (uint64_t)n_rows, nnz = (uint64_t)nnz_ub;
    L.cap_long = nnz / LONG_ITEM + 1;                                 // items with more than LONG_ITEM nonzeros
    const uint64_t by_min = nnz / chunk_floor(k);
    L.cap_split = by_min < n ? by_min : n;                            // rows longer than the smallest chunk size
    // one partial vector per chunk of a split row: at most nnz/chunk + (split rows) for the chunk size in use.
    // Large batches use MAX_CHUNK; a reserve lets small batches use smaller chunks (the device picks the size
    // that fits, see mh_reset_kernel).
    const uint64_t by_max = nnz / MAX_CHUNK;
    uint64_t reserve = reserve_bytes / (sizeof(uint32_t) * (uint64_t)k);
    if (reserve > SMALL_BATCH_PARTS) reserve = SMALL_BATCH_PARTS;
    uint64_t small_need = by_min + L.cap_split;                       // what the smallest chunk would need
    if (reserve > small_need) reserve = small_need;
    L.cap_parts = by_max + (by_max < n ? by_max : n);
    if (L.cap_parts < reserve) L.cap_parts = reserve;
    L.cap_short = n + L.cap_parts + 1;                                // whole rows, plus chunks not longer than LONG_ITEM
    L.items_off = sizeof(WorkHeader);
    L.split_rows_off = align_up(L.items_off + (L.cap_long + L.cap_short) * sizeof(Item), 256);
    L.partials_off = align_up(L.split_rows_off + L.cap_split * sizeof(SplitRow), 256);
    L.total = align_up(L.partials_off + L.cap_parts * (size_t)k * sizeof(uint32_t), 256);
    return L;
}

struct KArgs {
    const int64_t* row_ptr;
    const uint32_t* col_idx;
    const void* params;
    uint8_t* out;
    int64_t out_stride;
    int64_t perm_ld;
    WorkHeader* hdr;
    Item* items;
    SplitRow* split_rows;
    uint32_t* partials;                // [cap_parts][k] partial minima of chunks
    uint64_t D;
    uint64_t cap_long, cap_short, cap_split, cap_parts;
    uint64_t nnz_cap;                  // nonzeros the workspace was sized for (checked under VALIDATE)
    ModD md;
    int64_t n_rows;
    int32_t k, b;
    int32_t n_ftiles;
    int32_t log2_fl;                   // lanes covering one function tile = 1 << log2_fl
    int32_t ftile_size;                // functions per tile: (1 << log2_fl) * functions per lane (hash kernels), 256 (table)
    int32_t sig_bytes;
    uint32_t target_items;             // work items wanted for a balanced launch (a few per resident wavefront)
    uint32_t validate;
    uint32_t lane_pack;                // the hash kernel stores packed dwords from registers (see lane_pack_store)
    uint32_t min_chunk;                // chunk_floor(k); with packed input at least one tile
    uint64_t prime;                    // runtime modulus of the generic-% ablation kernels
    // packed input (minhash_signatures_packed): rows as tiles of differences instead of col_idx
    const uint32_t* pk_width;
    const int64_t* pk_word_ptr;
    const uint32_t* pk_words;
    int64_t pk_words_len;
};

// ------------------------------------------------------------------ small helpers
__device__ __forceinline__ uint32_t wave_bcast(uint32_t v, int src_lane)
{
    return (uint32_t)__shfl((int)v, src_lane, WAVE);
}
__device__ __forceinline__ uint32_t first_lane_value(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_readfirstlane((int)v);
}
// a 64-bit value that is the same in every lane, moved to scalar registers (an address built on it
// is then a scalar base, and the loads that use it need no copy per load)
__device__ __forceinline__ int64_t wave_uniform64(int64_t v)
{
    const uint32_t lo = first_lane_value((uint32_t)v), hi = first_lane_value((uint32_t)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

__device__ __forceinline__ void wave_sync_lds()
{
    // orders this wavefront's LDS writes before its later LDS reads (the hardware
    // executes a wavefront's LDS instructions in order; this stops the compiler)
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
// Hands work units to a persistent wavefront by ticket (TicketMap of mh_arith.h
// says which run of consecutive units a ticket stands for, 32 at most).  The first
// ticket of a wavefront is its own index in the grid, later ones come from an atomic
// counter that starts behind the grid, so a call with fewer units than resident
// wavefronts costs no atomic at all.  When a run starts, its item records are fetched
// with one coalesced load, lane i taking unit i of the run, and parked in the
// wavefront's LDS; a unit's fields then come from there, so that within a run the next
// unit is known without waiting on memory and its first nonzeros can be requested
// while the current unit is still being worked on.  All values are wavefront-uniform.
constexpr int MAX_RUN = 32;
// (Two forms of each structure: with packed input a unit also carries where its words start and
// how wide its differences are.  The form without is kept exactly as it was, so that the kernels for
// plain col_idx input compile to the same code whether or not the packed form exists.)
template <bool PACKED>
struct RunItemsT;
template <>
struct RunItemsT<false> {              // LDS of one wavefront
    uint4 rec[MAX_RUN];                // begin (low, high word), len, row
    uint2 meta[MAX_RUN];               // slot, function tile
};
template <>
struct RunItemsT<true> {
    uint4 rec[MAX_RUN];
    uint4 meta[MAX_RUN];               // slot, function tile, the item's first word (low, high)
    uint32_t width[MAX_RUN];           // bit width of the row's differences
};
template <bool PACKED>
struct UnitT;
template <>
struct UnitT<false> {
    int64_t begin;
    uint32_t len, row, slot;
    int ftile;
};
template <>
struct UnitT<true> {
    int64_t begin;
    uint32_t len, row, slot;
    int ftile;
    int64_t wbegin;                    // offset of the item's first tile in the word array,
    uint32_t w;                        // width of its differences
};
template <bool PACKED>
struct UnitStreamT {
    using RunItems = RunItemsT<PACKED>;
    using Unit = UnitT<PACKED>;
    TicketMap map;
    uint32_t grid_waves;
    uint32_t base, next, end;          // the run [base, end) has its records in LDS; next is the first unit not yet handed out

    __device__ __forceinline__ void load_run(const KArgs& a, uint32_t n_long, int lane, RunItems* lds) const
    {
        const uint32_t u = base + (uint32_t)lane;
        if (lane < MAX_RUN && u < end && u < map.n_units) {
            const uint32_t nft = (uint32_t)a.n_ftiles;
            const uint32_t item_idx = nft == 1u ? u : u / nft;
            const Item* p = item_idx < n_long ? a.items + item_idx : a.items + a.cap_long + (item_idx - n_long);
            const uint4 r = *reinterpret_cast<const uint4*>(p);
            if constexpr (PACKED) {
                const uint4 t = *(reinterpret_cast<const uint4*>(p) + 1);      // slot, first word (low, high), width
                lds->rec[lane] = r;
                lds->meta[lane] = uint4{t.x, u - item_idx * nft, t.y, t.z};
                lds->width[lane] = t.w;
            } else {
                const uint32_t slot = p->slot;
                lds->rec[lane] = r;
                lds->meta[lane] = uint2{slot, u - item_idx * nft};
            }
        }
        wave_sync_lds();
    }
    __device__ __forceinline__ void read(uint32_t unit, const RunItems* lds, Unit* out) const
    {
        const uint4 r = lds->rec[unit - base];
        const auto m = lds->meta[unit - base];
        out->begin = (int64_t)(((uint64_t)first_lane_value(r.y) << 32) | first_lane_value(r.x));
        out->len = first_lane_value(r.z);
        out->row = first_lane_value(r.w);
        out->slot = first_lane_value(m.x);
        out->ftile = (int)first_lane_value(m.y);
        if constexpr (PACKED) {
            out->wbegin = (int64_t)(((uint64_t)first_lane_value(m.w) << 32) | first_lane_value(m.z));
            out->w = first_lane_value(lds->width[unit - base]);
        }
    }
    // the first unit of this wavefront (its own index in the grid is its first ticket); false when there is none
    __device__ __forceinline__ bool init(const KArgs& a, uint64_t units, uint64_t single_units, uint32_t waves, uint32_t index,
                                         uint32_t n_long, int lane, RunItems* lds, Unit* out)
    {
        map = make_ticket_map(units, single_units, waves);
        grid_waves = waves;
        map.range(index, &base, &end);
        next = base;
        if (base >= map.n_units) return false;
        load_run(a, n_long, lane, lds);
        read(next++, lds, out);
        return true;
    }
    // the next unit, drawing a ticket and fetching its run when the current run is used up (this waits on
    // memory); false when nothing is left, where every wavefront gets because tickets only grow
    __device__ __forceinline__ bool advance(const KArgs& a, uint32_t n_long, int lane, RunItems* lds, Unit* out)
    {
        if (next >= end) {
            // Every unit had a wavefront of its own: no further ticket stands for anything, and a small batch is
            // spared some thousand atomics on one address at its end (15 of 42 microseconds for 1 000 rows).
            if (map.lg_run == 0u && map.n_units <= grid_waves) return false;
            uint32_t tk = 0;
            if (lane == 0) tk = grid_waves + atomicAdd(&a.hdr->ticket, 1u);
            map.range(first_lane_value(tk), &base, &end);
            next = base;
            if (base >= map.n_units) return false;
            wave_sync_lds();           // the records of the old run have all been read
            load_run(a, n_long, lane, lds);
        }
        read(next++, lds, out);
        return true;
    }
    // the next unit if it belongs to the current run: no waiting beyond the LDS
    __device__ __forceinline__ bool peek_and_take(const RunItems* lds, Unit* out)
    {
        if (next >= end || next >= map.n_units) return false;
        read(next++, lds, out);
        return true;
    }
};
// keeps a wave-uniform value in a vector register: integer instructions whose
// operands all sit in vector registers issue at twice the rate of those that
// read a scalar register
__device__ __forceinline__ uint32_t in_vgpr(uint32_t v)
{
    asm volatile("" : "+v"(v));
    return v;
}
// the same for a constant that only some kernels read: without "volatile" an
// unused copy is dropped instead of holding a register
__device__ __forceinline__ uint32_t in_vgpr_if_used(uint32_t v)
{
    asm("" : "+v"(v));
    return v;
}
// the mod-D constants of a launch plus the other wave-uniform constants the
// hand-ordered inner steps read, each held in a vector register
struct ModDV : ModD {
    uint32_t p31;    // 2^31 - 1
    uint32_t sign;   // 2^31
    uint32_t negD;   // 2^32 - D
    uint32_t kshift; // 32 - log2 D: left shift of the order-preserving keys of the negated forms
    uint32_t frot;   // 31 - log2 D: what the coefficients of the full-key form are rotated by
    uint32_t frac_m; // fractional keys (FracD of mh_arith.h): low word of the 33-bit multiplier,
    uint32_t frac_l; // and the bit at which the key starts
    uint32_t m61q;   // 61-bit residues modulo D in 32-bit steps (reduce61_mod_d of mh_arith.h): floor(2^61 / D'),
    uint32_t dp;     // D' = D 2^j in (2^29, 2^32 / 3],
    uint32_t mask29; // 2^29 - 1
    uint32_t negdp;  // and 2^32 - D'
};
__device__ __forceinline__ ModDV vector_constants(const ModD& src)
{
    ModDV v;
    v.pow2 = src.pow2;
    v.M64 = src.M64;
    v.M61q = src.M61q;
    v.D = in_vgpr(src.D);
    v.mask = in_vgpr(src.mask);
    v.M = in_vgpr(src.M);
    v.sh = in_vgpr_if_used(src.sh);
    v.p31 = in_vgpr_if_used(P31);
    v.sign = in_vgpr_if_used(0x80000000u);
    v.negD = in_vgpr_if_used(0u - src.D);
    v.kshift = src.pow2 ? neg_key_shift(src.mask) : 0u;
    v.frot = src.pow2 ? full_key_rotation(src.mask) : 0u;
    const bool frac = frac_key_serves(src.D);
    const FracD fd = frac ? make_frac_d(src.D) : FracD{0u, 0u, 0u};
    v.frac_m = in_vgpr_if_used(fd.m_low);
    v.frac_l = fd.l;
    v.m61q = in_vgpr_if_used(src.M61q);
    v.dp = in_vgpr_if_used(src.M61q ? scaled_up_d(src.D) : 0u);
    v.mask29 = in_vgpr_if_used(0x1FFFFFFFu);
    v.negdp = in_vgpr_if_used(0u - v.dp);
    return v;
}
// Issue priority of this wavefront among those of its SIMD.  The hand-ordered steps
// raise it for their runs of full-issue instructions (multiply-adds, three-operand
// adds and extrema, funnel shifts) and lower it for their runs of simple ones.  A
// SIMD issues the simple instructions of two wavefronts together, and a simple
// instruction alongside another wavefront's full-issue one (not alongside a
// 32-bit multiply, which issues alone), so the issue port should go to whoever
// has full-issue work while simple instructions fill in around it.  2U: 78-82 ms without, 67.5 ms with; the reverse assignment takes
// 96 ms; the level (1..3) makes no difference.  Without priorities the same loop
// ran anywhere between 78 and 87 ms depending on where the compiler placed it
// and on idle cycles inserted into an iteration; with them neither matters.
template <int P>
__device__ __forceinline__ void issue_priority()
{
    static_assert(P >= 0 && P <= 3, "priority");
    asm volatile("s_setprio %c0" : : "n"(P));
}
// three-operand extrema: one instruction folds two new values into the running one
__device__ __forceinline__ uint32_t umin3(uint32_t a, uint32_t b, uint32_t c)
{
    uint32_t d;
    asm("v_min3_u32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
    return d;
}
__device__ __forceinline__ uint32_t umax3(uint32_t a, uint32_t b, uint32_t c)
{
    uint32_t d;
    asm("v_max3_u32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
    return d;
}

// ------------------------------------------------------------------ reset / bin / fill
// Clears the header and picks the chunk size of this call: the largest power of two
// in [chunk_floor(k), MAX_CHUNK] that still yields target_items work items, as long as the
// partial vectors of the resulting chunks fit the workspace.  Large batches get
// MAX_CHUNK; a batch of a few hundred rows gets its long rows cut finely enough to
// occupy the whole GPU instead of waiting for one wavefront per row.
__device__ __forceinline__ uint32_t pick_chunk(const KArgs& a)      // one thread
{
    uint32_t chunk = MAX_CHUNK;
    const int64_t total = a.row_ptr[a.n_rows] - a.row_ptr[0];
    if (total > 0) {
        const uint64_t nnz = (uint64_t)total, n = (uint64_t)a.n_rows;
        while (chunk > a.min_chunk) {
            if (nnz / chunk >= a.target_items) break;
            const uint64_t by_next = nnz / (chunk / 2);
            if (by_next + (by_next < n ? by_next : n) > a.cap_parts) break;
            chunk /= 2;
        }
    }
    return chunk;
}
__device__ __forceinline__ void reset_header(const KArgs& a)          // threads 0..63 of one block
{
    uint32_t* words = reinterpret_cast<uint32_t*>(a.hdr);
    if (threadIdx.x < 64 && threadIdx.x != offsetof(WorkHeader, chunk) / 4) words[threadIdx.x] = 0;
    if (threadIdx.x == 0) a.hdr->chunk = pick_chunk(a);
}
__global__ void mh_reset_kernel(KArgs a) { reset_header(a); }

// One thread per row.  Prefix sums over the wavefront and then over the block's
// wavefronts make one atomic per block of 1024 rows and counter (one per
// wavefront made 31 000 atomics on one address for 2x10^6 rows, and those took
// all of the kernel's 0.36 ms).  Items longer than LONG_ITEM go to the front of
// the work list, the rest behind them: the persistent wavefronts draw tickets in
// list order, so the long items start first and the short ones fill the tail of
// the launch.
constexpr int BIN_BLOCK = 1024;
constexpr uint32_t MAX_ROW_PARTS = 512;    // chunks per row at most, unless the largest chunk size still leaves more
constexpr uint32_t BIN_TEAM_FROM = 32;     // rows of more chunks than this have their items written by the whole block,
constexpr int BIN_TEAM_ROWS = 64;          // up to this many rows per block (further ones by their own thread)
struct RowJob {                            // what writing the items of one row needs
    int64_t begin, nnz, pk_first;
    uint32_t row, first_part, first_lg, first_sh, n_it, pk_w, is_split, chunk;
};
// Item c of a row.  Full chunks are long items when the chunk size exceeds LONG_ITEM, so all items before a
// full chunk are long ones (or none is); the last or only item goes by its own length.
__device__ __forceinline__ void write_item(const KArgs& a, const RowJob& j, uint32_t c)
{
    const uint32_t CHUNK = j.chunk;
    Item it;
    it.begin = j.begin + (int64_t)c * CHUNK;
    const int64_t rest = j.nnz - (int64_t)c * CHUNK;
    it.len = j.is_split ? (uint32_t)(rest < (int64_t)CHUNK ? rest : (int64_t)CHUNK) : (uint32_t)j.nnz;
    it.row = j.row;
    it.slot = j.is_split ? j.first_part + c : NO_SLOT;
    const int64_t wbegin = j.pk_first + (int64_t)c * (int64_t)(CHUNK / PACKED_TILE) * (int64_t)packed_tile_words(PACKED_TILE, j.pk_w);
    it.wlo = (uint32_t)wbegin; it.whi = (uint32_t)((uint64_t)wbegin >> 32); it.w = j.pk_w;
    const uint32_t longs_before = CHUNK > LONG_ITEM ? c : 0u;
    if (it.len > LONG_ITEM) a.items[(uint64_t)j.first_lg + longs_before] = it;
    else a.items[a.cap_long + (uint64_t)j.first_sh + (c - longs_before)] = it;
}
__global__ __launch_bounds__(BIN_BLOCK) void mh_bin_rows_kernel(KArgs a)
{
    __shared__ uint32_t s_wave_tot[BIN_BLOCK / WAVE][4];     // totals per wavefront, then their exclusive prefix sums
    __shared__ uint32_t s_block_base[4];
    __shared__ RowJob s_jobs[BIN_TEAM_ROWS];
    __shared__ uint32_t s_n_jobs;
    const int lane = threadIdx.x & (WAVE - 1);
    const int wave = threadIdx.x >> 6;
    const int64_t row = (int64_t)blockIdx.x * BIN_BLOCK + threadIdx.x;
    __shared__ uint32_t s_chunk;
    if (threadIdx.x == 0) s_n_jobs = 0;                // (two barriers lie between this and the first use)
    // A batch of one block needs no header from an earlier launch and no atomics on it: the block's totals are the
    // call's, what it has to report collects in the LDS, and the whole header is written once, at the end.
    const bool own_reset = gridDim.x == 1;
    __shared__ uint32_t s_status;
    int64_t begin = 0, end = 0;
    if (row < a.n_rows) {                              // (requested before the chunk size is known: one wait for both)
        begin = a.row_ptr[row];
        end = a.row_ptr[row + 1];
    }
    if (own_reset) {
        if (threadIdx.x == 0) {
            s_chunk = pick_chunk(a);
            s_status = 0;
        }
        __syncthreads();
    }
    auto report = [&](uint32_t bits) {
        if (own_reset) atomicOr(&s_status, bits); else atomicOr(&a.hdr->status, bits);
    };
    uint32_t CHUNK = own_reset ? s_chunk : a.hdr->chunk;
    if (CHUNK < a.min_chunk || CHUNK > MAX_CHUNK) CHUNK = MAX_CHUNK;
    const uint32_t call_chunk = CHUNK;
    uint32_t n_it = 0, is_split = 0;
    int64_t nnz = 0;
    if (row < a.n_rows) {
        nnz = end - begin;
        // under VALIDATE the row must lie inside [row_ptr[0], row_ptr[n_rows]] and that range must not
        // hold more nonzeros than the workspace was sized for (row_extent_status of mh_arith.h)
        const int64_t lo = a.validate ? a.row_ptr[0] : 0, hi = a.validate ? a.row_ptr[a.n_rows] : 0;
        const uint32_t bad = row_extent_status(begin, end, lo, hi, a.nnz_cap, a.validate != 0);
        if (bad && a.validate) report(bad);
        if (bad) nnz = 0;              // treated as an empty row
        // a very long row of a small batch gets larger chunks than the call's: no more than MAX_ROW_PARTS of them
        while (nnz > (int64_t)CHUNK * MAX_ROW_PARTS && CHUNK < MAX_CHUNK) CHUNK *= 2;
        is_split = nnz > (int64_t)CHUNK ? 1u : 0u;
        n_it = is_split ? (uint32_t)((nnz + CHUNK - 1) / CHUNK) : 1u;
    }
    // length of the last (or only) item of the row, and how many of its items are long
    const int64_t last_len = row < a.n_rows ? nnz - (int64_t)(n_it - 1) * CHUNK : 0;
    const uint32_t last_long = last_len > (int64_t)LONG_ITEM ? 1u : 0u;
    const uint32_t full_long = CHUNK > LONG_ITEM ? 1u : 0u;                  // are full chunks long items?
    const uint32_t n_lg = row < a.n_rows ? (n_it - 1) * full_long + last_long : 0u;
    const uint32_t n_sh = row < a.n_rows ? n_it - n_lg : 0u;
    const uint32_t n_pt = is_split ? n_it : 0u;
    // inclusive scans over the wavefront: long items, short items, split rows, partial vectors
    uint32_t inc_lg = n_lg, inc_sh = n_sh, inc_sp = is_split, inc_pt = n_pt;
    for (int d = 1; d < WAVE; d <<= 1) {
        uint32_t v0 = (uint32_t)__shfl_up((int)inc_lg, d, WAVE);
        uint32_t v1 = (uint32_t)__shfl_up((int)inc_sh, d, WAVE);
        uint32_t v2 = (uint32_t)__shfl_up((int)inc_sp, d, WAVE);
        uint32_t v3 = (uint32_t)__shfl_up((int)inc_pt, d, WAVE);
        if (lane >= d) { inc_lg += v0; inc_sh += v1; inc_sp += v2; inc_pt += v3; }
    }
    if (lane == WAVE - 1) {
        s_wave_tot[wave][0] = inc_lg; s_wave_tot[wave][1] = inc_sh;
        s_wave_tot[wave][2] = inc_sp; s_wave_tot[wave][3] = inc_pt;
    }
    __syncthreads();
    uint32_t block_total = 0;          // thread c < 4: counter c of the block
    if (threadIdx.x < 4) {
        uint32_t* const counter = &a.hdr->n_long + threadIdx.x;   // n_long, n_short, n_split, n_parts lie in a row
        for (int w = 0; w < BIN_BLOCK / WAVE; ++w) {
            const uint32_t t = s_wave_tot[w][threadIdx.x];
            s_wave_tot[w][threadIdx.x] = block_total;
            block_total += t;
        }
        s_block_base[threadIdx.x] = block_total && !own_reset ? atomicAdd(counter, block_total) : 0u;
    }
    __syncthreads();
    const uint32_t base_lg = s_block_base[0] + s_wave_tot[wave][0];
    const uint32_t base_sh = s_block_base[1] + s_wave_tot[wave][1];
    const uint32_t base_sp = s_block_base[2] + s_wave_tot[wave][2];
    const uint32_t base_pt = s_block_base[3] + s_wave_tot[wave][3];
    const uint64_t first_lg = (uint64_t)base_lg + inc_lg - n_lg;
    const uint64_t first_sh = (uint64_t)base_sh + inc_sh - n_sh;
    const uint64_t first_part = (uint64_t)base_pt + inc_pt - n_pt;
    bool todo = row < a.n_rows;
    // An overflow can only happen when the workspace was sized for fewer nonzeros than
    // row_ptr describes.  Every allocated work-list entry inside the capacity is still
    // written (as an empty row), so that the consumer never reads an undefined entry.
    bool overflow = todo && (first_lg + n_lg > a.cap_long || first_sh + n_sh > a.cap_short);
    uint64_t sidx = 0;
    if (todo && is_split) {
        sidx = (uint64_t)base_sp + inc_sp - 1;
        overflow = overflow || sidx >= a.cap_split || first_part + n_it > a.cap_parts;
    }
    Item* long_items = a.items;
    Item* short_items = a.items + a.cap_long;
    if (overflow) {
        report(4u);
        Item it; it.begin = begin; it.len = 0; it.row = (uint32_t)row; it.slot = NO_SLOT; it.wlo = 0; it.whi = 0; it.w = 0;
        for (uint32_t c = 0; c < n_lg && first_lg + c < a.cap_long; ++c) long_items[first_lg + c] = it;
        for (uint32_t c = 0; c < n_sh && first_sh + c < a.cap_short; ++c) short_items[first_sh + c] = it;
        if (is_split && sidx < a.cap_split) {
            SplitRow sr; sr.row = (uint32_t)row; sr.first_part = 0; sr.n_parts = 0; sr.pad = 1;
            a.split_rows[sidx] = sr;
        }
        todo = false;
    }
    RowJob job;
    job.begin = begin; job.nnz = nnz; job.pk_first = 0; job.row = (uint32_t)row; job.first_part = (uint32_t)first_part;
    job.first_lg = (uint32_t)first_lg; job.first_sh = (uint32_t)first_sh; job.n_it = n_it; job.pk_w = 0; job.is_split = is_split; job.chunk = CHUNK;
    if (todo) {
        if (is_split) {
            SplitRow sr; sr.row = (uint32_t)row; sr.first_part = (uint32_t)first_part; sr.n_parts = n_it; sr.pad = 0;
            a.split_rows[sidx] = sr;
        }
        // packed input: where the row's words start and how wide its differences are (chunks are whole numbers of tiles)
        if (a.pk_words) {
            job.pk_first = a.pk_word_ptr[row];
            job.pk_w = a.pk_width[row];
            if (job.pk_w > 32u) {          // not a width: the row is reported and read as if its differences were 0 bits wide
                report(1u);
                job.pk_w = 0;
            }
        }
        // a row of many chunks is left to the whole block (a row of 10^5 nonzeros in a small batch has 1 500 of them)
        if (n_it > BIN_TEAM_FROM) {
            const uint32_t q = atomicAdd(&s_n_jobs, 1u);
            if (q < (uint32_t)BIN_TEAM_ROWS) {
                s_jobs[q] = job;
                todo = false;
            }
        }
    }
    if (todo)
        for (uint32_t c = 0; c < n_it; ++c) write_item(a, job, c);
    __syncthreads();
    if (own_reset && threadIdx.x < 64) {               // the header of the call: counters, chunk size, status, zeros elsewhere (the ticket counter among them)
        uint32_t word = threadIdx.x < 4 ? block_total : 0u;
        if (threadIdx.x == offsetof(WorkHeader, chunk) / 4) word = call_chunk;
        if (threadIdx.x == offsetof(WorkHeader, status) / 4) word = s_status;
        reinterpret_cast<uint32_t*>(a.hdr)[threadIdx.x] = word;
    }
    const uint32_t n_jobs = s_n_jobs < (uint32_t)BIN_TEAM_ROWS ? s_n_jobs : (uint32_t)BIN_TEAM_ROWS;
    for (uint32_t q = 0; q < n_jobs; ++q) {
        const RowJob j = s_jobs[q];
        for (uint32_t c = threadIdx.x; c < j.n_it; c += BIN_BLOCK) write_item(a, j, c);
    }
}

// ------------------------------------------------------------------ truncate + pack + store (one wavefront)
// mins[0 .. nf) are the full minima of functions j0 .. j0+nf of `row`; j0 is a
// multiple of ftile, so the bits start at a byte offset that is a multiple of 4.
// Value j takes bits [j b, (j+1) b) of the row's little-endian bit string
// (Section 1.1: only the lowest b bits of each hashed value are stored).
__device__ __forceinline__ void wave_pack_store(const KArgs& a, const uint32_t* mins, uint32_t row, int j0, int nf,
                                                bool last_tile, int lane)
{
    const int b = a.b;
    const uint32_t maskb = b >= 32 ? 0xFFFFFFFFu : ((1u << b) - 1u);
    uint8_t* dst = a.out + (int64_t)row * a.out_stride;
    const int64_t byte0 = ((int64_t)j0 * b) >> 3;
    const int nbytes = (int)((((int64_t)nf * b) + 7) >> 3);
    const int ndw = (nbytes + 3) >> 2;
    uint8_t* base = dst + byte0;
    const bool aligned = ((reinterpret_cast<uintptr_t>(base) & 3u) == 0);
    const bool b_pow2 = (b & (b - 1)) == 0;                 // 1, 2, 4, 8, 16, 32: fields do not straddle words
    const int lg_b = __builtin_ctz((unsigned)b);
    for (int w = lane; w < ndw; w += WAVE) {
        uint32_t word = 0;
        if (b_pow2) {
            const int per = 32 >> lg_b;
            const int j = w << (5 - lg_b);
            for (int i = 0; i < per && j + i < nf; ++i) word |= (mins[j + i] & maskb) << (i << lg_b);
        } else {
            const int bit_lo = w * 32;
            for (int j = bit_lo / b; j < nf && j * b < bit_lo + 32; ++j) {
                uint32_t v = mins[j] & maskb;
                int pos = j * b - bit_lo;
                word |= pos >= 0 ? (v << pos) : (v >> (-pos));
            }
        }
        if (aligned && 4 * w + 3 < nbytes) {
            *reinterpret_cast<uint32_t*>(base + 4 * w) = word;
        } else {
            for (int q = 0; q < 4; ++q)
                if (4 * w + q < nbytes) base[4 * w + q] = (uint8_t)(word >> (8 * q));
        }
    }
    if (last_tile) {                   // pad bytes up to the row pitch are zero
        for (int64_t q = a.sig_bytes + lane; q < a.out_stride; q += WAVE) dst[q] = 0;
    }
}

// The same for the shapes in which the fields of one lane fill whole dwords: eight
// functions per lane and b = 8, 16 or 32, a row pitch and an output pointer that are
// multiples of four (the host checks all of it once per call).  The lane that holds the
// minima packs them in its own registers and stores its 2, 4 or 8 dwords itself: no trip
// through the LDS, no loop over fields.  m[0 .. 8) are the minima of functions
// j_base .. j_base + 7; functions from k on do not exist and are not stored.
__device__ __forceinline__ void lane_pack_store(const KArgs& a, const uint32_t (&m)[HASH_ACC], uint32_t row, int j_base,
                                                bool holder)
{
    const int valid = a.k - j_base < HASH_FPL ? a.k - j_base : HASH_FPL;
    if (!holder || valid <= 0) return;
    const int b = a.b;
    uint8_t* dst = a.out + (int64_t)row * a.out_stride + (((int64_t)j_base * b) >> 3);
    uint32_t* dw = reinterpret_cast<uint32_t*>(dst);
    const int nbytes = (valid * b) >> 3;
    uint32_t w[HASH_FPL];
    int nd;
    if (b == 8) {          // byte 0 of four values per dword
        w[0] = __builtin_amdgcn_perm(m[1], m[0], 0x0c0c0400u) | __builtin_amdgcn_perm(m[3], m[2], 0x04000c0cu);
        w[1] = __builtin_amdgcn_perm(m[5], m[4], 0x0c0c0400u) | __builtin_amdgcn_perm(m[7], m[6], 0x04000c0cu);
        nd = 2;
    } else if (b == 16) {  // the low halves of two values per dword
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = __builtin_amdgcn_perm(m[2 * i + 1], m[2 * i], 0x05040100u);
        nd = 4;
    } else {               // b = 32: the minima as they are
#pragma unroll
        for (int i = 0; i < HASH_FPL; ++i) w[i] = m[i];
        nd = HASH_FPL;
    }
#pragma unroll
    for (int i = 0; i < HASH_FPL; ++i)
        if (i < nd && 4 * i + 4 <= nbytes) dw[i] = w[i];
    if (nbytes & 3) {      // the last lane of a k that ends inside a dword: its remaining bytes one by one
        const int i0 = nbytes >> 2;
        uint32_t word = 0;
#pragma unroll
        for (int i = 0; i < HASH_FPL; ++i)
            if (i == i0) word = w[i];
        for (int q = 0; q < (nbytes & 3); ++q) dst[4 * i0 + q] = (uint8_t)(word >> (8 * q));
    }
}

// ------------------------------------------------------------------ hash-family policies
template <class Pol, int NF>
__device__ __forceinline__ void pair_generic(const typename Pol::Fn (&fn)[HASH_FPL], uint32_t (&m)[HASH_ACC],
                                             const uint32_t* wa, const uint32_t* wb, const ModDV& md, uint64_t D);

// A policy evaluates one function on one staged nonzero and returns a value that
// the kernel folds into a running extremum: the hashed location itself (running
// minimum), or, when TRACK_MAX, its complement mask - h(t) (running maximum),
// which saves one instruction per evaluation for power-of-two D.
// FORM_ANY_D: exact quotient.  Power-of-two D: the coefficients are rotated so that the folded
// value itself is the key (prep_2u31_full).  FORM_FULL keeps one unsigned running maximum of the
// doubled value (key_full2_2u31), which needs a second look at a value with probability
// (D / 2^31)^n, n the evaluations behind it, so the host picks it for D <= 2^26; FORM_FULL_TWO
// keeps a signed and an unsigned maximum of the value (finish_full_keys), nothing to look at twice.
// FORM_FRAC_D (D below 2^28, not a power of two): the running minimum of fractional keys
// (frac_key), one multiply-add and one funnel shift after the canonical residue, instead of the
// exact quotient's multiply-high, shift and multiply-add; the location comes back once per row.
// The function keeps a register pair {bias, r} per slot whose low word stays put.
// FORM_BIG_D (D of at least p / 3): the quotient is 0, 1 or 2, so r mod D is the smallest of r,
// r - D and r - 2D (reduce_small_quotient): two subtractions and a three-operand minimum.
struct Fn2U31F : Fn2U31 {
    mutable u32x2 bq;
};
constexpr int FORM_ANY_D = 0, FORM_FULL_TWO = 1, FORM_FULL = 2, FORM_FRAC_D = 3, FORM_BIG_D = 4;
template <int FORM>
struct Pol2U31 {
    static constexpr bool POW2 = FORM == FORM_FULL || FORM == FORM_FULL_TWO;
    static constexpr bool FRAC_KEY = FORM == FORM_FRAC_D;   // the running minimum is a fractional key (finish_frac_key)
    static constexpr int NW = 1;
    static constexpr int MIN_WAVES = POW2 ? 5 : 4;   // wavefronts per SIMD the register allocation must leave room for
    static constexpr bool TRACK_MAX = POW2;
    static constexpr bool SHIFTED_KEY = false;
    static constexpr bool DOUBLED_KEY = FORM == FORM_FULL;   // one unsigned maximum of twice the folded value
    static constexpr bool TWO_MAXIMA = FORM == FORM_FULL_TWO;
    static constexpr bool SHIFT_END = false;
    static constexpr bool GUARDED = FORM == FORM_FULL;   // a single maximum can say that it may be wrong
    static constexpr bool VARIABLE_NF = true;    // hand-ordered steps exist for 5..8 functions per lane
    using Fn = std::conditional_t<FRAC_KEY, Fn2U31F, Fn2U31>;
    static __device__ __forceinline__ Fn load(const uint64_t* c, bool valid, const KArgs& a)
    {
        if constexpr (FRAC_KEY) {
            Fn f;
            static_cast<Fn2U31&>(f) = valid ? prep_2u31_raw(c[0], c[1]) : prep_2u31_raw(0, 0);
            f.bq = u32x2{make_frac_d(a.D).bias, 0u};
            return f;
        } else if constexpr (!POW2) {
            return valid ? prep_2u31_raw(c[0], c[1]) : prep_2u31_raw(0, 0);
        } else {
            const uint32_t rotation = full_key_rotation(a.md.mask);
            return valid ? prep_2u31_full(c[0], c[1], rotation) : prep_2u31_full(0, 0, rotation);
        }
    }
    static __device__ __forceinline__ void stage(uint32_t t, uint32_t* w) { w[0] = stage_2u31(t); }
    static __device__ __forceinline__ uint32_t key(const Fn& f, const uint32_t* w, const ModDV& md, uint64_t)
    {
        if (FORM == FORM_FULL) return key_full2_2u31(f, w[0]);
        if (POW2) return (uint32_t)key_full_2u31(f, w[0]);
        if (FRAC_KEY) {
            const uint32_t x = fold_2u31(f, w[0]), y = x - (uint32_t)P31;
            return frac_key(y < x ? y : x, make_frac_d(md.D));
        }
        if (FORM == FORM_BIG_D) {
            const uint32_t x = fold_2u31(f, w[0]), y = x - (uint32_t)P31;
            return reduce_small_quotient(y < x ? y : x, md.D);
        }
        return hash_2u31_raw(f, w[0], md);
    }
    // a running maximum below this is doubtful (full2_key_doubtful): one comparison of a lane's
    // smallest maximum says whether any of its values is
    static __device__ __forceinline__ uint32_t doubt_below(const ModDV& md) { return 2u * md.mask; }
    template <int NF>
    static __device__ __forceinline__ uint32_t doubtful(const uint32_t (&m)[HASH_ACC], const ModDV& md)
    {
        uint32_t bits = 0;
#pragma unroll
        for (int r = 0; r < NF; ++r) bits |= full2_key_doubtful(m[r], md.mask) ? 1u << r : 0u;
        return bits;
    }
    // the hashed location from the definition's arithmetic (canonical residue, then mod D)
    static __device__ __forceinline__ uint32_t exact_hash(const uint64_t* c, uint32_t t, const ModD& md, uint64_t)
    {
        return hash_2u31<POW2>(prep_2u31(c[0], c[1]), stage_2u31(t), md);
    }
    template <int NF>
    static __device__ __forceinline__ void pair(const Fn (&fn)[HASH_FPL], uint32_t (&m)[HASH_ACC], const uint32_t* wa,
                                                const uint32_t* wb, const ModDV& md, uint64_t D);
    static constexpr int DEG = 2;
};

// FULL (power-of-two D only): the coefficients are rotated so that the folded value itself
// is the key, kept as a signed and an unsigned running maximum (prep_4u31_full,
// finish_full_keys): no instruction after the fold, nothing to look at twice.  Without FULL
// the key is the shifted one of key_neg_4u31, one shift and one add-then-shift after the
// fold; the host picks it only when asked for the evaluation-by-evaluation form.
// FRAC (D below 2^28, not a power of two): fractional keys as in Pol2U31<FORM_FRAC_D>.
struct Fn4U31F : Fn4U31 {
    mutable u32x2 bq;
};
// MODE, for D that is not a power of two: 0 exact quotient, 1 fractional keys, 2 the quotient of
// at most 2 of Pol2U31<FORM_BIG_D>.
template <bool POW2, bool FULL = false, int MODE = 0>
struct Pol4U31 {
    static constexpr bool FRAC = MODE == 1;
    static_assert(POW2 || !FULL, "full keys are for power-of-two D");
    static_assert(!POW2 || MODE == 0, "the modes are for D that is not a power of two");
    static constexpr int NW = 3;
    static constexpr int MIN_WAVES = POW2 ? 4 : 3;
    static constexpr bool TRACK_MAX = POW2;
    static constexpr bool SHIFTED_KEY = POW2 && !FULL;  // the running maximum is a key shifted left by md.kshift
    static constexpr bool DOUBLED_KEY = false;
    static constexpr bool TWO_MAXIMA = FULL;            // ... or the folded value itself, kept as a signed and an unsigned maximum
    static constexpr bool SHIFT_END = false;
    static constexpr bool FRAC_KEY = FRAC;
    static constexpr bool GUARDED = false;
    static constexpr bool VARIABLE_NF = true;    // hand-ordered steps exist for 5..8 functions per lane
    using Fn = std::conditional_t<FRAC, Fn4U31F, Fn4U31>;
    static __device__ __forceinline__ Fn load(const uint64_t* c, bool valid, const KArgs& a)
    {
        if constexpr (FRAC) {
            Fn f;
            static_cast<Fn4U31&>(f) = valid ? prep_4u31(c[0], c[1], c[2], c[3]) : prep_4u31(0, 0, 0, 0);
            f.bq = u32x2{make_frac_d(a.D).bias, 0u};
            return f;
        } else if constexpr (FULL) {
            const uint32_t rotation = full_key_rotation(a.md.mask);
            return valid ? prep_4u31_full(c[0], c[1], c[2], c[3], rotation) : prep_4u31_full(0, 0, 0, 0, rotation);
        } else if constexpr (POW2) {
            return valid ? prep_4u31_neg(c[0], c[1], c[2], c[3]) : prep_4u31_neg(0, 0, 0, 0);
        } else {
            return valid ? prep_4u31(c[0], c[1], c[2], c[3]) : prep_4u31(0, 0, 0, 0);
        }
    }
    static __device__ __forceinline__ void stage(uint32_t t, uint32_t* w)
    {
        Pow4U31 p = stage_4u31(t);
        w[0] = (uint32_t)p.t1; w[1] = (uint32_t)p.t2; w[2] = (uint32_t)p.t3;
    }
    static __device__ __forceinline__ uint32_t key(const Fn& f, const uint32_t* w, const ModDV& md, uint64_t)
    {
        Pow4U31 p;
        p.t1 = (int32_t)w[0]; p.t2 = (int32_t)w[1]; p.t3 = (int32_t)w[2];
        if (FULL) return fold_4u31(f, p);
        if (MODE != 0) {
            const uint32_t x = fold_4u31(f, p), u = x - 1u, v = x ^ 0x80000000u, r = v < u ? v : u;
            return FRAC ? frac_key(r, make_frac_d(md.D)) : reduce_small_quotient(r, md.D);
        }
        if (POW2) return key_neg_4u31(f, p, md.kshift);
        return hash_4u31_np2(f, p, md);
    }
    template <int NF>
    static __device__ __forceinline__ void pair(const Fn (&fn)[HASH_FPL], uint32_t (&m)[HASH_ACC], const uint32_t* wa,
                                                const uint32_t* wb, const ModDV& md, uint64_t D);
    static constexpr int DEG = 4;
};

// The power-of-two path of 2U with p = 2^61-1 keeps, per function, a register pair
// whose high word stays zero: the second multiply-add takes {high word of L, 0}
// as its 64-bit addend, and only the low word is rewritten per evaluation.
struct Fn2U61V : Fn2U61 {
    mutable u32x2 hz;
};

// For power-of-two D <= 2^31 the fast path evaluates the negated, rotated function
// without carries (key_neg_2u61 of mh_arith.h) and keeps the unsigned running maximum
// of the keys; a maximum below GUARD61_FLOOR, which about one value in 2^n with n
// evaluations behind it has, is computed again from the exact arithmetic (GUARDED,
// see the kernel).
// STEPS32: other D of at most 2^32 / 3, the residue modulo D taken in 32-bit steps, ordered by hand (half_2u61_steps32).
template <bool POW2, bool STEPS32 = false>
struct Pol2U61 {
    static_assert(!(POW2 && STEPS32), "one form or the other");
    static constexpr int NW = 1;
    static constexpr int MIN_WAVES = POW2 || STEPS32 ? 4 : 5;
    static constexpr bool TRACK_MAX = POW2;
    static constexpr bool SHIFTED_KEY = POW2;
    static constexpr bool DOUBLED_KEY = false;
    static constexpr bool TWO_MAXIMA = false;
    static constexpr bool SHIFT_END = false;
    static constexpr bool FRAC_KEY = false;
    static constexpr bool GUARDED = POW2;
    static constexpr bool VARIABLE_NF = POW2 || STEPS32;    // hand-ordered steps exist for 5..8 functions per lane
    using Fn = std::conditional_t<POW2 || STEPS32, Fn2U61V, Fn2U61>;
    static __device__ __forceinline__ Fn load(const uint64_t* c, bool valid, const KArgs& a)
    {
        Fn f;
        if constexpr (POW2) {
            const uint32_t shift = neg_key_shift(a.md.mask);
            static_cast<Fn2U61&>(f) = valid ? prep_2u61_neg(c[0], c[1], shift) : prep_2u61_neg(0, 0, shift);
            f.hz = u32x2{0u, 0u};
        } else if constexpr (STEPS32) {
            static_cast<Fn2U61&>(f) = valid ? prep_2u61(c[0], c[1]) : prep_2u61(0, 0);
            f.hz = u32x2{0u, 0u};
        } else {
            static_cast<Fn2U61&>(f) = valid ? prep_2u61(c[0], c[1]) : prep_2u61(0, 0);
        }
        return f;
    }
    static __device__ __forceinline__ void stage(uint32_t t, uint32_t* w) { w[0] = t; }
    // the exact hashed location (the fast path of POW2 does not come through here)
    static __device__ __forceinline__ uint32_t key(const Fn& f, const uint32_t* w, const ModD& md, uint64_t D)
    {
        return hash_2u61<POW2>(f, w[0], md, D);
    }
    static __device__ __forceinline__ uint32_t doubt_below(const ModDV&) { return GUARD61_FLOOR; }
    template <int NF>
    static __device__ __forceinline__ uint32_t doubtful(const uint32_t (&m)[HASH_ACC], const ModDV&)
    {
        uint32_t bits = 0;
#pragma unroll
        for (int r = 0; r < NF; ++r) bits |= m[r] < GUARD61_FLOOR ? 1u << r : 0u;
        return bits;
    }
    static __device__ __forceinline__ uint32_t exact_hash(const uint64_t* c, uint32_t t, const ModD& md, uint64_t D)
    {
        return hash_2u61<POW2>(prep_2u61(c[0], c[1]), t, md, D);
    }
    template <int NF>
    static __device__ __forceinline__ void pair(const Fn (&fn)[HASH_FPL], uint32_t (&m)[HASH_ACC], const uint32_t* wa,
                                                const uint32_t* wb, const ModDV& md, uint64_t D);
    static constexpr int DEG = 2;
};

// 4U with p = 2^61-1: three Horner steps per evaluation on the raw index (any t <
// 2^32, so one policy serves every D).  Eight functions hold 64 coefficient words.
template <bool POW2>
struct Pol4U61 {
    static constexpr int NW = 1;
    static constexpr int MIN_WAVES = 2;
    static constexpr bool TRACK_MAX = false;
    static constexpr bool SHIFTED_KEY = false;
    static constexpr bool DOUBLED_KEY = false;
    static constexpr bool TWO_MAXIMA = false;
    static constexpr bool SHIFT_END = false;
    static constexpr bool FRAC_KEY = false;
    static constexpr bool GUARDED = false;
    static constexpr bool VARIABLE_NF = false;
    using Fn = Fn4U61;
    static __device__ __forceinline__ Fn load(const uint64_t* c, bool valid, const KArgs&)
    {
        return valid ? prep_4u61(c[0], c[1], c[2], c[3]) : prep_4u61(0, 0, 0, 0);
    }
    static __device__ __forceinline__ void stage(uint32_t t, uint32_t* w) { w[0] = t; }
    static __device__ __forceinline__ uint32_t key(const Fn& f, const uint32_t* w, const ModD& md, uint64_t D)
    {
        return hash_4u61<POW2>(f, w[0], md, D);
    }
    template <int NF>
    static __device__ __forceinline__ void pair(const Fn (&fn)[HASH_FPL], uint32_t (&m)[HASH_ACC], const uint32_t* wa,
                                                const uint32_t* wb, const ModDV& md, uint64_t D)
    {
        pair_generic<Pol4U61<POW2>, NF>(fn, m, wa, wb, md, D);
    }
    static constexpr int DEG = 4;
};

// 4U with p = 2^61-1 and t < 2^31, the three Horner steps ordered by hand: a power-of-two D <= 2^31
// (half_4u61_pow2), or another D of at most 2^32 / 3 (half_4u61_steps32).  A function keeps c3 as two words and c2, c1, c0 + 1 as register pairs, the 64-bit addends
// of the steps' first multiply-adds, and a pair whose high word stays zero for the second ones.
struct Fn4U61H {
    uint32_t lo3, hi3;
    u32x2 c2, c1, a0;
    mutable u32x2 hz;
};
template <bool POW2>
struct Pol4U61Hand {
    static constexpr int NW = 1;
    static constexpr int MIN_WAVES = 3;          // 168 registers: the coefficients take 80 of them
    static constexpr bool TRACK_MAX = false;
    static constexpr bool SHIFTED_KEY = false;
    static constexpr bool DOUBLED_KEY = false;
    static constexpr bool TWO_MAXIMA = false;
    static constexpr bool SHIFT_END = false;
    static constexpr bool FRAC_KEY = false;
    static constexpr bool GUARDED = false;
    static constexpr bool VARIABLE_NF = true;    // hand-ordered steps exist for 5..8 functions per lane
    using Fn = Fn4U61H;
    static __device__ __forceinline__ Fn load(const uint64_t* c, bool valid, const KArgs&)
    {
        const uint64_t c0 = valid ? c[0] : 0, c1 = valid ? c[1] : 0, c2 = valid ? c[2] : 0, c3 = valid ? c[3] : 0;
        Fn f;
        f.lo3 = (uint32_t)c3; f.hi3 = (uint32_t)(c3 >> 32);
        f.c2 = u32x2{(uint32_t)c2, (uint32_t)(c2 >> 32)};
        f.c1 = u32x2{(uint32_t)c1, (uint32_t)(c1 >> 32)};
        f.a0 = u32x2{(uint32_t)(c0 + 1), (uint32_t)((c0 + 1) >> 32)};
        f.hz = u32x2{0u, 0u};
        return f;
    }
    static __device__ __forceinline__ void stage(uint32_t t, uint32_t* w) { w[0] = t; }
    static __device__ __forceinline__ uint32_t key(const Fn& f, const uint32_t* w, const ModD& md, uint64_t D)
    {
        Fn4U61 g;
        g.c3lo = f.lo3; g.c3hi = f.hi3; g.c2lo = f.c2.x; g.c2hi = f.c2.y; g.c1lo = f.c1.x; g.c1hi = f.c1.y; g.a0lo = f.a0.x; g.a0hi = f.a0.y;
        return hash_4u61<POW2>(g, w[0], md, D);
    }
    template <int NF>
    static __device__ __forceinline__ void pair(const Fn (&fn)[HASH_FPL], uint32_t (&m)[HASH_ACC], const uint32_t* wa,
                                                const uint32_t* wb, const ModDV& md, uint64_t D);
    static constexpr int DEG = 4;
};

// ------------------------------------------------------------------ two nonzeros x 8 functions
// The unit of the hot loop: fold the 16 evaluations of two staged nonzeros into
// the 8 running extrema.  The generic form leaves the schedule to the compiler.
template <class Pol, int NF>
__device__ __forceinline__ void pair_generic(const typename Pol::Fn (&fn)[HASH_FPL], uint32_t (&m)[HASH_ACC],
                                             const uint32_t* wa, const uint32_t* wb, const ModDV& md, uint64_t D)
{
#pragma unroll
    for (int r = 0; r < NF; ++r) {
        uint32_t k0 = Pol::key(fn[r], wa, md, D);
        uint32_t k1 = Pol::key(fn[r], wb, md, D);
        m[r] = Pol::TRACK_MAX ? umax3(m[r], k0, k1) : umin3(m[r], k0, k1);
    }
}

// Widening multiply-add of function slot SLOT.  The
// carry-out it must name is never read; each slot sends it to a scalar register
// pair of its own, s[84:85] to s[98:99].  With one destination for all (a pair of the compiler's choice,
// or vcc) the compiler sees each statement redefine a register of the one before
// and, not knowing what the text holds, puts a wait state between any two of
// them: 28 per step of the 2U loop (with four pairs in turn it still put one before
// every fifth).
#define MH_MAD_TEXT(KIND, SDST, LAST) "v_mad_" #KIND " %0, " SDST ", %1, %2, " LAST
#define MH_MAD(SLOT, KIND, DST, A, B, C)                                                                                 \
    do {                                                                                                           \
        if (((SLOT) & 7) == 0) asm volatile(MH_MAD_TEXT(KIND, "s[84:85]", "%3") : "=v"(DST) : "v"(A), "v"(B), "v"(C) : "s84", "s85"); \
        else if (((SLOT) & 7) == 1) asm volatile(MH_MAD_TEXT(KIND, "s[86:87]", "%3") : "=v"(DST) : "v"(A), "v"(B), "v"(C) : "s86", "s87"); \
        else if (((SLOT) & 7) == 2) asm volatile(MH_MAD_TEXT(KIND, "s[88:89]", "%3") : "=v"(DST) : "v"(A), "v"(B), "v"(C) : "s88", "s89"); \
        else if (((SLOT) & 7) == 3) asm volatile(MH_MAD_TEXT(KIND, "s[90:91]", "%3") : "=v"(DST) : "v"(A), "v"(B), "v"(C) : "s90", "s91"); \
        else if (((SLOT) & 7) == 4) asm volatile(MH_MAD_TEXT(KIND, "s[92:93]", "%3") : "=v"(DST) : "v"(A), "v"(B), "v"(C) : "s92", "s93"); \
        else if (((SLOT) & 7) == 5) asm volatile(MH_MAD_TEXT(KIND, "s[94:95]", "%3") : "=v"(DST) : "v"(A), "v"(B), "v"(C) : "s94", "s95"); \
        else if (((SLOT) & 7) == 6) asm volatile(MH_MAD_TEXT(KIND, "s[96:97]", "%3") : "=v"(DST) : "v"(A), "v"(B), "v"(C) : "s96", "s97"); \
        else asm volatile(MH_MAD_TEXT(KIND, "s[98:99]", "%3") : "=v"(DST) : "v"(A), "v"(B), "v"(C) : "s98", "s99"); \
    } while (0)
#define MH_MAD_ACC(SLOT, KIND, ACC, A, B)                                                                                \
    do {                                                                                                           \
        if (((SLOT) & 7) == 0) asm volatile(MH_MAD_TEXT(KIND, "s[84:85]", "%0") : "+v"(ACC) : "v"(A), "v"(B) : "s84", "s85"); \
        else if (((SLOT) & 7) == 1) asm volatile(MH_MAD_TEXT(KIND, "s[86:87]", "%0") : "+v"(ACC) : "v"(A), "v"(B) : "s86", "s87"); \
        else if (((SLOT) & 7) == 2) asm volatile(MH_MAD_TEXT(KIND, "s[88:89]", "%0") : "+v"(ACC) : "v"(A), "v"(B) : "s88", "s89"); \
        else if (((SLOT) & 7) == 3) asm volatile(MH_MAD_TEXT(KIND, "s[90:91]", "%0") : "+v"(ACC) : "v"(A), "v"(B) : "s90", "s91"); \
        else if (((SLOT) & 7) == 4) asm volatile(MH_MAD_TEXT(KIND, "s[92:93]", "%0") : "+v"(ACC) : "v"(A), "v"(B) : "s92", "s93"); \
        else if (((SLOT) & 7) == 5) asm volatile(MH_MAD_TEXT(KIND, "s[94:95]", "%0") : "+v"(ACC) : "v"(A), "v"(B) : "s94", "s95"); \
        else if (((SLOT) & 7) == 6) asm volatile(MH_MAD_TEXT(KIND, "s[96:97]", "%0") : "+v"(ACC) : "v"(A), "v"(B) : "s96", "s97"); \
        else asm volatile(MH_MAD_TEXT(KIND, "s[98:99]", "%0") : "+v"(ACC) : "v"(A), "v"(B) : "s98", "s99"); \
    } while (0)

// 2U, p = 2^31-1, power-of-two D, with the instruction order fixed by hand.
// On gfx950 a SIMD issues the simple integer instructions (shift right, add,
// sub, and) of two different wavefronts together, but only while neither
// depends on its predecessor; a three-operand instruction issues alone but lets
// another wavefront's simple instruction go beside it, and a multiply lets
// nothing go beside it.  The eight evaluations of one nonzero are therefore
// emitted stage by stage, so that neighbouring instructions never depend on each
// other: eight multiply-adds at raised priority, the simple instructions at the
// normal one (see issue_priority); two such halves, then eight three-operand
// maxima.  half_2u31_pow2 is key_full_2u31 of mh_arith.h, instruction for
// instruction, for the form with two maxima.
template <int NF>
__device__ __forceinline__ void half_2u31_pow2(const Fn2U31 (&fn)[HASH_FPL], uint32_t (&x)[HASH_FPL], uint32_t t)
{
    uint64_t p[HASH_FPL];
    issue_priority<1>();
#pragma unroll
    for (int g = 0; g < NF; ++g) MH_MAD(g, u64_u32, p[g], fn[g].c1, t, fn[g].add);
    issue_priority<0>();
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_lshrrev_b32 %0, 1, %1" : "=v"(x[g]) : "v"((uint32_t)p[g]));
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_add_u32 %0, %0, %1" : "+v"(x[g]) : "v"((uint32_t)(p[g] >> 32)));
    issue_priority<1>();
}
// The doubled key 2 hi + lo (key_full2_2u31), formed with two simple instructions
// (SIMPLE) or with one shift-then-add.  A pair uses one form for each of its nonzeros:
// per evaluation that is one simple and one full-issue instruction (half a maximum
// included), which issue beside each other, where either form alone leaves one class
// without partners.
template <int NF, bool SIMPLE>
__device__ __forceinline__ void half_2u31_doubled(const Fn2U31 (&fn)[HASH_FPL], uint32_t (&x)[HASH_FPL], uint32_t t)
{
    uint64_t p[HASH_FPL];
    issue_priority<1>();
#pragma unroll
    for (int g = 0; g < NF; ++g) MH_MAD(g, u64_u32, p[g], fn[g].c1, t, fn[g].add);
    if constexpr (SIMPLE) {
        issue_priority<0>();
#pragma unroll
        for (int g = 0; g < NF; ++g) asm volatile("v_add_u32 %0, %1, %1" : "=v"(x[g]) : "v"((uint32_t)(p[g] >> 32)));
#pragma unroll
        for (int g = 0; g < NF; ++g) asm volatile("v_add_u32 %0, %0, %1" : "+v"(x[g]) : "v"((uint32_t)p[g]));
        issue_priority<1>();
    } else {
#pragma unroll
        for (int g = 0; g < NF; ++g)
            asm volatile("v_lshl_add_u32 %0, %1, 1, %2" : "=v"(x[g]) : "v"((uint32_t)(p[g] >> 32)), "v"((uint32_t)p[g]));
    }
}
template <int NF, bool TWO>
__device__ __forceinline__ void pair_2u31_pow2(const Fn2U31 (&fn)[HASH_FPL], uint32_t (&m)[HASH_ACC], uint32_t ta, uint32_t tb)
{
    uint32_t xa[HASH_FPL], xb[HASH_FPL];
    if constexpr (TWO) {
        half_2u31_pow2<NF>(fn, xa, ta);
        half_2u31_pow2<NF>(fn, xb, tb);
#pragma unroll
        for (int g = 0; g < NF; ++g)
            asm volatile("v_max3_i32 %0, %0, %1, %2" : "+v"(m[g]) : "v"(xa[g]), "v"(xb[g]));
#pragma unroll
        for (int g = 0; g < NF; ++g)
            asm volatile("v_max3_u32 %0, %0, %1, %2" : "+v"(m[HASH_FPL + g]) : "v"(xa[g]), "v"(xb[g]));
    } else {
        half_2u31_doubled<NF, true>(fn, xa, ta);
        half_2u31_doubled<NF, false>(fn, xb, tb);
#pragma unroll
        for (int g = 0; g < NF; ++g)
            asm volatile("v_max3_u32 %0, %0, %1, %2" : "+v"(m[g]) : "v"(xa[g]), "v"(xb[g]));
    }
}

// 4U, p = 2^31-1, power-of-two D, same idea: three chained multiply-adds per
// evaluation are issued function-major so that each waits for a result that is
// 16 instructions old; the fold of nonzero A overlaps the last multiply-adds of
// nonzero B.  Arithmetic of fold_4u31 (mh_arith.h), instruction for instruction; FULL
// ends there and keeps two maxima, otherwise key_neg_4u31's two instructions follow.
template <int NF, bool FULL>
__device__ __forceinline__ void half_4u31_pow2(const Fn4U31 (&fn)[HASH_FPL], uint32_t (&y)[HASH_FPL], const uint32_t* w,
                                               uint32_t amount, uint32_t p31)
{
    uint64_t acc[HASH_FPL];
    uint32_t u[HASH_FPL], v[HASH_FPL];
    issue_priority<1>();
#pragma unroll
    for (int g = 0; g < NF; ++g)
        MH_MAD(g, i64_i32, acc[g], fn[g].c1, w[0], fn[g].add);
#pragma unroll
    for (int g = 0; g < NF; ++g)
        MH_MAD_ACC(g, i64_i32, acc[g], fn[g].c2, w[1]);
#pragma unroll
    for (int g = 0; g < NF; ++g)
        MH_MAD_ACC(g, i64_i32, acc[g], fn[g].c3, w[2]);
    issue_priority<0>();
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_lshrrev_b32 %0, 1, %1" : "=v"(y[g]) : "v"((uint32_t)acc[g]));
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_and_b32 %0, %1, %2" : "=v"(u[g]) : "v"((uint32_t)(acc[g] >> 32)), "v"(p31));
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_lshrrev_b32 %0, 31, %1" : "=v"(v[g]) : "v"((uint32_t)(acc[g] >> 32)));
    issue_priority<1>();       // one three-operand add (full issue) instead of two simple adds: fewer instructions in all
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_add3_u32 %0, %0, %1, %2" : "+v"(y[g]) : "v"(u[g]), "v"(v[g]));
    if constexpr (!FULL) {      // key_neg_4u31: amount = 32 - log2 D; the full key is the folded value as it stands
        issue_priority<0>();
#pragma unroll
        for (int g = 0; g < NF; ++g) asm volatile("v_lshrrev_b32 %0, 31, %1" : "=v"(u[g]) : "v"(y[g]));
        issue_priority<1>();
#pragma unroll
        for (int g = 0; g < NF; ++g) asm volatile("v_add_lshl_u32 %0, %0, %1, %2" : "+v"(y[g]) : "v"(u[g]), "s"(amount));
    }
}

template <int NF, bool FULL>
__device__ __forceinline__ void pair_4u31_pow2(const Fn4U31 (&fn)[HASH_FPL], uint32_t (&m)[HASH_ACC],
                                               const uint32_t* wa, const uint32_t* wb, uint32_t amount, uint32_t p31)
{
    uint32_t ya[HASH_FPL], yb[HASH_FPL];
    half_4u31_pow2<NF, FULL>(fn, ya, wa, amount, p31);
    half_4u31_pow2<NF, FULL>(fn, yb, wb, amount, p31);
    if constexpr (FULL) {
#pragma unroll
        for (int g = 0; g < NF; ++g)
            asm volatile("v_max3_i32 %0, %0, %1, %2" : "+v"(m[g]) : "v"(ya[g]), "v"(yb[g]));
#pragma unroll
        for (int g = 0; g < NF; ++g)
            asm volatile("v_max3_u32 %0, %0, %1, %2" : "+v"(m[HASH_FPL + g]) : "v"(ya[g]), "v"(yb[g]));
        return;
    }
#pragma unroll
    for (int g = 0; g < NF; ++g)
        asm volatile("v_max3_u32 %0, %0, %1, %2" : "+v"(m[g]) : "v"(ya[g]), "v"(yb[g]));
}

// Other D, p = 2^31-1: the same stage-major order with the exact quotient of
// mh_arith.h appended.  The canonical residue r is written into the low word of
// the register pair that held the product, so that the closing multiply-add
// r + q (2^32 - D) can take the pair as its 64-bit addend (only the low word of
// its result is used).  Arithmetic of hash_2u31_raw / hash_4u31_np2.

template <int NF>
__device__ __forceinline__ void half_2u31_np2(const Fn2U31 (&fn)[HASH_FPL], u32x2 (&p)[HASH_FPL], uint32_t t, const ModDV& md)
{
    uint32_t x[HASH_FPL], y[HASH_FPL], r;
    issue_priority<1>();
#pragma unroll
    for (int g = 0; g < NF; ++g) MH_MAD(g, u64_u32, p[g], fn[g].c1, t, fn[g].add);
    issue_priority<0>();
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_lshrrev_b32 %0, 1, %1" : "=v"(x[g]) : "v"(p[g].x));
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_add_u32 %0, %0, %1" : "+v"(x[g]) : "v"(p[g].y));
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_sub_u32 %0, %1, %2" : "=v"(y[g]) : "v"(x[g]), "v"(md.p31));
    issue_priority<1>();
#pragma unroll
    for (int g = 0; g < NF; ++g) {
        asm volatile("v_min_u32 %0, %1, %2" : "=v"(r) : "v"(x[g]), "v"(y[g]));
        p[g].x = r;
    }
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_mul_hi_u32 %0, %1, %2" : "=v"(x[g]) : "v"(p[g].x), "v"(md.M));
    issue_priority<0>();
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_lshrrev_b32 %0, %1, %0" : "+v"(x[g]) : "v"(md.sh));
    issue_priority<1>();
#pragma unroll
    for (int g = 0; g < NF; ++g) MH_MAD_ACC(g, u64_u32, p[g], x[g], md.negD);
}
// The same up to the canonical residue, which is written into the high word of the
// function's {bias, r} pair; one multiply-add r m_low + {bias, r} and one funnel shift
// give the fractional key (frac_key of mh_arith.h).
template <int NF>
__device__ __forceinline__ void half_2u31_frac(const Fn2U31F (&fn)[HASH_FPL], uint32_t (&key)[HASH_FPL], uint32_t t, const ModDV& md)
{
    u32x2 p[HASH_FPL];
    uint32_t x[HASH_FPL], y[HASH_FPL], r;
    issue_priority<1>();
#pragma unroll
    for (int g = 0; g < NF; ++g) MH_MAD(g, u64_u32, p[g], fn[g].c1, t, fn[g].add);
    issue_priority<0>();
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_lshrrev_b32 %0, 1, %1" : "=v"(x[g]) : "v"(p[g].x));
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_add_u32 %0, %0, %1" : "+v"(x[g]) : "v"(p[g].y));
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_sub_u32 %0, %1, %2" : "=v"(y[g]) : "v"(x[g]), "v"(md.p31));
    issue_priority<1>();
#pragma unroll
    for (int g = 0; g < NF; ++g) {
        asm volatile("v_min_u32 %0, %1, %2" : "=v"(r) : "v"(x[g]), "v"(y[g]));
        fn[g].bq.y = r;
    }
#pragma unroll
    for (int g = 0; g < NF; ++g) MH_MAD(g, u64_u32, p[g], fn[g].bq.y, md.frac_m, fn[g].bq);
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_alignbit_b32 %0, %1, %2, %3" : "=v"(key[g]) : "v"(p[g].y), "v"(p[g].x), "s"(md.frac_l));
}
template <int NF>
__device__ __forceinline__ void pair_2u31_frac(const Fn2U31F (&fn)[HASH_FPL], uint32_t (&m)[HASH_ACC], uint32_t ta,
                                               uint32_t tb, const ModDV& md)
{
    uint32_t ka[HASH_FPL], kb[HASH_FPL];
    half_2u31_frac<NF>(fn, ka, ta, md);
    half_2u31_frac<NF>(fn, kb, tb, md);
#pragma unroll
    for (int g = 0; g < NF; ++g)
        asm volatile("v_min3_u32 %0, %0, %1, %2" : "+v"(m[g]) : "v"(ka[g]), "v"(kb[g]));
}

// D of at least p / 3: the same up to the canonical residue r, then r - D, r - 2D and the
// smallest of the three (reduce_small_quotient of mh_arith.h).
template <int NF>
__device__ __forceinline__ void half_2u31_bigd(const Fn2U31 (&fn)[HASH_FPL], uint32_t (&v)[HASH_FPL], uint32_t t, const ModDV& md)
{
    u32x2 p[HASH_FPL];
    uint32_t x[HASH_FPL], y[HASH_FPL];
    issue_priority<1>();
#pragma unroll
    for (int g = 0; g < NF; ++g) MH_MAD(g, u64_u32, p[g], fn[g].c1, t, fn[g].add);
    issue_priority<0>();
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_lshrrev_b32 %0, 1, %1" : "=v"(x[g]) : "v"(p[g].x));
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_add_u32 %0, %0, %1" : "+v"(x[g]) : "v"(p[g].y));
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_sub_u32 %0, %1, %2" : "=v"(y[g]) : "v"(x[g]), "v"(md.p31));
    issue_priority<1>();
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_min_u32 %0, %1, %2" : "=v"(v[g]) : "v"(x[g]), "v"(y[g]));
    issue_priority<0>();
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_add_u32 %0, %1, %2" : "=v"(x[g]) : "v"(v[g]), "v"(md.negD));
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_add_u32 %0, %1, %2" : "=v"(y[g]) : "v"(x[g]), "v"(md.negD));
    issue_priority<1>();
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_min3_u32 %0, %0, %1, %2" : "+v"(v[g]) : "v"(x[g]), "v"(y[g]));
}
template <int NF>
__device__ __forceinline__ void pair_2u31_bigd(const Fn2U31 (&fn)[HASH_FPL], uint32_t (&m)[HASH_ACC], uint32_t ta,
                                               uint32_t tb, const ModDV& md)
{
    uint32_t va[HASH_FPL], vb[HASH_FPL];
    half_2u31_bigd<NF>(fn, va, ta, md);
    half_2u31_bigd<NF>(fn, vb, tb, md);
#pragma unroll
    for (int g = 0; g < NF; ++g)
        asm volatile("v_min3_u32 %0, %0, %1, %2" : "+v"(m[g]) : "v"(va[g]), "v"(vb[g]));
}

template <int NF>
__device__ __forceinline__ void pair_2u31_np2(const Fn2U31 (&fn)[HASH_FPL], uint32_t (&m)[HASH_ACC], uint32_t ta,
                                              uint32_t tb, const ModDV& md)
{
    u32x2 pa[HASH_FPL], pb[HASH_FPL];
    half_2u31_np2<NF>(fn, pa, ta, md);
    half_2u31_np2<NF>(fn, pb, tb, md);
#pragma unroll
    for (int g = 0; g < NF; ++g)
        asm volatile("v_min3_u32 %0, %0, %1, %2" : "+v"(m[g]) : "v"(pa[g].x), "v"(pb[g].x));
}

template <int NF, int MODE, class FnT>      // MODE 0: exact quotient, 1: fractional key, 2: quotient of at most 2
__device__ __forceinline__ void half_4u31_np2(const FnT (&fn)[HASH_FPL], u32x2 (&acc)[HASH_FPL], const uint32_t* w,
                                              const ModDV& md)
{
    uint32_t y[HASH_FPL], u[HASH_FPL], v[HASH_FPL], r;
    issue_priority<1>();
#pragma unroll
    for (int g = 0; g < NF; ++g)
        MH_MAD(g, i64_i32, acc[g], fn[g].c1, w[0], fn[g].add);
#pragma unroll
    for (int g = 0; g < NF; ++g)
        MH_MAD_ACC(g, i64_i32, acc[g], fn[g].c2, w[1]);
#pragma unroll
    for (int g = 0; g < NF; ++g)
        MH_MAD_ACC(g, i64_i32, acc[g], fn[g].c3, w[2]);
    issue_priority<0>();
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_lshrrev_b32 %0, 1, %1" : "=v"(y[g]) : "v"(acc[g].x));
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_and_b32 %0, %1, %2" : "=v"(u[g]) : "v"(acc[g].y), "v"(md.p31));
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_lshrrev_b32 %0, 31, %1" : "=v"(v[g]) : "v"(acc[g].y));
    issue_priority<1>();       // one three-operand add (full issue) instead of two simple adds: fewer instructions in all
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_add3_u32 %0, %0, %1, %2" : "+v"(y[g]) : "v"(u[g]), "v"(v[g]));
    issue_priority<0>();
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_add_u32 %0, -1, %1" : "=v"(u[g]) : "v"(y[g]));
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_xor_b32 %0, %0, %1" : "+v"(y[g]) : "v"(md.sign));
    issue_priority<1>();
#pragma unroll
    for (int g = 0; g < NF; ++g) {
        asm volatile("v_min_u32 %0, %1, %2" : "=v"(r) : "v"(u[g]), "v"(y[g]));
        if constexpr (MODE == 1) fn[g].bq.y = r; else acc[g].x = r;
    }
    if constexpr (MODE == 2) {        // reduce_small_quotient: the smallest of r, r - D, r - 2D
        issue_priority<0>();
#pragma unroll
        for (int g = 0; g < NF; ++g) asm volatile("v_add_u32 %0, %1, %2" : "=v"(u[g]) : "v"(acc[g].x), "v"(md.negD));
#pragma unroll
        for (int g = 0; g < NF; ++g) asm volatile("v_add_u32 %0, %1, %2" : "=v"(y[g]) : "v"(u[g]), "v"(md.negD));
        issue_priority<1>();
#pragma unroll
        for (int g = 0; g < NF; ++g) {
            r = acc[g].x;
            asm volatile("v_min3_u32 %0, %0, %1, %2" : "+v"(r) : "v"(u[g]), "v"(y[g]));
            acc[g].x = r;
        }
    } else if constexpr (MODE == 1) { // frac_key: r m_low + {bias, r}, then the 32 bits from bit l up
#pragma unroll
        for (int g = 0; g < NF; ++g) MH_MAD(g, u64_u32, acc[g], fn[g].bq.y, md.frac_m, fn[g].bq);
#pragma unroll
        for (int g = 0; g < NF; ++g) {
            asm volatile("v_alignbit_b32 %0, %1, %2, %3" : "=v"(r) : "v"(acc[g].y), "v"(acc[g].x), "s"(md.frac_l));
            acc[g].x = r;
        }
    } else {
#pragma unroll
        for (int g = 0; g < NF; ++g) asm volatile("v_mul_hi_u32 %0, %1, %2" : "=v"(u[g]) : "v"(acc[g].x), "v"(md.M));
#pragma unroll
        for (int g = 0; g < NF; ++g) asm volatile("v_lshrrev_b32 %0, %1, %0" : "+v"(u[g]) : "v"(md.sh));
#pragma unroll
        for (int g = 0; g < NF; ++g)
            MH_MAD_ACC(g, u64_u32, acc[g], u[g], md.negD);
    }
}

template <int NF, int MODE, class FnT>
__device__ __forceinline__ void pair_4u31_np2(const FnT (&fn)[HASH_FPL], uint32_t (&m)[HASH_ACC], const uint32_t* wa,
                                              const uint32_t* wb, const ModDV& md)
{
    u32x2 ya[HASH_FPL], yb[HASH_FPL];
    half_4u31_np2<NF, MODE>(fn, ya, wa, md);
    half_4u31_np2<NF, MODE>(fn, yb, wb, md);
#pragma unroll
    for (int g = 0; g < NF; ++g)
        asm volatile("v_min3_u32 %0, %0, %1, %2" : "+v"(m[g]) : "v"(ya[g].x), "v"(yb[g].x));
}

// 2U, p = 2^61-1, power-of-two D <= 2^31: key_neg_2u61 of mh_arith.h, eight
// functions on one nonzero, stage by stage: two multiply-adds, the funnel shift
// H >> 29, one add for the key (the coefficients were rotated so that it needs no
// shift).
template <int NF>
__device__ __forceinline__ void half_2u61_pow2(const Fn2U61V (&fn)[HASH_FPL], uint32_t (&y)[HASH_FPL], uint32_t t)
{
    u32x2 L[HASH_FPL], H[HASH_FPL];
    uint32_t s[HASH_FPL], r;
    issue_priority<1>();
#pragma unroll
    for (int g = 0; g < NF; ++g) MH_MAD(g, u64_u32, L[g], fn[g].e0, t, fn[g].add);
    issue_priority<0>();
#pragma unroll
    for (int g = 0; g < NF; ++g) {
        asm volatile("v_mov_b32 %0, %1" : "=v"(r) : "v"(L[g].y));
        fn[g].hz.x = r;
    }
    issue_priority<1>();
#pragma unroll
    for (int g = 0; g < NF; ++g) MH_MAD(g, u64_u32, H[g], fn[g].e1, t, fn[g].hz);
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_alignbit_b32 %0, %1, %2, 29" : "=v"(s[g]) : "v"(H[g].y), "v"(H[g].x));
    issue_priority<0>();
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_add_u32 %0, %1, %2" : "=v"(y[g]) : "v"(L[g].x), "v"(s[g]));
    issue_priority<1>();
}

// 2U, p = 2^61-1, other D of at most 2^32 / 3 (so t < 2^31): the folded value x = y + (H >> 29) in [1, 2^61 +
// 2^32), congruent to X + 1 (residue_2u61 of mh_arith.h), with bit 61 folded once more x' = (X mod p) + 1 in
// [1, p]; then reduce61_mod_d's 32-bit steps on x' (the quotient estimate from bits 29..60 of x, which only
// makes it a hair smaller; the low word of x' exact), and at the end the 1 comes off: of u = (x' mod D') - 1
// and u + D' the smaller as unsigned words.  A carry links the two words of x.
// The two halves of a 64-bit addition.  The carry is an operand of both statements (a scalar pair of the
// compiler's choice, one per function slot), so that nothing the compiler places between them can take its
// register.
__device__ __forceinline__ void add_carry_out(uint32_t& d, uint64_t& carry, uint32_t a, uint32_t b)
{
    asm volatile("v_add_co_u32 %0, %1, %2, %3" : "=v"(d), "=s"(carry) : "v"(a), "v"(b));
}
__device__ __forceinline__ void add_carry_in(uint32_t& d, uint64_t& carry)       // d += carry (0 or 1)
{
    asm volatile("v_addc_co_u32 %0, %1, 0, %0, %1" : "+v"(d), "+s"(carry));
}
template <int NF, class FnT>
__device__ __forceinline__ void residue_mod_d_steps32(const FnT (&fn)[HASH_FPL], uint32_t (&xlo)[HASH_FPL], uint32_t (&xhi)[HASH_FPL],
                                                      uint32_t (&y)[HASH_FPL], const ModDV& md);
template <int NF>
__device__ __forceinline__ void half_2u61_steps32(const Fn2U61V (&fn)[HASH_FPL], uint32_t (&y)[HASH_FPL], uint32_t t, const ModDV& md)
{
    u32x2 L[HASH_FPL], H[HASH_FPL];
    uint32_t s[HASH_FPL], xlo[HASH_FPL], xhi[HASH_FPL], r;
    uint64_t carry[HASH_FPL];
    issue_priority<1>();
#pragma unroll
    for (int g = 0; g < NF; ++g) MH_MAD(g, u64_u32, L[g], fn[g].e0, t, fn[g].add);
    issue_priority<0>();
#pragma unroll
    for (int g = 0; g < NF; ++g) {
        asm volatile("v_mov_b32 %0, %1" : "=v"(r) : "v"(L[g].y));
        fn[g].hz.x = r;
    }
    issue_priority<1>();
#pragma unroll
    for (int g = 0; g < NF; ++g) MH_MAD(g, u64_u32, H[g], fn[g].e1, t, fn[g].hz);
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_alignbit_b32 %0, %1, %2, 29" : "=v"(s[g]) : "v"(H[g].y), "v"(H[g].x));
#pragma unroll
    for (int g = 0; g < NF; ++g) add_carry_out(xlo[g], carry[g], L[g].x, s[g]);                    // low word of x
    issue_priority<0>();
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_and_b32 %0, %1, %2" : "=v"(xhi[g]) : "v"(H[g].x), "v"(md.mask29));
    issue_priority<1>();
#pragma unroll
    for (int g = 0; g < NF; ++g) add_carry_in(xhi[g], carry[g]);                                  // high word: bits 32..61 of x
    residue_mod_d_steps32<NF>(fn, xlo, xhi, y, md);
}
// The second part: from the folded value x = (xhi : xlo) in [1, 2^61 + 2^32), congruent to X + 1, to (X mod p) mod D.
// Entered and left at raised priority.  (4U with p = 2^61-1 ends its Horner steps on the same kind of value.)
template <int NF, class FnT>
__device__ __forceinline__ void residue_mod_d_steps32(const FnT (&fn)[HASH_FPL], uint32_t (&xlo)[HASH_FPL], uint32_t (&xhi)[HASH_FPL],
                                                      uint32_t (&y)[HASH_FPL], const ModDV& md)
{
    u32x2 L[HASH_FPL];
    uint32_t s[HASH_FPL], q[HASH_FPL], r;
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_alignbit_b32 %0, %1, %2, 29" : "=v"(s[g]) : "v"(xhi[g]), "v"(xlo[g]));   // bits 29..60 of x
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_mul_hi_u32 %0, %1, %2" : "=v"(q[g]) : "v"(s[g]), "v"(md.m61q));
    issue_priority<0>();
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_lshrrev_b32 %0, 29, %1" : "=v"(xhi[g]) : "v"(xhi[g]));         // bit 61
#pragma unroll
    for (int g = 0; g < NF; ++g) {                      // low word of x', into the pair whose high word is zero
        asm volatile("v_add_u32 %0, %1, %2" : "=v"(r) : "v"(xlo[g]), "v"(xhi[g]));
        fn[g].hz.x = r;
    }
    issue_priority<1>();
    // x' - q D' in [0, 3 D') is the low word of q (2^32 - D') + x': a widening multiply-add again (the 32-bit
    // multiply that keeps the low word takes four issue slots, this one takes one)
#pragma unroll
    for (int g = 0; g < NF; ++g) MH_MAD(g, u64_u32, L[g], q[g], md.negdp, fn[g].hz);
    issue_priority<0>();
#pragma unroll
    for (int g = 0; g < NF; ++g) xlo[g] = L[g].x;
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_sub_u32 %0, %1, %2" : "=v"(s[g]) : "v"(xlo[g]), "v"(md.dp));
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_sub_u32 %0, %1, %2" : "=v"(q[g]) : "v"(s[g]), "v"(md.dp));
    issue_priority<1>();
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_min3_u32 %0, %0, %1, %2" : "+v"(xlo[g]) : "v"(s[g]), "v"(q[g]));   // x' mod D'
    issue_priority<0>();
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_add_u32 %0, -1, %0" : "+v"(xlo[g]));
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_add_u32 %0, %1, %2" : "=v"(s[g]) : "v"(xlo[g]), "v"(md.dp));
    issue_priority<1>();
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_min_u32 %0, %1, %2" : "=v"(y[g]) : "v"(xlo[g]), "v"(s[g]));   // (X mod p) mod D'
    if (md.dp != md.D) {               // D' is a multiple of D: the exact quotient by an invariant divisor finishes it (values below 2^30)
#pragma unroll
        for (int g = 0; g < NF; ++g) asm volatile("v_mul_hi_u32 %0, %1, %2" : "=v"(q[g]) : "v"(y[g]), "v"(md.M));
        issue_priority<0>();
#pragma unroll
        for (int g = 0; g < NF; ++g) asm volatile("v_lshrrev_b32 %0, %1, %0" : "+v"(q[g]) : "v"(md.sh));
#pragma unroll
        for (int g = 0; g < NF; ++g) {
            asm volatile("v_mov_b32 %0, %1" : "=v"(r) : "v"(y[g]));
            fn[g].hz.x = r;
        }
        issue_priority<1>();
#pragma unroll
        for (int g = 0; g < NF; ++g) MH_MAD(g, u64_u32, L[g], q[g], md.negD, fn[g].hz);      // low word: y - q D
#pragma unroll
        for (int g = 0; g < NF; ++g) y[g] = L[g].x;
    }
}

// One Horner step of horner_step_61 (mh_arith.h) for t < 2^31, eight functions stage by stage: the value
// (hi : lo), hi <= 2^29, times t plus a 64-bit coefficient is L = lo t + c (the coefficient is the 64-bit addend:
// below 2^63 + 2^61) and H = hi t + (L >> 32) < 2^61; bits 61 and up, H >> 29, are added to the 61 bits below
// them, with a carry from the low word to the high one.
template <int NF, class LoOf, class HiOf, class COf>
__device__ __forceinline__ void horner_step_4u61(const Fn4U61H (&fn)[HASH_FPL], uint32_t (&lo)[HASH_FPL], uint32_t (&hi)[HASH_FPL],
                                                 LoOf lo_in, HiOf hi_in, COf c, uint32_t t, const ModDV& md)
{
    u32x2 L[HASH_FPL], H[HASH_FPL];
    uint32_t s[HASH_FPL], r;
    uint64_t carry[HASH_FPL];
    issue_priority<1>();
#pragma unroll
    for (int g = 0; g < NF; ++g) MH_MAD(g, u64_u32, L[g], lo_in(g), t, c(g));
    issue_priority<0>();
#pragma unroll
    for (int g = 0; g < NF; ++g) {
        asm volatile("v_mov_b32 %0, %1" : "=v"(r) : "v"(L[g].y));
        fn[g].hz.x = r;
    }
    issue_priority<1>();
#pragma unroll
    for (int g = 0; g < NF; ++g) MH_MAD(g, u64_u32, H[g], hi_in(g), t, fn[g].hz);
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_alignbit_b32 %0, %1, %2, 29" : "=v"(s[g]) : "v"(H[g].y), "v"(H[g].x));
#pragma unroll
    for (int g = 0; g < NF; ++g) add_carry_out(lo[g], carry[g], L[g].x, s[g]);
    issue_priority<0>();
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_and_b32 %0, %1, %2" : "=v"(hi[g]) : "v"(H[g].x), "v"(md.mask29));
    issue_priority<1>();
#pragma unroll
    for (int g = 0; g < NF; ++g) add_carry_in(hi[g], carry[g]);
}
// residue_lo_4u61 of mh_arith.h and the mask: lo + (hi >> 29) - 1, lowest s bits
template <int NF>
__device__ __forceinline__ void half_4u61_pow2(const Fn4U61H (&fn)[HASH_FPL], uint32_t (&y)[HASH_FPL], uint32_t t, const ModDV& md)
{
    uint32_t lo[HASH_FPL], hi[HASH_FPL], lo2[HASH_FPL], hi2[HASH_FPL];
    horner_step_4u61<NF>(fn, lo, hi, [&](int g) { return fn[g].lo3; }, [&](int g) { return fn[g].hi3; }, [&](int g) { return fn[g].c2; }, t, md);
    horner_step_4u61<NF>(fn, lo2, hi2, [&](int g) { return lo[g]; }, [&](int g) { return hi[g]; }, [&](int g) { return fn[g].c1; }, t, md);
    horner_step_4u61<NF>(fn, lo, hi, [&](int g) { return lo2[g]; }, [&](int g) { return hi2[g]; }, [&](int g) { return fn[g].a0; }, t, md);
    issue_priority<0>();
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_lshrrev_b32 %0, 29, %0" : "+v"(hi[g]));
    issue_priority<1>();
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_add3_u32 %0, %0, %1, -1" : "+v"(lo[g]) : "v"(hi[g]));
    issue_priority<0>();
#pragma unroll
    for (int g = 0; g < NF; ++g) asm volatile("v_and_b32 %0, %1, %2" : "=v"(y[g]) : "v"(lo[g]), "v"(md.mask));
    issue_priority<1>();
}
// the same for another D of at most 2^32 / 3: the Horner steps end on the value that residue_mod_d_steps32 starts from
template <int NF>
__device__ __forceinline__ void half_4u61_steps32(const Fn4U61H (&fn)[HASH_FPL], uint32_t (&y)[HASH_FPL], uint32_t t, const ModDV& md)
{
    uint32_t lo[HASH_FPL], hi[HASH_FPL], lo2[HASH_FPL], hi2[HASH_FPL];
    horner_step_4u61<NF>(fn, lo, hi, [&](int g) { return fn[g].lo3; }, [&](int g) { return fn[g].hi3; }, [&](int g) { return fn[g].c2; }, t, md);
    horner_step_4u61<NF>(fn, lo2, hi2, [&](int g) { return lo[g]; }, [&](int g) { return hi[g]; }, [&](int g) { return fn[g].c1; }, t, md);
    horner_step_4u61<NF>(fn, lo, hi, [&](int g) { return lo2[g]; }, [&](int g) { return hi2[g]; }, [&](int g) { return fn[g].a0; }, t, md);
    residue_mod_d_steps32<NF>(fn, lo, hi, y, md);
}
template <bool POW2>
template <int NF>
__device__ __forceinline__ void Pol4U61Hand<POW2>::pair(const Fn (&fn)[HASH_FPL], uint32_t (&m)[HASH_ACC], const uint32_t* wa,
                                                        const uint32_t* wb, const ModDV& md, uint64_t)
{
    uint32_t ya[HASH_FPL], yb[HASH_FPL];
    if constexpr (POW2) {
        half_4u61_pow2<NF>(fn, ya, wa[0], md);
        half_4u61_pow2<NF>(fn, yb, wb[0], md);
    } else {
        half_4u61_steps32<NF>(fn, ya, wa[0], md);
        half_4u61_steps32<NF>(fn, yb, wb[0], md);
    }
#pragma unroll
    for (int g = 0; g < NF; ++g)
        asm volatile("v_min3_u32 %0, %0, %1, %2" : "+v"(m[g]) : "v"(ya[g]), "v"(yb[g]));
}

// Ablation: the definition evaluated with the % operator on runtime moduli (Horner
// form keeps every product below 2^62).  This is what Section 3.4's shift/mask
// routine replaces; it exists only to be timed against the Mersenne kernels.
template <int DEGREE>
struct PolGenericMod {
    static constexpr int NW = 1;
    static constexpr int MIN_WAVES = 3;        // no spills, so that the ablation times the arithmetic only
    static constexpr bool TRACK_MAX = false;
    static constexpr bool SHIFTED_KEY = false;
    static constexpr bool DOUBLED_KEY = false;
    static constexpr bool TWO_MAXIMA = false;
    static constexpr bool SHIFT_END = false;
    static constexpr bool FRAC_KEY = false;
    static constexpr bool GUARDED = false;
    static constexpr bool VARIABLE_NF = false;
    static constexpr int DEG = DEGREE;
    struct Fn { uint64_t c[DEGREE]; uint64_t p; };
    static __device__ __forceinline__ Fn load(const uint64_t* c, bool valid, const KArgs& a)
    {
        Fn f;
#pragma unroll
        for (int i = 0; i < DEGREE; ++i) f.c[i] = valid ? c[i] : 0;
        f.p = a.prime;                 // a kernel argument, so that the compiler cannot specialise the % on it
        return f;
    }
    static __device__ __forceinline__ void stage(uint32_t t, uint32_t* w) { w[0] = t; }
    static __device__ __forceinline__ uint32_t key(const Fn& f, const uint32_t* w, const ModD&, uint64_t D)
    {
        const uint64_t t = w[0];
        uint64_t acc = f.c[DEGREE - 1];
#pragma unroll
        for (int i = DEGREE - 2; i >= 0; --i) acc = (acc * t + f.c[i]) % f.p;
        return (uint32_t)(acc % D);
    }
    template <int NF>
    static __device__ __forceinline__ void pair(const Fn (&fn)[HASH_FPL], uint32_t (&m)[HASH_ACC], const uint32_t* wa,
                                                const uint32_t* wb, const ModDV& md, uint64_t D)
    {
        pair_generic<PolGenericMod<DEGREE>, NF>(fn, m, wa, wb, md, D);
    }
};

// multiply-shift 2U: md.M = 32 - log2(D).  The kernel tracks the minimum of an
// order-preserving 32-bit key and shifts it down once per row (mh_arith.h), so
// the unit of the hot loop is 16 multiply-adds and 8 three-operand minima.
template <bool HIGH>
struct Pol2UMS32 {
    static constexpr int NW = 1;
    static constexpr int MIN_WAVES = 5;
    static constexpr bool TRACK_MAX = false;
    static constexpr bool SHIFTED_KEY = false;
    static constexpr bool DOUBLED_KEY = false;
    static constexpr bool TWO_MAXIMA = false;
    static constexpr bool SHIFT_END = true;
    static constexpr bool FRAC_KEY = false;
    static constexpr bool GUARDED = false;
    static constexpr bool VARIABLE_NF = true;    // hand-ordered steps exist for 5..8 functions per lane
    using Fn = Fn2UMS32;
    static __device__ __forceinline__ Fn load(const uint64_t* c, bool valid, const KArgs& a)
    {
        return valid ? prep_2ums32_key<HIGH>(c[0], c[1], a.md.M) : prep_2ums32_key<HIGH>(0, 0, a.md.M);
    }
    static __device__ __forceinline__ void stage(uint32_t t, uint32_t* w) { w[0] = t; }
    static __device__ __forceinline__ uint32_t key(const Fn& f, const uint32_t* w, const ModD&, uint64_t)
    {
        return key_2ums32(f, w[0]);
    }
    template <int NF>
    static __device__ __forceinline__ void pair(const Fn (&fn)[HASH_FPL], uint32_t (&m)[HASH_ACC], const uint32_t* wa,
                                                const uint32_t* wb, const ModDV&, uint64_t)
    {
        uint64_t pa[HASH_FPL], pb[HASH_FPL];
#pragma unroll
        for (int g = 0; g < NF; ++g)
            MH_MAD(g, u64_u32, pa[g], fn[g].c1, wa[0], fn[g].add);
#pragma unroll
        for (int g = 0; g < NF; ++g)
            MH_MAD(g, u64_u32, pb[g], fn[g].c1, wb[0], fn[g].add);
#pragma unroll
        for (int g = 0; g < NF; ++g)
            asm volatile("v_min3_u32 %0, %0, %1, %2" : "+v"(m[g]) : "v"((uint32_t)pa[g]), "v"((uint32_t)pb[g]));
    }
    static constexpr int DEG = 2;
};

template <>
template <int NF>
__device__ __forceinline__ void Pol2U31<FORM_FULL_TWO>::pair(const Fn (&fn)[HASH_FPL], uint32_t (&m)[HASH_ACC], const uint32_t* wa,
                                                             const uint32_t* wb, const ModDV&, uint64_t)
{
    pair_2u31_pow2<NF, true>(fn, m, wa[0], wb[0]);
}
template <>
template <int NF>
__device__ __forceinline__ void Pol2U31<FORM_FULL>::pair(const Fn (&fn)[HASH_FPL], uint32_t (&m)[HASH_ACC], const uint32_t* wa,
                                                         const uint32_t* wb, const ModDV&, uint64_t)
{
    pair_2u31_pow2<NF, false>(fn, m, wa[0], wb[0]);
}
template <>
template <int NF>
__device__ __forceinline__ void Pol2U31<FORM_FRAC_D>::pair(const Fn (&fn)[HASH_FPL], uint32_t (&m)[HASH_ACC], const uint32_t* wa,
                                                           const uint32_t* wb, const ModDV& md, uint64_t)
{
    pair_2u31_frac<NF>(fn, m, wa[0], wb[0], md);
}
template <>
template <int NF>
__device__ __forceinline__ void Pol2U31<FORM_BIG_D>::pair(const Fn (&fn)[HASH_FPL], uint32_t (&m)[HASH_ACC], const uint32_t* wa,
                                                          const uint32_t* wb, const ModDV& md, uint64_t)
{
    pair_2u31_bigd<NF>(fn, m, wa[0], wb[0], md);
}
template <>
template <int NF>
__device__ __forceinline__ void Pol2U31<FORM_ANY_D>::pair(const Fn (&fn)[HASH_FPL], uint32_t (&m)[HASH_ACC], const uint32_t* wa,
                                                     const uint32_t* wb, const ModDV& md, uint64_t)
{
    pair_2u31_np2<NF>(fn, m, wa[0], wb[0], md);
}

template <>
template <int NF>
__device__ __forceinline__ void Pol4U31<true, true>::pair(const Fn (&fn)[HASH_FPL], uint32_t (&m)[HASH_ACC], const uint32_t* wa,
                                                          const uint32_t* wb, const ModDV& md, uint64_t)
{
    pair_4u31_pow2<NF, true>(fn, m, wa, wb, 0u, md.p31);
}
template <>
template <int NF>
__device__ __forceinline__ void Pol4U31<true, false>::pair(const Fn (&fn)[HASH_FPL], uint32_t (&m)[HASH_ACC], const uint32_t* wa,
                                                           const uint32_t* wb, const ModDV& md, uint64_t)
{
    pair_4u31_pow2<NF, false>(fn, m, wa, wb, md.kshift, md.p31);
}
template <>
template <int NF>
__device__ __forceinline__ void Pol4U31<false>::pair(const Fn (&fn)[HASH_FPL], uint32_t (&m)[HASH_ACC], const uint32_t* wa,
                                                     const uint32_t* wb, const ModDV& md, uint64_t)
{
    pair_4u31_np2<NF, 0>(fn, m, wa, wb, md);
}
template <>
template <int NF>
__device__ __forceinline__ void Pol4U31<false, false, 2>::pair(const Fn (&fn)[HASH_FPL], uint32_t (&m)[HASH_ACC], const uint32_t* wa,
                                                               const uint32_t* wb, const ModDV& md, uint64_t)
{
    pair_4u31_np2<NF, 2>(fn, m, wa, wb, md);
}
template <>
template <int NF>
__device__ __forceinline__ void Pol4U31<false, false, 1>::pair(const Fn (&fn)[HASH_FPL], uint32_t (&m)[HASH_ACC], const uint32_t* wa,
                                                                  const uint32_t* wb, const ModDV& md, uint64_t)
{
    pair_4u31_np2<NF, 1>(fn, m, wa, wb, md);
}

template <>
template <int NF>
__device__ __forceinline__ void Pol2U61<true, false>::pair(const Fn (&fn)[HASH_FPL], uint32_t (&m)[HASH_ACC], const uint32_t* wa,
                                                           const uint32_t* wb, const ModDV&, uint64_t)
{
    uint32_t ya[HASH_FPL], yb[HASH_FPL];
    half_2u61_pow2<NF>(fn, ya, wa[0]);
    half_2u61_pow2<NF>(fn, yb, wb[0]);
#pragma unroll
    for (int g = 0; g < NF; ++g)
        asm volatile("v_max3_u32 %0, %0, %1, %2" : "+v"(m[g]) : "v"(ya[g]), "v"(yb[g]));
}
template <>
template <int NF>
__device__ __forceinline__ void Pol2U61<false, false>::pair(const Fn (&fn)[HASH_FPL], uint32_t (&m)[HASH_ACC], const uint32_t* wa,
                                                            const uint32_t* wb, const ModDV& md, uint64_t D)
{
    pair_generic<Pol2U61<false, false>, NF>(fn, m, wa, wb, md, D);
}
template <>
template <int NF>
__device__ __forceinline__ void Pol2U61<false, true>::pair(const Fn (&fn)[HASH_FPL], uint32_t (&m)[HASH_ACC], const uint32_t* wa,
                                                           const uint32_t* wb, const ModDV& md, uint64_t)
{
    uint32_t ya[HASH_FPL], yb[HASH_FPL];
    half_2u61_steps32<NF>(fn, ya, wa[0], md);
    half_2u61_steps32<NF>(fn, yb, wb[0], md);
#pragma unroll
    for (int g = 0; g < NF; ++g)
        asm volatile("v_min3_u32 %0, %0, %1, %2" : "+v"(m[g]) : "v"(ya[g]), "v"(yb[g]));
}

// ------------------------------------------------------------------ staging
// Requests the nonzeros [begin+off, begin+off+extent) of a row of `len` nonzeros
// (off < len) into 4 registers per lane (element lane + 64 q), coalesced.  Entries
// past the end of the row repeat its last nonzero: the minimum is idempotent, so
// duplicates change nothing and the inner loops need no masks.  Groups of 64 entries
// from `extent` on are not read by the caller and not loaded.
__device__ __forceinline__ void load_tile(const uint32_t* col, int64_t begin, uint32_t len, uint32_t off, int extent,
                                          int lane, uint32_t (&r)[4])
{
    const uint32_t* src = col + begin;
    const uint32_t last = len - 1u;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        if (WAVE * q < extent) {       // wavefront-uniform: a short row issues no load for the groups it lacks
            const uint32_t e = off + (uint32_t)lane + (uint32_t)(WAVE * q);
            r[q] = __builtin_nontemporal_load(src + (e < last ? e : last));
        }
    }
}
// The same for a tile that lies wholly inside the row (off + 256 <= len): no entry needs the clamp,
// and the four loads share one lane offset.
__device__ __forceinline__ void load_full_tile(const uint32_t* col, int64_t begin, uint32_t off, int lane, uint32_t (&r)[4])
{
    const uint32_t* src = col + begin + off;
#pragma unroll
    for (int q = 0; q < 4; ++q) r[q] = __builtin_nontemporal_load(src + lane + WAVE * q);
}
// How the steps of the hash kernel walk a tile of in_tile nonzeros with n_slices lane slices: a
// step takes four nonzeros per slice (two pairs); when the last step would hold at most two per
// slice it is done as a single pair.  extent = tile entries read (repeats of the last one included).
struct TileWalk {
    int n_steps, odd_pair, extent;
};
__device__ __forceinline__ TileWalk walk_of(uint32_t in_tile, int n_slices)
{
    TileWalk t;
    const int n_pairs = (int)((in_tile + 2u * n_slices - 1u) / (2u * n_slices));
    t.n_steps = n_pairs >> 1;
    t.odd_pair = n_pairs & 1;
    t.extent = (t.n_steps * 4 + t.odd_pair * 2) * n_slices;
    return t;
}

// Packed input: requests the words of the tile that starts `off` nonzeros into an item (off a multiple of
// 256) into 4 registers per lane (word lane + 64 q).  A tile that would leave the word array is reported
// and read as zeros.
__device__ __forceinline__ void load_packed_tile(const KArgs& a, int64_t wbegin, uint32_t w, uint32_t len, uint32_t off, int lane,
                                                 uint32_t (&r)[4])
{
    const uint32_t m = len - off < PACKED_TILE ? len - off : PACKED_TILE;
    const uint32_t nw = packed_tile_words(m, w);
    const int64_t at = wbegin + (int64_t)(off / PACKED_TILE) * (int64_t)packed_tile_words(PACKED_TILE, w);
    const bool inside = at >= 0 && at + (int64_t)nw <= a.pk_words_len;
    if (!inside && lane == 0) atomicOr(&a.hdr->status, 1u);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t j = (uint32_t)lane + (uint32_t)(WAVE * q);
        r[q] = 0;
        if ((uint32_t)(WAVE * q) < nw && inside && j < nw) r[q] = __builtin_nontemporal_load(a.pk_words + at + j);
    }
}
// The 256 indices of such a tile from its words: lane l gets indices 4l .. 4l+3 in v.  The words pass
// through `buf` (LDS of this wavefront, at least 258 words); a field is w bits at bit (i - 1) w of the
// bit string that starts at word 1, the index is the first word plus the running sum of the fields.
// Indices past the end of the item repeat its last one (their fields read as 0).
__device__ __forceinline__ void decode_packed_tile(uint32_t* buf, const uint32_t (&r)[4], uint32_t w, uint32_t len, uint32_t off, int lane_in,
                                                   uint32_t (&v)[4])
{
    // Everything below that depends on the lane number alone would otherwise be worked out once, ahead of
    // the loops over units and tiles, and sit in registers through the steps where they are scarcest.
    int lane = lane_in;
    asm volatile("" : "+v"(lane));
    const uint32_t m = len - off < PACKED_TILE ? len - off : PACKED_TILE;
    const uint32_t nw = packed_tile_words(m, w);
#pragma unroll
    for (int q = 0; q < 4; ++q)
        if ((uint32_t)(WAVE * q) < nw + 2u) buf[lane + WAVE * q] = r[q];     // words from nw on are zeros: a field may reach one word further
    if (lane < 2) buf[PACKED_TILE + lane] = 0;
    wave_sync_lds();
    const uint32_t mask = w >= 32u ? 0xFFFFFFFFu : (1u << w) - 1u;
    uint32_t run = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t i = 4u * (uint32_t)lane + (uint32_t)q;
        uint32_t d = 0;
        if (i == 0) {
            d = buf[0];
        } else if (i < m && w > 0) {
            const uint32_t bit = (i - 1u) * w, j = 1u + (bit >> 5), sh = bit & 31u;
            d = (uint32_t)((((uint64_t)buf[j + 1] << 32) | buf[j]) >> sh) & mask;
        }
        run += d;
        v[q] = run;
    }
    // Inclusive sums of the lanes' totals over the wavefront with data-parallel shifts: within each row of
    // 16 lanes by 1, 2, 4 and 8 (a lane without a source adds 0), then lane 15 of rows 0 and 2 goes to the
    // row after it, then lane 31 to the upper 32 lanes.
    uint32_t below = run;
    below += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)below, 0x111, 0xf, 0xf, false);    // row_shr:1
    below += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)below, 0x112, 0xf, 0xf, false);    // row_shr:2
    below += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)below, 0x114, 0xf, 0xf, false);    // row_shr:4
    below += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)below, 0x118, 0xf, 0xf, false);    // row_shr:8
    below += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)below, 0x142, 0xa, 0xf, false);    // row_bcast:15 into rows 1 and 3
    below += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)below, 0x143, 0xc, 0xf, false);    // row_bcast:31 into rows 2 and 3
    below -= run;
#pragma unroll
    for (int q = 0; q < 4; ++q) v[q] += below;
    wave_sync_lds();
}

// Minimum over lanes that are a power of two apart, without the LDS: the upper half of the
// wavefront comes down with a lane swap, the upper 16 of 32 lanes with a swizzle, smaller
// distances with data-parallel row shifts.  After min_from_above<D> lane i (i mod 2D < D) holds
// the minimum of its own value and that of lane i + D; the other lanes hold nothing of use.
template <int D>
__device__ __forceinline__ uint32_t min_from_above(uint32_t v)
{
    uint32_t o;
    if constexpr (D == 32) {
        o = __builtin_amdgcn_permlane32_swap(v, v, false, false)[1];      // lanes 0..31 receive lanes 32..63
    } else if constexpr (D == 16) {
        o = (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, 0x401F);        // swap neighbouring groups of 16 lanes
    } else {
        static_assert(D == 8 || D == 4 || D == 2 || D == 1, "distance");
        o = (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x100 + D, 0xf, 0xf, false);   // row_shl:D, lanes without a source keep v
    }
    return o < v ? o : v;
}
// the minimum of v over all 64 lanes, in every lane
__device__ __forceinline__ uint32_t wave_min(uint32_t v)
{
    v = min_from_above<32>(v);
    v = min_from_above<16>(v);
    v = min_from_above<8>(v);
    v = min_from_above<4>(v);
    v = min_from_above<2>(v);
    v = min_from_above<1>(v);
    return first_lane_value(v);
}

// ------------------------------------------------------------------ the hash kernel
// PACKED: the rows arrive as tiles of differences (a.pk_*) instead of a.col_idx; a tile of that form is a
// staging tile, so its words are what is requested ahead and it is decoded while it is staged.
template <class Pol, int NF, bool PACKED>
__global__ __launch_bounds__(BLOCK) __attribute__((amdgpu_waves_per_eu(Pol::MIN_WAVES, 8))) void mh_hash_kernel(KArgs a)
{
    __shared__ uint32_t s_tile[WAVES_PER_BLOCK][Pol::NW][TILE];
    __shared__ uint32_t s_mins[WAVES_PER_BLOCK][HASH_FTILE];
    using RunItems = RunItemsT<PACKED>;
    using Unit = UnitT<PACKED>;
    __shared__ RunItems s_items[WAVES_PER_BLOCK];

    const int lane = threadIdx.x & (WAVE - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);      // wave-uniform: keep it in a scalar register
    uint32_t(*tile)[TILE] = s_tile[wave];
    uint32_t* mins = s_mins[wave];
    RunItems* run_items = &s_items[wave];

    const int fl_lanes = 1 << a.log2_fl;            // lanes that cover one function tile
    const int n_slices = WAVE >> a.log2_fl;         // the other lane bits take slices of the nonzeros
    const int fl = lane & (fl_lanes - 1);
    const int slice = lane >> a.log2_fl;

    const uint32_t n_long = a.hdr->n_long < a.cap_long ? a.hdr->n_long : (uint32_t)a.cap_long;
    const uint32_t n_short = a.hdr->n_short < a.cap_short ? a.hdr->n_short : (uint32_t)a.cap_short;
    const uint64_t n_units = ((uint64_t)n_long + n_short) * (uint64_t)a.n_ftiles;

    const ModDV md = vector_constants(a.md);

    typename Pol::Fn fn[HASH_FPL];
    int cur_ftile = -1;

    // The first nonzeros of a unit are requested before the unit starts: for the first unit
    // right here, for later ones during the last tile of the unit before (when the next unit
    // belongs to the same run of the work list) or after a new run has been fetched.
    UnitStreamT<PACKED> units;
    Unit cur;
    uint32_t regs[4];
    // the first tile of a unit: its nonzeros, or the words they are packed in
    auto request_first_tile = [&](const Unit& u) {
        if (u.len == 0) return;
        if constexpr (PACKED) load_packed_tile(a, u.wbegin, u.w, u.len, 0, lane, regs);
        else load_tile(a.col_idx, wave_uniform64(u.begin), u.len, 0, walk_of(u.len < (uint32_t)TILE ? u.len : (uint32_t)TILE, n_slices).extent, lane, regs);
    };
    bool have = units.init(a, n_units, (uint64_t)n_long * (uint64_t)a.n_ftiles, gridDim.x * WAVES_PER_BLOCK,
                           blockIdx.x * WAVES_PER_BLOCK + wave, n_long, lane, run_items, &cur);
    if (have) request_first_tile(cur);
    while (have) {
        const int ftile = cur.ftile;
        const int j_base = ftile * a.ftile_size + fl * NF;
        if (ftile != cur_ftile) {
            const uint64_t* coeffs = static_cast<const uint64_t*>(a.params);
#pragma unroll
            for (int r = 0; r < NF; ++r) {
                int j = j_base + r;
                bool valid = j < a.k;
                fn[r] = Pol::load(coeffs + (size_t)(valid ? j : 0) * Pol::DEG, valid, a);
            }
            cur_ftile = ftile;
        }
        const int64_t begin = cur.begin;
        const uint32_t len = cur.len;
        const uint32_t unit_row = cur.row, unit_slot = cur.slot;
        int64_t unit_wbegin = 0;
        uint32_t unit_w = 0;
        if constexpr (PACKED) {
            unit_wbegin = cur.wbegin;
            unit_w = cur.w;
        }
        Unit nxt;
        bool have_next = false;        // the next unit is known and its first tile is on its way

        uint32_t m[HASH_ACC];
#pragma unroll
        for (int r = 0; r < NF; ++r) m[r] = Pol::TWO_MAXIMA ? (uint32_t)FULL_KEY_INIT : Pol::TRACK_MAX ? 0u : EMPTY_MIN;
        if (Pol::TWO_MAXIMA) {
#pragma unroll
            for (int r = 0; r < NF; ++r) m[HASH_FPL + r] = FULL_KEY_INIT_UNSIGNED;
        }

        if (len > 0) {
            for (uint32_t off = 0; off < len; off += TILE) {
                const uint32_t in_tile = len - off < (uint32_t)TILE ? len - off : (uint32_t)TILE;
                const TileWalk walk = walk_of(in_tile, n_slices);
                const int n_steps = walk.n_steps, extent = walk.extent;
                // stage: pre-compute what depends on t alone
                if constexpr (PACKED) {
                    uint32_t vals[4];  // lane l decodes nonzeros 4l .. 4l+3 of the tile (all 256 entries get a value)
                    decode_packed_tile(mins, regs, unit_w, len, off, lane, vals);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        uint32_t t = vals[q];
                        if (a.validate && (uint64_t)t >= a.D) {
                            atomicOr(&a.hdr->status, 2u);
                            t = 0;
                        }
                        uint32_t w[Pol::NW];
                        Pol::stage(t, w);
#pragma unroll
                        for (int i = 0; i < Pol::NW; ++i) tile[i][4 * lane + q] = w[i];
                    }
                } else if (in_tile == (uint32_t)TILE && !a.validate) {      // the usual tile: whole, and nothing to check
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        uint32_t w[Pol::NW];
                        Pol::stage(regs[q], w);
#pragma unroll
                        for (int i = 0; i < Pol::NW; ++i) tile[i][lane + WAVE * q] = w[i];
                    }
                } else if (!a.validate) {                                   // a partial tile, nothing to check
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        if (WAVE * q >= extent) break;               // wavefront-uniform: never read, not staged
                        uint32_t w[Pol::NW];
                        Pol::stage(regs[q], w);
#pragma unroll
                        for (int i = 0; i < Pol::NW; ++i) tile[i][lane + WAVE * q] = w[i];
                    }
                } else {               // one nonzero per lane and register
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        if (WAVE * q >= extent) break;               // wavefront-uniform: never read, not staged
                        uint32_t t = regs[q];
                        if ((uint64_t)t >= a.D) {
                            atomicOr(&a.hdr->status, 2u);
                            t = 0;
                        }
                        uint32_t w[Pol::NW];
                        Pol::stage(t, w);
#pragma unroll
                        for (int i = 0; i < Pol::NW; ++i) tile[i][lane + WAVE * q] = w[i];
                    }
                }
                wave_sync_lds();
                if (off + TILE < len) {
                    if constexpr (PACKED) {
                        load_packed_tile(a, unit_wbegin, unit_w, len, off + TILE, lane, regs);
                    } else {
                        const uint32_t rest = len - off - TILE;
                        if (rest >= (uint32_t)TILE) load_full_tile(a.col_idx, begin, off + TILE, lane, regs);
                        else load_tile(a.col_idx, begin, len, off + TILE, walk_of(rest, n_slices).extent, lane, regs);
                    }
                } else {               // last tile: the registers are free for the first tile of the next unit
                    have_next = units.peek_and_take(run_items, &nxt);
                    if (have_next) request_first_tile(nxt);
                }

                for (int s = 0; s < n_steps; ++s) {
                    const int e = 4 * (s * n_slices + slice);
                    uint32_t w[4][Pol::NW];
#pragma unroll
                    for (int i = 0; i < Pol::NW; ++i) {
                        uint4 v = *reinterpret_cast<const uint4*>(&tile[i][e]);
                        w[0][i] = v.x; w[1][i] = v.y; w[2][i] = v.z; w[3][i] = v.w;
                    }
                    Pol::template pair<NF>(fn, m, w[0], w[1], md, a.D);
                    Pol::template pair<NF>(fn, m, w[2], w[3], md, a.D);
                }
                if (walk.odd_pair) {
                    const int e = 4 * n_steps * n_slices + 2 * slice;     // the slices share what is left, two nonzeros each
                    uint32_t w[2][Pol::NW];
#pragma unroll
                    for (int i = 0; i < Pol::NW; ++i) {
                        uint2 v = *reinterpret_cast<const uint2*>(&tile[i][e]);
                        w[0][i] = v.x; w[1][i] = v.y;
                    }
                    Pol::template pair<NF>(fn, m, w[0], w[1], md, a.D);
                }
                wave_sync_lds();
            }
            // A GUARDED policy keeps keys that are exact unless the running value itself, or a guard
            // word beside it, says otherwise (rarely); bit r of `doubt` marks such a value.
            uint32_t doubt = 0;
            if constexpr (Pol::GUARDED) {
                // hardly ever: the smallest of the lane's maxima decides with one comparison, and the
                // bit mask is only worked out when some lane of the wavefront has a doubtful value
                uint32_t lowest = m[0];
#pragma unroll
                for (int r = 1; r + 1 < NF; r += 2) lowest = umin3(lowest, m[r], m[r + 1]);
                if ((NF & 1) == 0) lowest = lowest < m[NF - 1] ? lowest : m[NF - 1];
                if (__builtin_amdgcn_ballot_w64(lowest < Pol::doubt_below(md)) != 0ull) doubt = Pol::template doubtful<NF>(m, md);
            }
            if (Pol::TRACK_MAX) {      // back from keys to the minimum location
#pragma unroll
                for (int r = 0; r < NF; ++r) {
                    if (Pol::TWO_MAXIMA) m[r] = finish_full_keys((int32_t)m[r], m[HASH_FPL + r], md.frot, md.mask);
                    else if (Pol::DOUBLED_KEY) m[r] = finish_full2_key(m[r], md.frot, md.mask);
                    else m[r] = Pol::SHIFTED_KEY ? finish_neg_key(m[r], md.kshift, md.mask) : md.mask - m[r];
                }
            }
            if (Pol::FRAC_KEY) {       // from the fractional key back to the hashed location
#pragma unroll
                for (int r = 0; r < NF; ++r) m[r] = finish_frac_key(m[r], (uint32_t)a.D);
            }
            if (Pol::SHIFT_END) {      // from the order-preserving key back to the hashed location
#pragma unroll
                for (int r = 0; r < NF; ++r) m[r] = finish_2ums32(m[r], a.md.M);
            }
            if constexpr (Pol::GUARDED) {
                // Every doubtful value is computed again from the definition: the whole wavefront
                // evaluates that one function on all nonzeros of the item, a lane each, and the
                // owner takes the minimum (over the whole item, which its slice is part of).
                uint64_t owners = __builtin_amdgcn_ballot_w64(doubt != 0u);      // doubt is 0 in every lane unless the test above fired
                if (!PACKED && owners != 0ull && len <= SHORT_ITEM) {
                    // A short item makes many of its values doubtful (few evaluations stand behind
                    // each) and is cheap to go through: every lane sees to its own values.
                    for (uint32_t which = doubt; which; which &= which - 1) {
                        const int r = __builtin_ctz(which);
                        if (j_base + r >= a.k) continue;
                        const uint64_t* src = static_cast<const uint64_t*>(a.params) + (size_t)(j_base + r) * Pol::DEG;
                        uint64_t c[Pol::DEG];
#pragma unroll
                        for (int i = 0; i < Pol::DEG; ++i) c[i] = src[i];
                        uint32_t best = EMPTY_MIN;
                        for (uint32_t e = 0; e < len; ++e) {
                            uint32_t t = a.col_idx[begin + e];
                            if (a.validate && (uint64_t)t >= a.D) t = 0;
                            const uint32_t h = Pol::exact_hash(c, t, a.md, a.D);
                            best = h < best ? h : best;
                        }
#pragma unroll
                        for (int q = 0; q < NF; ++q)
                            if (q == r) m[q] = best;
                    }
                    owners = 0ull;
                }
                while (owners) {
                    const int owner = __builtin_ctzll(owners);
                    owners &= owners - 1;
                    uint32_t which = (uint32_t)__builtin_amdgcn_readlane((int)doubt, owner);
                    const int j0 = __builtin_amdgcn_readlane(j_base, owner);
                    while (which) {
                        const int r = __builtin_ctz(which);
                        which &= which - 1;
                        if (j0 + r >= a.k) continue;                    // an unused slot: never stored
                        const uint64_t* c = static_cast<const uint64_t*>(a.params) + (size_t)(j0 + r) * Pol::DEG;
                        uint32_t best = EMPTY_MIN;
                        if constexpr (PACKED) {    // the item's tiles once more (the registers of the main loop may hold the next unit's words)
                            for (uint32_t off2 = 0; off2 < len; off2 += TILE) {
                                uint32_t words2[4], vals[4];
                                load_packed_tile(a, unit_wbegin, unit_w, len, off2, lane, words2);
                                decode_packed_tile(mins, words2, unit_w, len, off2, lane, vals);
                                *reinterpret_cast<uint4*>(&tile[0][4 * lane]) = uint4{vals[0], vals[1], vals[2], vals[3]};
                                wave_sync_lds();
#pragma unroll 1
                                for (int e = lane; e < TILE; e += WAVE) {      // entries past the end repeat the last nonzero: harmless
                                    uint32_t t = tile[0][e];
                                    if (a.validate && (uint64_t)t >= a.D) t = 0;
                                    const uint32_t h = Pol::exact_hash(c, t, a.md, a.D);
                                    best = h < best ? h : best;
                                }
                                wave_sync_lds();
                            }
                        } else {
                            for (uint32_t e = (uint32_t)lane; e < len; e += WAVE) {
                                uint32_t t = a.col_idx[begin + e];
                                if (a.validate && (uint64_t)t >= a.D) t = 0;
                                const uint32_t h = Pol::exact_hash(c, t, a.md, a.D);
                                best = h < best ? h : best;
                            }
                        }
                        best = wave_min(best);
                        if (lane == owner) {
#pragma unroll
                            for (int q = 0; q < NF; ++q)
                                if (q == r) m[q] = best;
                        }
                    }
                }
            }
        } else if (Pol::TRACK_MAX) {
#pragma unroll
            for (int r = 0; r < NF; ++r) m[r] = EMPTY_MIN;
        }
        // merge the slices of nonzeros (lanes that share fl): the values come down to slice 0, which stores them
        if (n_slices >= 2) {
#pragma unroll
            for (int r = 0; r < NF; ++r) m[r] = min_from_above<32>(m[r]);
        }
        if (n_slices >= 4) {
#pragma unroll
            for (int r = 0; r < NF; ++r) m[r] = min_from_above<16>(m[r]);
        }
        if (n_slices >= 8) {
#pragma unroll
            for (int r = 0; r < NF; ++r) m[r] = min_from_above<8>(m[r]);
        }
        if (n_slices >= 16) {
#pragma unroll
            for (int r = 0; r < NF; ++r) m[r] = min_from_above<4>(m[r]);
        }
        if (n_slices >= 32) {
#pragma unroll
            for (int r = 0; r < NF; ++r) m[r] = min_from_above<2>(m[r]);
        }
        if (n_slices >= 64) {
#pragma unroll
            for (int r = 0; r < NF; ++r) m[r] = min_from_above<1>(m[r]);
        }
        const int nf_tile = a.k - ftile * a.ftile_size < a.ftile_size ? a.k - ftile * a.ftile_size : a.ftile_size;
        if (unit_slot == NO_SLOT) {
            bool stored = false;
            if constexpr (NF == HASH_FPL) {
                if (a.lane_pack) {
                    lane_pack_store(a, m, unit_row, j_base, slice == 0);
                    if (ftile == a.n_ftiles - 1) {     // pad bytes up to the row pitch are zero
                        uint8_t* dst = a.out + (int64_t)unit_row * a.out_stride;
                        for (int64_t q = a.sig_bytes + lane; q < a.out_stride; q += WAVE) dst[q] = 0;
                    }
                    stored = true;
                }
            }
            if (!stored) {
                if (slice == 0) {
#pragma unroll
                    for (int r = 0; r < NF; ++r) mins[fl * NF + r] = m[r];
                }
                wave_sync_lds();
                wave_pack_store(a, mins, unit_row, ftile * a.ftile_size, nf_tile, ftile == a.n_ftiles - 1, lane);
                wave_sync_lds();
            }
        } else if (slice == 0) {
            uint32_t* part = a.partials + (size_t)unit_slot * (size_t)a.k;
#pragma unroll
            for (int r = 0; r < NF; ++r)
                if (j_base + r < a.k) part[j_base + r] = m[r];
        }
        // on to the next unit: already under way, or drawn now (which waits for the ticket and the run's records)
        if (have_next) {
            cur = nxt;
        } else {
            have = units.advance(a, n_long, lane, run_items, &cur);
            if (have) request_first_tile(cur);
        }
    }
}

// ------------------------------------------------------------------ the permutation-table kernel
// table[t][j] = pi_j(t), index-major (Section 1.5: a permutation matrix of size
// D x k): the k values of one nonzero are contiguous, so each nonzero costs one
// coalesced read of 4k bytes.  VEC4: lane l reads entries 4l..4l+3 with one
// 16-byte load (needs perm_ld % 4 == 0 and a 16-byte aligned table); otherwise
// lane l reads entries l, l+64, l+128, l+192.
template <bool VEC4>
__global__ __launch_bounds__(BLOCK) void mh_perm_kernel(KArgs a)
{
    __shared__ uint32_t s_tile[WAVES_PER_BLOCK][TILE];
    __shared__ uint32_t s_mins[WAVES_PER_BLOCK][PERM_FTILE];
    using RunItems = RunItemsT<false>;
    using Unit = UnitT<false>;
    __shared__ RunItems s_items[WAVES_PER_BLOCK];
    const int lane = threadIdx.x & (WAVE - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint32_t* tile = s_tile[wave];
    uint32_t* mins = s_mins[wave];
    RunItems* run_items = &s_items[wave];
    const uint32_t* table = static_cast<const uint32_t*>(a.params);

    const uint32_t n_long = a.hdr->n_long < a.cap_long ? a.hdr->n_long : (uint32_t)a.cap_long;
    const uint32_t n_short = a.hdr->n_short < a.cap_short ? a.hdr->n_short : (uint32_t)a.cap_short;
    const uint64_t n_units = ((uint64_t)n_long + n_short) * (uint64_t)a.n_ftiles;
    constexpr int U = 8;               // nonzeros in flight per lane

    // the steps read whole groups of U entries: what a tile of n nonzeros needs staged
    auto extent_of = [](uint32_t n) { return (int)(((n < (uint32_t)TILE ? n : (uint32_t)TILE) + U - 1) / U * U); };
    UnitStreamT<false> units;
    Unit cur;
    uint32_t regs[4];
    bool have = units.init(a, n_units, (uint64_t)n_long * (uint64_t)a.n_ftiles, gridDim.x * WAVES_PER_BLOCK,
                           blockIdx.x * WAVES_PER_BLOCK + wave, n_long, lane, run_items, &cur);
    if (have && cur.len > 0) load_tile(a.col_idx, cur.begin, cur.len, 0, extent_of(cur.len), lane, regs);
    while (have) {
        const int ftile = cur.ftile;
        const int64_t begin = cur.begin;
        const uint32_t len = cur.len;
        const uint32_t unit_row = cur.row, unit_slot = cur.slot;
        Unit nxt;
        bool have_next = false;
        const int j0 = ftile * PERM_FTILE;
        const int nf_tile = a.k - j0 < PERM_FTILE ? a.k - j0 : PERM_FTILE;

        // function slots of this lane and whether they exist
        int jl[PERM_FPL];
        bool ok[PERM_FPL];
#pragma unroll
        for (int r = 0; r < PERM_FPL; ++r) {
            jl[r] = VEC4 ? lane * PERM_FPL + r : lane + WAVE * r;
            ok[r] = jl[r] < nf_tile;
        }
        uint32_t m[PERM_FPL];
#pragma unroll
        for (int r = 0; r < PERM_FPL; ++r) m[r] = EMPTY_MIN;

        if (len > 0) {
            for (uint32_t off = 0; off < len; off += TILE) {
                const int extent = extent_of(len - off);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if (WAVE * q >= extent) break;               // wavefront-uniform: never read, not staged
                    uint32_t t = regs[q];
                    if (a.validate && (uint64_t)t >= a.D) {
                        atomicOr(&a.hdr->status, 2u);
                        t = 0;
                    }
                    tile[lane + WAVE * q] = t;
                }
                wave_sync_lds();
                if (off + TILE < len) {
                    load_tile(a.col_idx, begin, len, off + TILE, extent_of(len - off - TILE), lane, regs);
                } else {               // last tile: request the first tile of the next unit of this run
                    have_next = units.peek_and_take(run_items, &nxt);
                    if (have_next && nxt.len > 0) load_tile(a.col_idx, nxt.begin, nxt.len, 0, extent_of(nxt.len), lane, regs);
                }
                const uint32_t in_tile = len - off < (uint32_t)TILE ? len - off : (uint32_t)TILE;
                const int n_steps = (int)((in_tile + U - 1) / U);
                for (int s = 0; s < n_steps; ++s) {
                    uint32_t tt[U];
#pragma unroll
                    for (int u = 0; u < U; u += 4) {
                        uint4 v = *reinterpret_cast<const uint4*>(&tile[s * U + u]);
                        tt[u] = v.x; tt[u + 1] = v.y; tt[u + 2] = v.z; tt[u + 3] = v.w;
                    }
                    if (VEC4) {
                        u32x4 g[U];
                        const bool lane_ok = lane * PERM_FPL < nf_tile;
#pragma unroll
                        for (int u = 0; u < U; ++u) {
                            const uint32_t t = first_lane_value(tt[u]);
                            const uint32_t* rowp = table + (size_t)t * (size_t)a.perm_ld + j0;
                            const u32x4 none = {EMPTY_MIN, EMPTY_MIN, EMPTY_MIN, EMPTY_MIN};
                            g[u] = lane_ok ? __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(rowp) + lane) : none;
                        }
#pragma unroll
                        for (int u = 0; u < U; ++u) {
                            m[0] = g[u].x < m[0] ? g[u].x : m[0];
                            m[1] = g[u].y < m[1] ? g[u].y : m[1];
                            m[2] = g[u].z < m[2] ? g[u].z : m[2];
                            m[3] = g[u].w < m[3] ? g[u].w : m[3];
                        }
                    } else {
                        uint32_t g[U][PERM_FPL];
#pragma unroll
                        for (int u = 0; u < U; ++u) {
                            const uint32_t t = first_lane_value(tt[u]);
                            const uint32_t* rowp = table + (size_t)t * (size_t)a.perm_ld + j0;
#pragma unroll
                            for (int r = 0; r < PERM_FPL; ++r)
                                g[u][r] = ok[r] ? __builtin_nontemporal_load(rowp + jl[r]) : EMPTY_MIN;
                        }
#pragma unroll
                        for (int u = 0; u < U; ++u)
#pragma unroll
                            for (int r = 0; r < PERM_FPL; ++r) m[r] = g[u][r] < m[r] ? g[u][r] : m[r];
                    }
                }
                wave_sync_lds();
            }
        }
        if (unit_slot == NO_SLOT) {
#pragma unroll
            for (int r = 0; r < PERM_FPL; ++r) mins[jl[r]] = m[r];
            wave_sync_lds();
            wave_pack_store(a, mins, unit_row, j0, nf_tile, ftile == a.n_ftiles - 1, lane);
            wave_sync_lds();
        } else {
            uint32_t* part = a.partials + (size_t)unit_slot * (size_t)a.k + j0;
#pragma unroll
            for (int r = 0; r < PERM_FPL; ++r)
                if (ok[r]) part[jl[r]] = m[r];
        }
        if (have_next) {
            cur = nxt;
        } else {
            have = units.advance(a, n_long, lane, run_items, &cur);
            if (have && cur.len > 0) load_tile(a.col_idx, cur.begin, cur.len, 0, extent_of(cur.len), lane, regs);
        }
    }
}

// ------------------------------------------------------------------ finalize split rows
// The minimum over the vectors of partial minima of every split row and function tile (a unit), packed
// and stored.  A block takes 16 units at a time, one per wavefront; a unit of up to FIN_ALONE vectors is
// its wavefront's alone (large batches have tens of thousands of such rows), a larger one waits until the
// whole block turns to it: wavefront w then takes vectors w, w + 16, ..., the 16 results meet in the LDS and
// the first wavefront packs and stores (a row of 10^5 nonzeros in a small batch has some hundred vectors; one
// wavefront going through them alone, four loads at a time, took 120 microseconds).  Either way two vectors
// are in flight per round, a lane reading its up to eight functions of each.
constexpr int FIN_WAVES = 16;
constexpr int FIN_BLOCK = FIN_WAVES * WAVE;
constexpr uint32_t FIN_ALONE = 8;
constexpr int FIN_FPL = MAX_FTILE / WAVE;
// v[i] = minimum over vectors first, first + step, ... (below n) of function j0 + lane + 64 i; nf functions in the tile
__device__ __forceinline__ void merge_parts(const KArgs& a, const uint32_t* first_vec, uint32_t first, uint32_t step, uint32_t n, int j0,
                                            int nf, int lane, uint32_t (&v)[FIN_FPL])
{
    // (a function past the end of the tile reads the tile's last one instead: loads without conditions all go out together)
    int at[FIN_FPL];
#pragma unroll
    for (int i = 0; i < FIN_FPL; ++i) {
        at[i] = lane + WAVE * i < nf ? lane + WAVE * i : nf - 1;
        v[i] = EMPTY_MIN;
    }
    const size_t pitch = (size_t)step * (size_t)a.k;
    const uint32_t* p = first_vec + (size_t)first * (size_t)a.k + j0;
    for (uint32_t c = first; c < n; c += 2 * step) {           // two vectors a round (the last one perhaps twice)
        const uint32_t* q = c + step < n ? p + pitch : p;
        uint32_t o[FIN_FPL], o2[FIN_FPL];
#pragma unroll
        for (int i = 0; i < FIN_FPL; ++i) {
            o[i] = p[at[i]];
            o2[i] = q[at[i]];
        }
#pragma unroll
        for (int i = 0; i < FIN_FPL; ++i) v[i] = umin3(v[i], o[i], o2[i]);
        p += 2 * pitch;
    }
}
__global__ __launch_bounds__(FIN_BLOCK) void mh_finalize_kernel(KArgs a, int ftile_size)
{
    __shared__ uint32_t s_part[FIN_WAVES][MAX_FTILE];
    __shared__ uint32_t s_mins[MAX_FTILE];
    __shared__ uint32_t s_big[FIN_WAVES];
    const int lane = threadIdx.x & (WAVE - 1);
    const int wave = threadIdx.x >> 6;
    const uint32_t n_split = a.hdr->n_split < a.cap_split ? a.hdr->n_split : (uint32_t)a.cap_split;
    const uint64_t n_units = (uint64_t)n_split * (uint64_t)a.n_ftiles;
    for (uint64_t base = (uint64_t)blockIdx.x * FIN_WAVES; base < n_units; base += (uint64_t)gridDim.x * FIN_WAVES) {
        uint32_t big = 0;
        if (base + wave < n_units) {
            const uint64_t u = base + wave;
            const uint32_t sidx = (uint32_t)(u / (uint64_t)a.n_ftiles);
            const int ftile = (int)(u - (uint64_t)sidx * (uint64_t)a.n_ftiles);
            const int j0 = ftile * ftile_size;
            const int nf = a.k - j0 < ftile_size ? a.k - j0 : ftile_size;
            const SplitRow sr = a.split_rows[sidx];
            if (sr.n_parts <= FIN_ALONE) {
                uint32_t v[FIN_FPL];
                merge_parts(a, a.partials + (size_t)sr.first_part * (size_t)a.k, 0u, 1u, sr.n_parts, j0, nf, lane, v);
#pragma unroll
                for (int i = 0; i < FIN_FPL; ++i)
                    if (lane + WAVE * i < nf) s_part[wave][lane + WAVE * i] = v[i];
                wave_sync_lds();
                wave_pack_store(a, s_part[wave], sr.row, j0, nf, ftile == a.n_ftiles - 1, lane);
                wave_sync_lds();
            } else {
                big = 1;
            }
        }
        if (lane == 0) s_big[wave] = big;
        __syncthreads();
        for (int w = 0; w < FIN_WAVES; ++w) {
            if (!s_big[w]) continue;                       // the same for every thread of the block
            const uint64_t u = base + w;
            const uint32_t sidx = (uint32_t)(u / (uint64_t)a.n_ftiles);
            const int ftile = (int)(u - (uint64_t)sidx * (uint64_t)a.n_ftiles);
            const int j0 = ftile * ftile_size;
            const int nf = a.k - j0 < ftile_size ? a.k - j0 : ftile_size;
            const SplitRow sr = a.split_rows[sidx];
            uint32_t v[FIN_FPL];
            merge_parts(a, a.partials + (size_t)sr.first_part * (size_t)a.k, (uint32_t)wave, (uint32_t)FIN_WAVES, sr.n_parts, j0, nf, lane, v);
#pragma unroll
            for (int i = 0; i < FIN_FPL; ++i)
                if (lane + WAVE * i < nf) s_part[wave][lane + WAVE * i] = v[i];
            __syncthreads();
            for (int j = threadIdx.x; j < nf; j += FIN_BLOCK) {
                uint32_t m = s_part[0][j];
#pragma unroll
                for (int x = 1; x < FIN_WAVES; ++x) m = s_part[x][j] < m ? s_part[x][j] : m;
                s_mins[j] = m;
            }
            __syncthreads();
            if (wave == 0) wave_pack_store(a, s_mins, sr.row, j0, nf, ftile == a.n_ftiles - 1, lane);
            __syncthreads();
        }
        __syncthreads();                                   // before s_big is written again
    }
}

// Copies the deferred status of a call to where the caller wants it (a caller that
// may not synchronise reads it later, from its own memory).
__global__ void mh_export_status_kernel(const WorkHeader* hdr, int32_t* status_out)
{
    const uint32_t st = hdr->status;
    *status_out = (st & 4u) ? MINHASH_ERR_WORKSPACE : st ? MINHASH_ERR_DATA : MINHASH_OK;
}

__global__ void mh_store_ok_kernel(int32_t* status_out) { *status_out = MINHASH_OK; }

// ------------------------------------------------------------------ host side
thread_local char g_hip_error[256] = "";

int hip_fail(hipError_t e, const char* what)
{
    snprintf(g_hip_error, sizeof(g_hip_error), "%s: %s", what, hipGetErrorString(e));
    return MINHASH_ERR_HIP;
}

bool is_multiply_shift(int32_t family) { return family == MINHASH_2U_MS32 || family == MINHASH_2U_MS32_HIGH; }

bool family_prime(int32_t family, uint64_t* p, int* deg)
{
    switch (family) {
    case MINHASH_2U_MS32:
    case MINHASH_2U_MS32_HIGH: *p = 1ull << 32; *deg = 2; return true;     // modulus 2^32, not a prime
    case MINHASH_2U_M31: *p = P31; *deg = 2; return true;
    case MINHASH_4U_M31: *p = P31; *deg = 4; return true;
    case MINHASH_2U_M61: *p = P61; *deg = 2; return true;
    case MINHASH_4U_M61: *p = P61; *deg = 4; return true;
    default: return false;
    }
}

int validate_shape(int64_t n_rows, int64_t nnz_ub, int32_t k, int32_t family)
{
    if (n_rows < 0 || n_rows >= (1ll << 31) || nnz_ub < 0) return MINHASH_ERR_ARG;
    if (family != MINHASH_PERM) {
        uint64_t p; int deg;
        if (!family_prime(family, &p, &deg)) return MINHASH_ERR_FAMILY;
    }
    if (k < 1 || k > MINHASH_MAX_K) return MINHASH_ERR_KB;
    return MINHASH_OK;
}

// Launch constants are kept per device (the library may be called with any device
// current): the number of compute units, and per kernel instantiation the number of
// blocks that are resident at once.  Slots are filled on first use; two threads that
// fill one at the same time write the same value.
constexpr int MAX_DEVICES = 64;

int current_device()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return 0;
    return dev;
}
int device_cus(int dev)
{
    static std::atomic<int> cache[MAX_DEVICES];
    int cus = cache[dev].load(std::memory_order_relaxed);
    if (cus > 0) return cus;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
    cache[dev].store(cus, std::memory_order_relaxed);
    return cus;
}

// persistent grid: as many blocks as are resident at once, no more
template <class K>
int resident_blocks(K kernel, int dev, int cus, std::atomic<int>* cache)
{
    int blocks = cache[dev].load(std::memory_order_relaxed);
    if (blocks > 0) return blocks;
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, BLOCK, 0) != hipSuccess || per_cu < 1) per_cu = 2;
    blocks = cus * per_cu;
    cache[dev].store(blocks, std::memory_order_relaxed);
    return blocks;
}

struct Launch {                        // where a call's kernels go
    int dev, cus;
    hipStream_t s;
};

template <class Pol, int NF, bool PACKED>
void launch_hash_form(const KArgs& a, const Launch& l)
{
    static std::atomic<int> cache[MAX_DEVICES];
    const int blocks = resident_blocks(mh_hash_kernel<Pol, NF, PACKED>, l.dev, l.cus, cache);
    hipLaunchKernelGGL((mh_hash_kernel<Pol, NF, PACKED>), dim3(blocks), dim3(BLOCK), 0, l.s, a);
}
template <class Pol, int NF>
void launch_hash_nf(const KArgs& a, const Launch& l)
{
    if (a.pk_words) launch_hash_form<Pol, NF, true>(a, l);       // rows given as tiles of differences
    else launch_hash_form<Pol, NF, false>(a, l);
}
// nf = functions per lane of this launch (see functions_per_lane); the hand-ordered
// policies exist for 5..8, the compiler-scheduled ones for 8 only
template <class Pol>
void launch_hash(const KArgs& a, int nf, const Launch& l)
{
    if constexpr (Pol::VARIABLE_NF) {
        switch (nf) {
        case 5: launch_hash_nf<Pol, 5>(a, l); return;
        case 6: launch_hash_nf<Pol, 6>(a, l); return;
        case 7: launch_hash_nf<Pol, 7>(a, l); return;
        default: break;
        }
    }
    launch_hash_nf<Pol, HASH_FPL>(a, l);
}
template <bool VEC4>
void launch_perm(const KArgs& a, const Launch& l)
{
    static std::atomic<int> cache[MAX_DEVICES];
    const int blocks = resident_blocks(mh_perm_kernel<VEC4>, l.dev, l.cus, cache);
    hipLaunchKernelGGL(mh_perm_kernel<VEC4>, dim3(blocks), dim3(BLOCK), 0, l.s, a);
}

// How many of its HASH_FPL function slots a lane uses.  A tile of functions spans
// 2^log2_fl lanes; with 8 functions per lane k = 300 would occupy 64 lanes x 8 = 512
// slots and k = 200 32 x 8 = 256, although 64 x 5 and 32 x 7 suffice.  For k up to
// one tile the pair (lanes, functions per lane) with the fewest slots is taken,
// functions per lane in 5..8 (fewer would only halve the lanes again).
void functions_per_lane(int k, bool variable, int* nf, int* log2_fl)
{
    *nf = HASH_FPL;
    int lanes_needed = ((k < HASH_FTILE ? k : HASH_FTILE) + HASH_FPL - 1) / HASH_FPL;
    int lg = 0;
    while ((1 << lg) < lanes_needed) ++lg;
    *log2_fl = lg;
    if (!variable || k > HASH_FTILE) return;
    int best = (1 << lg) * HASH_FPL;
    for (int f = HASH_FPL - 1; f >= 5; --f) {
        int need = (k + f - 1) / f, l = 0;
        while ((1 << l) < need) ++l;
        if ((1 << l) > WAVE) continue;
        if ((1 << l) * f < best) { best = (1 << l) * f; *nf = f; *log2_fl = l; }
    }
}

// What a call needs beyond its arguments, all of it worked out on the host without
// touching the GPU.
struct Plan {
    KArgs a;
    int nf;                            // functions per lane (hash families)
    int ftile_size;
    bool generic_mod, full4, guarded61, has_split;
};

// Everything that can be rejected without touching the GPU.  MINHASH_OK with
// *empty set means a successful no-op.
int check_arguments(const int64_t* row_ptr, int64_t n_rows, uint64_t D, int32_t k, int32_t b, int32_t family,
                    const void* params, int64_t perm_ld, const uint8_t* out, int64_t out_stride, uint32_t flags,
                    bool* empty)
{
    *empty = false;
    int rc = validate_shape(n_rows, 0, k, family);
    if (rc != MINHASH_OK) return rc;
    if (b < 1 || b > 32) return MINHASH_ERR_KB;
    if (D < 1 || D > (1ull << 32)) return MINHASH_ERR_D;
    if (is_multiply_shift(family)) {
        if ((D & (D - 1)) != 0) return MINHASH_ERR_D;                   // D = 2^s
        if (family == MINHASH_2U_MS32_HIGH && D < 2) return MINHASH_ERR_D;
        if (perm_ld != 0) return MINHASH_ERR_STRIDE;
    } else if (family != MINHASH_PERM) {
        uint64_t p; int deg;
        family_prime(family, &p, &deg);
        if (D >= p) return MINHASH_ERR_D;
        if (perm_ld != 0) return MINHASH_ERR_STRIDE;
    } else if (perm_ld < k) {
        return MINHASH_ERR_STRIDE;
    }
    const int64_t sig_bytes = ((int64_t)k * b + 7) / 8;
    if (out_stride < sig_bytes) return MINHASH_ERR_STRIDE;
    if (flags & ~(MINHASH_FLAG_VALIDATE | MINHASH_FLAG_GENERIC_MOD | MINHASH_FLAG_EXACT_FOLD)) return MINHASH_ERR_ARG;
    const bool generic_mod = (flags & MINHASH_FLAG_GENERIC_MOD) != 0;
    if (generic_mod && family != MINHASH_2U_M31 && family != MINHASH_4U_M31) return MINHASH_ERR_ARG;
    if ((flags & MINHASH_FLAG_EXACT_FOLD) && family != MINHASH_2U_M61 && family != MINHASH_4U_M31 &&
        family != MINHASH_2U_M31)
        return MINHASH_ERR_ARG;
    if (n_rows == 0) { *empty = true; return MINHASH_OK; }
    if (!row_ptr || !params || !out) return MINHASH_ERR_ARG;
    return MINHASH_OK;
}

// Fills the plan for a workspace at `ws` laid out for at most nnz_cap nonzeros.
int make_plan(Plan* plan, const int64_t* row_ptr, const uint32_t* col_idx, int64_t n_rows, uint64_t D, int32_t k, int32_t b,
              int32_t family, const void* params, int64_t perm_ld, uint8_t* out, int64_t out_stride, void* workspace,
              int64_t nnz_cap, uint32_t flags, uint64_t reserve_bytes = SMALL_BATCH_BYTES)
{
    const Layout L = make_layout(n_rows, nnz_cap, k, reserve_bytes);
    char* ws = static_cast<char*>(workspace);
    KArgs& a = plan->a;
    memset(&a, 0, sizeof(a));
    a.row_ptr = row_ptr; a.col_idx = col_idx; a.params = params; a.out = out;
    a.out_stride = out_stride; a.perm_ld = perm_ld;
    a.hdr = reinterpret_cast<WorkHeader*>(ws);
    a.items = reinterpret_cast<Item*>(ws + L.items_off);
    a.split_rows = reinterpret_cast<SplitRow*>(ws + L.split_rows_off);
    a.partials = reinterpret_cast<uint32_t*>(ws + L.partials_off);
    a.D = D; a.cap_long = L.cap_long; a.cap_short = L.cap_short; a.cap_split = L.cap_split; a.cap_parts = L.cap_parts;
    a.nnz_cap = (uint64_t)nnz_cap;
    a.min_chunk = chunk_floor(k);
    a.md = make_mod_d(D);
    if (is_multiply_shift(family)) {
        int sbits = 0;
        while ((1ull << sbits) < D) ++sbits;
        a.md.M = (uint32_t)(32 - sbits);                                // shift that keeps the s highest bits
    }
    a.n_rows = n_rows; a.k = k; a.b = b;
    a.sig_bytes = (int32_t)(((int64_t)k * b + 7) / 8);
    a.validate = (flags & MINHASH_FLAG_VALIDATE) ? 1u : 0u;
    a.prime = P31;
    a.target_items = 0;

    const bool pow2 = a.md.pow2 != 0;
    plan->generic_mod = (flags & MINHASH_FLAG_GENERIC_MOD) != 0;
    // 4U: two maxima of the folded value for every power-of-two D, unless the caller asks for the
    // form that yields the location evaluation by evaluation
    plan->full4 = pow2 && !(flags & MINHASH_FLAG_EXACT_FOLD);
    // 2U with p = 2^61-1: the guarded fast path needs a power-of-two D and t < 2^31
    plan->guarded61 = pow2 && D <= (1ull << 31) && !(flags & MINHASH_FLAG_EXACT_FOLD);
    plan->has_split = L.cap_split > 0;
    plan->nf = HASH_FPL;
    plan->ftile_size = PERM_FTILE;
    if (family != MINHASH_PERM) {
        // the kernels ordered by hand come with 5..8 functions per lane
        const bool hand4u61 = family == MINHASH_4U_M61 && ((pow2 && D <= (1ull << 31)) || a.md.M61q != 0);
        const bool hand2u61 = family == MINHASH_2U_M61 && (plan->guarded61 || a.md.M61q != 0);
        const bool variable = !plan->generic_mod && (family != MINHASH_4U_M61 || hand4u61) &&
                              (family != MINHASH_2U_M61 || hand2u61);
        int lg = 0;
        functions_per_lane(k, variable, &plan->nf, &lg);
        a.log2_fl = lg;
        plan->ftile_size = k > HASH_FTILE ? HASH_FTILE : (1 << lg) * plan->nf;
    } else {
        a.log2_fl = 6;
    }
    a.ftile_size = plan->ftile_size;
    a.n_ftiles = (k + plan->ftile_size - 1) / plan->ftile_size;
    a.lane_pack = family != MINHASH_PERM && plan->nf == HASH_FPL && (b == 8 || b == 16 || b == 32) && out_stride % 4 == 0 &&
                  reinterpret_cast<uintptr_t>(out) % 4 == 0;

    // tickets and unit numbers are 32 bits wide; tickets run past the last unit by one per resident wavefront
    if ((L.cap_long + L.cap_short) * (uint64_t)a.n_ftiles >= (1ull << 32) - (1ull << 24)) return MINHASH_ERR_ARG;
    return MINHASH_OK;
}

// Enqueues the kernels of a planned call.  Events of the profiled variant exist
// before the first launch, so that a failure to create them leaves nothing enqueued.
int enqueue(Plan& plan, int32_t family, uint64_t D, uint32_t flags, void* stream, float* kernel_ms, bool profiled,
            int32_t* status_out)
{
    KArgs& a = plan.a;
    Launch l;
    l.dev = current_device();
    l.cus = device_cus(l.dev);
    l.s = static_cast<hipStream_t>(stream);
    (void)hipGetLastError();           // an error left behind by an earlier, unrelated call is not this call's

    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (profiled) {
        hipError_t e = hipEventCreate(&e0);
        if (e != hipSuccess) return hip_fail(e, "hipEventCreate");
        e = hipEventCreate(&e1);
        if (e != hipSuccess) { (void)hipEventDestroy(e0); return hip_fail(e, "hipEventCreate"); }
    }
    a.target_items = (uint32_t)l.cus * 24u * 2u;   // two items per wavefront of a fully occupied launch
    const int bin_blocks = (int)((a.n_rows + BIN_BLOCK - 1) / BIN_BLOCK);
    if (bin_blocks > 1) hipLaunchKernelGGL(mh_reset_kernel, dim3(1), dim3(64), 0, l.s, a);   // one block of rows resets for itself
    hipLaunchKernelGGL(mh_bin_rows_kernel, dim3(bin_blocks), dim3(BIN_BLOCK), 0, l.s, a);

    hipError_t r0 = profiled ? hipEventRecord(e0, l.s) : hipSuccess;
    const bool pow2 = a.md.pow2 != 0;
    const int nf = plan.nf;
    switch (plan.generic_mod ? -family - 1 : family) {
    case -MINHASH_2U_M31 - 1: launch_hash<PolGenericMod<2>>(a, nf, l); break;
    case -MINHASH_4U_M31 - 1: launch_hash<PolGenericMod<4>>(a, nf, l); break;
    case MINHASH_2U_M31:
        // power-of-two D: one maximum of the doubled key for D <= 2^26, where a value asks for a second
        // look with probability (D / 2^31)^n, n the evaluations behind it; a signed and an unsigned
        // maximum of the key beyond, or when the caller asks for the form that needs no second look
        if (pow2 && D <= (1ull << FULL_KEY_MAX_LOG2_D) && !(flags & MINHASH_FLAG_EXACT_FOLD))
            launch_hash<Pol2U31<FORM_FULL>>(a, nf, l);
        else if (pow2) launch_hash<Pol2U31<FORM_FULL_TWO>>(a, nf, l);
        else if (frac_key_serves(D)) launch_hash<Pol2U31<FORM_FRAC_D>>(a, nf, l);
        else if (small_quotient_serves(D)) launch_hash<Pol2U31<FORM_BIG_D>>(a, nf, l);
        else launch_hash<Pol2U31<FORM_ANY_D>>(a, nf, l);
        break;
    case MINHASH_4U_M31:
        if (plan.full4) launch_hash<Pol4U31<true, true>>(a, nf, l);
        else if (pow2) launch_hash<Pol4U31<true, false>>(a, nf, l);
        else if (frac_key_serves(D)) launch_hash<Pol4U31<false, false, 1>>(a, nf, l);
        else if (small_quotient_serves(D)) launch_hash<Pol4U31<false, false, 2>>(a, nf, l);
        else launch_hash<Pol4U31<false>>(a, nf, l);
        break;
    case MINHASH_2U_M61:
        if (plan.guarded61) launch_hash<Pol2U61<true>>(a, nf, l);
        else if (a.md.M61q) launch_hash<Pol2U61<false, true>>(a, nf, l);     // other D of at most 2^32 / 3
        else launch_hash<Pol2U61<false>>(a, nf, l);
        break;
    case MINHASH_4U_M61:
        if (pow2 && D <= (1ull << 31)) launch_hash<Pol4U61Hand<true>>(a, nf, l);       // t < 2^31: the Horner steps ordered by hand
        else if (a.md.M61q) launch_hash<Pol4U61Hand<false>>(a, nf, l);                // (M61q is 0 for a power of two)
        else if (pow2) launch_hash<Pol4U61<true>>(a, nf, l);
        else launch_hash<Pol4U61<false>>(a, nf, l);
        break;
    case MINHASH_2U_MS32: launch_hash<Pol2UMS32<false>>(a, nf, l); break;
    case MINHASH_2U_MS32_HIGH: launch_hash<Pol2UMS32<true>>(a, nf, l); break;
    case MINHASH_PERM: {
        const bool vec4 = (a.perm_ld % 4 == 0) && (reinterpret_cast<uintptr_t>(a.params) % 16 == 0);
        if (vec4) launch_perm<true>(a, l); else launch_perm<false>(a, l);
        break;
    }
    default: break;                                // unreachable: the family was validated before planning
    }
    hipError_t r1 = profiled ? hipEventRecord(e1, l.s) : hipSuccess;
    if (plan.has_split)
        hipLaunchKernelGGL(mh_finalize_kernel, dim3(l.cus * 2), dim3(FIN_BLOCK), 0, l.s, a, plan.ftile_size);   // latency-bound: fill the chip
    if (status_out) hipLaunchKernelGGL(mh_export_status_kernel, dim3(1), dim3(1), 0, l.s, a.hdr, status_out);

    hipError_t le = hipGetLastError();
    if (profiled) {
        hipError_t se = hipStreamSynchronize(l.s);
        float ms = 0.0f;
        hipError_t te = hipSuccess;
        if (se == hipSuccess && le == hipSuccess && r0 == hipSuccess && r1 == hipSuccess) te = hipEventElapsedTime(&ms, e0, e1);
        (void)hipEventDestroy(e0);
        (void)hipEventDestroy(e1);
        if (le != hipSuccess) return hip_fail(le, "kernel launch");
        if (se != hipSuccess) return hip_fail(se, "hipStreamSynchronize");
        if (r0 != hipSuccess) return hip_fail(r0, "hipEventRecord");
        if (r1 != hipSuccess) return hip_fail(r1, "hipEventRecord");
        if (te != hipSuccess) return hip_fail(te, "hipEventElapsedTime");
        if (kernel_ms) *kernel_ms = ms;
    }
    if (le != hipSuccess) return hip_fail(le, "kernel launch");
    return MINHASH_OK;
}

// The device address of the built-in work space on the GPU that is current, looked
// up once per device.  `scratch` names the array for the compiler; on the host that
// name is a stand-in and not a device address, so host code only ever hands out the
// pointer found here.
int static_scratch(void** ptr)
{
    static std::mutex lock;
    static void* address[MAX_DEVICES];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= MAX_DEVICES) return MINHASH_ERR_ARG;
    std::lock_guard<std::mutex> hold(lock);
    if (!address[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress");
        if (!p || (reinterpret_cast<uintptr_t>(p) % MINHASH_WORKSPACE_ALIGN) != 0) return MINHASH_ERR_WORKSPACE;
        address[dev] = p;
    }
    *ptr = address[dev];
    return MINHASH_OK;
}

int run(const int64_t* row_ptr, const uint32_t* col_idx, int64_t n_rows, uint64_t D, int32_t k, int32_t b,
        int32_t family, const void* params, int64_t perm_ld, uint8_t* out, int64_t out_stride, void* workspace,
        size_t workspace_bytes, void* stream, uint32_t flags, float* kernel_ms, bool profiled)
{
    if (kernel_ms) *kernel_ms = 0.0f;
    bool empty = false;
    int rc = check_arguments(row_ptr, n_rows, D, k, b, family, params, perm_ld, out, out_stride, flags, &empty);
    if (rc != MINHASH_OK || empty) return rc;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % MINHASH_WORKSPACE_ALIGN) != 0) return MINHASH_ERR_WORKSPACE;
    // The nonzero bound the workspace was sized for is not passed in; recover the
    // largest bound this workspace can serve and let the device-side capacity
    // checks refuse anything beyond it.
    if (workspace_bytes < make_layout(n_rows, 0, k).total) return MINHASH_ERR_WORKSPACE;
    int64_t lo = 0, hi = (int64_t)1 << 46;
    while (lo < hi) {                              // largest nnz bound whose layout fits
        int64_t mid = lo + (hi - lo + 1) / 2;
        if (make_layout(n_rows, mid, k).total <= workspace_bytes) lo = mid; else hi = mid - 1;
    }
    Plan plan;
    rc = make_plan(&plan, row_ptr, col_idx, n_rows, D, k, b, family, params, perm_ld, out, out_stride, workspace, lo, flags);
    if (rc != MINHASH_OK) return rc;
    return enqueue(plan, family, D, flags, stream, kernel_ms, profiled, nullptr);
}

}  // namespace

namespace mh {
int report_hip_error(hipError_t e, const char* what) { return hip_fail(e, what); }
int launches_ok()
{
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? MINHASH_OK : hip_fail(e, "kernel launch");
}
}  // namespace mh

// ==================================================================== C ABI
extern "C" {

int minhash_signatures(const int64_t* row_ptr, const uint32_t* col_idx, int64_t n_rows, uint64_t D, int32_t k,
                       int32_t b, int32_t family, const void* params, int64_t perm_ld, uint8_t* out,
                       int64_t out_stride, void* workspace, size_t workspace_bytes, void* stream, uint32_t flags)
{
    return run(row_ptr, col_idx, n_rows, D, k, b, family, params, perm_ld, out, out_stride, workspace,
               workspace_bytes, stream, flags, nullptr, false);
}

int minhash_signatures_profiled(const int64_t* row_ptr, const uint32_t* col_idx, int64_t n_rows, uint64_t D,
                                int32_t k, int32_t b, int32_t family, const void* params, int64_t perm_ld,
                                uint8_t* out, int64_t out_stride, void* workspace, size_t workspace_bytes,
                                void* stream, uint32_t flags, float* kernel_ms)
{
    return run(row_ptr, col_idx, n_rows, D, k, b, family, params, perm_ld, out, out_stride, workspace,
               workspace_bytes, stream, flags, kernel_ms, true);
}

int minhash_signatures_static(const int64_t* row_ptr, const uint32_t* col_idx, int64_t n_rows, int64_t nnz_upper_bound,
                              uint64_t D, int32_t k, int32_t b, int32_t family, const void* params, int64_t perm_ld,
                              uint8_t* out, int64_t out_stride, int32_t* status, void* stream, uint32_t flags)
{
    bool empty = false;
    int rc = check_arguments(row_ptr, n_rows, D, k, b, family, params, perm_ld, out, out_stride, flags, &empty);
    if (rc != MINHASH_OK) return rc;
    if (nnz_upper_bound < 0) return MINHASH_ERR_ARG;
    if (nnz_upper_bound > ((int64_t)1 << 46)) return MINHASH_ERR_TOO_LARGE;
    // The reserve of partial vectors that lets small batches cut their long rows finely is
    // what a caller-sized workspace spends most of its bytes on; here it shrinks until the
    // layout fits the built-in buffer (the device picks the chunk size that the vectors allow).
    uint64_t reserve = SMALL_BATCH_BYTES;
    while (make_layout(n_rows, nnz_upper_bound, k, reserve).total > (size_t)MINHASH_STATIC_SCRATCH_BYTES) {
        if (reserve == 0) return MINHASH_ERR_TOO_LARGE;
        reserve = reserve > (1u << 20) ? reserve / 2 : 0;
    }
    void* ws = nullptr;
    rc = static_scratch(&ws);          // the device address of `scratch` on the current GPU, never its host-side name
    if (rc != MINHASH_OK) return rc;
    if (empty) {                       // nothing to hash; the caller's status word still gets its value
        if (status) {
            (void)hipGetLastError();
            hipLaunchKernelGGL(mh_store_ok_kernel, dim3(1), dim3(1), 0, static_cast<hipStream_t>(stream), status);
            hipError_t le = hipGetLastError();
            if (le != hipSuccess) return hip_fail(le, "kernel launch");
        }
        return MINHASH_OK;
    }
    Plan plan;
    rc = make_plan(&plan, row_ptr, col_idx, n_rows, D, k, b, family, params, perm_ld, out, out_stride, ws,
                   nnz_upper_bound, flags, reserve);
    if (rc != MINHASH_OK) return rc;
    return enqueue(plan, family, D, flags, stream, nullptr, false, status);
}

int minhash_signatures_packed(const int64_t* row_ptr, const uint32_t* width, const int64_t* word_ptr, const uint32_t* words,
                              int64_t words_len, int64_t n_rows, uint64_t D, int32_t k, int32_t b, int32_t family,
                              const void* params, uint8_t* out, int64_t out_stride, void* workspace, size_t workspace_bytes,
                              void* stream, uint32_t flags)
{
    if (family == MINHASH_PERM) return MINHASH_ERR_FAMILY;       // the table kernel takes col_idx: unpack first
    bool empty = false;
    int rc = check_arguments(row_ptr, n_rows, D, k, b, family, params, 0, out, out_stride, flags, &empty);
    if (rc != MINHASH_OK) return rc;
    if (words_len < 0) return MINHASH_ERR_ARG;
    if (empty) return MINHASH_OK;
    if (!width || !word_ptr || (!words && words_len > 0)) return MINHASH_ERR_ARG;
    if (!words) words = reinterpret_cast<const uint32_t*>(word_ptr);      // no words at all (every row empty): any address will do, none is read
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % MINHASH_WORKSPACE_ALIGN) != 0) return MINHASH_ERR_WORKSPACE;
    if (workspace_bytes < make_layout(n_rows, 0, k).total) return MINHASH_ERR_WORKSPACE;
    int64_t lo = 0, hi = (int64_t)1 << 46;
    while (lo < hi) {                              // largest nnz bound whose layout fits
        int64_t mid = lo + (hi - lo + 1) / 2;
        if (make_layout(n_rows, mid, k).total <= workspace_bytes) lo = mid; else hi = mid - 1;
    }
    Plan plan;
    rc = make_plan(&plan, row_ptr, nullptr, n_rows, D, k, b, family, params, 0, out, out_stride, workspace, lo, flags);
    if (rc != MINHASH_OK) return rc;
    plan.a.pk_width = width;
    plan.a.pk_word_ptr = word_ptr;
    plan.a.pk_words = words;
    plan.a.pk_words_len = words_len;
    if (plan.a.min_chunk < PACKED_TILE) plan.a.min_chunk = PACKED_TILE;       // a chunk starts at a tile
    return enqueue(plan, family, D, flags, stream, nullptr, false, nullptr);
}

size_t minhash_workspace_bytes(int64_t n_rows, int64_t nnz_upper_bound, int32_t k, int32_t family)
{
    if (validate_shape(n_rows, nnz_upper_bound, k, family) != MINHASH_OK) return 0;
    if (nnz_upper_bound > ((int64_t)1 << 46)) return 0;
    return make_layout(n_rows, nnz_upper_bound, k).total;
}

int minhash_check_coeffs(const uint64_t* host_coeffs, int32_t k, int32_t family)
{
    uint64_t p; int deg;
    if (!family_prime(family, &p, &deg)) return MINHASH_ERR_FAMILY;
    if (k < 1 || k > MINHASH_MAX_K) return MINHASH_ERR_KB;
    if (!host_coeffs) return MINHASH_ERR_ARG;
    for (int64_t i = 0; i < (int64_t)k * deg; ++i)
        if (host_coeffs[i] >= p) return MINHASH_ERR_COEFF;
    if (is_multiply_shift(family))
        for (int64_t j = 0; j < k; ++j)
            if ((host_coeffs[2 * j + 1] & 1u) == 0) return MINHASH_ERR_COEFF;   // the multiplier must be odd
    return MINHASH_OK;
}

int minhash_status(const void* workspace, void* stream)
{
    if (!workspace) return MINHASH_ERR_ARG;
    hipError_t e = hipStreamSynchronize(static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e, "hipStreamSynchronize");
    WorkHeader h;
    e = hipMemcpy(&h, workspace, sizeof(uint32_t) * 8, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_fail(e, "hipMemcpy");
    if (h.status & 4u) return MINHASH_ERR_WORKSPACE;
    return h.status ? MINHASH_ERR_DATA : MINHASH_OK;
}

int minhash_status_async(const void* workspace, int32_t* status_out, void* stream)
{
    if (!workspace || !status_out) return MINHASH_ERR_ARG;
    (void)hipGetLastError();
    hipLaunchKernelGGL(mh_export_status_kernel, dim3(1), dim3(1), 0, static_cast<hipStream_t>(stream),
                       static_cast<const WorkHeader*>(workspace), status_out);
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? MINHASH_OK : hip_fail(e, "mh_export_status_kernel");
}

const char* minhash_error_string(int code)
{
    switch (code) {
    case MINHASH_OK: return "ok";
    case MINHASH_ERR_ARG: return "invalid argument";
    case MINHASH_ERR_FAMILY: return "unknown hash family";
    case MINHASH_ERR_D: return "D out of range (need 1 <= D <= 2^32 and D < p for hash families)";
    case MINHASH_ERR_KB: return "k or b out of range";
    case MINHASH_ERR_STRIDE: return "out_stride or perm_ld too small";
    case MINHASH_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case MINHASH_ERR_HIP: return "HIP runtime error";
    case MINHASH_ERR_COEFF: return "hash coefficient not below the prime";
    case MINHASH_ERR_DATA: return "input data invalid (index >= D or decreasing row_ptr)";
    case MINHASH_ERR_TOO_LARGE: return "batch needs more work space than the built-in buffer of minhash_signatures_static holds";
    default: return "unknown error code";
    }
}

const char* minhash_last_hip_error(void) { return g_hip_error; }

int minhash_version(void) { return MINHASH_VERSION; }

}  // extern "C"
