// Roofline denominators measured on the device: what the integer ALUs and the
// memory system of this GPU deliver to loops of the shapes the signature kernels
// are made of.  Built into a library of its own (libminhash_probe.so); the
// signature library does not depend on it.  bench.py --probe runs everything
// and prints the table that the issue model of the hash kernels and the
// ceilings quoted for the permutation-table gather rest on.
//
//   mh_probe_issue        a loop of 8 independent instructions of one kind
//                         followed by n x 8 independent simple adds, with or
//                         without the wave priorities the hash kernels use:
//                         how many issue slots one group costs
//   mh_probe_stream_read  a plain coalesced read of a buffer (16 bytes per lane
//                         and load, several loads in flight): streaming GB/s
//   mh_probe_copy         reads and writes a known number of bytes: the kernel
//                         FETCH_SIZE / WRITE_SIZE counters are scaled by
//   mh_probe_gather_rows  reads whole rows of a table at random row numbers,
//                         one row per wavefront and load (the access pattern of
//                         the permutation-table kernel without any of its other
//                         work): gather GB/s for that row size
//
// All pointers are device pointers owned by the caller; every function
// synchronises the stream and returns 0 or a negative number (-1 bad argument,
// -7 HIP error).  Durations are averages over `reps` launches, measured with HIP
// events on the given stream.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int BLOCK = 256;
constexpr int ISSUE_ITERS = 1000;      // iterations of the probe loop
constexpr int ISSUE_UNROLL = 4;        // groups per iteration

// One group = 8 instructions of the probed kind (text FASM(SD), operating on a 32-bit
// register v[i] and a 64-bit pair q[i], reading b and c; SD is the scalar pair a
// widening multiply-add names for its unused carry-out, a different one for each of the
// eight so that the compiler puts no wait states between them) + NS x 8 simple adds.
// Results feed a store that never happens, so nothing is optimised away.
#define MH_PROBE_ONE(FASM, I, SD, S0, S1) \
    asm volatile(FASM(SD) : "+v"(v[I]), "+v"(q[I]) : "v"(b), "v"(c) : S0, S1)
#define MH_PROBE_KERNEL(NAME, FASM, NS, PRIO)                                                             \
    __global__ __launch_bounds__(BLOCK) void NAME(uint32_t* out, uint32_t s1, uint32_t s2)                \
    {                                                                                                     \
        uint32_t v[8], w[8];                                                                              \
        uint64_t q[8];                                                                                    \
        for (int i = 0; i < 8; ++i) {                                                                     \
            v[i] = threadIdx.x * 7 + i + s1;                                                              \
            w[i] = v[i] ^ s2;                                                                             \
            q[i] = v[i] * 3ull;                                                                           \
        }                                                                                                 \
        uint32_t b = s2 | 1, c = s1 + 3;                                                                  \
        asm volatile("" : "+v"(b), "+v"(c));                                                              \
        for (int it = 0; it < ISSUE_ITERS; ++it) {                                                        \
            _Pragma("unroll") for (int u = 0; u < ISSUE_UNROLL; ++u)                                      \
            {                                                                                             \
                if (PRIO) asm volatile("s_setprio 1");                                                    \
                MH_PROBE_ONE(FASM, 0, "s[40:41]", "s40", "s41");                                          \
                MH_PROBE_ONE(FASM, 1, "s[42:43]", "s42", "s43");                                          \
                MH_PROBE_ONE(FASM, 2, "s[44:45]", "s44", "s45");                                          \
                MH_PROBE_ONE(FASM, 3, "s[46:47]", "s46", "s47");                                          \
                MH_PROBE_ONE(FASM, 4, "s[48:49]", "s48", "s49");                                          \
                MH_PROBE_ONE(FASM, 5, "s[50:51]", "s50", "s51");                                          \
                MH_PROBE_ONE(FASM, 6, "s[52:53]", "s52", "s53");                                          \
                MH_PROBE_ONE(FASM, 7, "s[54:55]", "s54", "s55");                                          \
                if (PRIO) asm volatile("s_setprio 0");                                                    \
                _Pragma("unroll") for (int f = 0; f < NS; ++f)                                            \
                    _Pragma("unroll") for (int i = 0; i < 8; ++i)                                         \
                        asm volatile("v_add_u32 %0, %0, %1" : "+v"(w[i]) : "v"(b));                       \
            }                                                                                             \
        }                                                                                                 \
        uint32_t s = 0;                                                                                   \
        for (int i = 0; i < 8; ++i) s ^= v[i] ^ w[i] ^ (uint32_t)q[i] ^ (uint32_t)(q[i] >> 32);           \
        if (s == 0x12345678u && s1 == 0xFFFFFFFFu) out[threadIdx.x] = s;                                  \
    }

#define MH_PROBE_KIND(TAG, FASM)                                                                           \
    MH_PROBE_KERNEL(probe_##TAG##_0, FASM, 0, 0)                                                           \
    MH_PROBE_KERNEL(probe_##TAG##_1, FASM, 1, 0)                                                           \
    MH_PROBE_KERNEL(probe_##TAG##_2, FASM, 2, 0)                                                           \
    MH_PROBE_KERNEL(probe_##TAG##_3, FASM, 3, 0)                                                           \
    MH_PROBE_KERNEL(probe_##TAG##_5, FASM, 5, 0)                                                           \
    MH_PROBE_KERNEL(probe_##TAG##_1p, FASM, 1, 1)                                                          \
    MH_PROBE_KERNEL(probe_##TAG##_2p, FASM, 2, 1)                                                          \
    MH_PROBE_KERNEL(probe_##TAG##_3p, FASM, 3, 1)                                                          \
    MH_PROBE_KERNEL(probe_##TAG##_5p, FASM, 5, 1)

// the instruction kinds of the hash kernels' inner steps
#define F_MAD64(SD) "v_mad_u64_u32 %1, " SD ", %2, %3, %1"           // widening multiply-add (the evaluation itself)
#define F_MULHI(SD) "v_mul_hi_u32 %0, %0, %2"                        // quotient by an invariant divisor
#define F_MIN3(SD) "v_min3_u32 %0, %0, %2, %3"                       // three-operand extremum (running minimum of two values)
#define F_ADD3(SD) "v_add3_u32 %0, %0, %2, %3"                       // three-operand add (fold of the cubic)
#define F_LSHLADD(SD) "v_lshl_add_u32 %0, %0, 1, %2"                 // shift-then-add (doubled key)
#define F_ALIGNBIT(SD) "v_alignbit_b32 %0, %0, %2, 29"               // funnel shift (fold modulo 2^61-1, fractional key)
#define F_MIN2(SD) "v_min_u32 %0, %0, %2"                            // two-operand minimum (canonical residue)
#define F_ADD(SD) "v_add_u32 %0, %0, %2"                             // a simple instruction in the probed slot: all-simple loops
#define F_LSHR(SD) "v_lshrrev_b32 %0, 1, %0"                         // shift right (simple)
MH_PROBE_KIND(mad64, F_MAD64)
MH_PROBE_KIND(mulhi, F_MULHI)
MH_PROBE_KIND(min3, F_MIN3)
MH_PROBE_KIND(add3, F_ADD3)
MH_PROBE_KIND(lshladd, F_LSHLADD)
MH_PROBE_KIND(alignbit, F_ALIGNBIT)
MH_PROBE_KIND(min2, F_MIN2)
MH_PROBE_KIND(add, F_ADD)
MH_PROBE_KIND(lshr, F_LSHR)

typedef void (*probe_fn)(uint32_t*, uint32_t, uint32_t);
#define MH_PROBE_ROW(TAG)                                                                                  \
    { probe_##TAG##_0, probe_##TAG##_1, probe_##TAG##_2, probe_##TAG##_3, probe_##TAG##_5,                 \
      nullptr, probe_##TAG##_1p, probe_##TAG##_2p, probe_##TAG##_3p, probe_##TAG##_5p }
const probe_fn PROBES[][10] = {MH_PROBE_ROW(mad64), MH_PROBE_ROW(mulhi), MH_PROBE_ROW(min3), MH_PROBE_ROW(add3),
                               MH_PROBE_ROW(lshladd), MH_PROBE_ROW(alignbit), MH_PROBE_ROW(min2), MH_PROBE_ROW(add),
                               MH_PROBE_ROW(lshr)};
constexpr int N_KINDS = sizeof(PROBES) / sizeof(PROBES[0]);
const char* const KIND_NAMES[N_KINDS] = {"v_mad_u64_u32", "v_mul_hi_u32", "v_min3_u32", "v_add3_u32", "v_lshl_add_u32",
                                         "v_alignbit_b32", "v_min_u32", "v_add_u32", "v_lshrrev_b32"};

// ------------------------------------------------------------------ memory probes
// Every lane reads 16 bytes per load, U loads in flight, blocks stride over the
// buffer; the loaded words are folded into a value that is stored only if it
// has an impossible value (the compiler cannot drop the loads).
template <int U>
__global__ __launch_bounds__(BLOCK) void probe_stream_read_kernel(const u32x4* src, size_t n_vec, uint32_t* sink)
{
    const size_t stride = (size_t)gridDim.x * BLOCK;
    size_t i = (size_t)blockIdx.x * BLOCK + threadIdx.x;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (; i + (U - 1) * stride < n_vec; i += U * stride) {
        u32x4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= v[u];
    }
    for (; i < n_vec; i += stride) acc ^= __builtin_nontemporal_load(src + i);
    const uint32_t f = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (f == 0x9E3779B9u && n_vec == 1) sink[threadIdx.x] = f;
}

__global__ __launch_bounds__(BLOCK) void probe_copy_kernel(const u32x4* src, u32x4* dst, size_t n_vec)
{
    const size_t stride = (size_t)gridDim.x * BLOCK;
    for (size_t i = (size_t)blockIdx.x * BLOCK + threadIdx.x; i < n_vec; i += stride) {
        u32x4 v = __builtin_nontemporal_load(src + i);
        v.x += 1u;
        __builtin_nontemporal_store(v, dst + i);
    }
}

// One wavefront per row and load: lane l reads bytes [16 l, 16 l + 16) of row
// rows[j] when they exist (row_bytes / 16 lanes are active), U rows in flight.
// Persistent wavefronts stride over the list of row numbers.
template <int U>
__global__ __launch_bounds__(BLOCK) void probe_gather_rows_kernel(const uint32_t* table, size_t pitch_words, int row_vecs,
                                                                  const uint32_t* rows, size_t n_idx, uint32_t* sink)
{
    const int lane = threadIdx.x & 63;
    const size_t wave = ((size_t)blockIdx.x * BLOCK + threadIdx.x) >> 6;
    const size_t n_waves = ((size_t)gridDim.x * BLOCK) >> 6;
    const bool lane_ok = lane < row_vecs;
    u32x4 acc = {0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu};
    for (size_t j = wave * U; j + U <= n_idx; j += n_waves * U) {
        u32x4 g[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t r = __builtin_amdgcn_readfirstlane(rows[j + u]);
            const u32x4* p = reinterpret_cast<const u32x4*>(table + (size_t)r * pitch_words);
            g[u] = lane_ok ? __builtin_nontemporal_load(p + lane) : acc;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            acc.x = g[u].x < acc.x ? g[u].x : acc.x;
            acc.y = g[u].y < acc.y ? g[u].y : acc.y;
            acc.z = g[u].z < acc.z ? g[u].z : acc.z;
            acc.w = g[u].w < acc.w ? g[u].w : acc.w;
        }
    }
    const uint32_t f = acc.x & acc.y & acc.z & acc.w;
    if (f == 0x9E3779B9u && n_idx == 1) sink[threadIdx.x] = f;
}

int device_cus()
{
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return 256;
    return cus;
}

// Runs `launch` once untimed and `reps` times between two events; average ms.
template <class F>
int timed(F launch, int reps, hipStream_t s, float* ms_avg)
{
    if (reps < 1) return -1;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess) return -7;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return -7; }
    launch();
    hipError_t e = hipStreamSynchronize(s);
    if (e == hipSuccess) e = hipEventRecord(e0, s);
    if (e == hipSuccess) {
        for (int r = 0; r < reps; ++r) launch();
        e = hipEventRecord(e1, s);
    }
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e == hipSuccess) e = hipGetLastError();
    float ms = 0.0f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess) return -7;
    if (ms_avg) *ms_avg = ms / (float)reps;
    return 0;
}

}  // namespace

extern "C" {

int mh_probe_n_kinds(void) { return N_KINDS; }
const char* mh_probe_kind_name(int kind) { return kind >= 0 && kind < N_KINDS ? KIND_NAMES[kind] : ""; }

// kind: index below mh_probe_n_kinds(); n_simple in {0, 1, 2, 3, 5}; prio: 1 raises the
// wave priority for the run of probed instructions and lowers it for the simple ones;
// waves_per_simd in 1..8 (blocks of 4 wavefronts, one per SIMD).  scratch: device, at
// least 1 KiB (never written).  *ms: average duration; *slots: issue slots per
// (1 probed + n_simple simple) instructions per SIMD at `clock_ghz`, one slot = one
// 64-lane instruction at 16 lanes per clock.
int mh_probe_issue(int kind, int n_simple, int prio, int waves_per_simd, double clock_ghz, void* scratch, void* stream,
                   int reps, float* ms, double* slots)
{
    if (kind < 0 || kind >= N_KINDS || waves_per_simd < 1 || waves_per_simd > 8 || !scratch || clock_ghz <= 0.0) return -1;
    int col;
    switch (n_simple) {
    case 0: col = 0; break;
    case 1: col = 1; break;
    case 2: col = 2; break;
    case 3: col = 3; break;
    case 5: col = 4; break;
    default: return -1;
    }
    if (prio && n_simple == 0) prio = 0;                 // nothing to prioritise against
    const probe_fn fn = PROBES[kind][col + (prio ? 5 : 0)];
    if (!fn) return -1;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int blocks = device_cus() * waves_per_simd;
    float t = 0.0f;
    int rc = timed([&] { hipLaunchKernelGGL(fn, dim3(blocks), dim3(BLOCK), 0, s, static_cast<uint32_t*>(scratch), 1u, 2u); },
                   reps, s, &t);
    if (rc != 0) return rc;
    if (ms) *ms = t;
    // per SIMD: waves_per_simd wavefronts, ISSUE_ITERS * ISSUE_UNROLL groups each; a slot is 4 clocks
    if (slots)
        *slots = (double)t * 1e-3 * clock_ghz * 1e9 / 4.0 / ((double)ISSUE_ITERS * ISSUE_UNROLL * 8.0 * waves_per_simd);
    return 0;
}

int mh_probe_stream_read(const void* buf, size_t bytes, int blocks_per_cu, void* stream, int reps, float* ms)
{
    if (!buf || bytes < 4096 || (reinterpret_cast<uintptr_t>(buf) & 15u) || blocks_per_cu < 1 || blocks_per_cu > 32) return -1;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int blocks = device_cus() * blocks_per_cu;
    const u32x4* src = static_cast<const u32x4*>(buf);
    uint32_t* sink = const_cast<uint32_t*>(static_cast<const uint32_t*>(buf));     // never written: the guard cannot hold
    return timed([&] { hipLaunchKernelGGL(probe_stream_read_kernel<8>, dim3(blocks), dim3(BLOCK), 0, s, src, bytes / 16, sink); },
                 reps, s, ms);
}

int mh_probe_copy(const void* src, void* dst, size_t bytes, void* stream, int reps, float* ms)
{
    if (!src || !dst || bytes < 16 || ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15u)) return -1;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int blocks = device_cus() * 8;
    return timed([&] {
        hipLaunchKernelGGL(probe_copy_kernel, dim3(blocks), dim3(BLOCK), 0, s, static_cast<const u32x4*>(src),
                           static_cast<u32x4*>(dst), bytes / 16);
    }, reps, s, ms);
}

// table: n_table_rows rows, pitch_bytes apart (a multiple of 16, table 16-byte aligned), of which
// the first row_bytes (a multiple of 16, at most 1024) are read; rows: n_idx row numbers, each
// below n_table_rows (checked by the caller; the kernel trusts them); in_flight: 8 or 16.
int mh_probe_gather_rows(const void* table, size_t n_table_rows, size_t pitch_bytes, int row_bytes, const uint32_t* rows,
                         size_t n_idx, int in_flight, int blocks_per_cu, void* stream, int reps, float* ms)
{
    if (!table || !rows || n_table_rows < 1 || (reinterpret_cast<uintptr_t>(table) & 15u) || (pitch_bytes & 15u) ||
        row_bytes < 16 || row_bytes > 1024 || (row_bytes & 15) || (size_t)row_bytes > pitch_bytes ||
        (in_flight != 8 && in_flight != 16) || n_idx < (size_t)in_flight || blocks_per_cu < 1 || blocks_per_cu > 32)
        return -1;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int blocks = device_cus() * blocks_per_cu;
    const uint32_t* t = static_cast<const uint32_t*>(table);
    uint32_t* sink = const_cast<uint32_t*>(rows);                                  // never written
    if (in_flight == 8)
        return timed([&] {
            hipLaunchKernelGGL(probe_gather_rows_kernel<8>, dim3(blocks), dim3(BLOCK), 0, s, t, pitch_bytes / 4, row_bytes / 16,
                               rows, n_idx, sink);
        }, reps, s, ms);
    return timed([&] {
        hipLaunchKernelGGL(probe_gather_rows_kernel<16>, dim3(blocks), dim3(BLOCK), 0, s, t, pitch_bytes / 4, row_bytes / 16,
                           rows, n_idx, sink);
    }, reps, s, ms);
}

}  // extern "C"
