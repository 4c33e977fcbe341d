// Consumers of packed b-bit signatures on MI355X: the 2^b x k expansion, the
// number of equal b-bit values of two rows, and the resemblance estimator
// (Section 1.1: Theorem 1, eq. eqn_R_b and the paragraph after it).
//
// All three are memory-bound: a signature row is read once per use, with
// coalesced dword loads when rows are 4-byte aligned.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "minhash.h"
#include "mh_host.h"

namespace {

constexpr int WAVE = 64;
constexpr int BLOCK = 256;

struct SigView {
    const uint8_t* base;
    int64_t stride;
    int32_t k, b;
    int32_t sig_bytes;
    int32_t aligned;      // base and stride are multiples of 4
};

// value j of a row: bits [j b, (j+1) b) of its little-endian bit string
__device__ __forceinline__ uint32_t load_field(const SigView& s, const uint8_t* row, int j)
{
    const int64_t bit = (int64_t)j * s.b;
    const uint32_t mask = s.b >= 32 ? 0xFFFFFFFFu : ((1u << s.b) - 1u);
    if (s.aligned) {
        const uint32_t* r32 = reinterpret_cast<const uint32_t*>(row);
        const int w = (int)(bit >> 5), sh = (int)(bit & 31);
        const int ndw = (s.sig_bytes + 3) >> 2;          // a 4-aligned pitch covers the rounded-up dwords
        uint32_t lo = r32[w];
        uint32_t v = lo >> sh;
        if (sh + s.b > 32 && w + 1 < ndw) v |= r32[w + 1] << (32 - sh);
        return v & mask;
    }
    const int byte = (int)(bit >> 3), sh = (int)(bit & 7);
    uint64_t acc = 0;
    const int need = (sh + s.b + 7) >> 3;                // 1..5 bytes
    for (int i = 0; i < need; ++i) acc |= (uint64_t)row[byte + i] << (8 * i);
    return (uint32_t)(acc >> sh) & mask;
}

__global__ __launch_bounds__(BLOCK) void mh_expand_kernel(SigView s, int64_t n_rows, uint32_t* out)
{
    const int lane = threadIdx.x & (WAVE - 1);
    const int64_t wave = ((int64_t)blockIdx.x * BLOCK + threadIdx.x) >> 6;
    const int64_t n_waves = ((int64_t)gridDim.x * BLOCK) >> 6;
    for (int64_t i = wave; i < n_rows; i += n_waves) {
        const uint8_t* row = s.base + i * s.stride;
        uint32_t* dst = out + i * (int64_t)s.k;
        for (int j = lane; j < s.k; j += WAVE)
            dst[j] = (uint32_t)(((uint64_t)j << s.b) + load_field(s, row, j));
    }
}

// number of all-zero b-bit fields of x for b dividing 32 (x = XOR of two packed dwords)
__device__ __forceinline__ uint32_t zero_fields(uint32_t x, int b)
{
    switch (b) {
    case 1: return __popc(~x);
    case 2: x |= x >> 1; return __popc(~x & 0x55555555u);
    case 4: x |= x >> 1; x |= x >> 2; return __popc(~x & 0x11111111u);
    case 8: x |= x >> 1; x |= x >> 2; x |= x >> 4; return __popc(~x & 0x01010101u);
    case 16: return ((x & 0xFFFFu) == 0) + ((x >> 16) == 0);
    default: return x == 0;
    }
}

__global__ __launch_bounds__(BLOCK) void mh_match_kernel(SigView s, int64_t n_rows, const int64_t* pairs, int64_t n_pairs,
                                                         uint32_t* counts)
{
    const int lane = threadIdx.x & (WAVE - 1);
    const int64_t wave = ((int64_t)blockIdx.x * BLOCK + threadIdx.x) >> 6;
    const int64_t n_waves = ((int64_t)gridDim.x * BLOCK) >> 6;
    const bool dword_path = s.aligned && (32 % s.b == 0);
    const int per_dw = dword_path ? 32 / s.b : 1;
    for (int64_t q = wave; q < n_pairs; q += n_waves) {
        const int64_t r1 = pairs[2 * q], r2 = pairs[2 * q + 1];
        if (r1 < 0 || r1 >= n_rows || r2 < 0 || r2 >= n_rows) {      // no access outside the signatures
            if (lane == 0) counts[q] = 0xFFFFFFFFu;
            continue;
        }
        const uint8_t* a = s.base + r1 * s.stride;
        const uint8_t* c = s.base + r2 * s.stride;
        uint32_t n = 0;
        if (dword_path) {
            const uint32_t* a32 = reinterpret_cast<const uint32_t*>(a);
            const uint32_t* c32 = reinterpret_cast<const uint32_t*>(c);
            const int full = s.k / per_dw;                            // dwords made of whole fields of real values
            for (int w = lane; w < full; w += WAVE) n += zero_fields(a32[w] ^ c32[w], s.b);
            for (int j = full * per_dw + lane; j < s.k; j += WAVE) n += load_field(s, a, j) == load_field(s, c, j);
        } else {
            for (int j = lane; j < s.k; j += WAVE) n += load_field(s, a, j) == load_field(s, c, j);
        }
        for (int d = WAVE / 2; d > 0; d >>= 1) n += (uint32_t)__shfl_xor((int)n, d, WAVE);
        if (lane == 0) counts[q] = n;
    }
}

// A of Theorem 1: r (1-r)^(2^b - 1) / (1 - (1-r)^(2^b))
__device__ __forceinline__ double theorem1_A(double r, int b)
{
    const double n = ldexp(1.0, b);
    return r * pow(1.0 - r, n - 1.0) / (1.0 - pow(1.0 - r, n));
}

__global__ __launch_bounds__(BLOCK) void mh_estimate_kernel(const uint32_t* counts, const int64_t* f1, const int64_t* f2,
                                                            int64_t n_pairs, double D, int k, int b, double* r_hat)
{
    const int64_t q = (int64_t)blockIdx.x * BLOCK + threadIdx.x;
    if (q >= n_pairs) return;
    const double r1 = (double)f1[q] / D, r2 = (double)f2[q] / D;
    const double A1 = theorem1_A(r1, b), A2 = theorem1_A(r2, b);
    const double C1 = A1 * r2 / (r1 + r2) + A2 * r1 / (r1 + r2);
    const double C2 = A1 * r1 / (r1 + r2) + A2 * r2 / (r1 + r2);
    const double P = (double)counts[q] / (double)k;
    r_hat[q] = (P - C1) / (1.0 - C2);
}

int check_sig(const uint8_t* sig, int64_t n_rows, int64_t sig_stride, int32_t k, int32_t b, SigView* v)
{
    if (n_rows < 0) return MINHASH_ERR_ARG;
    if (k < 1 || k > MINHASH_MAX_K || b < 1 || b > 32) return MINHASH_ERR_KB;
    const int64_t sig_bytes = ((int64_t)k * b + 7) / 8;
    if (sig_stride < sig_bytes) return MINHASH_ERR_STRIDE;
    v->base = sig; v->stride = sig_stride; v->k = k; v->b = b; v->sig_bytes = (int32_t)sig_bytes;
    v->aligned = (reinterpret_cast<uintptr_t>(sig) % 4 == 0 && sig_stride % 4 == 0) ? 1 : 0;
    return MINHASH_OK;
}

int grid_for(int64_t waves_wanted)
{
    int64_t blocks = (waves_wanted + 3) / 4;
    const int64_t cap = 256 * 32;
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    return (int)blocks;
}

}  // namespace

extern "C" {

int minhash_expand_indices(const uint8_t* sig, int64_t n_rows, int64_t sig_stride, int32_t k, int32_t b,
                           uint32_t* out_idx, void* stream)
{
    SigView v;
    int rc = check_sig(sig, n_rows, sig_stride, k, b, &v);
    if (rc != MINHASH_OK) return rc;
    if (((unsigned __int128)k << b) > ((unsigned __int128)1 << 32)) return MINHASH_ERR_KB;
    if (n_rows == 0) return MINHASH_OK;
    if (!sig || !out_idx) return MINHASH_ERR_ARG;
    (void)hipGetLastError();           // an error left by an earlier, unrelated call is not this call's
    hipLaunchKernelGGL(mh_expand_kernel, dim3(grid_for(n_rows)), dim3(BLOCK), 0, static_cast<hipStream_t>(stream), v,
                       n_rows, out_idx);
    return mh::launches_ok();
}

int minhash_match_counts(const uint8_t* sig, int64_t n_rows, int64_t sig_stride, int32_t k, int32_t b,
                         const int64_t* pairs, int64_t n_pairs, uint32_t* counts, void* stream)
{
    SigView v;
    int rc = check_sig(sig, n_rows, sig_stride, k, b, &v);
    if (rc != MINHASH_OK) return rc;
    if (n_pairs < 0) return MINHASH_ERR_ARG;
    if (n_pairs == 0) return MINHASH_OK;
    if (!sig || !pairs || !counts) return MINHASH_ERR_ARG;
    (void)hipGetLastError();           // an error left by an earlier, unrelated call is not this call's
    hipLaunchKernelGGL(mh_match_kernel, dim3(grid_for(n_pairs)), dim3(BLOCK), 0, static_cast<hipStream_t>(stream), v,
                       n_rows, pairs, n_pairs, counts);
    return mh::launches_ok();
}

int minhash_resemblance_estimates(const uint32_t* counts, const int64_t* f1, const int64_t* f2, int64_t n_pairs,
                                  uint64_t D, int32_t k, int32_t b, double* r_hat, void* stream)
{
    if (n_pairs < 0) return MINHASH_ERR_ARG;
    if (k < 1 || k > MINHASH_MAX_K || b < 1 || b > 32) return MINHASH_ERR_KB;
    if (D < 1 || D > (1ull << 32)) return MINHASH_ERR_D;
    if (n_pairs == 0) return MINHASH_OK;
    if (!counts || !f1 || !f2 || !r_hat) return MINHASH_ERR_ARG;
    const int blocks = (int)((n_pairs + BLOCK - 1) / BLOCK);
    (void)hipGetLastError();           // an error left by an earlier, unrelated call is not this call's
    hipLaunchKernelGGL(mh_estimate_kernel, dim3(blocks), dim3(BLOCK), 0, static_cast<hipStream_t>(stream), counts, f1,
                       f2, n_pairs, (double)D, k, b, r_hat);
    return mh::launches_ok();
}

}  // extern "C"
