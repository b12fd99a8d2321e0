// Device-side seeded partition of a buffer into mini-batches.
//
// Algorithm 1 draws a fresh random partition of the buffer at the start of every pass; Section 2.2
// asks for disjoint parts that cover the buffer.  The generator is a keyed 8-round balanced Feistel
// network on 2h bits (2^(2h) < 4 * rows) restricted to [0, rows) by cycle walking, in uint32 arithmetic
// only, so that the index arrays are reproducible bit for bit.  Mini-batch m is
// perm[(m-1) n : min(m n, rows)).
#include "bmgd_internal.h"

#include <algorithm>

namespace bmgd {

namespace {

__host__ __device__ inline uint32_t mix32(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x7FEB352Du;
    x ^= x >> 15;
    x *= 0x846CA68Bu;
    x ^= x >> 16;
    return x;
}

struct KeyRow {
    uint32_t k[kPermRounds];
};

__device__ inline uint32_t feistel(uint32_t x, const KeyRow& key, uint32_t h, uint32_t mask)
{
    uint32_t left = x >> h, right = x & mask;
#pragma unroll
    for (int i = 0; i < kPermRounds; ++i) {
        const uint32_t f = mix32(right ^ key.k[i]) & mask;
        const uint32_t t = left ^ f;
        left = right;
        right = t;
    }
    return (left << h) | right;
}

// With `subset` the partition is one of the rows subset[0 .. rows) of a larger buffer: out holds subset[PERM[j]].
// An entry outside [0, limit) is replaced by row 0 and reported through *bad (the host turns that into an error).
__global__ void __launch_bounds__(256) perm_kernel(int32_t* __restrict__ out, uint32_t rows, uint32_t h,
                                                   PermKeys keys, const int32_t* __restrict__ subset, uint32_t limit,
                                                   unsigned* bad)
{
    const uint32_t pass = blockIdx.y;
    const uint32_t j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= rows) return;
    KeyRow key;
#pragma unroll
    for (int i = 0; i < kPermRounds; ++i) key.k[i] = keys.key[pass][i];
    const uint32_t mask = (1u << h) - 1u;
    // j < rows lies on a cycle of the bijection that returns to j, so the walk always re-enters [0, rows).
    uint32_t x = feistel(j, key, h, mask);
    while (x >= rows) x = feistel(x, key, h, mask);
    if (subset) {
        const uint32_t v = (uint32_t)subset[x];
        if (v >= limit) __hip_atomic_store(bad, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        x = v < limit ? v : 0u;
    }
    out[(size_t)pass * rows + j] = (int32_t)x;
}

__global__ void __launch_bounds__(256) fill_zero_kernel(uint4* __restrict__ dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = make_uint4(0, 0, 0, 0);
}

// avg <- theta for the first snapshot, else avg + (theta - avg) * inv with inv = 1 / (snapshots so far + 1)
__global__ void __launch_bounds__(256) running_mean_kernel(float* __restrict__ avg, const float* __restrict__ theta, size_t n,
                                                           float inv, int first)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const float t = theta[i];
        avg[i] = first ? t : avg[i] + (t - avg[i]) * inv;
    }
}

}  // namespace

hipError_t launch_running_mean(float* avg, const float* theta, size_t n, float inv, bool first, hipStream_t stream)
{
    if (n == 0) return hipSuccess;
    const unsigned blocks = (unsigned)std::min<size_t>((n + 255) / 256, 2048);
    hipLaunchKernelGGL(running_mean_kernel, dim3(blocks), dim3(256), 0, stream, avg, theta, n, inv, first ? 1 : 0);
    return hipGetLastError();
}

hipError_t launch_fill_zero(void* dst, size_t bytes, hipStream_t stream)
{
    if (bytes == 0) return hipSuccess;
    if ((reinterpret_cast<uintptr_t>(dst) % 16) != 0 || bytes % 16 != 0) return hipErrorInvalidValue;
    const size_t n16 = bytes / 16;
    const unsigned blocks = (unsigned)std::min<size_t>((n16 + 255) / 256, 2048);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, stream, static_cast<uint4*>(dst), n16);
    return hipGetLastError();
}

void perm_round_keys(uint64_t seed, uint32_t b, uint32_t t, uint32_t out[kPermRounds])
{
    uint32_t a = mix32((uint32_t)(seed & 0xFFFFFFFFu) ^ 0x9E3779B9u);
    a = mix32(a ^ (uint32_t)(seed >> 32));
    a = mix32(a + b);
    a = mix32(a ^ t);
    for (int i = 0; i < kPermRounds; ++i) out[i] = mix32(a + (uint32_t)i * 0x9E3779B9u);
}

int perm_half_width(int64_t rows)
{
    int bits = 0;
    for (uint64_t v = (uint64_t)(rows - 1); v != 0; v >>= 1) ++bits;
    const int h = (bits + 1) / 2;
    return h < 1 ? 1 : h;
}

hipError_t launch_perm(int32_t* out, int64_t rows, int npass, const PermKeys& keys, hipStream_t stream, const int32_t* subset,
                       int64_t limit, unsigned* bad)
{
    if (rows <= 0 || npass <= 0) return hipSuccess;
    if (npass > kMaxPassesPerLaunch || rows > (int64_t(1) << 30)) return hipErrorInvalidValue;
    if (subset && (!bad || limit < rows || limit > (int64_t(1) << 30))) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((rows + 255) / 256), (unsigned)npass);
    hipLaunchKernelGGL(perm_kernel, grid, dim3(256), 0, stream, out, (uint32_t)rows,
                       (uint32_t)perm_half_width(rows), keys, subset, (uint32_t)limit, bad);
    return hipGetLastError();
}

}  // namespace bmgd
