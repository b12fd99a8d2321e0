// Layout of the moment matrices of a mini-batch in device memory, shared by the kernel that forms them, the chain
// that reads them step by step (gram_kernels.hip) and the kernel that multiplies the steps of a pass together
// (gram_products.hip).
#pragma once

#include <hip/hip_runtime.h>

namespace bmgd {
namespace {

// Where the chain kernel wants entry (r, c) of Sxx_m: thread t = r * tpr + seg of the chain owns, of row r, the
// float4 chunks seg + tpr k (k < kq) and the single columns 4 tpr kq + tpr j + seg (j < ks); all threads' k-th
// chunks are contiguous ("plane" k), so every load instruction of a wavefront reads one contiguous KiB.
struct GramLayout {
    int p, tpr, nthr, kq, ks;
    int b_off;          // Sxy_m: p floats
    int step_floats;    // floats per mini-batch, multiple of 4
};

__device__ __host__ __forceinline__ int gram_pos(const GramLayout& L, int r, int c)
{
    const int wide = 4 * L.tpr * L.kq;
    if (c < wide) {
        const int chunk = c >> 2, k = chunk / L.tpr, seg = chunk % L.tpr;
        return ((k * L.nthr + r * L.tpr + seg) << 2) + (c & 3);
    }
    const int cc = c - wide, j = cc / L.tpr, seg = cc % L.tpr;
    return 4 * L.kq * L.nthr + j * L.nthr + r * L.tpr + seg;
}

inline GramLayout make_layout(int p)
{
    GramLayout L{};
    L.p = p;
    L.tpr = p <= 64 ? 16 : 8;
    L.nthr = (p * L.tpr + 63) / 64 * 64;
    L.kq = p / (4 * L.tpr);
    const int rem = p - 4 * L.tpr * L.kq;
    L.ks = (rem + L.tpr - 1) / L.tpr;
    L.b_off = 4 * L.kq * L.nthr + L.ks * L.nthr;
    L.step_floats = (L.b_off + p + 3) & ~3;
    return L;
}

}  // namespace
}  // namespace bmgd
