// Least squares with few features: the steps of a launch multiplied together instead of applied one by one.
//
// A step of eq. (3.1) is an affine map, theta <- (I - alpha_s Sxx_s) theta + alpha_s Sxy_s, which in homogeneous
// coordinates is the (p + 1) x (p + 1) matrix A_s = [[I - alpha_s Sxx_s, alpha_s Sxy_s], [0, 1]].  None of the A_s
// depends on theta, so the estimate after the N steps of a launch is [theta; 1] <- A_{N-1} ... A_1 A_0 [theta; 1]
// (the products of eq. (3.2)), and the product can be formed as a tree: N / 2 independent products of neighbours, then
// N / 4, ... -- log2 N launches of small dense products on the matrix cores (fp32 in, fp32 accumulate) in place of a
// chain of N dependent steps in one workgroup.  Same arithmetic as the chain up to the order of the fp32 operations;
// intermediate estimates are not formed.
#include "bmgd_internal.h"
#include "glm_device.h"
#include "gram_layout.h"

#include <hip/hip_ext.h>

#include <algorithm>

namespace bmgd {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kPairThreads = 256;
constexpr int kMaxTilesPerWave = 3;                  // Q <= 144: nine tile columns over four wavefronts

struct FirstLevel {                                  // where the steps' moment matrices are, and their learning rates
    const float* dense;                              // per mini-batch [Sxx | -Sxy], dense of order Q (gram_launch_moments, dense)
    int p;
    int period;                                      // step s uses matrix s % period
    float alpha;
    const float* lr_tab;                             // optional: step s uses lr_tab[min(lr_base + s, lr_len - 1)]
    int lr_base, lr_len;
};

constexpr int kMaxOrder = (kGramMaxP + 1 + 15) / 16 * 16;                       // 144
constexpr int kMaxRightVec = (kMaxOrder * kMaxOrder / 4 + kPairThreads - 1) / kPairThreads;   // float4 of the right factor per thread
constexpr int kTileRows = 2;                          // 16-row tile rows of a product per workgroup (the right factor is staged once for both)
constexpr int kMaxLeftVec = (16 * kTileRows * kMaxOrder / 4 + kPairThreads - 1) / kPairThreads;   // of the left factor's rows

// out[j] = in[2 j + 1] * in[2 j] (the later step on the left); a missing in[2 j + 1] counts as the identity.  Dense
// Q x Q matrices, row-major, Q a multiple of 16.  Workgroup (x, y) computes the tile rows 2 x and 2 x + 1 of out[y]: it stages
// their 32 rows of the left factor and the whole right factor in shared memory and each wavefront takes every fourth 16 x 16
// tile of both rows.  Everything a thread stages is requested first and stored afterwards (unconditional loads from clamped
// addresses), so the staging costs one trip to memory, not one per element; row and column of a float4 come from a
// multiplication (qv_inv = 2^20 / (Q / 4) + 1: exact for the 5184 float4 of the largest matrix).  MFMA operand layout
// (v_mfma_f32_16x16x4_f32): a = A[lane % 16][lane / 16], b = B[lane / 16][lane % 16], c[v] = C[4 (lane / 16) + v][lane % 16].
// FIRST: the factors are the steps themselves, A_s = [[I - alpha_s Sxx_s, alpha_s Sxy_s], [0, 1]] padded with zeros:
// entry (r, c) is (r == c and r <= p) - alpha_s D_s(r, c) with D_s the dense matrix the moments kernel wrote.
// CHAIN_OUT: the product P goes out as [I - P | last column of P] in the layout the chain kernel reads (GramLayout), so
// that the chain's step theta - 1 * ((I - P) theta - d) applies it.
template <bool FIRST, bool CHAIN_OUT = false>
__global__ void __launch_bounds__(kPairThreads) affine_pair_kernel(FirstLevel f, const float* __restrict__ in, float* __restrict__ out,
                                                                   int count_in, int Q, int rs, unsigned qv_inv, GramLayout L)
{
    extern __shared__ __align__(16) float lds[];
    const int ls = Q + 4;                            // row stride of the left factor's rows: float4 stores stay aligned, and a
    float* Ls = lds;                                 // column read (16 rows, one k) meets each bank at most twice
    float* Rs = lds + 16 * kTileRows * ls;           // right factor, row stride rs = 16 (mod 32): four rows of 16 columns apart
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int NT = Q / 16, QV = Q / 4;
    const int tr = kTileRows * blockIdx.x, j = blockIdx.y;   // first tile row of this workgroup
    const int nrows = 16 * min(kTileRows, NT - tr);  // rows of the left factor it needs
    const int right = 2 * j, left = 2 * j + 1;
    const bool has_left = left < count_in;
    const int lc = has_left ? left : right;          // (clamped: not used when the left factor is the identity)

    const float* Rm;
    const float* Lm;
    float a_r = 0.f, a_l = 0.f;
    if constexpr (FIRST) {
        Rm = f.dense + (size_t)(right % f.period) * Q * Q;
        Lm = f.dense + (size_t)(lc % f.period) * Q * Q + (size_t)16 * tr * Q;
        a_r = f.lr_tab ? f.lr_tab[min(f.lr_base + right, f.lr_len - 1)] : f.alpha;
        a_l = f.lr_tab ? f.lr_tab[min(f.lr_base + lc, f.lr_len - 1)] : f.alpha;
    } else {
        Rm = in + (size_t)right * Q * Q;
        Lm = in + (size_t)lc * Q * Q + (size_t)16 * tr * Q;        // its 16 rows are contiguous
    }
    const int nR = Q * QV, nL = nrows * QV;
    float4 rv[kMaxRightVec], lv[kMaxLeftVec];
#pragma unroll
    for (int i = 0; i < kMaxRightVec; ++i)
        rv[i] = *reinterpret_cast<const float4*>(Rm + (size_t)4 * min(tid + kPairThreads * i, nR - 1));
#pragma unroll
    for (int i = 0; i < kMaxLeftVec; ++i)
        lv[i] = *reinterpret_cast<const float4*>(Lm + (size_t)4 * min(tid + kPairThreads * i, nL - 1));
    // entry (r, c .. c + 3) of a factor from what was loaded for it
    auto entry = [&](float4 v, float alpha, int r, int c) {
        if constexpr (FIRST) {
            const bool in_map = r <= f.p;
            v.x = (in_map && r == c ? 1.f : 0.f) - alpha * v.x;
            v.y = (in_map && r == c + 1 ? 1.f : 0.f) - alpha * v.y;
            v.z = (in_map && r == c + 2 ? 1.f : 0.f) - alpha * v.z;
            v.w = (in_map && r == c + 3 ? 1.f : 0.f) - alpha * v.w;
        }
        return v;
    };
#pragma unroll
    for (int i = 0; i < kMaxRightVec; ++i) {
        const int e = tid + kPairThreads * i;
        if (e < nR) {
            const int r = (int)(((unsigned)e * qv_inv) >> 20), c = 4 * (e - r * QV);
            const float4 v = entry(rv[i], a_r, r, c);
            *reinterpret_cast<float4*>(Rs + r * rs + c) = v;
        }
    }
#pragma unroll
    for (int i = 0; i < kMaxLeftVec; ++i) {
        const int e = tid + kPairThreads * i;
        if (e < nL) {
            const int ii = (int)(((unsigned)e * qv_inv) >> 20), c = 4 * (e - ii * QV), r = 16 * tr + ii;
            float4 v = entry(lv[i], a_l, r, c);
            if (!has_left) v = make_float4(r == c ? 1.f : 0.f, r == c + 1 ? 1.f : 0.f, r == c + 2 ? 1.f : 0.f, r == c + 3 ? 1.f : 0.f);
            *reinterpret_cast<float4*>(Ls + ii * ls + c) = v;
        }
    }
    __syncthreads();

    floatx4 acc[kTileRows][kMaxTilesPerWave];
#pragma unroll
    for (int h = 0; h < kTileRows; ++h)
#pragma unroll
        for (int t = 0; t < kMaxTilesPerWave; ++t) acc[h][t] = floatx4{0.f, 0.f, 0.f, 0.f};
    const float* ap = Ls + (lane & 15) * ls + (lane >> 4);
    const float* bp = Rs + (lane >> 4) * rs + (lane & 15);
    const bool two = nrows > 16;                     // (the same for the whole workgroup)
    // (Q is a multiple of 16: four K steps per trip, their operand reads issued together)
    for (int k0 = 0; k0 < Q; k0 += 16) {
        float a[4][kTileRows], b[4][kMaxTilesPerWave];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
#pragma unroll
            for (int h = 0; h < kTileRows; ++h) a[q][h] = ap[(two ? 16 * h : 0) * ls + k0 + 4 * q];
#pragma unroll
            for (int t = 0; t < kMaxTilesPerWave; ++t) b[q][t] = bp[(k0 + 4 * q) * rs + 16 * min(wave + 4 * t, NT - 1)];
        }
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int t = 0; t < kMaxTilesPerWave; ++t)
                if (wave + 4 * t < NT) {             // (the same for the whole wavefront)
                    acc[0][t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[q][0], b[q][t], acc[0][t], 0, 0, 0);
                    if (two) acc[1][t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[q][1], b[q][t], acc[1][t], 0, 0, 0);
                }
    }
    float* o = out + (size_t)j * (CHAIN_OUT ? (size_t)L.step_floats : (size_t)Q * Q);
#pragma unroll
    for (int h = 0; h < kTileRows; ++h) {
        if (16 * h >= nrows) break;
#pragma unroll
        for (int t = 0; t < kMaxTilesPerWave; ++t) {
            const int tc = wave + 4 * t;
            if (tc < NT) {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int r = 16 * (tr + h) + 4 * (lane >> 4) + v, c = 16 * tc + (lane & 15);
                    if constexpr (CHAIN_OUT) {
                        if (r < L.p && c < L.p) o[gram_pos(L, r, c)] = (r == c ? 1.f : 0.f) - acc[h][t][v];
                        else if (r < L.p && c == L.p) o[L.b_off + r] = acc[h][t][v];
                    } else {
                        o[(size_t)r * Q + c] = acc[h][t][v];
                    }
                }
            }
        }
    }
}

// theta <- P[0 .. p) [theta; 1]: one workgroup; wavefront w takes rows w, w + 4, ..., its lanes the columns (all of a
// wavefront's rows are requested before any is summed).
__global__ void __launch_bounds__(256) affine_apply_kernel(const float* __restrict__ P, float* __restrict__ theta, int p, int Q)
{
    __shared__ float th[kMaxOrder + 64], nv[kGramMaxP];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int RPW = (kGramMaxP + 3) / 4, CPL = (kMaxOrder + 63) / 64;      // rows per wavefront, columns per lane
    float v[RPW][CPL];
#pragma unroll
    for (int i = 0; i < RPW; ++i)
#pragma unroll
        for (int k = 0; k < CPL; ++k)
            v[i][k] = P[(size_t)min(wave + 4 * i, p - 1) * Q + min(lane + 64 * k, Q - 1)];
    for (int c = tid; c < kMaxOrder + 64; c += 256) th[c] = c < p ? theta[c] : (c == p ? 1.f : 0.f);
    __syncthreads();
#pragma unroll
    for (int i = 0; i < RPW; ++i) {
        float s = 0.f;
#pragma unroll
        for (int k = 0; k < CPL; ++k) s = fmaf(v[i][k], th[lane + 64 * k], s);   // columns beyond p meet zeros
        s = group_sum(s, 64);                        // (lane butterflies: a shuffle through shared memory per stage and row would dominate)
        const int r = wave + 4 * i;
        if (lane == 0 && r < p) nv[r] = s;
    }
    __syncthreads();
    for (int c = tid; c < p; c += 256) theta[c] = nv[c];
}

int padded_order(int p) { return gram_dense_order(p); }

}  // namespace

size_t gram_products_scratch_floats(int64_t p, int64_t max_steps)
{
    const size_t Q = (size_t)padded_order((int)p);
    const size_t half = (size_t)(max_steps + 1) / 2, quarter = (half + 1) / 2;
    const size_t per = std::max(Q * Q, (size_t)make_layout((int)p).step_floats);       // dense, or in the chain's layout
    return (half + quarter) * per;
}

hipError_t gram_launch_apply(const float* product, float* theta, int p, hipStream_t stream, hipEvent_t start, hipEvent_t stop)
{
    if (p < 1 || p > kGramMaxP) return hipErrorInvalidValue;
    hipExtLaunchKernelGGL(affine_apply_kernel, dim3(1), dim3(256), 0u, stream, start, stop, 0u, product, theta, p, padded_order(p));
    return hipGetLastError();
}

namespace {

// what every launch of the pair kernel needs
struct PairSetup {
    int N, Q, NT, rs;
    size_t lds;
    unsigned qv_inv;
    FirstLevel f;
};

hipError_t pair_setup(const float* gram, int rows, int p, int n, int npass, int perm_stride, float alpha, const float* lr_tab,
                      int lr_base, int lr_len, PairSetup* out)
{
    if (p < 1 || p > kGramMaxP) return hipErrorInvalidValue;
    const int M = (rows + n - 1) / n;
    PairSetup s{};
    s.N = M * npass;
    s.Q = padded_order(p);
    s.NT = s.Q / 16;
    if (s.NT > 4 * kMaxTilesPerWave) return hipErrorInvalidValue;
    s.rs = s.Q % 32 == 0 ? s.Q + 16 : s.Q;
    s.lds = sizeof(float) * (size_t)(16 * kTileRows * (s.Q + 4) + s.Q * s.rs);
    s.qv_inv = (1u << 20) / (unsigned)(s.Q / 4) + 1u;
    s.f.dense = gram;
    s.f.p = p;
    s.f.period = perm_stride == 0 ? M : s.N;
    s.f.alpha = alpha;
    s.f.lr_tab = lr_tab;
    s.f.lr_base = lr_base;
    s.f.lr_len = lr_len;
    *out = s;
    return hipSuccess;
}

}  // namespace

hipError_t gram_products_prepare()
{
    // the pair kernel stages up to 92 KB in shared memory (order 144): above the default limit of a launch
    const int bytes = 160 * 1024 - 64;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(affine_pair_kernel<true>), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(affine_pair_kernel<false>), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(affine_pair_kernel<true, true>), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    return e;
}

hipError_t gram_launch_pairs(const float* gram, float* pairs_out, int rows, int p, int n, int npass, int perm_stride, float alpha,
                             const float* lr_tab, int lr_base, int lr_len, hipStream_t stream, hipEvent_t start, hipEvent_t stop)
{
    PairSetup s;
    hipError_t e = pair_setup(gram, rows, p, n, npass, perm_stride, alpha, lr_tab, lr_base, lr_len, &s);
    if (e != hipSuccess) return e;
    hipExtLaunchKernelGGL((affine_pair_kernel<true, true>), dim3((s.NT + kTileRows - 1) / kTileRows, (s.N + 1) / 2), dim3(kPairThreads), (uint32_t)s.lds, stream, start,
                          stop, 0u, s.f, static_cast<const float*>(nullptr), pairs_out, s.N, s.Q, s.rs, s.qv_inv, make_layout(p));
    return hipGetLastError();
}

hipError_t gram_launch_products(const float* gram, float* theta, float* scratch, float* product_out, int rows, int p, int n, int npass,
                                int perm_stride, float alpha, const float* lr_tab, int lr_base, int lr_len, hipStream_t stream,
                                hipEvent_t start, hipEvent_t stop, bool pairs_then_chain)
{
    PairSetup ps;
    {
        hipError_t e0 = pair_setup(gram, rows, p, n, npass, perm_stride, alpha, lr_tab, lr_base, lr_len, &ps);
        if (e0 != hipSuccess) return e0;
    }
    const int N = ps.N, Q = ps.Q, NT = ps.NT, rs = ps.rs;
    const size_t lds = ps.lds;
    const unsigned qv_inv = ps.qv_inv;
    const FirstLevel f = ps.f;
    const GramLayout L = make_layout(p);
    if (pairs_then_chain) {
        // one round of products into the chain's layout, then the chain over half as many steps, each applied with rate 1
        hipError_t e = gram_launch_pairs(gram, scratch, rows, p, n, npass, perm_stride, alpha, lr_tab, lr_base, lr_len, stream, start,
                                         nullptr);
        if (e != hipSuccess) return e;
        OptArgs none{};
        none.kind = kOptSgd;
        const int half = (N + 1) / 2;
        return gram_launch_chain_steps(scratch, theta, p, half, half, 1.0f, nullptr, 0, 0, none, stream, nullptr, stop);
    }
    float* buf[2] = {scratch, scratch + (size_t)((N + 1) / 2) * Q * Q};
    // the round that leaves one matrix writes it where the caller wants the product of the launch
    float* fin = product_out ? product_out : buf[0];
    int count = N, which = 0;
    // round 0 reads the moment matrices; the start event rides on its dispatch, the stop event on the last one's
    hipExtLaunchKernelGGL(affine_pair_kernel<true>, dim3((NT + kTileRows - 1) / kTileRows, (count + 1) / 2), dim3(kPairThreads), (uint32_t)lds, stream, start, nullptr,
                          0u, f, static_cast<const float*>(nullptr), count <= 2 ? fin : buf[0], count, Q, rs, qv_inv, L);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const float* cur = count <= 2 ? fin : buf[0];
    count = (count + 1) / 2;
    while (count > 1) {
        float* dst = count <= 2 ? fin : buf[which ^ 1];
        if (dst == cur) dst = buf[which ^ 1];        // (no product_out: the last round must not write what it reads)
        hipLaunchKernelGGL(affine_pair_kernel<false>, dim3((NT + kTileRows - 1) / kTileRows, (count + 1) / 2), dim3(kPairThreads), lds, stream, f, cur, dst, count, Q,
                           rs, qv_inv, L);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        cur = dst;
        count = (count + 1) / 2;
        which ^= 1;
    }
    return gram_launch_apply(cur, theta, p, stream, nullptr, stop);
}

}  // namespace bmgd
