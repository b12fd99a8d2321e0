// Least squares with few features: the update in its linear-system form.
//
// For the squared loss the mini-batch update of eq. (2.1) is eq. (3.1):
//     theta <- (I - alpha Sxx_m) theta + alpha Sxy_m,   Sxx_m = n_b^-1 sum x x',  Sxy_m = n_b^-1 sum x y
// over the rows of mini-batch m.  Sxx_m and Sxy_m do not depend on theta, so when p is small (p^2 << n p)
// they are formed for every mini-batch of a pass by a fully parallel pre-pass over the buffer -- a dense
// contraction [X y]' [X y] per mini-batch, on the matrix cores in fp32 -- and the strictly sequential chain
// then costs p^2 multiply-adds and 4 p^2 bytes per step inside ONE workgroup: no exchange between workgroups
// at all.  Same arithmetic as the row form up to the order of summation.
#include "bmgd_internal.h"
#include "gram_layout.h"

#include <hip/hip_ext.h>

#include <algorithm>

namespace bmgd {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v)
{
    return __builtin_bit_cast(float,
                              __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

struct GramTiles {
    int ntiles;                     // upper-triangle 16 x 16 tiles of the (p + 1) x (p + 1) moment matrix
    int tsplit;                     // workgroups per mini-batch; each takes TPW consecutive entries of `tile`
    unsigned short tile[48];        // I | J << 8, I <= J; padding entries repeat tile 0 and are not written out
};

constexpr int kRowsPerChunk = 16;   // rows staged per wavefront at a time: four K = 4 matrix instructions
constexpr int kGramWaves = 4;

// Moment matrices of one mini-batch (one pass): the wavefronts take 16-row chunks in turn and accumulate
// their TPW tiles of [X y]' [X y]; the four partial sums meet in LDS, are divided by n_b and written in the
// chain's layout (both triangles).  MFMA operand layout (v_mfma_f32_16x16x4_f32): a = A[lane % 16][lane / 16],
// b = B[lane / 16][lane % 16], c[v] = C[4 (lane / 16) + v][lane % 16]; here A = (staged rows)' and B = staged rows.
// VEC: p is a multiple of 4 and rows are moved as float4 (a quarter of the load, address and store instructions; the
// kernel is bound by instruction issue, not by any one unit).
template <int TPW, bool WIDE, bool VEC>
__global__ void __launch_bounds__(64 * kGramWaves) gram_mfma_kernel(const float* __restrict__ X, const float* __restrict__ y,
                                                                     const int* __restrict__ perm, float* __restrict__ out,
                                                                     int rows, int n, int perm_stride, int M, int n_items,
                                                                     int stride, GramLayout L, GramTiles T, int dense_q)
{
    extern __shared__ __align__(16) float lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // Workgroups go to the eight XCDs in turn (blockIdx % 8), each with an L2 of its own: the tsplit workgroups
    // that read the same mini-batch are consecutive on one XCD, so all but the first find its rows in that L2.
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int part = slot % T.tsplit;
    const int mb = (slot / T.tsplit) * 8 + xcd;
    if (mb >= n_items) return;
    const int m = mb % M, pass = mb / M;
    const int p = L.p;
    const int nb = min(n, rows - m * n);
    const int* idx = perm + (size_t)pass * perm_stride + (size_t)m * n;
    float* xs = lds + wave * kRowsPerChunk * stride;             // this wavefront's staging area
    constexpr int CL = WIDE ? 2 : 1;                              // 64-column groups of a row

    for (int e = lane; e < kRowsPerChunk * stride; e += 64) xs[e] = 0.f;   // padding columns stay zero

    int tI[TPW], tJ[TPW];
#pragma unroll
    for (int t = 0; t < TPW; ++t) {
        const int g = part * TPW + t;
        const unsigned short code = T.tile[g < T.ntiles ? g : 0];
        tI[t] = 16 * (code & 0xFF);
        tJ[t] = 16 * (code >> 8);
    }
    floatx4 acc[TPW];
#pragma unroll
    for (int t = 0; t < TPW; ++t) acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};

    const int nchunks = (nb + kRowsPerChunk - 1) / kRowsPerChunk;
    float v[kRowsPerChunk][CL];                      // (not VEC)
    float yv = 0.f;
    // VEC: the 16 * p / 4 float4 of a chunk are dealt to the lanes in turn; which row and which columns lane l's i-th
    // float4 belongs to does not change from chunk to chunk
    constexpr int NV = WIDE ? 8 : 4;                 // float4 per lane and chunk: 16 * (p / 4) / 64 rounded up for the largest p
    float4 v4[VEC ? NV : 1];
    int vrow[VEC ? NV : 1], vcol[VEC ? NV : 1];      // row of the chunk (as a byte offset of its lane for the shuffle), first column
    if constexpr (VEC) {
        const int p4 = p >> 2;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int e = min(lane + 64 * i, kRowsPerChunk * p4 - 1);    // (beyond the chunk: the last float4 again, same value)
            const int r = e / p4;
            vrow[i] = r;
            vcol[i] = 4 * (e - r * p4);
        }
    }
    auto request = [&](int chunk) {
        if constexpr (VEC) {
            const int i = min(chunk * kRowsPerChunk + (lane & 15), nb - 1);
            const int row = idx[i];
            yv = y[row];
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                const int rr = __builtin_amdgcn_ds_bpermute(4 * vrow[q], row);   // the row index held by lane vrow[q]
                v4[q] = *reinterpret_cast<const float4*>(X + (size_t)rr * p + vcol[q]);
            }
        } else {
            // unconditional loads from clamped rows and columns; what lies outside the mini-batch is zeroed on use
            const int i = min(chunk * kRowsPerChunk + (lane & 15), nb - 1);
            const int row = idx[i];
            yv = y[row];
#pragma unroll
            for (int r = 0; r < kRowsPerChunk; ++r) {
                const int rr = __builtin_amdgcn_readlane(row, r);
                const float* src = X + (size_t)rr * p;
#pragma unroll
                for (int j = 0; j < CL; ++j) v[r][j] = src[min(lane + 64 * j, p - 1)];
            }
        }
    };
    auto stage = [&](int chunk) {
        const int left = nb - chunk * kRowsPerChunk;              // rows of this chunk inside the mini-batch
        if constexpr (VEC) {
            if (left < kRowsPerChunk) {                           // (uniform) the last chunk: rows beyond the mini-batch are zeroed
#pragma unroll
                for (int q = 0; q < NV; ++q)
                    if (vrow[q] >= left) v4[q] = make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int q = 0; q < NV; ++q) *reinterpret_cast<float4*>(xs + vrow[q] * stride + vcol[q]) = v4[q];
            __builtin_amdgcn_wave_barrier();
            if (lane < kRowsPerChunk) xs[lane * stride + p] = lane < left ? yv : 0.f;
        } else {
#pragma unroll
            for (int r = 0; r < kRowsPerChunk; ++r) {
#pragma unroll
                for (int j = 0; j < CL; ++j) {
                    // no branch: lanes beyond p write a zero into a padding column (or into the column of y, which
                    // the store below then overwrites)
                    const int c = lane + 64 * j;
                    xs[r * stride + min(c, stride - 1)] = (c < p && r < left) ? v[r][j] : 0.f;
                }
            }
            __builtin_amdgcn_wave_barrier();
            if (lane < kRowsPerChunk) xs[lane * stride + p] = lane < left ? yv : 0.f;
        }
    };

    if (wave < nchunks) request(wave);
    for (int chunk = wave; chunk < nchunks; chunk += kGramWaves) {
        __builtin_amdgcn_wave_barrier();
        stage(chunk);
        __builtin_amdgcn_wave_barrier();
        if (chunk + kGramWaves < nchunks) request(chunk + kGramWaves);
#pragma unroll
        for (int kk = 0; kk < kRowsPerChunk / 4; ++kk) {
            const float* rowp = xs + (4 * kk + (lane >> 4)) * stride + (lane & 15);
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                const float a = rowp[tI[t]];
                const float b = rowp[tJ[t]];
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[t], 0, 0, 0);
            }
        }
    }

    // sum over the wavefronts, scale, write out
    __syncthreads();
    floatx4* red = reinterpret_cast<floatx4*>(lds);               // [wave][TPW][64]
#pragma unroll
    for (int t = 0; t < TPW; ++t) red[(wave * TPW + t) * 64 + lane] = acc[t];
    __syncthreads();
    const float inv = 1.f / (float)nb;
    // dense_q > 0: the matrix [Sxx_m | -Sxy_m] goes out dense, row-major with row stride dense_q, for the kernel that
    // multiplies steps together (gram_products.hip); rows and columns beyond it are never written (they stay zero)
    float* o = out + (size_t)(pass * M + m) * (dense_q > 0 ? (size_t)dense_q * dense_q : (size_t)L.step_floats);
    const int my_tiles = min(TPW, T.ntiles - part * TPW);
    for (int t = wave; t < my_tiles; t += kGramWaves) {
        floatx4 s = red[t * 64 + lane];
#pragma unroll
        for (int w = 1; w < kGramWaves; ++w) s += red[(w * TPW + t) * 64 + lane];
        const unsigned short code = T.tile[part * TPW + t];
        const int I = 16 * (code & 0xFF), J = 16 * (code >> 8);
        const int c = J + (lane & 15);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int r = I + 4 * (lane >> 4) + q;
            const float val = s[q] * inv;
            if (dense_q > 0) {
                if (r < p && c < p) {
                    o[r * dense_q + c] = val;
                    if (I != J) o[c * dense_q + r] = val;
                } else if (r < p && c == p) {
                    o[r * dense_q + p] = -val;
                }
            } else if (r < p && c < p) {
                o[gram_pos(L, r, c)] = val;
                if (I != J) o[gram_pos(L, c, r)] = val;
            } else if (r < p && c == p) {
                o[L.b_off + r] = val;
            }
        }
    }
}

// The chain: one workgroup, theta in LDS (two copies, alternating), the matrices of the coming AHEAD steps
// already in registers.  Thread (i, seg) = (t / TPR, t % TPR); the TPR lanes of a row add up their parts.
// OPT: an update rule other than the plain step: separate instantiations, the plain path carries none of it.
template <int TPR, int KQ, int KS, int AHEAD, bool TAB, bool OPT>
__global__ void __launch_bounds__(1024) gram_chain_kernel(const float* __restrict__ gram, float* __restrict__ theta,
                                                          GramLayout L, int nsteps, int period, float alpha,
                                                          const float* __restrict__ lr_tab, int lr_base, int lr_len, OptArgs opt)
{
    __shared__ __align__(16) float th[2][kGramMaxP + 4 * 16];
    const int t = threadIdx.x;
    const int i = t / TPR, seg = t % TPR;
    const int p = L.p;
    const bool row_ok = i < p;
    constexpr int NQ = KQ > 0 ? KQ : 1, NS = KS > 0 ? KS : 1;
    float4 sq[AHEAD][NQ];
    float ss[AHEAD][NS];
    float bb[AHEAD];
    float aa[AHEAD];                                  // learning rate of the step, from the optional table
    const int ib = row_ok ? i : 0;
    int fidx = 0;                                     // matrices to request next; wraps when passes share one partition
    // Addresses are a wavefront-uniform base (scalar registers) plus a 32-bit per-thread byte offset that never
    // changes: no vector arithmetic per request.
    const unsigned off16 = (unsigned)t * 16u, off4 = (unsigned)t * 4u, offb = (unsigned)ib * 4u;
    // TAB: the learning rate of a step comes from lr_tab (requested with the step's matrices), else it is alpha.
    const int lr_last = lr_len - 1;
    int lr_next = lr_base;
    auto fetch = [&](float4 (&q)[NQ], float (&sc)[NS], float& bv, float& av) {
        const char* g = reinterpret_cast<const char*>(gram + (size_t)fidx * L.step_floats);
        fidx = fidx + 1 == period ? 0 : fidx + 1;
#pragma unroll
        for (int k = 0; k < KQ; ++k) q[k] = *reinterpret_cast<const float4*>(g + (size_t)k * L.nthr * 16 + off16);
#pragma unroll
        for (int j = 0; j < KS; ++j) sc[j] = *reinterpret_cast<const float*>(g + (size_t)(4 * KQ + j) * L.nthr * 4 + off4);
        bv = *reinterpret_cast<const float*>(g + (size_t)L.b_off * 4 + offb);
        if constexpr (TAB) {
            av = lr_tab[min(lr_next, lr_last)];
            lr_next += 1;
        }
    };
#pragma unroll
    for (int d = 0; d + 1 < AHEAD; ++d) fetch(sq[d], ss[d], bb[d], aa[d]);
    for (int c = t; c < kGramMaxP + 64; c += blockDim.x) { th[0][c] = c < p ? theta[c] : 0.f; th[1][c] = 0.f; }
    // The compiler is free to reorder these first requests; with all of them landed before the loop, the waits
    // it places inside the loop count only the requests of the loop itself, which are issued oldest slot first.
    __builtin_amdgcn_s_waitcnt(0x0F70);               // vmcnt(0)
    __syncthreads();

    // Steps are taken AHEAD at a time without any branch around the loads (a branch would make the compiler
    // wait for every outstanding load); steps past the last one run with a zero learning rate.
    // optimizer state of coordinate i lives in the registers of the lane that updates it
    const bool owner = seg == 0 && row_ok;
    float om = 0.f, os = 0.f;
    if (OPT && owner) {
        om = opt.m[i];
        if (opt.kind == kOptAdam) os = opt.s[i];
    }
    int cur = 0;
    for (int sb = 0; sb < nsteps; sb += AHEAD) {
#pragma unroll
        for (int d = 0; d < AHEAD; ++d) {
            const float a_eff = sb + d < nsteps ? (TAB ? aa[d] : alpha) : 0.f;
            // Request step s + AHEAD - 1 into the ring slot the previous step has just used up, before this step's
            // arithmetic: the memory pipeline works on the requests of all wavefronts while they compute.
            const int prev = (d + AHEAD - 1) % AHEAD;
            fetch(sq[prev], ss[prev], bb[prev], aa[prev]);
            float dot0 = 0.f, dot1 = 0.f;
#pragma unroll
            for (int k = 0; k < KQ; ++k) {
                const float4 tv = *reinterpret_cast<const float4*>(&th[cur][4 * (seg + TPR * k)]);
                dot0 = fmaf(sq[d][k].x, tv.x, dot0);
                dot1 = fmaf(sq[d][k].y, tv.y, dot1);
                dot0 = fmaf(sq[d][k].z, tv.z, dot0);
                dot1 = fmaf(sq[d][k].w, tv.w, dot1);
            }
#pragma unroll
            for (int j = 0; j < KS; ++j) {
                const float tv = th[cur][4 * TPR * KQ + TPR * j + seg];
                if (j & 1) dot1 = fmaf(ss[d][j], tv, dot1); else dot0 = fmaf(ss[d][j], tv, dot0);
            }
            float dot = dot0 + dot1;
            const float base = fmaf(a_eff, bb[d], th[cur][ib]);
            if (TPR >= 2) dot += dpp_mov<0xB1>(dot);      // lanes ^1
            if (TPR >= 4) dot += dpp_mov<0x4E>(dot);      // lanes ^2
            if (TPR >= 8) dot += dpp_mov<0x141>(dot);     // mirror within 8
            if (TPR >= 16) dot += dpp_mov<0x140>(dot);    // mirror within 16
            if constexpr (!OPT) {
                if (owner) th[cur ^ 1][i] = fmaf(-a_eff, dot, base);
            } else if (owner) {
                float nv = th[cur][i];
                if (sb + d < nsteps) {               // steps past the last one leave theta and the state alone
                    float c1 = 1.f, c2 = 1.f;
                    if (opt.kind == kOptAdam) opt_corrections(opt, opt.k_base + sb + d + 1, c1, c2);
                    nv = opt_update(opt, nv, dot - bb[d], a_eff, om, os, c1, c2);
                }
                th[cur ^ 1][i] = nv;
            }
            __syncthreads();
            cur ^= 1;
        }
    }
    for (int c = t; c < p; c += blockDim.x) theta[c] = th[cur][c];
    if (OPT && owner) {
        opt.m[i] = om;
        if (opt.kind == kOptAdam) opt.s[i] = os;
    }
}

// tiles per workgroup for NT tile rows: {few workgroups, many workgroups}
void tile_split(int ntiles, int wgs_per_split, int* tsplit, int* tpw)
{
    // at most 10 tiles per workgroup: measured faster than wider workgroups (more of them, two per SIMD)
    static const int options[10][3] = {{1, 1, 1}, {3, 1, 1}, {6, 1, 1}, {10, 1, 2}, {15, 3, 3},
                                       {21, 3, 3}, {28, 4, 4}, {36, 4, 4}, {45, 5, 5}, {0, 0, 0}};
    for (int i = 0; options[i][0]; ++i)
        if (options[i][0] == ntiles) {
            const int few = options[i][1], many = options[i][2];
            *tsplit = wgs_per_split * few >= 256 ? few : many;
            *tpw = (ntiles + *tsplit - 1) / *tsplit;
            return;
        }
    *tsplit = 0;
    *tpw = 0;
}

template <int TPW>
hipError_t launch_gram_mfma(bool wide, dim3 grid, size_t lds, hipStream_t stream, const float* X, const float* y, const int32_t* perm,
                            float* out, int rows, int n, int perm_stride, int M, int n_items, int stride, const GramLayout& L,
                            const GramTiles& T, int dense_q, hipEvent_t start, hipEvent_t stop)
{
    // the events ride on the dispatch itself: no separate markers in the queue
    const bool vec = L.p % 4 == 0;
#define GRAM_LAUNCH(W, V)                                                                                                          \
    hipExtLaunchKernelGGL((gram_mfma_kernel<TPW, W, V>), grid, dim3(64 * kGramWaves), (uint32_t)lds, stream, start, stop, 0u, X, y,  \
                          perm, out, rows, n, perm_stride, M, n_items, stride, L, T, dense_q)
    if (wide && vec) GRAM_LAUNCH(true, true);
    else if (wide) GRAM_LAUNCH(true, false);
    else if (vec) GRAM_LAUNCH(false, true);
    else GRAM_LAUNCH(false, false);
#undef GRAM_LAUNCH
    return hipGetLastError();
}

template <int TPR, int KQ, int KS>
hipError_t launch_chain(const GramLayout& L, const float* gram, float* theta, int nsteps, int period, float alpha, const float* lr_tab,
                        int lr_base, int lr_len, const OptArgs& opt, hipStream_t stream, hipEvent_t start, hipEvent_t stop)
{
    constexpr int per_step = 4 * KQ + KS + 1;
    constexpr int AHEAD = per_step <= 9 ? 8 : per_step <= 14 ? 6 : 4;
    auto go = [&](auto kernel) {
        hipExtLaunchKernelGGL(kernel, dim3(1), dim3(L.nthr), 0u, stream, start, stop, 0u, gram, theta, L, nsteps, period, alpha, lr_tab,
                              lr_base, lr_len, opt);
    };
    const bool with_opt = opt.kind != kOptSgd;
    if (lr_tab && with_opt) go(gram_chain_kernel<TPR, KQ, KS, AHEAD, true, true>);
    else if (lr_tab) go(gram_chain_kernel<TPR, KQ, KS, AHEAD, true, false>);
    else if (with_opt) go(gram_chain_kernel<TPR, KQ, KS, AHEAD, false, true>);
    else go(gram_chain_kernel<TPR, KQ, KS, AHEAD, false, false>);
    return hipGetLastError();
}

template <int TPR, int KQ>
hipError_t launch_chain_ks(const GramLayout& L, const float* gram, float* theta, int nsteps, int period, float alpha,
                           const float* lr_tab, int lr_base, int lr_len, const OptArgs& opt, hipStream_t stream, hipEvent_t start,
                           hipEvent_t stop)
{
    switch (L.ks) {
    case 0: return launch_chain<TPR, KQ, 0>(L, gram, theta, nsteps, period, alpha, lr_tab, lr_base, lr_len, opt, stream, start, stop);
    case 1: return launch_chain<TPR, KQ, 1>(L, gram, theta, nsteps, period, alpha, lr_tab, lr_base, lr_len, opt, stream, start, stop);
    case 2: return launch_chain<TPR, KQ, 2>(L, gram, theta, nsteps, period, alpha, lr_tab, lr_base, lr_len, opt, stream, start, stop);
    case 3: return launch_chain<TPR, KQ, 3>(L, gram, theta, nsteps, period, alpha, lr_tab, lr_base, lr_len, opt, stream, start, stop);
    case 4: return launch_chain<TPR, KQ, 4>(L, gram, theta, nsteps, period, alpha, lr_tab, lr_base, lr_len, opt, stream, start, stop);
    }
    return hipErrorInvalidValue;
}

}  // namespace

bool gram_eligible(int model, int64_t p, int64_t n)
{
    return model == 0 && p <= kGramMaxP && n >= 2 * p;
}

size_t gram_bytes_per_batch(int64_t p)
{
    return (size_t)make_layout((int)p).step_floats * sizeof(float);
}

int gram_dense_order(int64_t p) { return (int)((p + 1 + 15) / 16 * 16); }

size_t gram_dense_bytes_per_batch(int64_t p)
{
    const size_t q = (size_t)gram_dense_order(p);
    return q * q * sizeof(float);
}

int gram_chain_threads(int64_t p)
{
    return make_layout((int)p).nthr;
}

hipError_t gram_launch_moments(const float* X, const float* y, const int32_t* perm, float* gram, int rows, int p, int n, int npass,
                               int perm_stride, hipStream_t stream, hipEvent_t start, hipEvent_t stop, bool dense)
{
    const int dense_q = dense ? gram_dense_order(p) : 0;
    if (p < 1 || p > kGramMaxP) return hipErrorInvalidValue;
    const GramLayout L = make_layout(p);
    const int M = (rows + n - 1) / n;
    const int gpass = perm_stride == 0 ? 1 : npass;      // one partition for all passes: one set of matrices
    const int NT = (p + 1 + 15) / 16;                    // tile rows of the moment matrix of [X y]
    GramTiles T{};
    T.ntiles = NT * (NT + 1) / 2;
    int tpw = 0;
    tile_split(T.ntiles, M * gpass, &T.tsplit, &tpw);
    if (T.tsplit == 0) return hipErrorInvalidValue;
    {
        int k = 0;
        for (int I = 0; I < NT; ++I)
            for (int J = I; J < NT; ++J) T.tile[k++] = (unsigned short)(I | (J << 8));
        for (; k < 48; ++k) T.tile[k] = 0;
    }
    int stride = NT * 16;
    if (stride % 32 == 0) stride += 16;                  // rows k and k + 1 of an operand read fall on different banks
    const size_t lds = sizeof(float) * (size_t)std::max(kGramWaves * kRowsPerChunk * stride, kGramWaves * tpw * 64 * 4);
    const int n_items = M * gpass;
    const dim3 grid((unsigned)((n_items + 7) / 8 * 8 * T.tsplit));
    const bool wide = p > 64;
    hipError_t e = hipErrorInvalidValue;
#define GRAM_CASE(N) case N: e = launch_gram_mfma<N>(wide, grid, lds, stream, X, y, perm, gram, rows, n, perm_stride, M, n_items, stride, L, T, dense_q, start, stop); break
    switch (tpw) {
        GRAM_CASE(1); GRAM_CASE(3); GRAM_CASE(5); GRAM_CASE(6); GRAM_CASE(7); GRAM_CASE(9); GRAM_CASE(10);
    }
#undef GRAM_CASE
    return e;
}

hipError_t gram_launch_chain(const float* gram, float* theta, int rows, int p, int n, int npass, int perm_stride, float alpha,
                             const float* lr_tab, int lr_base, int lr_len, const OptArgs& opt, hipStream_t stream,
                             hipEvent_t start, hipEvent_t stop)
{
    const int M = (rows + n - 1) / n;
    const int nsteps = M * npass, period = perm_stride == 0 ? M : nsteps;
    return gram_launch_chain_steps(gram, theta, p, nsteps, period, alpha, lr_tab, lr_base, lr_len, opt, stream, start, stop);
}

hipError_t gram_launch_chain_steps(const float* gram, float* theta, int p, int nsteps, int period, float alpha, const float* lr_tab,
                                   int lr_base, int lr_len, const OptArgs& opt, hipStream_t stream, hipEvent_t start,
                                   hipEvent_t stop)
{
    if (p < 1 || p > kGramMaxP || nsteps < 1 || period < 1) return hipErrorInvalidValue;
    const GramLayout L = make_layout(p);
    if (L.tpr == 16) {
        switch (L.kq) {
        case 0: return launch_chain_ks<16, 0>(L, gram, theta, nsteps, period, alpha, lr_tab, lr_base, lr_len, opt, stream, start, stop);
        case 1: return launch_chain_ks<16, 1>(L, gram, theta, nsteps, period, alpha, lr_tab, lr_base, lr_len, opt, stream, start, stop);
        }
    } else {
        switch (L.kq) {
        case 2: return launch_chain_ks<8, 2>(L, gram, theta, nsteps, period, alpha, lr_tab, lr_base, lr_len, opt, stream, start, stop);
        case 3: return launch_chain_ks<8, 3>(L, gram, theta, nsteps, period, alpha, lr_tab, lr_base, lr_len, opt, stream, start, stop);
        case 4: return launch_chain_ks<8, 4>(L, gram, theta, nsteps, period, alpha, lr_tab, lr_base, lr_len, opt, stream, start, stop);
        }
    }
    return hipErrorInvalidValue;
}

}  // namespace bmgd
