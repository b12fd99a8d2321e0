// Softmax regression step on the matrix cores (bf16 inputs, fp32 accumulation and master weights).
//
// One mini-batch update of eq. (2.1) for the C-class member of the GLM family of Section 3.2.3:
//     U = X_b W            (n_b x C logits)                       -- MFMA, bf16 x bf16 -> fp32
//     R = softmax_rows(U) - onehot(y)                             -- fp32, stored as bf16
//     W <- W - (alpha / n_b) X_b' R                               -- MFMA, fused with the update
// with W kept in fp32 (the "master") and a bf16 copy refreshed by the update's epilogue.
//
// Both contractions run through one "NT" tile kernel, C[m][n] = sum_k A[m][k] B[n][k], whose two operands
// are read along their contiguous K axis.  The data is laid out so that this is always possible:
//   logits    A = gathered rows of X (K = features),          B = WbT [C_pad][p]  (bf16 copy, transposed)
//   gradient  A = XT [p][n_pad] (the batch, transposed once per pass, K = rows), B = Rt [C_pad][n_pad]
// XT is written by a permute-and-transpose pass over the slot that does not depend on W, so it sits outside
// the sequential chain.  Tiles are 128 x 128 x 32 per workgroup of four wavefronts, each wavefront owning a
// 64 x 64 quadrant as 2 x 2 v_mfma_f32_32x32x16_bf16 tiles.
#include "bmgd_internal.h"

namespace bmgd {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int TM = 128, TN = 128, TK = 32;
constexpr int LDS_STRIDE = 40;                     // bf16 elements per tile row in LDS (80 bytes: 16-byte aligned, spreads banks)

__device__ __forceinline__ unsigned short f32_to_bf16_rne(float f)
{
    unsigned u = __builtin_bit_cast(unsigned, f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}

// ---------------------------------------------------------------------------------------------------
// XT[m][c][j] = X[perm[m * n + j]][c] for every mini-batch m of one pass (zero for j beyond the batch).
__global__ void __launch_bounds__(256) permute_transpose_kernel(const unsigned short* __restrict__ X,
                                                                const int* __restrict__ perm,
                                                                unsigned short* __restrict__ XT, int rows, int p, int n,
                                                                int n_pad, int jtiles)
{
    // 64 rows x 64 features per workgroup, moved 16 bytes at a time in both directions (p and n_pad are
    // multiples of 8): a thread reads 8 features of one row, and writes 8 rows of one feature.
    constexpr int TS = 72;                           // tile row stride in elements: 16-byte aligned rows
    __shared__ __align__(16) unsigned short tile[64 * TS];
    const int m = blockIdx.x / jtiles, jt = blockIdx.x % jtiles;
    const int j0 = jt * 64, c0 = blockIdx.y * 64;
    const int nb = min(n, rows - m * n);
    const int seg = threadIdx.x & 7, rq = threadIdx.x >> 3;      // 8 chunks x 32
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int r = rq + 32 * h, j = j0 + r, c = c0 + 8 * seg;
        // unconditional load from a clamped row and chunk; zeroed below if it lies outside
        const int row = perm[m * n + min(j, nb - 1)];
        uint4 v = *reinterpret_cast<const uint4*>(X + (size_t)row * p + min(c, p - 8));
        if (j >= nb || c >= p) v = make_uint4(0, 0, 0, 0);
        *reinterpret_cast<uint4*>(&tile[r * TS + 8 * seg]) = v;
    }
    __syncthreads();
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int cl = rq + 32 * h, c = c0 + cl, j = j0 + 8 * seg;
        unsigned short e[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) e[q] = tile[(8 * seg + q) * TS + cl];
        uint4 w;
        w.x = e[0] | ((unsigned)e[1] << 16);
        w.y = e[2] | ((unsigned)e[3] << 16);
        w.z = e[4] | ((unsigned)e[5] << 16);
        w.w = e[6] | ((unsigned)e[7] << 16);
        if (c < p && j < n_pad) *reinterpret_cast<uint4*>(&XT[((size_t)m * p + c) * n_pad + j]) = w;
    }
}

// ---------------------------------------------------------------------------------------------------
struct GemmArgs {
    const unsigned short* A;    // rows of K contiguous bf16
    const int* a_idx;           // optional gather: row m is A + a_idx[m] * a_stride
    long long a_stride;
    int M;                      // valid rows of A (others read as zero)
    const unsigned short* B;
    long long b_stride;
    int N;                      // valid rows of B
    int K;                      // valid K (multiple of 8)
    int k_per_split;            // multiple of TK
    // epilogue: logits
    float* U;                   // [splits][m_pad][ldu]
    int ldu, m_pad;
    // epilogue: update
    float* W;                   // [p][ldw] fp32 master
    unsigned short* WbT;        // [ldw][ldwt] bf16 copy, transposed
    int ldw, ldwt;
    float inv_nb;               // 1 / n_b
    // The learning rate and the update count come from device memory, so that a captured sequence of launches can be
    // replayed: update number u (within the pass: a constant of the launch) uses
    // lr_tab[min(state->lr_pos + u, lr_len - 1)], or state->alpha without a table, and Adam's count state->opt_k + u + 1.
    const SoftmaxState* state;
    int u;
    const float* lr_tab;
    int lr_len;
    OptArgs opt;                // state arrays [p][ldw] like W; plain steps if kind == kOptSgd (k_base unused)
    int tiles_m, tiles_n, splits;   // work items = splits * tiles_m * tiles_n, dealt to XCDs in contiguous runs
};

// K tiles are pipelined: up to kDepth tiles are requested ahead into registers, one tile sits in each of two
// LDS buffers, and one is being multiplied.  A tile's arithmetic takes ~0.1 us while a trip to L2/HBM takes
// ~1 us, so the loop would otherwise run at memory latency.
constexpr int kDepth = 4;
// Eight wavefronts per workgroup, two per SIMD, each with a 64 x 32 part of the 128 x 128 tile: a wavefront's waits (global ->
// register -> shared memory -> register -> MFMA) are covered by its SIMD mate.
constexpr int kGemmThreads = 512;
constexpr int kWN = 32;                             // columns of the tile per wavefront (one MFMA tile wide, two high)

// OPT (with UPDATE): an update rule other than the plain step, in an instantiation of its own.
template <bool UPDATE, bool OPT = false>
__global__ void __launch_bounds__(kGemmThreads) gemm_nt_kernel(GemmArgs g)
{
    __shared__ __align__(16) unsigned short As[2][TM * LDS_STRIDE];
    __shared__ __align__(16) unsigned short Bs[2][TN * LDS_STRIDE];
    __shared__ __align__(16) unsigned short Ts[UPDATE ? TN * (TM + 8) : 8];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // Workgroups are handed to the 8 XCDs round robin, each XCD with its own L2.  Work items are ordered
    // (split, tile row, tile column) and XCD x takes the x-th contiguous eighth, so the tiles that share
    // rows of A and the whole of B for one K range meet in one L2.
    const int total = g.splits * g.tiles_m * g.tiles_n;
    const int per = (total + 7) / 8;
    const int item = (int)(blockIdx.x % 8) * per + (int)(blockIdx.x / 8);
    if (item >= total) return;
    const int split = item / (g.tiles_m * g.tiles_n);
    const int tile = item - split * (g.tiles_m * g.tiles_n);
    const int m0 = (tile / g.tiles_n) * TM, n0 = (tile % g.tiles_n) * TN;
    const int kb = split * g.k_per_split;
    const int ke = min(g.K, kb + g.k_per_split);
    const int ntiles = (ke - kb + TK - 1) / TK;

    // Each thread moves one 16-byte chunk of A and one of B per K tile.  Every request is unconditional, from a
    // clamped row and a clamped K offset; what lies outside the operands is zeroed when the chunk goes to LDS.
    // (A branch or a select next to the load would make the compiler wait for the load on the spot.)
    constexpr int CPT = TM * (TK / 8) / kGemmThreads;   // chunks per thread and operand
    const unsigned short* a_ptr[CPT];
    const unsigned short* b_ptr[CPT];
    int lds_off[CPT], kc[CPT];
    bool a_ok[CPT], b_ok[CPT];
#pragma unroll
    for (int h = 0; h < CPT; ++h) {
        const int chunk = tid + h * kGemmThreads;
        const int row = chunk >> 2;
        kc[h] = (chunk & 3) * 8;
        lds_off[h] = row * LDS_STRIDE + kc[h];
        const int am = m0 + row, bn = n0 + row;
        a_ok[h] = am < g.M;
        b_ok[h] = bn < g.N;
        const int amc = min(am, g.M - 1), bnc = min(bn, g.N - 1);
        a_ptr[h] = g.A + (size_t)(g.a_idx ? g.a_idx[amc] : amc) * g.a_stride;
        b_ptr[h] = g.B + (size_t)bnc * g.b_stride;
    }
    const int klast = g.K - 8;                       // K is a multiple of 8
    auto fetch = [&](int tile_k, uint4 (&ra)[CPT], uint4 (&rb)[CPT]) {
        const int k0 = kb + tile_k * TK;
#pragma unroll
        for (int h = 0; h < CPT; ++h) {
            const int k = min(k0 + kc[h], klast);
            ra[h] = *reinterpret_cast<const uint4*>(a_ptr[h] + k);
            rb[h] = *reinterpret_cast<const uint4*>(b_ptr[h] + k);
        }
    };
    auto masked = [](uint4 v, bool ok) { return ok ? v : make_uint4(0, 0, 0, 0); };

    constexpr int NJ = kWN / 32;                     // MFMA tiles side by side per wavefront
    f32x16 acc[2][NJ];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    constexpr int WCOLS = TN / kWN;                  // wavefronts side by side
    const int wm = (wave / WCOLS) * 64, wn = (wave % WCOLS) * kWN;
    const int frow = lane & 31, fk = (lane >> 5) * 8;

    // Ring of kDepth register slots.  A slot goes to LDS, and only then is requested again, so no copy of it is
    // ever live across a request; the first requests are waited for before the loop (the compiler is free to
    // reorder them) so that the waits inside the loop count the loop's own requests, oldest slot first.  The
    // loop has no branch: tiles past the last one are all zeros and add nothing.
    uint4 ra[kDepth][CPT], rb[kDepth][CPT];
#pragma unroll
    for (int d = 0; d < kDepth; ++d) fetch(d, ra[d], rb[d]);
    __builtin_amdgcn_s_waitcnt(0x0F70);              // vmcnt(0)
    for (int tb = 0; tb < ntiles; tb += kDepth) {
#pragma unroll
        for (int d = 0; d < kDepth; ++d) {
            const int t = tb + d;
            const int buf = d & 1;                   // kDepth is even, so tile t uses buffer t % 2
            const int k0 = kb + t * TK;
#pragma unroll
            for (int h = 0; h < CPT; ++h) {
                const bool kin = k0 + kc[h] < ke;
                *reinterpret_cast<uint4*>(&As[buf][lds_off[h]]) = masked(ra[d][h], a_ok[h] && kin);
                *reinterpret_cast<uint4*>(&Bs[buf][lds_off[h]]) = masked(rb[d][h], b_ok[h] && kin);
            }
            fetch(t + kDepth, ra[d], rb[d]);
            __syncthreads();                         // tile t visible; the other buffer was last read before this point
#pragma unroll
            for (int ks = 0; ks < TK; ks += 16) {
                bf16x8 fa[2], fb[NJ];
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    fa[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(&As[buf][(wm + i * 32 + frow) * LDS_STRIDE + ks + fk]));
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    fb[j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(&Bs[buf][(wn + j * 32 + frow) * LDS_STRIDE + ks + fk]));
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
            }
        }
    }

    // accumulator layout of the 32 x 32 tile: lane holds column (lane % 32); value v is row
    // 8 * (v / 4) + 4 * (lane / 32) + (v % 4)
    const int ccol = lane & 31, rbase = (lane >> 5) * 4;
    if constexpr (!UPDATE) {
        float* U = g.U + (size_t)split * g.m_pad * g.ldu;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int r = m0 + wm + i * 32 + 8 * (v >> 2) + rbase + (v & 3);
                    const int c = n0 + wn + j * 32 + ccol;
                    if (r < g.m_pad && c < g.ldu) U[(size_t)r * g.ldu + c] = acc[i][j][v];
                }
    } else {
        const float alpha = g.lr_tab ? g.lr_tab[min(g.state->lr_pos + g.u, g.lr_len - 1)] : g.state->alpha;
        const float scale = alpha * g.inv_nb;
        float oc1 = 1.f, oc2 = 1.f;
        if (OPT && g.opt.kind == kOptAdam) opt_corrections(g.opt, g.state->opt_k + g.u + 1, oc1, oc2);
        // rows are features, columns are classes: W[r][c] -= scale * acc; bf16 copy goes out transposed.
        // The 32 master weights of a half-quadrant are requested together, from clamped addresses and without a
        // branch, and only then combined and stored (a branch around each load would wait for it on the spot).
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            float wv[NJ][16];
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int r = min(m0 + wm + i * 32 + 8 * (v >> 2) + rbase + (v & 3), g.M - 1);
                    const int c = min(n0 + wn + j * 32 + ccol, g.ldw - 1);
                    wv[j][v] = g.W[(size_t)r * g.ldw + c];
                }
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int lr = wm + i * 32 + 8 * (v >> 2) + rbase + (v & 3);
                    const int lc = wn + j * 32 + ccol;
                    const int r = m0 + lr, c = n0 + lc;
                    const bool ok = r < g.M && c < g.ldw;
                    float w = 0.f;
                    if constexpr (!OPT) {
                        w = ok ? wv[j][v] - scale * acc[i][j][v] : 0.f;
                    } else if (ok) {
                        // the state is read here, element by element: this path trades speed for the extra arrays
                        const size_t at = (size_t)r * g.ldw + c;
                        float m = g.opt.m[at], sv = g.opt.kind == kOptAdam ? g.opt.s[at] : 0.f;
                        w = opt_update(g.opt, wv[j][v], acc[i][j][v] * g.inv_nb, alpha, m, sv, oc1, oc2);
                        g.opt.m[at] = m;
                        if (g.opt.kind == kOptAdam) g.opt.s[at] = sv;
                    }
                    if (ok) g.W[(size_t)r * g.ldw + c] = w;
                    Ts[lc * (TM + 8) + lr] = f32_to_bf16_rne(w);
                }
        }
        __syncthreads();
        // 128 class rows x 128 features: 16 chunks of 8 features per class row
        for (int chunk = tid; chunk < TN * (TM / 8); chunk += kGemmThreads) {
            const int lc = chunk >> 4, lr = (chunk & 15) * 8;
            const int c = n0 + lc, r = m0 + lr;
            if (c < g.ldw && r < g.ldwt)
                *reinterpret_cast<uint4*>(&g.WbT[(size_t)c * g.ldwt + r]) = *reinterpret_cast<const uint4*>(&Ts[lc * (TM + 8) + lr]);
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// R = softmax(U) - onehot(y) for SM_ROWS rows per workgroup, one row per wavefront with the row's logits
// held in registers so U is read once (lane l owns classes 4l .. 4l+3 of every block of 256); written
// transposed as Rt[c][j] (bf16), 16 bytes per class and workgroup.  U is the sum of `splits` partial logit
// buffers; classes >= C are padding and get probability 0.
constexpr int SM_ROWS = 8;
constexpr int SM_THREADS = SM_ROWS * 64;
constexpr int SM_MAXB = 8;                         // blocks of 256 classes per row: c_pad <= 2048

// KB = blocks of 256 classes a row spans (rounded up to a power of two), SPLITS = partial logit buffers: both
// compile-time so that every load of a row is issued up front, unconditionally and from clamped addresses
// (a branch or a loop around the loads would turn them into SPLITS * KB round trips to memory, one after another).
template <int KB, int SPLITS>
__global__ void __launch_bounds__(SM_THREADS) softmax_residual_kernel(const float* __restrict__ U, int m_pad, int ldu,
                                                                      const int* __restrict__ y, const int* __restrict__ idx,
                                                                      int nb, int n_pad, int C, unsigned short* __restrict__ Rt)
{
    extern __shared__ __align__(16) unsigned short rl[];      // [SM_ROWS][ldu + 8]
    const int lds_stride = ldu + 8;
    const int lane = threadIdx.x & 63, rr = threadIdx.x >> 6;
    const int i0 = blockIdx.x * SM_ROWS;
    const int i = i0 + rr;
    unsigned short* out = rl + rr * lds_stride;
    if (i >= nb) {                                   // padding rows of the K axis of the gradient contraction
        for (int c = lane; c < ldu; c += 64) out[c] = 0;
    } else {
        const int row = idx[i];
        float4 q[SPLITS][KB];
#pragma unroll
        for (int sp = 0; sp < SPLITS; ++sp)
#pragma unroll
            for (int k = 0; k < KB; ++k)
                q[sp][k] = *reinterpret_cast<const float4*>(U + ((size_t)sp * m_pad + i) * ldu + min(4 * lane + 256 * k, ldu - 4));
        const int label = y[row];
        float u[KB][4];
        float mx = -INFINITY;
#pragma unroll
        for (int k = 0; k < KB; ++k) {
            const int c = 4 * lane + 256 * k;
            float4 t = q[0][k];
#pragma unroll
            for (int sp = 1; sp < SPLITS; ++sp) { t.x += q[sp][k].x; t.y += q[sp][k].y; t.z += q[sp][k].z; t.w += q[sp][k].w; }
            const float tv[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                u[k][v] = c + v < C ? tv[v] : -INFINITY;      // padding classes (and clamped reads) count as -inf
                mx = fmaxf(mx, u[k][v]);
            }
        }
        for (int o = 32; o >= 1; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
        float sum = 0.f;
#pragma unroll
        for (int k = 0; k < KB; ++k)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                u[k][v] = expf(u[k][v] - mx);        // exp(-inf) = 0 for padding classes
                sum += u[k][v];
            }
        for (int o = 32; o >= 1; o >>= 1) sum += __shfl_xor(sum, o);
        const float inv = 1.f / sum;
#pragma unroll
        for (int k = 0; k < KB; ++k) {
            const int c = 4 * lane + 256 * k;
            if (c < ldu) {
                unsigned short h[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) h[v] = f32_to_bf16_rne(u[k][v] * inv - (c + v == label ? 1.f : 0.f));
                uint2 w;
                w.x = h[0] | ((unsigned)h[1] << 16);
                w.y = h[2] | ((unsigned)h[3] << 16);
                *reinterpret_cast<uint2*>(out + c) = w;
            }
        }
    }
    __syncthreads();
    // transposed store: for class c, SM_ROWS consecutive j (16 bytes)
    for (int c = threadIdx.x; c < ldu; c += SM_THREADS) {
        unsigned short v[SM_ROWS];
#pragma unroll
        for (int q = 0; q < SM_ROWS; ++q) v[q] = rl[q * lds_stride + c];
        uint4 w;
        w.x = v[0] | ((unsigned)v[1] << 16);
        w.y = v[2] | ((unsigned)v[3] << 16);
        w.z = v[4] | ((unsigned)v[5] << 16);
        w.w = v[6] | ((unsigned)v[7] << 16);
        *reinterpret_cast<uint4*>(Rt + (size_t)c * n_pad + i0) = w;
    }
}

// Evaluation: cross-entropy -log softmax(u)[label] of SM_ROWS rows per workgroup from the (split) logits, one row per
// wavefront, summed in fp64 into partial[blockIdx.x].  Not on the hot path: plain loops.
__global__ void __launch_bounds__(SM_THREADS) softmax_loss_kernel(const float* __restrict__ U, int splits, int m_pad, int ldu,
                                                                  const int* __restrict__ y, int nb, int C,
                                                                  double* __restrict__ partial)
{
    __shared__ double wsum[SM_ROWS];
    const int lane = threadIdx.x & 63, rr = threadIdx.x >> 6;
    const int i = blockIdx.x * SM_ROWS + rr;
    double l = 0.0;
    if (i < nb) {
        const int label = y[i];
        float u[SM_MAXB][4];
        float mx = -INFINITY, ul = 0.f;
#pragma unroll
        for (int k = 0; k < SM_MAXB; ++k) {
            const int c = 4 * lane + 256 * k;
#pragma unroll
            for (int v = 0; v < 4; ++v) u[k][v] = -INFINITY;
            if (c < ldu) {
                float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
                for (int sp = 0; sp < splits; ++sp) {
                    const float4 q = *reinterpret_cast<const float4*>(U + ((size_t)sp * m_pad + i) * ldu + c);
                    t.x += q.x; t.y += q.y; t.z += q.z; t.w += q.w;
                }
                const float tv[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (c + v < C) {
                        u[k][v] = tv[v];
                        mx = fmaxf(mx, tv[v]);
                        if (c + v == label) ul = tv[v];
                    }
            }
        }
        for (int o = 32; o >= 1; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
        float sum = 0.f;
#pragma unroll
        for (int k = 0; k < SM_MAXB; ++k)
#pragma unroll
            for (int v = 0; v < 4; ++v) sum += expf(u[k][v] - mx);
        for (int o = 32; o >= 1; o >>= 1) {
            sum += __shfl_xor(sum, o);
            ul += __shfl_xor(ul, o);                 // only the lane that owns the label holds a non-zero value
        }
        l = (double)(mx + logf(sum) - ul);
    }
    if (lane == 0) wsum[rr] = l;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int q = 0; q < SM_ROWS; ++q) t += wsum[q];
        partial[blockIdx.x] = t;
    }
}

// WbT[c][r] = bf16(W[r][c]) for the whole matrix (after bmgd_set_theta / at creation).
__global__ void __launch_bounds__(256) shadow_kernel(const float* __restrict__ W, unsigned short* __restrict__ WbT, int p,
                                                     int ldw, int ldwt)
{
    __shared__ float tile[32][33];
    const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;      // 32 x 8
    for (int rr = ty; rr < 32; rr += 8) {
        const int r = r0 + rr, c = c0 + tx;
        tile[rr][tx] = (r < p && c < ldw) ? W[(size_t)r * ldw + c] : 0.f;
    }
    __syncthreads();
    for (int cc = ty; cc < 32; cc += 8) {
        const int c = c0 + cc, r = r0 + tx;
        if (c < ldw && r < ldwt) WbT[(size_t)c * ldwt + r] = f32_to_bf16_rne(tile[tx][cc]);
    }
}

__global__ void softmax_state_kernel(SoftmaxState* st, float alpha, int lr_pos, int opt_k)
{
    st->alpha = alpha;
    st->lr_pos = lr_pos;
    st->opt_k = opt_k;
}

}  // namespace

hipError_t softmax_set_state(SoftmaxState* state, float alpha, int lr_pos, int opt_k, hipStream_t stream)
{
    hipLaunchKernelGGL(softmax_state_kernel, dim3(1), dim3(1), 0, stream, state, alpha, lr_pos, opt_k);
    return hipGetLastError();
}

SoftmaxDims softmax_dims(int64_t p, int64_t n, int64_t C)
{
    SoftmaxDims d;
    d.c_pad = (int)((C + TN - 1) / TN * TN);
    d.n_pad = (int)((n + TK - 1) / TK * TK);
    d.m_pad = (int)((n + TM - 1) / TM * TM);
    d.p_pad = (int)((p + TM - 1) / TM * TM);
    const int tiles = (d.m_pad / TM) * (d.c_pad / TN);
    int splits = 1;
    const int ktiles = (int)((p + TK - 1) / TK);
    while (tiles * splits < 256 && splits < 8 && ktiles / (splits * 2) >= 8) splits *= 2;
    d.splits = splits;
    d.k_per_split = ((ktiles + splits - 1) / splits) * TK;
    return d;
}

hipError_t softmax_permute_transpose(const void* X, const int32_t* perm, void* XT, int rows, int p, int n,
                                     const SoftmaxDims& d, hipStream_t stream)
{
    const int M = (rows + n - 1) / n;
    const int jtiles = (d.n_pad + 63) / 64;
    dim3 grid((unsigned)(M * jtiles), (unsigned)((p + 63) / 64));
    hipLaunchKernelGGL(permute_transpose_kernel, grid, dim3(256), 0, stream, static_cast<const unsigned short*>(X), perm,
                       static_cast<unsigned short*>(XT), rows, p, n, d.n_pad, jtiles);
    return hipGetLastError();
}

namespace {

template <int KB, int SPLITS>
hipError_t launch_residual_ks(const SoftmaxDims& d, size_t lds, hipStream_t stream, const SoftmaxStep& s)
{
    hipLaunchKernelGGL((softmax_residual_kernel<KB, SPLITS>), dim3(d.n_pad / SM_ROWS), dim3(SM_THREADS), lds, stream, s.U, d.m_pad,
                       d.c_pad, s.y, s.idx, s.nb, d.n_pad, s.C, static_cast<unsigned short*>(s.Rt));
    return hipGetLastError();
}

template <int KB>
hipError_t launch_residual_k(const SoftmaxDims& d, size_t lds, hipStream_t stream, const SoftmaxStep& s)
{
    switch (d.splits) {
    case 1: return launch_residual_ks<KB, 1>(d, lds, stream, s);
    case 2: return launch_residual_ks<KB, 2>(d, lds, stream, s);
    case 4: return launch_residual_ks<KB, 4>(d, lds, stream, s);
    case 8: return launch_residual_ks<KB, 8>(d, lds, stream, s);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_residual(const SoftmaxDims& d, size_t lds, hipStream_t stream, const SoftmaxStep& s)
{
    const int blocks = (d.c_pad + 255) / 256;
    if (blocks <= 1) return launch_residual_k<1>(d, lds, stream, s);
    if (blocks <= 2) return launch_residual_k<2>(d, lds, stream, s);
    if (blocks <= 4) return launch_residual_k<4>(d, lds, stream, s);
    return launch_residual_k<8>(d, lds, stream, s);
}

}  // namespace

hipError_t softmax_step(const SoftmaxStep& s, const SoftmaxDims& d, hipStream_t stream)
{
    // 1. logits
    GemmArgs g{};
    g.A = static_cast<const unsigned short*>(s.X);
    g.a_idx = s.idx;
    g.a_stride = s.p;
    g.M = s.nb;
    g.B = static_cast<const unsigned short*>(s.WbT);
    g.b_stride = d.p_pad;
    g.N = d.c_pad;
    g.K = s.p;
    g.k_per_split = d.k_per_split;
    g.U = s.U;
    g.ldu = d.c_pad;
    g.m_pad = d.m_pad;
    g.tiles_m = (s.nb + TM - 1) / TM;
    g.tiles_n = d.c_pad / TN;
    g.splits = d.splits;
    hipLaunchKernelGGL(gemm_nt_kernel<false>, dim3((g.tiles_m * g.tiles_n * g.splits + 7) / 8 * 8), dim3(kGemmThreads), 0, stream, g);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // 2. residual
    const size_t lds = (size_t)SM_ROWS * (d.c_pad + 8) * sizeof(unsigned short);
    if ((e = launch_residual(d, lds, stream, s)) != hipSuccess) return e;
    // 3. gradient + update
    GemmArgs h{};
    h.A = static_cast<const unsigned short*>(s.XT);
    h.a_idx = nullptr;
    h.a_stride = d.n_pad;
    h.M = s.p;
    h.B = static_cast<const unsigned short*>(s.Rt);
    h.b_stride = d.n_pad;
    h.N = d.c_pad;
    h.K = d.n_pad;
    h.k_per_split = d.n_pad;
    h.W = s.W;
    h.WbT = static_cast<unsigned short*>(s.WbT);
    h.ldw = d.c_pad;
    h.ldwt = d.p_pad;
    h.inv_nb = 1.f / (float)s.nb;
    h.state = s.state;
    h.u = s.u;
    h.lr_tab = s.lr_tab;
    h.lr_len = s.lr_len;
    h.opt = s.opt;
    h.tiles_m = d.p_pad / TM;
    h.tiles_n = d.c_pad / TN;
    h.splits = 1;
    if (s.opt.kind != kOptSgd)
        hipLaunchKernelGGL((gemm_nt_kernel<true, true>), dim3((h.tiles_m * h.tiles_n + 7) / 8 * 8), dim3(kGemmThreads), 0, stream, h);
    else
        hipLaunchKernelGGL((gemm_nt_kernel<true, false>), dim3((h.tiles_m * h.tiles_n + 7) / 8 * 8), dim3(kGemmThreads), 0, stream, h);
    return hipGetLastError();
}

hipError_t softmax_launch_loss(const void* X, const int32_t* y, int nb, int p, int C, const void* WbT, float* U,
                               const SoftmaxDims& d, double* partial, hipStream_t stream)
{
    GemmArgs g{};
    g.A = static_cast<const unsigned short*>(X);
    g.a_idx = nullptr;
    g.a_stride = p;
    g.M = nb;
    g.B = static_cast<const unsigned short*>(WbT);
    g.b_stride = d.p_pad;
    g.N = d.c_pad;
    g.K = p;
    g.k_per_split = d.k_per_split;
    g.U = U;
    g.ldu = d.c_pad;
    g.m_pad = d.m_pad;
    g.tiles_m = (nb + TM - 1) / TM;
    g.tiles_n = d.c_pad / TN;
    g.splits = d.splits;
    hipLaunchKernelGGL(gemm_nt_kernel<false>, dim3((g.tiles_m * g.tiles_n * g.splits + 7) / 8 * 8), dim3(kGemmThreads), 0, stream, g);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(softmax_loss_kernel, dim3((nb + SM_ROWS - 1) / SM_ROWS), dim3(SM_THREADS), 0, stream, U, d.splits, d.m_pad,
                       d.c_pad, y, nb, C, partial);
    return hipGetLastError();
}

hipError_t softmax_prepare(const SoftmaxDims& d)
{
    // every kernel here stays within the default 64 KiB of LDS (residual kernel: 8 rows of at most 2056 bf16)
    return d.c_pad <= 256 * SM_MAXB ? hipSuccess : hipErrorInvalidValue;
}

hipError_t softmax_refresh_shadow(const float* W, void* WbT, int p, const SoftmaxDims& d, hipStream_t stream)
{
    dim3 grid((unsigned)(d.c_pad / 32), (unsigned)(d.p_pad / 32));
    hipLaunchKernelGGL(shadow_kernel, grid, dim3(256), 0, stream, W, static_cast<unsigned short*>(WbT), p, d.c_pad, d.p_pad);
    return hipGetLastError();
}

}  // namespace bmgd
