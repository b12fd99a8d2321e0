// Fused mini-batch gradient + update for least squares and logistic regression.
//
// One step of eq. (2.1): theta <- theta - alpha/n_b * sum_{i in batch} (b'(x_i'theta) - y_i) x_i, with
// b' the identity (eq. (3.1)) or the sigmoid (Section 3.2.3).  The steps of a pass, and the passes of a
// buffer, depend on each other through theta (Algorithm 1's inner loops), so the whole chain for one
// buffer runs inside ONE persistent kernel: all workgroups are resident at once, each mini-batch is spread over all
// of them, and a grid-wide barrier per step stands where a kernel boundary would otherwise be.
//
// Data path of a step (per row, read from HBM exactly once):
//   * a row is held in the registers of L cooperating lanes (L a power of two, 64/L rows per wavefront);
//     lane l owns the columns V*(l + L*k) .. +V-1, k < CPL, and keeps its slice of theta and of the
//     gradient accumulator for exactly those columns;
//   * u = x'theta is finished with DPP / permlane-swap butterflies inside the wavefront, the residual
//     is formed, and the same registers feed acc += r * x;
//   * accumulators are summed over the row slots of a wavefront (lane shuffles), over wavefronts (LDS)
//     and over workgroups (global partial sums, fixed order, so results are reproducible run to run);
//   * rows of the next step do not depend on theta: their loads are issued before the barrier wait and
//     are in flight while the barrier resolves.
//
// Reduction across workgroups, two forms:
//   redundant  every workgroup sums all partials itself and keeps its own copy of theta (one barrier per
//              step; for small p * G);
//   sliced     workgroup g sums a slice of the columns, writes that slice of theta, second barrier, all
//              re-read theta (for large p).
#include "bmgd_internal.h"

#include <stdio.h>

#include <algorithm>

namespace bmgd {

namespace {

enum { kLinear = 0, kLogistic = 1 };

template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v)
{
    return __builtin_bit_cast(float,
                              __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

// lane i of an even 16-lane row + lane i of the odd row next to it, result in both
__device__ __forceinline__ float swap16_sum(float v)
{
    // Both registers are rewritten by the instruction, so it is issued as inline assembly with two
    // read-write operands (the compiler builtin hands back only one of the two results).  The s_nop
    // covers the wait states the instruction needs after a VALU write of its operands.
    float a = v, b = v;
    asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
    return a + b;
}

// lane i of the lower half-wave + lane i of the upper half-wave, result in both
__device__ __forceinline__ float swap32_sum(float v)
{
    // Both registers are rewritten by the instruction, so it is issued as inline assembly with two
    // read-write operands (the compiler builtin hands back only one of the two results).  The s_nop
    // covers the wait states the instruction needs after a VALU write of its operands.
    float a = v, b = v;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
    return a + b;
}

// Sum over each aligned group of L consecutive lanes; every lane of the group receives the sum.
__device__ __forceinline__ float group_sum(float v, int L)
{
    if (L >= 2) v += dpp_mov<0xB1>(v);    // quad_perm [1,0,3,2]
    if (L >= 4) v += dpp_mov<0x4E>(v);    // quad_perm [2,3,0,1]
    if (L >= 8) v += dpp_mov<0x141>(v);   // row_half_mirror (both quads already hold their sums)
    if (L >= 16) v += dpp_mov<0x140>(v);  // row_mirror
    if (L >= 32) v = swap16_sum(v);
    if (L >= 64) v = swap32_sum(v);
    return v;
}

// Sum over the lanes that share lane % L (one per row slot of the wavefront); valid in lanes < L.
__device__ __forceinline__ float slot_sum(float v, int L)
{
    if (L <= 1) v += dpp_mov<0x121>(v);   // row_ror 1
    if (L <= 2) v += dpp_mov<0x122>(v);   // row_ror 2
    if (L <= 4) v += dpp_mov<0x124>(v);   // row_ror 4
    if (L <= 8) v += dpp_mov<0x128>(v);   // row_ror 8
    if (L <= 16) v = swap16_sum(v);
    if (L <= 32) v = swap32_sum(v);
    return v;
}

template <int V>
__device__ __forceinline__ void load_vec(const float* __restrict__ src, float* dst)
{
    if constexpr (V == 4) {
        const float4 t = *reinterpret_cast<const float4*>(src);
        dst[0] = t.x; dst[1] = t.y; dst[2] = t.z; dst[3] = t.w;
    } else if constexpr (V == 2) {
        const float2 t = *reinterpret_cast<const float2*>(src);
        dst[0] = t.x; dst[1] = t.y;
    } else {
        dst[0] = *src;
    }
}

__device__ __forceinline__ float residual(int model, float u, float y)
{
    if (model == kLogistic) {
        const float e = expf(-fabsf(u));
        const float s = (u >= 0.f) ? 1.f / (1.f + e) : e / (1.f + e);
        return s - y;
    }
    return u - y;
}

// Exchange between workgroups: "flagged words".  A value travels as one 64-bit word {tag : float bits}
// written with a single 8-byte store; a reader polls the word until it carries the tag of the step it
// waits for.  Data and readiness arrive together, so a step needs no separate barrier, fence or counter.
// Tags grow monotonically over the life of a context and 0 is never used, hence stale words never match.
__device__ __forceinline__ void ll_store(unsigned long long* dst, float v, unsigned tag)
{
    const unsigned long long w = ((unsigned long long)tag << 32) | (unsigned long long)__builtin_bit_cast(unsigned, v);
    __hip_atomic_store(dst, w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ unsigned long long ll_load(const unsigned long long* src)
{
    return __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Four flagged words requested back to back and awaited together.  (Written as inline assembly because
// the compiler waits for each atomic load before issuing the next; the instruction is the one it emits
// for an agent-scope load.)  The wait also covers this wavefront's older loads.
__device__ __forceinline__ void ll_load4(const unsigned long long* const (&src)[4], unsigned long long (&w)[4])
{
    asm volatile("global_load_dwordx2 %0, %4, off sc1\n\t"
                 "global_load_dwordx2 %1, %5, off sc1\n\t"
                 "global_load_dwordx2 %2, %6, off sc1\n\t"
                 "global_load_dwordx2 %3, %7, off sc1\n\t"
                 "s_waitcnt vmcnt(0)"
                 : "=&v"(w[0]), "=&v"(w[1]), "=&v"(w[2]), "=&v"(w[3])
                 : "v"(src[0]), "v"(src[1]), "v"(src[2]), "v"(src[3])
                 : "memory");
}

// The same with eight words per trip (wide rows: a thread has eight words to fetch per exchange, and two trips of four
// cost twice the latency of the fabric).
__device__ __forceinline__ void ll_load8(const unsigned long long* const (&src)[8], unsigned long long (&w)[8])
{
    asm volatile("global_load_dwordx2 %0, %8, off sc1\n\t"
                 "global_load_dwordx2 %1, %9, off sc1\n\t"
                 "global_load_dwordx2 %2, %10, off sc1\n\t"
                 "global_load_dwordx2 %3, %11, off sc1\n\t"
                 "global_load_dwordx2 %4, %12, off sc1\n\t"
                 "global_load_dwordx2 %5, %13, off sc1\n\t"
                 "global_load_dwordx2 %6, %14, off sc1\n\t"
                 "global_load_dwordx2 %7, %15, off sc1\n\t"
                 "s_waitcnt vmcnt(0)"
                 : "=&v"(w[0]), "=&v"(w[1]), "=&v"(w[2]), "=&v"(w[3]), "=&v"(w[4]), "=&v"(w[5]), "=&v"(w[6]), "=&v"(w[7])
                 : "v"(src[0]), "v"(src[1]), "v"(src[2]), "v"(src[3]), "v"(src[4]), "v"(src[5]), "v"(src[6]), "v"(src[7])
                 : "memory");
}

template <int U>
__device__ __forceinline__ void ll_load_n(const unsigned long long* const (&src)[U], unsigned long long (&w)[U])
{
    static_assert(U == 4 || U == 8, "four or eight words per trip");
    if constexpr (U == 4) ll_load4(src, w);
    else ll_load8(src, w);
}

// Every wait is bounded: a poll that has failed for `timeout` ticks of the 100 MHz wall clock raises the
// abort flag, which every other poller checks, and the kernel exits.
struct PollGuard {
    unsigned* flag;
    long long timeout;
    long long t0;
    unsigned misses;
    // Called after a failed poll: backs off briefly (polls travel over the fabric; a storm of them slows
    // the very stores they wait for), and reports true when the wait must be given up.
    __device__ __forceinline__ bool expired()
    {
        __builtin_amdgcn_s_sleep(2);
        ++misses;
        if (misses > 2u && (misses & 31u) != 0u) return false;   // clock and flag: first misses, then every 32nd
        if (__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) return true;
        const long long now = wall_clock64();
        if (t0 == 0) t0 = now;
        if (now - t0 > timeout) {
            __hip_atomic_store(flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return true;
        }
        return false;
    }
    __device__ __forceinline__ void arm() { t0 = 0; misses = 0; }
};

// What the cross-workgroup sum needs to know about its caller.
struct ExchangeCtx {
    int G, p, pp, tid, block;
    float* red;                 // [block] LDS scratch
    int* s_abort;               // LDS flag
    PollGuard* guard;
};

// Sum over workgroups, in fixed order, of the flagged words of columns [c_lo, c_hi) for `tag`; then
// `apply(c, sum)` runs once per column.  Leaves *s_abort set if a wait ran out.
// Thread (gs, cj) fetches column c_lo + cj of workgroups gs, gs + NG, ...: four words are requested back to
// back and awaited together, so a thread pays one trip over the fabric per four workgroups.
template <int U = 4, class F>
__device__ __forceinline__ void gather_columns_impl(const ExchangeCtx& x, const unsigned long long* words, int c_lo,
                                                    int c_hi, unsigned tag, F&& apply)
{
    const int width = c_hi - c_lo;
    if (width <= 0) return;
    const int W = min(width, x.block);
    const int NG = min(x.block / W, x.G);            // groups that have a workgroup to fetch
    const int cj = x.tid % W, gs = x.tid / W;
    float* red = x.red;
    for (int cb = c_lo; cb < c_hi; cb += W) {
        const int c = cb + cj;
        if (gs < NG && c < c_hi) {
            float t = 0.f;
            bool dead = false;
            for (int g0 = gs; g0 < x.G && !dead; g0 += NG * U) {
                const unsigned long long* src[U];
#pragma unroll
                for (int u = 0; u < U; ++u) src[u] = words + (size_t)min(g0 + u * NG, x.G - 1) * x.pp + c;
                unsigned long long w[U];
                for (;;) {
                    ll_load_n<U>(src, w);
                    bool ready = true;
#pragma unroll
                    for (int u = 0; u < U; ++u)
                        ready = ready && ((unsigned)(w[u] >> 32) == tag || g0 + u * NG >= x.G);
                    if (ready) break;
                    if (x.guard->expired()) { dead = true; break; }
                }
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if (g0 + u * NG < x.G) t += __builtin_bit_cast(float, (unsigned)w[u]);
            }
            if (dead) *x.s_abort = 1;
            red[gs * W + cj] = t;
        }
        __syncthreads();
        if (*x.s_abort) return;
        if (x.tid < W && cb + x.tid < c_hi) {
            float t0 = 0.f, t1 = 0.f, t2 = 0.f, t3 = 0.f;   // fixed association, four loads in flight
            int q = 0;
            for (; q + 4 <= NG; q += 4) {
                t0 += red[q * W + x.tid];
                t1 += red[(q + 1) * W + x.tid];
                t2 += red[(q + 2) * W + x.tid];
                t3 += red[(q + 3) * W + x.tid];
            }
            for (; q < NG; ++q) t0 += red[q * W + x.tid];
            apply(cb + x.tid, (t0 + t1) + (t2 + t3));
        }
        __syncthreads();
    }
}

// Sliced reduction: workgroup j sums a 16-column-aligned slice, applies the update to it and publishes the
// new values in kThetaCopies copies (a workgroup polls copy (its index mod kThetaCopies), so no single set
// of words is polled by the whole grid); then everyone collects the whole updated theta into th_lds.
// Returns true when a wait ran out.
template <int U = 4, class F>
__device__ __forceinline__ bool sliced_update(const ExchangeCtx& x, const unsigned long long* words,
                                              unsigned long long* thw, float* th_lds, unsigned tag, F&& new_theta)
{
    const int cw = ((x.p + x.G - 1) / x.G + 15) & ~15;   // slices are whole lines of 16 words
    const int c_lo = min(x.p, (int)blockIdx.x * cw), c_hi = min(x.p, c_lo + cw);
    const int pp = x.pp;
    gather_columns_impl<U>(x, words, c_lo, c_hi, tag, [&](int c, float t) {
        const float v = new_theta(c, t);
#pragma unroll
        for (int r = 0; r < kThetaCopies; ++r) ll_store(thw + (size_t)r * pp + c, v, tag);
    });
    __syncthreads();
    if (*x.s_abort) return true;
    const unsigned long long* mine = thw + (size_t)(blockIdx.x % kThetaCopies) * pp;
    bool dead = false;
    for (int c0 = x.tid; c0 < x.p && !dead; c0 += U * x.block) {   // U words per trip over the fabric
        const unsigned long long* src[U];
#pragma unroll
        for (int u = 0; u < U; ++u) src[u] = mine + min(c0 + u * x.block, x.p - 1);
        unsigned long long w[U];
        for (;;) {
            ll_load_n<U>(src, w);
            bool ready = true;
#pragma unroll
            for (int u = 0; u < U; ++u) ready = ready && (unsigned)(w[u] >> 32) == tag;
            if (ready) break;
            if (x.guard->expired()) { dead = true; break; }
        }
        if (dead) break;
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (c0 + u * x.block < x.p) th_lds[c0 + u * x.block] = __builtin_bit_cast(float, (unsigned)w[u]);
    }
    if (dead) *x.s_abort = 1;
    __syncthreads();
    return *x.s_abort != 0;
}

template <int V, int CPL, int PF>
struct RowGroup {
    float x[PF][CPL * V];
    float y[PF];
    bool ok[PF];
};

// PIPE selects how row loads are scheduled against the theta chain:
//   kPipeWide   one row per slot, no look-ahead inside a step; the first row of the next step is requested
//               before the exchange (wide rows: registers hold a single row);
//   kPipeGroups several groups per step with one group of look-ahead; first group of the next step requested
//               before the exchange;
//   kPipeAhead  a whole step fits one register-resident group: rows are requested TWO steps ahead, right
//               after an exchange completes, so neither the exchange (whose polls queue behind older loads
//               of the same wavefront) nor the compute ever waits for HBM latency.
enum { kPipeWide = 0, kPipeGroups = 1, kPipeAhead = 2 };

// OPT: an update rule other than the plain step (its state lives in global memory, see GlmArgs::opt); a separate
// instantiation so that the plain path carries none of it.
template <int V, int CPL, int PF, bool THL, int PIPE, int BLOCK, bool OPT>
__global__ void __launch_bounds__(BLOCK) glm_chain_kernel(GlmArgs a)
{
    extern __shared__ __align__(16) float smem[];
    __shared__ int s_abort;

    constexpr int NW = BLOCK / 64;
    constexpr int E = CPL * V;                       // floats of a row held per lane
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int L = a.L;
    const int lsub = lane & (L - 1);
    const int slot = lane >> a.logL;
    const int rpw = 64 >> a.logL;                    // rows per wavefront
    const int G = gridDim.x;
    const int p = a.p;
    const int S_total = G * NW * rpw;
    const int myslot = (blockIdx.x * NW + wave) * rpw + slot;
    const int pp = (p + 15) & ~15;                   // stride of flagged-word rows: writers own whole 128-byte lines
    const int th_len = max((p + 63) & ~63, V * L * CPL);
    float* th_lds = smem;                            // [th_len]
    float* wpart = smem + th_len;                    // [NW][p] per-wavefront sums
    float* red = wpart + NW * p;                     // [BLOCK] scratch of the cross-workgroup sum
    const int M = (a.rows + a.n - 1) / a.n;
    const int first = a.single_step >= 0 ? a.single_step : a.s_begin;
    const int last = a.single_step >= 0 ? a.single_step + 1 : a.s_end;

    int col[CPL];
#pragma unroll
    for (int k = 0; k < CPL; ++k) col[k] = V * (lsub + L * k);

    for (int c = tid; c < th_len; c += BLOCK) th_lds[c] = c < p ? a.theta[c] : 0.f;
    if (tid == 0) s_abort = 0;
    __syncthreads();

    float th[THL ? 1 : E];
    auto load_theta_regs = [&]() {
        if constexpr (!THL) {
#pragma unroll
            for (int k = 0; k < CPL; ++k) load_vec<V>(th_lds + col[k], th + k * V);
        }
    };
    load_theta_regs();

    // Batch geometry of step s.
    // Step s is mini-batch m = s mod M of pass t = s / M.  The chain is latency bound, so the quotient comes
    // from a float reciprocal plus a correction (exact for s < 2^23, which the host guarantees) instead of
    // an integer division, and the two possible group counts are computed once.
    const float rcpM = 1.0f / (float)M;
    auto split = [&](int s, int& t, int& m) {
        t = (int)((float)s * rcpM);
        m = s - t * M;
        if (m >= M) { m -= M; ++t; }
        if (m < 0) { m += M; --t; }
    };
    const int n_tail = a.rows - (M - 1) * a.n;
    const int iters_full = (a.n + S_total * PF - 1) / (S_total * PF);
    const int iters_tail = (n_tail + S_total * PF - 1) / (S_total * PF);
    auto batch_rows = [&](int s) { int t, m; split(s, t, m); return m == M - 1 ? n_tail : a.n; };
    auto batch_base = [&](int s) { int t, m; split(s, t, m); return t * a.perm_stride + m * a.n; };
    auto batch_iters = [&](int s) { int t, m; split(s, t, m); return m == M - 1 ? iters_tail : iters_full; };

    // Row indices of group (s, it) for this lane's row slot; -1 where the slot has no row.
    // The loads are unconditional (positions beyond the batch read its first entry, steps beyond the launch
    // read the first step's) so that none of them waits for another; validity travels in `okn`, bit q.
    unsigned okn = 0u;
    auto load_idx = [&](int s, int it, int (&idx)[PF]) {
        const bool live = s < last;
        const int sc = live ? s : first;
        const int nb = batch_rows(sc), base = batch_base(sc);
        okn = 0u;
#pragma unroll
        for (int q = 0; q < PF; ++q) {
            const int j = (it * PF + q) * S_total + myslot;
            const bool ok = live && j < nb;
            idx[q] = a.perm[base + (ok ? j : 0)];
            okn |= ok ? (1u << q) : 0u;
        }
    };
    auto issue_rows = [&](const int (&idx)[PF], RowGroup<V, CPL, PF>& g) {
#pragma unroll
        for (int q = 0; q < PF; ++q) {
            // Loads are unconditional (a slot without a row reads some valid row, a chunk beyond p reads chunk 0) so
            // that they can all be in flight together; what they bring is neutralised where it is used:
            // theta is 0 on chunks beyond p and the residual of a missing row is forced to 0.
            const int i = idx[q];
            const float* row = a.X + (size_t)i * p;
            g.y[q] = a.y[i];
            g.ok[q] = (okn >> q) & 1u;
#pragma unroll
            for (int k = 0; k < CPL; ++k) load_vec<V>(row + (col[k] < p ? col[k] : 0), &g.x[q][k * V]);
        }
    };
    // Group (s, 0) into `g`, and the indices of the group that follows it into `idx`.
    auto prefetch_step = [&](int s, RowGroup<V, CPL, PF>& g, int (&idx)[PF]) {
        issue_rows(idx, g);
        const bool in_step = 1 < batch_iters(min(s, last - 1));
        load_idx(in_step ? s : s + 1, in_step ? 1 : 0, idx);
    };

    constexpr bool DB = PIPE == kPipeGroups;
    constexpr bool AHEAD = PIPE == kPipeAhead;
    RowGroup<V, CPL, PF> cur, nxt;                   // nxt is not live with kPipeWide
    int idxn[PF];
    load_idx(first, 0, idxn);
    prefetch_step(first, cur, idxn);
    if constexpr (AHEAD) prefetch_step(first + 1, nxt, idxn);
    // after the exchange of step s: bring the rows a later step needs
    auto advance_rows = [&](int s) {
        if constexpr (AHEAD) {
            cur = nxt;                               // rows of step s + 1, requested a whole step ago
            prefetch_step(s + 2, nxt, idxn);
        }
    };

    PollGuard guard{a.sync + 1, a.timeout_ticks, 0, 0};

    ExchangeCtx xc{G, p, pp, tid, BLOCK, red, &s_abort, &guard};
    auto gather_columns = [&](const unsigned long long* words, int c_lo, int c_hi, unsigned tag, auto&& apply) {
        gather_columns_impl(xc, words, c_lo, c_hi, tag, apply);
    };

    for (int s = first; s < last; ++s) {
        const int nb = batch_rows(s);
        const int iters = batch_iters(s);
        const unsigned tag = a.tag_base + (unsigned)(s - first) + 1u;
        // requested here (a scalar load), used after the rows of the step have been processed
        const float alpha_s = a.lr_tab ? a.lr_tab[min(a.lr_base + s, a.lr_len - 1)] : a.alpha;
        guard.arm();
        float acc[E];
#pragma unroll
        for (int e = 0; e < E; ++e) acc[e] = 0.f;

        for (int it = 0; it < iters; ++it) {
            const bool more = it + 1 < iters;
            const bool in_step = it + 2 < iters;
            if constexpr (DB) {
                if (more) {                          // rows of the next group fly while this one is used
                    issue_rows(idxn, nxt);
                    load_idx(in_step ? s : s + 1, in_step ? it + 2 : 0, idxn);
                }
            }
#pragma unroll
            for (int q = 0; q < PF; ++q) {
                float dot = 0.f;
#pragma unroll
                for (int k = 0; k < CPL; ++k) {
                    float t[V];
                    if constexpr (THL) load_vec<V>(th_lds + col[k], t);
#pragma unroll
                    for (int v = 0; v < V; ++v)
                        dot = fmaf(cur.x[q][k * V + v], THL ? t[v] : th[(THL ? 0 : k * V + v)], dot);
                    if constexpr (THL) {             // keep theta reads from LDS from piling up in registers
                        if ((k & 3) == 3) __builtin_amdgcn_sched_barrier(0);
                    }
                }
                dot = group_sum(dot, L);
                const float r = cur.ok[q] ? residual(a.model, dot, cur.y[q]) : 0.f;
#pragma unroll
                for (int e = 0; e < E; ++e) acc[e] = fmaf(r, cur.x[q][e], acc[e]);
            }
            if (more) {
                if constexpr (DB) {
                    cur = nxt;
                } else {                             // other wavefronts cover the latency
                    issue_rows(idxn, cur);
                    load_idx(in_step ? s : s + 1, in_step ? it + 2 : 0, idxn);
                }
            }
        }

        // wavefront partial: sum the row slots, lanes < L hold it
#pragma unroll
        for (int e = 0; e < E; ++e) acc[e] = slot_sum(acc[e], L);
        if (lane < L) {
#pragma unroll
            for (int k = 0; k < CPL; ++k)
                if (col[k] < p) {
#pragma unroll
                    for (int v = 0; v < V; ++v) wpart[wave * p + col[k] + v] = acc[k * V + v];
                }
        }
        __syncthreads();

        const float scale = alpha_s / (float)nb;
        // new value of theta[c] from the batch sum t of column c; `si` is where that coordinate's optimizer state lives
        float oc1 = 1.f, oc2 = 1.f;
        if constexpr (OPT) {
            if (a.opt.kind == kOptAdam) opt_corrections(a.opt, a.opt.k_base + (s - first) + 1, oc1, oc2);
        }
        auto apply_update = [&](int c, int si, float t) -> float {
            if constexpr (!OPT) return th_lds[c] - scale * t;
            float m = a.opt.m[si], sv = a.opt.kind == kOptAdam ? a.opt.s[si] : 0.f;
            const float v = opt_update(a.opt, th_lds[c], t / (float)nb, alpha_s, m, sv, oc1, oc2);
            a.opt.m[si] = m;
            if (a.opt.kind == kOptAdam) a.opt.s[si] = sv;
            return v;
        };
        if (a.single_step >= 0) {
            // step-per-launch: plain partial sums, a second kernel reduces and updates
            float* part = a.partial + (size_t)(s & 1) * G * p;
            for (int c = tid; c < p; c += BLOCK) {
                float t = 0.f;
                for (int w = 0; w < NW; ++w) t += wpart[w * p + c];
                part[(size_t)blockIdx.x * p + c] = t;
            }
            return;
        }
        if (G == 1) {
            // single workgroup: the workgroup sum is the batch sum
            for (int c = tid; c < p; c += BLOCK) {
                float t = 0.f;
                for (int w = 0; w < NW; ++w) t += wpart[w * p + c];
                th_lds[c] = apply_update(c, c, t);
            }
            __syncthreads();
            if constexpr (AHEAD) advance_rows(s);
            else if (s + 1 < last) prefetch_step(s + 1, cur, idxn);
            load_theta_regs();
            continue;
        }

        // next step's rows do not depend on theta: in flight while the exchange resolves
        if constexpr (PIPE == kPipeGroups) {
            if (s + 1 < last) prefetch_step(s + 1, cur, idxn);
        }
        // publish this workgroup's sums as flagged words
        unsigned long long* words = a.ll_part + (size_t)(s & 1) * G * pp;
        for (int c = tid; c < p; c += BLOCK) {
            float t = 0.f;
            for (int w = 0; w < NW; ++w) t += wpart[w * p + c];
            ll_store(words + (size_t)blockIdx.x * pp + c, t, tag);
        }
        if constexpr (PIPE == kPipeWide) {           // wide rows: sums first, they are what the others wait for
            if (s + 1 < last) prefetch_step(s + 1, cur, idxn);
        }
        if (a.reduce_mode == kReduceRedundant) {
            // every workgroup applies the same update to its own copy of theta and of the optimizer's state
            gather_columns(words, 0, p, tag, [&](int c, float t) { th_lds[c] = apply_update(c, (int)blockIdx.x * pp + c, t); });
            if (s_abort) return;
        } else {
            if (sliced_update(xc, words, a.ll_theta + (size_t)(s & 1) * kThetaCopies * pp, th_lds, tag,
                              [&](int c, float t) { return apply_update(c, c, t); }))
                return;
        }
        if constexpr (AHEAD) advance_rows(s);
        load_theta_regs();
    }

    if (blockIdx.x == 0 && a.single_step < 0) {
        for (int c = tid; c < p; c += BLOCK) a.theta[c] = th_lds[c];
    }
}

// Wide rows (1024 < p <= 4096), persistent chain over several workgroups.
//
// One wavefront holds one whole row (CPL float4 chunks per lane).  A step is bound by the time HBM needs for its rows,
// and nothing can be computed between the end of a step's rows and the arrival of the new theta; what can be done in
// that window is to have the rows of the next step on their way.  So each wavefront keeps TWO rows in flight at all
// times, in two register sets used in turn over the whole sequence of row groups (s, 0), (s, 1), ..., (s + 1, 0), ...:
// a set is refilled with the group two places ahead as soon as it has been used, also across a step's end, and half
// of a four-group step is then loaded while the exchange resolves.  To make room for the second row the gradient
// sums of a wavefront live in shared memory (its own p floats: plain read-add-write, no atomics) instead of registers.
// The barrier after a step's last rows waits for shared memory only: rows in flight do not hold it up.
// (The polls of the exchange still return behind the wavefront's older row loads - loads complete in order -, so
// the exchange ends no earlier than those rows land; that time is spent loading either way.)
constexpr int kWideBlock = 512;

__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <int CPL, bool OPT>
__global__ void __launch_bounds__(kWideBlock) glm_wide_kernel(GlmArgs a)
{
    extern __shared__ __align__(16) float smem[];
    __shared__ int s_abort;

    constexpr int BLOCK = kWideBlock;
    constexpr int NW = BLOCK / 64;
    constexpr int E = CPL * 4;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int G = gridDim.x;
    const int p = a.p;
    const int S_total = G * NW;                      // rows per group
    const int myslot = blockIdx.x * NW + wave;
    const int pp = (p + 15) & ~15;
    const int th_len = max((p + 63) & ~63, 256 * CPL);
    float* th_lds = smem;                            // [th_len]
    float* wpart = smem + th_len;                    // [NW][p] per-wavefront sums
    float* red = wpart + NW * p;                     // [BLOCK] scratch of the cross-workgroup sum
    float* wacc = wpart + wave * p;
    const int M = (a.rows + a.n - 1) / a.n;
    const int first = a.s_begin, last = a.s_end;

    for (int c = tid; c < th_len; c += BLOCK) th_lds[c] = c < p ? a.theta[c] : 0.f;
    if (tid == 0) s_abort = 0;
    __syncthreads();

    const float rcpM = 1.0f / (float)M;
    auto split = [&](int s, int& t, int& m) {        // s = t M + m, exact for s < 2^23
        t = (int)((float)s * rcpM);
        m = s - t * M;
        if (m >= M) { m -= M; ++t; }
        if (m < 0) { m += M; --t; }
    };
    const int n_tail = a.rows - (M - 1) * a.n;
    const int iters_full = (a.n + S_total - 1) / S_total;
    const int iters_tail = (n_tail + S_total - 1) / S_total;
    auto batch_rows = [&](int s) { int t, m; split(s, t, m); return m == M - 1 ? n_tail : a.n; };
    auto batch_base = [&](int s) { int t, m; split(s, t, m); return t * a.perm_stride + m * a.n; };
    auto batch_iters = [&](int s) { int t, m; split(s, t, m); return m == M - 1 ? iters_tail : iters_full; };

    struct Row {
        float x[E];
        float y;
        bool ok;
        int idx_next;                                // row this set takes at its next request, and whether that
        bool ok_next;                                // group has a row for this wavefront at all
    };
    Row A, B;

    // Each set carries the index of the row it will request next, loaded right after its previous request: by the
    // time it is needed it is older than the other set's rows in flight, so waiting for it waits for none of them
    // (loads complete in order).  Groups beyond the launch read the first step's rows and count as empty.
    int sq = first, iq = 0;                          // the group whose index is loaded next
    auto load_idx = [&](Row& r) {
        const bool live = sq < last;
        const int sc = live ? sq : first;
        const int j = iq * S_total + myslot;
        r.ok_next = live && j < batch_rows(sc);
        r.idx_next = a.perm[batch_base(sc) + (r.ok_next ? j : 0)];
        if (live) {
            if (iq + 1 < batch_iters(sq)) ++iq;
            else { ++sq; iq = 0; }
        }
    };
    // Request the rows of the set's next group (row `idx`: the set's idx_next, read into a scalar by the caller at
    // a point where waiting for it costs nothing), then the index for the request after that.
    auto request = [&](Row& r, int idx) {
        const float* row = a.X + (size_t)idx * p;
        r.y = a.y[idx];
        r.ok = r.ok_next;
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
            const int c = 4 * (lane + 64 * k);
            const float4 t = *reinterpret_cast<const float4*>(row + (c < p ? c : 0));   // chunks beyond p: theta is 0 there
            r.x[4 * k] = t.x; r.x[4 * k + 1] = t.y; r.x[4 * k + 2] = t.z; r.x[4 * k + 3] = t.w;
        }
        load_idx(r);
    };
    load_idx(A);
    load_idx(B);
    asm volatile("" ::: "memory");                   // A's rows are the older ones, as in every later round
    request(A, __builtin_amdgcn_readfirstlane(A.idx_next));
    asm volatile("" ::: "memory");
    request(B, __builtin_amdgcn_readfirstlane(B.idx_next));
    asm volatile("" ::: "memory");

    PollGuard guard{a.sync + 1, a.timeout_ticks, 0, 0};
    ExchangeCtx xc{G, p, pp, tid, BLOCK, red, &s_abort, &guard};

    int su = first, iu = 0;                          // the group that is used next
    int iters_u = batch_iters(min(su, last - 1));
    // learning rate of step su: requested when the step begins, so that it is older than the step's rows and
    // waiting for it at the step's end waits for none of them
    auto rate_of = [&](int s) { return a.lr_tab ? a.lr_tab[min(a.lr_base + min(s, last - 1), a.lr_len - 1)] : a.alpha; };
    float alpha_s = first < last ? rate_of(first) : a.alpha;

    // Use the rows in `r` (group (su, iu)), refill `r`, and end the step if that was its last group.
    // Returns true when the launch is over (all steps done, or a wait ran out).
    auto process = [&](Row& r) -> bool {
        float dot = 0.f;
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
            const float4 t = *reinterpret_cast<const float4*>(th_lds + 4 * (lane + 64 * k));
            dot = fmaf(r.x[4 * k], t.x, dot);
            dot = fmaf(r.x[4 * k + 1], t.y, dot);
            dot = fmaf(r.x[4 * k + 2], t.z, dot);
            dot = fmaf(r.x[4 * k + 3], t.w, dot);
        }
        dot = group_sum(dot, 64);
        const float res = r.ok ? residual(a.model, dot, r.y) : 0.f;
        // the set's next row: its index arrived right behind the rows just used (the same for all lanes)
        const int idx_s = __builtin_amdgcn_readfirstlane(r.idx_next);
        if (iu == 0) {
#pragma unroll
            for (int k = 0; k < CPL; ++k) {
                const int c = 4 * (lane + 64 * k);
                if (c < p)
                    *reinterpret_cast<float4*>(wacc + c) =
                        make_float4(res * r.x[4 * k], res * r.x[4 * k + 1], res * r.x[4 * k + 2], res * r.x[4 * k + 3]);
            }
        } else {
#pragma unroll
            for (int k = 0; k < CPL; ++k) {
                const int c = 4 * (lane + 64 * k);
                if (c < p) {
                    float4 t = *reinterpret_cast<float4*>(wacc + c);
                    t.x = fmaf(res, r.x[4 * k], t.x);
                    t.y = fmaf(res, r.x[4 * k + 1], t.y);
                    t.z = fmaf(res, r.x[4 * k + 2], t.z);
                    t.w = fmaf(res, r.x[4 * k + 3], t.w);
                    *reinterpret_cast<float4*>(wacc + c) = t;
                }
            }
        }
        const bool step_ends = iu + 1 >= iters_u;
        const int s = su;
        const unsigned tag = a.tag_base + (unsigned)(s - first) + 1u;
        unsigned long long* words = a.ll_part + (size_t)(s & 1) * G * pp;
        if (step_ends) {
            guard.arm();
            lds_barrier();
            // publish this workgroup's sums as flagged words: they are what the others wait for
            for (int c = tid; c < p; c += BLOCK) {
                float t = 0.f;
                for (int w = 0; w < NW; ++w) t += wpart[w * p + c];
                ll_store(words + (size_t)blockIdx.x * pp + c, t, tag);
            }
        }
        // The refill: one place in the code for both cases, so that what it loads has one home in registers (two
        // would be reconciled by copies, and a copy of a value in flight waits for everything in flight).  It stays
        // behind the last use of the set's registers and behind the publication of the sums.
        asm volatile("" ::: "memory");
        request(r, idx_s);
        asm volatile("" ::: "memory");
        if (!step_ends) {
            ++iu;
            return false;
        }

        // ---- the rest of the end of step su
        const int nb = batch_rows(s);
        const float scale = alpha_s / (float)nb;
        float oc1 = 1.f, oc2 = 1.f;
        if constexpr (OPT) {
            if (a.opt.kind == kOptAdam) opt_corrections(a.opt, a.opt.k_base + (s - first) + 1, oc1, oc2);
        }
        auto apply_update = [&](int c, int si, float t) -> float {
            if constexpr (!OPT) return th_lds[c] - scale * t;
            float m = a.opt.m[si], sv = a.opt.kind == kOptAdam ? a.opt.s[si] : 0.f;
            const float v = opt_update(a.opt, th_lds[c], t / (float)nb, alpha_s, m, sv, oc1, oc2);
            a.opt.m[si] = m;
            if (a.opt.kind == kOptAdam) a.opt.s[si] = sv;
            return v;
        };
        if (a.reduce_mode == kReduceRedundant) {
            gather_columns_impl<8>(xc, words, 0, p, tag,
                                   [&](int c, float t) { th_lds[c] = apply_update(c, (int)blockIdx.x * pp + c, t); });
            if (s_abort) return true;
        } else {
            if (sliced_update<8>(xc, words, a.ll_theta + (size_t)(s & 1) * kThetaCopies * pp, th_lds, tag,
                              [&](int c, float t) { return apply_update(c, c, t); }))
                return true;
        }
        // Everything this wavefront had in flight has landed (the polls waited for it); said in a form the compiler
        // sees, so that the waits it plans for the next rows start from a clean slate.
        __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0) only
        ++su;
        iu = 0;
        iters_u = batch_iters(min(su, last - 1));
        alpha_s = rate_of(su);
        return su >= last;
    };

    if (first < last) {
        // (not peeled or unrolled: every round of the loop then finds the two sets in the same order of age)
#pragma clang loop unroll(disable)
        for (;;) {
            if (process(A)) break;
            if (process(B)) break;
        }
    }
    // rows requested beyond the last step land in registers that die with the wavefront
    if (blockIdx.x == 0 && !s_abort) {
        for (int c = tid; c < p; c += BLOCK) a.theta[c] = th_lds[c];
    }
}

// Step-per-launch companion: one thread per column sums the workgroups' partial sums and applies the update
// (opt.k_base = updates made before this one).
__global__ void __launch_bounds__(256) glm_update_kernel(float* __restrict__ theta, const float* __restrict__ part,
                                                         int p, int G, float alpha, float inv_nb, OptArgs opt)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= p) return;
    float t = 0.f;
    for (int g = 0; g < G; ++g) t += part[(size_t)g * p + c];
    if (opt.kind == kOptSgd) {
        theta[c] -= alpha * inv_nb * t;
        return;
    }
    float c1 = 1.f, c2 = 1.f;
    if (opt.kind == kOptAdam) opt_corrections(opt, opt.k_base + 1, c1, c2);
    float m = opt.m[c], sv = opt.kind == kOptAdam ? opt.s[c] : 0.f;
    theta[c] = opt_update(opt, theta[c], t * inv_nb, alpha, m, sv, c1, c2);
    opt.m[c] = m;
    if (opt.kind == kOptAdam) opt.s[c] = sv;
}

// Evaluation: sum over rows of the per-sample loss at theta (least squares: (x'theta - y)^2 / 2; logistic:
// log(1 + e^u) - y u with u = x'theta), one row per wavefront at a time, fp64 sums, one partial sum per workgroup
// (the host adds them in index order: reproducible).
constexpr int kLossBlock = 256;

__global__ void __launch_bounds__(kLossBlock) glm_loss_kernel(const float* __restrict__ X, const float* __restrict__ y,
                                                              const float* __restrict__ theta, int rows, int p, int model,
                                                              double* __restrict__ partial)
{
    extern __shared__ __align__(16) float th[];      // [p]
    __shared__ double wsum[kLossBlock / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int c = threadIdx.x; c < p; c += kLossBlock) th[c] = theta[c];
    __syncthreads();
    double acc = 0.0;
    for (int i = blockIdx.x * (kLossBlock / 64) + wave; i < rows; i += gridDim.x * (kLossBlock / 64)) {
        const float* row = X + (size_t)i * p;
        float d = 0.f;
        for (int c = lane; c < p; c += 64) d = fmaf(row[c], th[c], d);
        const float u = group_sum(d, 64);
        const float yi = y[i];
        float l;
        if (model == kLogistic) l = fmaxf(u, 0.f) + log1pf(expf(-fabsf(u))) - yi * u;
        else l = 0.5f * (u - yi) * (u - yi);
        acc += (double)l;
    }
    if (lane == 0) wsum[wave] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int w = 0; w < kLossBlock / 64; ++w) t += wsum[w];
        partial[blockIdx.x] = t;
    }
}

using KernelFn = void (*)(GlmArgs);

// Rows in flight per row slot are limited by registers: CPL * V * PF <= 16 floats per group (two groups
// are live except with kPipeWide), at most 4 rows per group; wide rows (CPL >= 8) hold one row.
constexpr bool shape_ok(int v, int cpl, int pf, int pipe)
{
    const int e = v * cpl;
    if (cpl >= 8) return pf == 1 && pipe == kPipeWide;
    if (pipe == kPipeWide) return false;
    return e * pf <= 16 && pf <= 4;
}

int max_pf(int v, int cpl)
{
    int pf = 1;
    while (pf < 4 && shape_ok(v, cpl, pf * 2, kPipeGroups)) pf *= 2;
    return pf;
}

template <bool OPT, int V, int CPL, int PF, int PIPE>
KernelFn pick()
{
    if constexpr (!shape_ok(V, CPL, PF, PIPE)) {
        return nullptr;
    } else {
        constexpr bool wide = CPL >= 8;
        return glm_chain_kernel<V, CPL, PF, wide, PIPE, wide ? 512 : 1024, OPT>;
    }
}

template <bool OPT, int V, int CPL, int PF>
KernelFn pick_pipe(int pipe)
{
    switch (pipe) {
    case kPipeWide: return pick<OPT, V, CPL, PF, kPipeWide>();
    case kPipeGroups: return pick<OPT, V, CPL, PF, kPipeGroups>();
    case kPipeAhead: return pick<OPT, V, CPL, PF, kPipeAhead>();
    }
    return nullptr;
}

template <bool OPT, int V, int CPL>
KernelFn pick_pf(int pf, int pipe)
{
    switch (pf) {
    case 1: return pick_pipe<OPT, V, CPL, 1>(pipe);
    case 2: return pick_pipe<OPT, V, CPL, 2>(pipe);
    case 4: return pick_pipe<OPT, V, CPL, 4>(pipe);
    }
    return nullptr;
}

template <bool OPT, int V>
KernelFn pick_v(int cpl, int pf, int pipe)
{
    switch (cpl) {
    case 1: return pick_pf<OPT, V, 1>(pf, pipe);
    case 2: return pick_pf<OPT, V, 2>(pf, pipe);
    case 4: return pick_pf<OPT, V, 4>(pf, pipe);
    case 8: return pick_pf<OPT, V, 8>(pf, pipe);
    case 16: return pick_pf<OPT, V, 16>(pf, pipe);
    }
    return nullptr;
}

template <bool OPT>
KernelFn pick_kernel_opt(const GlmLaunchShape& s)
{
    switch (s.V) {
    case 1: return pick_v<OPT, 1>(s.CPL, s.PF, s.pipe);
    case 2: return pick_v<OPT, 2>(s.CPL, s.PF, s.pipe);
    case 4: return pick_v<OPT, 4>(s.CPL, s.PF, s.pipe);
    }
    return nullptr;
}

KernelFn pick_kernel(const GlmLaunchShape& s)
{
    return s.with_optimizer ? pick_kernel_opt<true>(s) : pick_kernel_opt<false>(s);
}


}  // namespace

bool glm_plan(int64_t p, int64_t n, int requested_G, int num_cus, GlmLaunchShape* out, char* why, size_t why_len)
{
    GlmLaunchShape s{};
    s.V = (p % 4 == 0) ? 4 : (p % 2 == 0) ? 2 : 1;
    const int64_t chunks = p / s.V;
    if (chunks <= 64) {
        s.L = 1;
        while (s.L < chunks) s.L *= 2;
        s.CPL = 1;
    } else {
        s.L = 64;
        const int64_t need = (chunks + 63) / 64;
        s.CPL = 1;
        while (s.CPL < need) s.CPL *= 2;
        if (s.CPL > 16) {
            snprintf(why, why_len, "p = %lld is above the supported maximum (%d for this alignment of p)",
                     (long long)p, 64 * 16 * s.V);
            return false;
        }
    }
    s.block = s.CPL >= 8 ? 512 : 1024;
    const int slots_per_group = (s.block / 64) * (64 / s.L);
    int G = requested_G;
    if (G <= 0) {
        // measured on MI355X: a compute unit sustains ~19 GB/s of gathered rows, one exchange costs 1.5-3 us;
        // about 12 KB of rows per workgroup and step balances the two
        const int64_t bytes = n * p * 4;
        G = (int)std::min<int64_t>((bytes + 12287) / 12288, 1 << 20);
    }
    if (G < 1) G = 1;
    if (G > num_cus) G = num_cus;
    s.G = G;
    // Rows each row slot must take per step.  If one register-resident group covers it, the whole next
    // batch is prefetched across the exchange (no look-ahead needed); otherwise iterate with look-ahead.
    const int64_t need = (n + (int64_t)G * slots_per_group - 1) / ((int64_t)G * slots_per_group);
    if (s.CPL >= 8) {
        s.PF = 1; s.pipe = kPipeWide;
    } else if (need <= max_pf(s.V, s.CPL)) {
        s.PF = 1; s.pipe = kPipeAhead;
        while (s.PF < need) s.PF *= 2;
    } else {
        s.PF = max_pf(s.V, s.CPL); s.pipe = kPipeGroups;
    }
    s.reduce_mode = ((int64_t)G * p <= 4096) ? kReduceRedundant : kReduceSliced;
    const int64_t th_len = std::max<int64_t>((p + 63) & ~int64_t(63), (int64_t)s.V * s.L * s.CPL);
    s.lds_bytes = (size_t)(th_len + (int64_t)(s.block / 64) * p + s.block + 64) * sizeof(float);
    *out = s;
    return true;
}

// The kernel of the persistent chain: wide rows over several workgroups have one of their own.
static KernelFn pick_chain_kernel(const GlmLaunchShape& s)
{
    if (s.pipe == kPipeWide && s.G > 1 && s.V == 4 && s.L == 64 && s.block == kWideBlock) {
        if (s.CPL == 8) return s.with_optimizer ? glm_wide_kernel<8, true> : glm_wide_kernel<8, false>;
        if (s.CPL == 16) return s.with_optimizer ? glm_wide_kernel<16, true> : glm_wide_kernel<16, false>;
    }
    return pick_kernel(s);
}

hipError_t glm_prepare(GlmLaunchShape* s)
{
    KernelFn fn = pick_kernel(*s);
    if (!fn) return hipErrorInvalidValue;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)s->lds_bytes);
    if (e != hipSuccess) return e;
    int per_cu = 0;
    e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(fn), s->block,
                                                     s->lds_bytes);
    if (e != hipSuccess) return e;
    int dev = 0;
    hipDeviceProp_t prop;
    if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
    if ((e = hipGetDeviceProperties(&prop, dev)) != hipSuccess) return e;
    s->max_G = per_cu * prop.multiProcessorCount;
    if (s->max_G < 1) return hipErrorLaunchOutOfResources;
    // one workgroup per compute unit at most: the barrier cost grows with the number of arrivals
    if (s->G > prop.multiProcessorCount) s->G = prop.multiProcessorCount;
    if (s->G > s->max_G) s->G = s->max_G;
    // the persistent chain may run another kernel for this shape: same shared memory, same residency test
    KernelFn chain = pick_chain_kernel(*s);
    if (chain != fn) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(chain), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)s->lds_bytes);
        if (e != hipSuccess) return e;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(chain), s->block, s->lds_bytes);
        if (e != hipSuccess) return e;
        if (per_cu < 1) return hipErrorLaunchOutOfResources;
        s->max_G = std::min(s->max_G, per_cu * prop.multiProcessorCount);
        if (s->G > s->max_G) s->G = s->max_G;
    }
    return hipSuccess;
}

hipError_t glm_launch_chain(const GlmLaunchShape& s, const GlmArgs& args, hipStream_t stream)
{
    KernelFn fn = pick_chain_kernel(s);
    if (!fn || s.G < 1 || s.G > s.max_G) return hipErrorInvalidValue;
    GlmArgs a = args;
    a.single_step = -1;
    // An ordinary launch: s.G <= s.max_G (checked above) means every workgroup fits on the device at once,
    // so all of them become resident as soon as compute units are free, and each device-side wait is
    // bounded anyway.  (The runtime's cooperative-launch path is avoided: it brings nothing more here and
    // its dedicated queue does not tear down cleanly under the profiler.)
    hipLaunchKernelGGL(fn, dim3(s.G), dim3(s.block), s.lds_bytes, stream, a);
    return hipGetLastError();
}

hipError_t glm_launch_step(const GlmLaunchShape& s, const GlmArgs& args, int nb, hipStream_t stream)
{
    KernelFn fn = pick_kernel(s);
    if (!fn || s.G < 1 || args.single_step < 0) return hipErrorInvalidValue;
    hipLaunchKernelGGL(fn, dim3(s.G), dim3(s.block), s.lds_bytes, stream, args);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const float* part = args.partial + (size_t)(args.single_step & 1) * s.G * args.p;
    hipLaunchKernelGGL(glm_update_kernel, dim3((args.p + 255) / 256), dim3(256), 0, stream, args.theta, part,
                       args.p, s.G, args.alpha, 1.f / (float)nb, args.opt);
    return hipGetLastError();
}

hipError_t glm_launch_loss(const float* X, const float* y, const float* theta, int rows, int p, int model, double* partial,
                           int nblocks, hipStream_t stream)
{
    hipLaunchKernelGGL(glm_loss_kernel, dim3(nblocks), dim3(kLossBlock), (size_t)p * sizeof(float), stream, X, y, theta, rows, p,
                       model, partial);
    return hipGetLastError();
}

}  // namespace bmgd
