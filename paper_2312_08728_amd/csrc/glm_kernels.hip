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
#include "glm_device.h"

#include <stdio.h>

#include <algorithm>

namespace bmgd {

namespace {

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
    // (in 64 bits: up to four partitions of up to 2^30 rows lie behind one another)
    auto batch_base = [&](int s) { int t, m; split(s, t, m); return (size_t)t * (size_t)a.perm_stride + (size_t)m * (size_t)a.n; };
    auto batch_iters = [&](int s) { int t, m; split(s, t, m); return m == M - 1 ? iters_tail : iters_full; };

    // Row indices of group (s, it) for this lane's row slot; -1 where the slot has no row.
    // The loads are unconditional (positions beyond the batch read its first entry, steps beyond the launch
    // read the first step's) so that none of them waits for another; validity travels in `okn`, bit q.
    unsigned okn = 0u;
    auto load_idx = [&](int s, int it, int (&idx)[PF]) {
        const bool live = s < last;
        const int sc = live ? s : first;
        const int nb = batch_rows(sc);
        const size_t base = batch_base(sc);
        okn = 0u;
#pragma unroll
        for (int q = 0; q < PF; ++q) {
            const int j = (it * PF + q) * S_total + myslot;
            const bool ok = live && j < nb;
            idx[q] = a.perm[base + (size_t)(ok ? j : 0)];
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
    // kPipeAhead: ga holds the rows of even steps (counted from `first`), gb those of odd steps.  Otherwise ga is
    // the group in use and gb the look-ahead of kPipeGroups (not live with kPipeWide).
    RowGroup<V, CPL, PF> ga, gb;
    int idxn[PF];
    load_idx(first, 0, idxn);
    prefetch_step(first, ga, idxn);
    if constexpr (AHEAD) prefetch_step(first + 1, gb, idxn);

    PollGuard guard{a.sync + 1, a.timeout_ticks, 0, 0};

    ExchangeCtx xc{G, p, pp, tid, BLOCK, red, &s_abort, &guard};
    auto gather_columns = [&](const unsigned long long* words, int c_lo, int c_hi, unsigned tag, auto&& apply) {
        gather_columns_impl(xc, words, c_lo, c_hi, tag, apply);
    };

    // Step s of the launch on the rows held in `cur`; false when the launch ends with it (a wait ran out, or the
    // step-per-launch form has written its sums).  With kPipeAhead `cur` is refilled, once theta is known, with the
    // rows of step s + 2: the caller alternates two groups, so that rows in flight are never copied from one set
    // of registers to another (a copy would have to wait for them).
    auto run_step = [&](int s, RowGroup<V, CPL, PF>& cur, RowGroup<V, CPL, PF>& nxt) __attribute__((always_inline)) -> bool {
        (void)nxt;
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
            return false;
        }
        if (G == 1) {
            // single workgroup: the workgroup sum is the batch sum
            for (int c = tid; c < p; c += BLOCK) {
                float t = 0.f;
                for (int w = 0; w < NW; ++w) t += wpart[w * p + c];
                th_lds[c] = apply_update(c, c, t);
            }
            __syncthreads();
            if constexpr (AHEAD) prefetch_step(s + 2, cur, idxn);
            else if (s + 1 < last) prefetch_step(s + 1, cur, idxn);
            load_theta_regs();
            return true;
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
            if (s_abort) return false;
        } else {
            if (sliced_update(xc, words, a.ll_theta + (size_t)(s & 1) * kThetaCopies * pp, th_lds, tag,
                              [&](int c, float t) { return apply_update(c, c, t); }))
                return false;
        }
        if constexpr (AHEAD) prefetch_step(s + 2, cur, idxn);
        load_theta_regs();
        return true;
    };

    if constexpr (AHEAD) {
        int s = first;
        for (; s + 1 < last; s += 2) {
            if (!run_step(s, ga, gb)) return;
            if (!run_step(s + 1, gb, ga)) return;
        }
        if (s < last && !run_step(s, ga, gb)) return;
    } else {
        for (int s = first; s < last; ++s)
            if (!run_step(s, ga, gb)) return;
    }

    if (blockIdx.x == 0 && a.single_step < 0) {
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
    // narrow rows on eight or more workgroups, a step's rows fitting the registers: the kernel with an exchange wavefront
    // (not where the sums of all workgroups are few enough for every workgroup to add them up itself: one trip
    // over the fabric per step instead of two)
    if (s.CPL < 8 && s.V >= 2 && G >= 8 && (int64_t)G * p > 4096) {
        const int pf = glm_narrow_rows_in_flight(s.V, s.CPL, s.L, G & ~7, n);
        if (pf > 0) {
            s.narrow = 1;
            s.narrow_pf = pf;
            G &= ~7;
        }
    }
    s.G = G;
    s.n = n;
    s.p = (int)p;
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
    s.chain_block = s.narrow ? glm_narrow_block() : s.block;
    if (s.CPL >= 8 && s.V == 4 && G >= 8) {
        // wide rows on eight or more workgroups: the kernel with an exchange wavefront and a two-level exchange
        s.split = 1;
        s.split_ch = s.CPL == 8 ? 1 : 2;
        s.G = G & ~7;
        s.chain_block = glm_split_block();
    }
    s.reduce_mode = ((int64_t)G * p <= 4096) ? kReduceRedundant : kReduceSliced;
    const int64_t th_len = std::max<int64_t>((p + 63) & ~int64_t(63), (int64_t)s.V * s.L * s.CPL);
    s.lds_bytes = (size_t)(th_len + (int64_t)(s.block / 64) * p + s.block + 64) * sizeof(float);
    *out = s;
    return true;
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
    if (s->split) {
        int cap = 0;
        e = glm_split_prepare(s->split_ch, s->with_optimizer != 0, &cap);
        if (e != hipSuccess) return e;
        cap = std::min(cap, prop.multiProcessorCount) & ~7;
        if (cap >= 8) {
            s->max_G = std::min(s->max_G, cap);
            s->G = std::min(s->G, cap) & ~7;
            return hipSuccess;
        }
        s->split = 0;                                // not even eight fit: the kernel below takes over
        s->chain_block = s->block;
    }
    if (s->narrow) {
        int cap = 0;
        e = glm_narrow_prepare(*s, s->p, &cap);
        if (e != hipSuccess) return e;
        cap = std::min(cap, prop.multiProcessorCount) & ~7;
        const int G = std::min(s->G, cap) & ~7;
        // fewer workgroups than planned hold fewer rows: only if the step still fits
        if (G >= 8 && glm_narrow_rows_in_flight(s->V, s->CPL, s->L, G, s->n) == s->narrow_pf) {
            s->max_G = std::min(s->max_G, cap);
            s->G = G;
        } else {
            s->narrow = 0;
            s->chain_block = s->block;
        }
    }
    return hipSuccess;
}

hipError_t glm_launch_chain(const GlmLaunchShape& s, const GlmArgs& args, hipStream_t stream)
{
    if (s.split) {
        if (s.G < 8 || s.G > s.max_G) return hipErrorInvalidValue;
        GlmArgs a = args;
        a.single_step = -1;
        return glm_split_launch(s.split_ch, s.with_optimizer != 0, s.G, a, stream);
    }
    if (s.narrow) {
        if (s.G > s.max_G) return hipErrorInvalidValue;
        GlmArgs a = args;
        a.single_step = -1;
        return glm_narrow_launch(s, a, stream);
    }
    KernelFn fn = pick_kernel(s);
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
