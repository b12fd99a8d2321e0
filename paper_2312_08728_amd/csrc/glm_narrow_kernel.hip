// Fused mini-batch gradient + update for rows of up to 1024 floats (least squares, logistic) when the rows a
// workgroup takes per step fit its registers; persistent over all steps of up to four passes, on G workgroups
// (G a multiple of 8, one per compute unit).
//
// A step of eq. (2.1) on such rows moves little data (a few KB per workgroup), so the chain of steps is bound by the
// exchange of the gradient sums between the workgroups, and the kernel's job is to put nothing else on that path:
//
//   * A row is held by L cooperating lanes of a row wavefront (L a power of two, 64 / L rows side by side, PF rows
//     one after the other per lane; lane l owns the columns V (l + L k) .. + V - 1, k < CPL).  Eight row wavefronts
//     per workgroup.
//   * Each row wavefront holds TWO groups of rows in registers and alternates between them: the group used in step
//     s is refilled, as soon as it has been used, with the rows of step s + 2 (rows do not depend on theta).  Rows
//     therefore have a whole step to arrive and are never copied between registers while in flight.  The loop over
//     steps is straight-line code (two steps per trip, one exit at the bottom, steps past the end run empty), so
//     that the compiler's count of loads in flight is exact and a step waits only for its own rows.
//   * The row wavefronts never touch global memory except for rows: their sums go to shared memory, and four
//     exchange wavefronts (glm_exchange.h), one per SIMD, carry them to the other workgroups and bring the new theta
//     back, two trips over the fabric per step.  Row wavefronts wait for theta on a flag in shared memory.
#include "glm_exchange.h"

#include <algorithm>

namespace bmgd {

namespace {

// Registers: two groups of PF rows of CPL * V floats per lane.  Loads: a group is PF * (CPL + 2) of them (chunks,
// response, next index), and the two groups' loads together must stay below the 63 that a wavefront's count of
// loads in flight can hold.
constexpr bool narrow_shape_ok(int v, int cpl, int pf)
{
    return v >= 2 && cpl <= 4 && pf <= 8 && v * cpl * pf <= 32 && pf * (cpl + 2) <= 24;
}

// Wavefronts 0 .. 3 are the exchange wavefronts (the hardware deals the wavefronts of a workgroup out to the four
// SIMDs in turn, so each SIMD gets one), wavefronts 4 .. 11 the row wavefronts.
constexpr int kXWaves = 4;
constexpr int kNarrowBlock = 64 * (kXWaves + kRowWaves);

template <int V, int CPL, int PF, bool OPT>
__global__ void __launch_bounds__(kNarrowBlock) glm_narrow_kernel(GlmArgs a)
{
    extern __shared__ __align__(16) float smem[];
    __shared__ int s_abort;                          // set by the exchange wavefront when a wait ran out
    __shared__ unsigned s_theta_version;             // versions of theta delivered to shared memory so far
    __shared__ unsigned s_published;                 // publications of row wavefronts, counted over all steps
    __shared__ unsigned s_xarrived[kXWaves], s_xconsumed;   // hand-over of partial sums between the exchange wavefronts

    constexpr int E = CPL * V;                       // floats of a row held per lane
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int G = gridDim.x;
    const int g = blockIdx.x;
    const int p = a.p;
    const int L = a.L;
    const int stride = max((p + 15) & ~15, V * L * CPL);          // of theta and of the sums in shared memory
    lds_f32* th = (lds_f32*)smem;                    // [2][stride]: theta, by version parity
    lds_f32* sums = th + 2 * stride;                 // [kRowWaves][stride]: each row wavefront's gradient sums of a step
    lds_f32* red = sums + kRowWaves * stride;        // scratch of the exchange wavefronts
    const int first = a.s_begin, last = a.s_end;

    // theta (version 0 in copy 0) and the sums; columns beyond p stay zero for good (rows are read at column 0 there)
    for (int c = tid; c < (2 + kRowWaves) * stride; c += kNarrowBlock) th[c] = c < p ? a.theta[c] : 0.f;
    if (tid == 0) { s_abort = 0; s_theta_version = 0u; s_published = 0u; s_xconsumed = 0u; }
    if (tid < kXWaves) s_xarrived[tid] = 0u;
    __syncthreads();                                 // the only barrier: from here on the wavefronts meet through flags

    const int rw = wave - kXWaves;
    if (rw >= 0) {
        // ------------------------------------------------------------------------------------ row wavefronts
        const StepGeometry geo(a);
        const int lsub = lane & (L - 1);
        const int slot = lane >> a.logL;
        const int rpw = 64 >> a.logL;                // rows side by side in a wavefront
        const int S_total = G * kRowWaves * rpw;     // row slots of the grid: row j of a mini-batch goes to slot j mod S_total
        const int myslot = (g * kRowWaves + rw) * rpw + slot;
        int col[CPL];
#pragma unroll
        for (int k = 0; k < CPL; ++k) col[k] = V * (lsub + L * k);

        // A group: the rows of one step.  Besides the rows it carries their responses and the indices of the rows
        // that take their place at the group's next request; both are loaded right behind the rows, so they have
        // arrived when the rows have (loads return in order) and waiting for them waits for nothing else.
        struct Group {
            float x[PF][E];
            float y[PF];
            int idx_next[PF];
            unsigned ok, ok_next;                    // bit q: row q exists
            int sq;                                  // the step whose row indices are loaded next
        };
        auto load_idx = [&](Group& S) {
            const bool live = S.sq < last;
            const int sc = live ? S.sq : first;      // beyond the end: the first step's rows again (valid addresses, not used)
            const int nb = geo.batch_rows(sc);
            const size_t base = geo.batch_base(sc);
            S.ok_next = 0u;
#pragma unroll
            for (int q = 0; q < PF; ++q) {
                const int j = q * S_total + myslot;
                const bool ok = live && j < nb;
                S.idx_next[q] = a.perm[base + (size_t)(ok ? j : 0)];
                S.ok_next |= ok ? (1u << q) : 0u;
            }
            S.sq += 2;
        };
        auto request = [&](Group& S) {
#pragma unroll
            for (int q = 0; q < PF; ++q) {
                const float* row = a.X + (size_t)S.idx_next[q] * (size_t)p;
#pragma unroll
                for (int k = 0; k < CPL; ++k) load_vec<V>(row + (col[k] < p ? col[k] : 0), &S.x[q][k * V]);   // beyond p: theta is 0 there
            }
#pragma unroll
            for (int q = 0; q < PF; ++q) S.y[q] = a.y[S.idx_next[q]];
            S.ok = S.ok_next;
            load_idx(S);
        };
        auto keep = [&](const Group& S) {
#pragma unroll
            for (int q = 0; q < PF; ++q) {
#pragma unroll
                for (int e = 0; e < E; ++e) asm volatile("" :: "v"(S.x[q][e]));
                asm volatile("" :: "v"(S.y[q]), "v"(S.idx_next[q]));
            }
        };
        Group A, B;
        A.sq = first; B.sq = first + 1;
        load_idx(A); load_idx(B);
        request(A); request(B);

        const unsigned abort_addr = (unsigned)(uintptr_t)(lds_u32*)&s_abort;
        const unsigned version_addr = (unsigned)(uintptr_t)(lds_u32*)&s_theta_version;
        lds_f32* my_sums = sums + rw * stride;
        // Step s on the rows in S, then S is refilled.  Straight-line code with one conditional (the publication).  A
        // step past the end uses rows requested beyond the end, publishes nothing and waits for the last version only.
        auto process = [&](Group& S, int s) {
            const bool live = s < last;
            const unsigned want = (unsigned)(min(s, last) - first);
            lds_wait_ge(version_addr, want * kXWaves, abort_addr);   // (every exchange wavefront raises it once per version)
            const lds_f32* src = th + (want & 1u) * stride;
            float thr[E], acc[E];
#pragma unroll
            for (int k = 0; k < CPL; ++k) {
#pragma unroll
                for (int v = 0; v < V; ++v) thr[k * V + v] = src[col[k] + v];
            }
#pragma unroll
            for (int e = 0; e < E; ++e) acc[e] = 0.f;
#pragma unroll
            for (int q = 0; q < PF; ++q) {
                float dot = 0.f;
#pragma unroll
                for (int e = 0; e < E; ++e) dot = fmaf(S.x[q][e], thr[e], dot);
                dot = group_sum_flat(dot, L);
                const float r = ((S.ok >> q) & 1u) != 0u ? residual(a.model, dot, S.y[q]) : 0.f;
#pragma unroll
                for (int e = 0; e < E; ++e) acc[e] = fmaf(r, S.x[q][e], acc[e]);
            }
            if (L < 64) {                            // (no loads inside: the branch does not disturb their count)
#pragma unroll
                for (int e = 0; e < E; ++e) acc[e] = slot_sum_flat(acc[e], L);
            }                                        // lanes < L: the wavefront's sums
            if (live) {
                if (lane < L) {
#pragma unroll
                    for (int k = 0; k < CPL; ++k)
                        if (col[k] < p) {
#pragma unroll
                            for (int v = 0; v < V; ++v) my_sums[col[k] + v] = acc[k * V + v];
                        }
                }
                // (shared memory serves a wavefront's requests in order: the count is raised after the sums are in place;
                // a release here would wait for the rows in flight as well)
                asm volatile("" ::: "memory");
                if (lane == 0) __hip_atomic_fetch_add(&s_published, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
            request(S);
        };
        int su = first;
#pragma clang loop unroll(disable)
        do {
            process(A, su);
            process(B, su + 1);
            su += 2;
        } while (su < last && __hip_atomic_load(&s_abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) == 0);
        // What was requested beyond the last step is still in flight.  It is named here as if it were needed, so that
        // the last requests stay where they are in the loop: moved behind the loop's exit test (they are dead when
        // the loop ends), their results would reach the registers of the next trip through copies, and a copy waits
        // for its load.
        keep(A); keep(B);
        return;
    }

    // ------------------------------------------------------------------------------------ exchange wavefronts
    // (p <= 1024: two loads per lane and trip collect theta; eight cover the slice for up to 256 workgroups)
    const ExchangeLds x{th, stride, red, sums, kRowWaves, stride, (unsigned)kRowWaves,
                        (lds_u32*)&s_published, (lds_u32*)&s_theta_version, (lds_i32*)&s_abort,
                        (lds_u32*)s_xarrived, (lds_u32*)&s_xconsumed};
    exchange_wavefront<OPT, kXWaves, 8, 2>(a, x, lane, wave);
}

using KernelFn = void (*)(GlmArgs);

template <bool OPT, int V, int CPL, int PF>
KernelFn pick()
{
    if constexpr (!narrow_shape_ok(V, CPL, PF)) return nullptr;
    else return glm_narrow_kernel<V, CPL, PF, OPT>;
}

template <bool OPT, int V, int CPL>
KernelFn pick_pf(int pf)
{
    switch (pf) {
    case 1: return pick<OPT, V, CPL, 1>();
    case 2: return pick<OPT, V, CPL, 2>();
    case 4: return pick<OPT, V, CPL, 4>();
    case 8: return pick<OPT, V, CPL, 8>();
    }
    return nullptr;
}

template <bool OPT, int V>
KernelFn pick_cpl(int cpl, int pf)
{
    switch (cpl) {
    case 1: return pick_pf<OPT, V, 1>(pf);
    case 2: return pick_pf<OPT, V, 2>(pf);
    case 4: return pick_pf<OPT, V, 4>(pf);
    }
    return nullptr;
}

KernelFn narrow_kernel(int v, int cpl, int pf, bool opt)
{
    if (v == 4) return opt ? pick_cpl<true, 4>(cpl, pf) : pick_cpl<false, 4>(cpl, pf);
    if (v == 2) return opt ? pick_cpl<true, 2>(cpl, pf) : pick_cpl<false, 2>(cpl, pf);
    return nullptr;
}

size_t narrow_lds_bytes(const GlmLaunchShape& s, int p)
{
    const int stride = std::max((p + 15) & ~15, s.V * s.L * s.CPL);
    return (size_t)((2 + kRowWaves) * stride + kExchangeScratch * kXWaves + 16) * sizeof(float);
}

}  // namespace

int glm_narrow_block() { return kNarrowBlock; }

int glm_narrow_rows_in_flight(int v, int cpl, int L, int G, int64_t n)
{
    const int64_t slots = (int64_t)G * kRowWaves * (64 / L);
    const int64_t need = (n + slots - 1) / slots;
    int pf = 1;
    while (pf < need && pf < 16) pf *= 2;
    return narrow_shape_ok(v, cpl, pf) ? pf : 0;
}

hipError_t glm_narrow_prepare(const GlmLaunchShape& s, int p, int* max_groups)
{
    KernelFn fn = narrow_kernel(s.V, s.CPL, s.narrow_pf, s.with_optimizer != 0);
    if (!fn) return hipErrorInvalidValue;
    const size_t lds = narrow_lds_bytes(s, p);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    int per_cu = 0;
    e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(fn), kNarrowBlock, lds);
    if (e != hipSuccess) return e;
    int dev = 0;
    hipDeviceProp_t prop;
    if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
    if ((e = hipGetDeviceProperties(&prop, dev)) != hipSuccess) return e;
    *max_groups = per_cu * prop.multiProcessorCount;
    return hipSuccess;
}

hipError_t glm_narrow_launch(const GlmLaunchShape& s, const GlmArgs& args, hipStream_t stream)
{
    KernelFn fn = narrow_kernel(s.V, s.CPL, s.narrow_pf, s.with_optimizer != 0);
    const int64_t slots = (int64_t)s.G * kRowWaves * (64 / s.L);
    // what the kernel assumes: whole vector chunks, every row of a step in a register slot, words in pairs
    if (!fn || s.G < 8 || s.G % 8 != 0 || args.s_begin >= args.s_end || args.p % s.V != 0 || args.p % 2 != 0 ||
        args.p > s.V * s.L * s.CPL || args.L != s.L || (1 << args.logL) != s.L || (int64_t)args.n > slots * s.narrow_pf)
        return hipErrorInvalidValue;
    hipLaunchKernelGGL(fn, dim3(s.G), dim3(kNarrowBlock), narrow_lds_bytes(s, args.p), stream, args);
    return hipGetLastError();
}

}  // namespace bmgd
