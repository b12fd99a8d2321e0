// The exchange wavefront of the persistent GLM kernels, and what they share around it.
//
// A workgroup of these kernels is a set of "row" wavefronts, which read rows and accumulate the gradient sums of a
// step of eq. (2.1), and one exchange wavefront, which carries those sums to the other workgroups and brings the
// new theta back.  The two kinds meet only through flags in shared memory:
//   s_published      counts publications of row wavefronts over all steps (each stores its sums to shared memory first);
//   s_theta_version  versions of theta the exchange wavefront has delivered to shared memory (version v = theta
//                    after v steps of the launch, kept in the copy v & 1);
//   s_abort          set by the exchange wavefront when a wait ran out: everybody leaves.
// A row wavefront must not poll global memory itself: loads return to a wavefront in the order it issued them, so
// its poll would come back behind the newest rows it has in flight.
//
// Per step the exchange wavefront makes two trips over the fabric, asking for everything a trip needs at once
// (32 loads of 16 bytes per lane in flight):
//   0. the workgroup's sums leave as flagged words {value : tag};
//   1. workgroup g adds up, for the g-th slice of the columns (whole 128-byte lines of words), the words of all G
//      workgroups in a fixed order, applies the update to its slice of theta and publishes the new values in
//      kThetaCopies copies of theta (a workgroup later reads copy g mod kThetaCopies, so no set of words is polled
//      by the whole grid);
//   2. it collects the whole new theta from its copy into shared memory and raises the version.
// Its polls are bounded by the wall clock (PollGuard).
#pragma once

#include "bmgd_internal.h"
#include "glm_device.h"

namespace bmgd {
namespace {

// Eleven wavefronts are launched and three roles handed out by wavefront index.  The hardware deals the wavefronts of a
// workgroup out to the four SIMDs of a compute unit in turn (0, 4, 8 share the first one), and every SIMD feeds its memory
// instructions into a queue of its own, in order.  The exchange wavefront must not stand in such a queue behind row
// loads, so it is wavefront 0 and its two SIMD mates (4 and 8) leave right after the start-up barrier; the other
// eight are the row wavefronts.  (Only speed depends on the dealing order; the roles are correct for any.)
constexpr int kRowWaves = 8;
constexpr int kRoleWaves = 11;
constexpr int kRoleBlock = 64 * kRoleWaves;
// wavefront index -> row wavefront 0 .. 7 (1, 2, 3, 5, 6, 7, 9, 10), -1 for the exchange wavefront, -2 for the two that leave
__device__ __forceinline__ int role_of(int wave) { return wave == 0 ? -1 : (wave & 3) == 0 ? -2 : wave - 1 - (wave >> 2); }

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
// (pointers into shared memory carry its address space, so that accesses through them are shared-memory
// instructions and are counted apart from the row loads)
typedef __attribute__((address_space(3))) float lds_f32;
typedef __attribute__((address_space(3))) unsigned lds_u32;
typedef __attribute__((address_space(3))) int lds_i32;

constexpr int kAgentScope = 0x10;                    // cache policy of a buffer instruction: sc1

__device__ __forceinline__ __amdgpu_buffer_rsrc_t words_rsrc(const void* base, size_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

// (A function, so that its argument is a scalar copy: bit-casting an element of a vector in place reads element 0.)
__device__ __forceinline__ float as_float(unsigned v) { return __builtin_bit_cast(float, v); }

// two flagged words next to each other: {value, tag, value, tag}
__device__ __forceinline__ u32x4 word_pair(float v0, float v1, unsigned tag)
{
    u32x4 w;
    w.x = __builtin_bit_cast(unsigned, v0); w.y = tag;
    w.z = __builtin_bit_cast(unsigned, v1); w.w = tag;
    return w;
}

// A wait of a row wavefront, written as one block of assembly.  The compiler must see no loop and no branch out of
// the row loop at such a place: it keeps count of the row loads in flight per path through the control-flow graph,
// and every extra path (a poll loop, an early exit, which the structuriser routes through the loop's latch) makes
// it wait for rows that the path actually taken does not need.
// Wait until the word at shared-memory address `addr` is >= want, or the word at `abort_addr` is non-zero.
__device__ __forceinline__ void lds_wait_ge(unsigned addr, unsigned want, unsigned abort_addr)
{
    unsigned t;
    asm volatile("1:\n\t"
                 "ds_read_b32 %0, %1\n\t"
                 "s_waitcnt lgkmcnt(0)\n\t"
                 "v_cmp_ge_u32_e32 vcc, %0, %2\n\t"
                 "s_cbranch_vccnz 2f\n\t"
                 "ds_read_b32 %0, %3\n\t"
                 "s_waitcnt lgkmcnt(0)\n\t"
                 "v_cmp_ne_u32_e32 vcc, 0, %0\n\t"
                 "s_cbranch_vccnz 2f\n\t"
                 "s_sleep 1\n\t"
                 "s_branch 1b\n"
                 "2:"
                 : "=&v"(t) : "v"(addr), "v"(want), "v"(abort_addr) : "vcc", "memory");
}

// Mini-batches of the steps of a launch: step s is mini-batch m = s mod M of pass t = s / M.
struct StepGeometry {
    int M, n, n_tail, perm_stride;
    float rcpM;
    __device__ __forceinline__ explicit StepGeometry(const GlmArgs& a)
    {
        M = (a.rows + a.n - 1) / a.n;
        n = a.n;
        n_tail = a.rows - (M - 1) * a.n;
        perm_stride = a.perm_stride;
        rcpM = 1.0f / (float)M;
    }
    // s = t M + m, from a float reciprocal plus a correction: exact for s < 2^23, which the host guarantees
    __device__ __forceinline__ void split(int s, int& t, int& m) const
    {
        t = (int)((float)s * rcpM);
        m = s - t * M;
        if (m >= M) { m -= M; ++t; }
        if (m < 0) { m += M; --t; }
    }
    __device__ __forceinline__ int batch_rows(int s) const { int t, m; split(s, t, m); return m == M - 1 ? n_tail : n; }
    // where the mini-batch of step s starts in the array of partitions
    __device__ __forceinline__ size_t batch_base(int s) const
    {
        int t, m;
        split(s, t, m);
        return (size_t)t * (size_t)perm_stride + (size_t)m * (size_t)n;
    }
};

// The exchange wavefronts' view of the workgroup's shared memory.
struct ExchangeLds {
    lds_f32* th;                  // [2][th_stride]: theta by version parity (th_stride even, >= p rounded up to even)
    int th_stride;
    lds_f32* red;                 // [kExchangeScratch * NX] scratch of the exchange wavefronts
    const lds_f32* sums;          // [nsum][sums_stride]: the workgroup's gradient sums of a step; column c is the sum over
    int nsum, sums_stride;        //   the nsum arrays, added in their order (columns [p, p rounded up to even) hold 0)
    unsigned publishers;          // publications of row wavefronts that complete a step
    lds_u32* s_published;
    lds_u32* s_theta_version;     // raised by every exchange wavefront once per step: NX v when version v is complete
    lds_i32* s_abort;
    lds_u32* s_xarrived;          // NX > 1: [NX] chunks of slices each exchange wavefront has handed its partial sums of to
    lds_u32* s_xconsumed;         //         the first one, and chunks that one has added up
};
constexpr int kExchangeScratch = 3 * 128;            // floats of `red` per exchange wavefront

// All steps [a.s_begin, a.s_end) of a launch, by exchange wavefront xw of NX of workgroup blockIdx.x of gridDim.x (a
// multiple of 8).  p is even.  Returns when the last version of theta has been delivered (workgroup 0 also writes it to
// a.theta), or with s_abort and the global abort flag set when a wait ran out.
// With NX > 1 the wavefronts share every phase: each sends a part of the workgroup's sums, adds up a part of the
// workgroups for the slice (the first one then adds the NX partial sums in their order and applies the update) and
// collects a part of theta.  A wavefront pulls freshly written lines at a fraction of what a compute unit can take,
// so where no row traffic competes (narrow rows) four wavefronts on the four SIMDs finish a trip sooner.
// U1, U2: pairs of words a lane requests per trip when it sums the slice / collects theta.
template <bool OPT, int NX, int U1, int U2>
__device__ __forceinline__ void exchange_wavefront(const GlmArgs& a, const ExchangeLds& x, int lane, int xw)
{
    const int G = gridDim.x;
    const int g = blockIdx.x;
    const int p = a.p;
    const int pp = (p + 15) & ~15;                   // stride of a row of words
    const int first = a.s_begin, last = a.s_end;
    const StepGeometry geo(a);
    const unsigned words_bytes = (unsigned)((size_t)G * pp * 8);
    const unsigned copies_bytes = (unsigned)((size_t)kThetaCopies * pp * 8);
    // Workgroup g owns the columns [c_lo, c_hi) of theta (whole 128-byte lines of words, so no line has two writers).
    const int cw = (((p + G - 1) / G) + 15) & ~15;
    const int c_lo = min(p, g * cw), c_hi = min(p, c_lo + cw);
    const int npair = cw / 2;                        // column pairs of a slice (a multiple of 8)
    const int PPc = min(npair, 64);                  // pairs taken side by side by the lanes ...
    const int SG = 64 / PPc;                         // ... by SG groups of lanes, each group taking every SG-th workgroup
    const int my_pair = lane % PPc, my_sg = lane / PPc;
    const bool lane_used = my_sg < SG;
    lds_f32* red = x.red + xw * 128;                 // [64][2]: this wavefront's own scratch
    lds_f32* xpart = x.red + NX * 128;               // [2][NX][64][2]: the wavefronts' partial sums of a chunk of the slice, by parity
    PollGuard guard{a.sync + 1, a.timeout_ticks, 0, 0};
    bool dead = false;
    unsigned phase = 0u;                             // chunks of slices summed so far (the same in all NX wavefronts)
    // A wait on shared memory alone (the wall clock and the global abort flag are looked at now and then: a load from
    // global memory would return after microseconds).  False: give up.
    auto spin_ge = [&](lds_u32* word, unsigned want) -> bool {
        long long t0 = 0;
        unsigned spins = 0u;
        while (__hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) < want) {
            __builtin_amdgcn_s_sleep(1);
            if constexpr (NX > 1) {
                if (__hip_atomic_load(x.s_abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) != 0) return false;
            }
            if ((++spins & 1023u) == 0u) {
                const long long now = wall_clock64();
                if (t0 == 0) t0 = now;
                if (now - t0 > a.timeout_ticks ||
                    __hip_atomic_load(a.sync + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) return false;
            }
        }
        return true;
    };
    for (int s = first; s < last && !dead; ++s) {
        const unsigned tag = a.tag_base + (unsigned)(s - first) + 1u;
        const float alpha_s = a.lr_tab ? a.lr_tab[min(a.lr_base + s, a.lr_len - 1)] : a.alpha;
        const int nb = geo.batch_rows(s);
        const float scale = alpha_s / (float)nb;
        const unsigned ver = (unsigned)(s - first);
        const lds_f32* th_old = x.th + (ver & 1u) * x.th_stride;
        lds_f32* th_new = x.th + ((ver + 1u) & 1u) * x.th_stride;
        float oc1 = 1.f, oc2 = 1.f;
        if constexpr (OPT) {
            if (a.opt.kind == kOptAdam) opt_corrections(a.opt, a.opt.k_base + (s - first) + 1, oc1, oc2);
        }
        // This workgroup's own rows first: until they have been summed nothing can be complete, and polling the
        // fabric meanwhile would only take bandwidth from the rows.
        if (!spin_ge(x.s_published, (ver + 1u) * x.publishers)) { dead = true; break; }
        guard.arm();
        const __amdgpu_buffer_rsrc_t part = words_rsrc(a.ll_part + (size_t)(s & 1) * G * pp, words_bytes);
        // 0. this workgroup's sums out of shared memory, as flagged words: what the others wait for
        asm volatile("" ::: "memory");
        if (x.nsum == 1) {
#pragma unroll 8
            for (int c = 2 * (lane + 64 * xw); c < p; c += 128 * NX)
                __builtin_amdgcn_raw_buffer_store_b128(word_pair(x.sums[c], x.sums[c + 1], tag), part, (unsigned)(((size_t)g * pp + c) * 8), 0, kAgentScope);
        } else {
            for (int c = 2 * (lane + 64 * xw); c < p; c += 128 * NX) {
                float v0 = 0.f, v1 = 0.f;
                for (int k = 0; k < x.nsum; ++k) {
                    v0 += x.sums[k * x.sums_stride + c];
                    v1 += x.sums[k * x.sums_stride + c + 1];
                }
                __builtin_amdgcn_raw_buffer_store_b128(word_pair(v0, v1, tag), part, (unsigned)(((size_t)g * pp + c) * 8), 0, kAgentScope);
            }
        }
        const __amdgpu_buffer_rsrc_t thw = words_rsrc(a.ll_theta + (size_t)(s & 1) * kThetaCopies * pp, copies_bytes);

        // 1. this workgroup's slice, if it has one: sum over all workgroups, in a fixed order; the update; the new
        //    values into every copy of theta
        for (int pb = 0; pb < npair && c_lo < c_hi && !dead; pb += PPc) {
            const int c = c_lo + 2 * (pb + my_pair);
            const bool mine = lane_used && c < c_hi;             // (a slice ends on a multiple of 16 or at p)
            // One address register per lane (its pair of columns in the row of words of workgroup my_sg); what differs
            // between a lane's loads is uniform and goes into the scalar offset.  Load u of wavefront xw takes the
            // workgroups SG (xw + NX u) + my_sg.  G is a multiple of SG, so whether a load is beyond the last
            // workgroup is uniform too (such loads repeat the last group and are not added).
            const unsigned voff = (unsigned)min(c, pp - 2) * 8u + (unsigned)my_sg * (unsigned)(pp * 8);
            float t0 = 0.f, t1 = 0.f;
            for (int i0 = 0; i0 < G && !dead; i0 += SG * NX * U1) {
                u32x4 w[U1];
                for (;;) {
                    asm volatile("" ::: "memory");
#pragma unroll
                    for (int u = 0; u < U1; ++u)
                        w[u] = __builtin_amdgcn_raw_buffer_load_b128(part, voff, (unsigned)min(i0 + SG * (xw + NX * u), G - SG) * (unsigned)(pp * 8), kAgentScope);
                    asm volatile("" ::: "memory");
                    unsigned miss = 0u;
#pragma unroll
                    for (int u = 0; u < U1; ++u) miss |= (w[u].y ^ tag) | (w[u].w ^ tag);
                    if (!mine) miss = 0u;
                    if (__builtin_amdgcn_ballot_w64(miss != 0u) == 0ull) break;
                    if (guard.expired()) { dead = true; break; }
                }
                if (dead) break;
#pragma unroll
                for (int u = 0; u < U1; ++u)
                    if (i0 + SG * (xw + NX * u) < G) {
                        t0 += as_float(w[u].x);
                        t1 += as_float(w[u].z);
                    }
            }
            if (dead) break;
            // the SG groups' sums meet in shared memory (this wavefront alone uses its `red`; its requests are served in order)
            if (lane_used) {
                red[(my_sg * PPc + my_pair) * 2] = t0;
                red[(my_sg * PPc + my_pair) * 2 + 1] = t1;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            const bool upd = lane < PPc && c < c_hi;             // this lane ends up with a pair of the slice
            float b0 = 0.f, b1 = 0.f;
            if (upd) {
                for (int q = 0; q < SG; ++q) {
                    b0 += red[(q * PPc + lane) * 2];
                    b1 += red[(q * PPc + lane) * 2 + 1];
                }
            }
            if constexpr (NX > 1) {
                // the NX wavefronts' sums meet in the first one (two sets of partial sums alternate; a wavefront does
                // not overwrite a set before the first one has added it up)
                if (phase >= 2u && !spin_ge(x.s_xconsumed, phase - 1u)) { dead = true; break; }
                lds_f32* out = xpart + ((phase & 1u) * NX + xw) * 128;
                if (upd) { out[lane * 2] = b0; out[lane * 2 + 1] = b1; }
                asm volatile("" ::: "memory");
                if (lane == 0) __hip_atomic_store(x.s_xarrived + xw, phase + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                if (xw == 0) {
                    // (also: every wavefront has delivered its part of the theta this update starts from)
                    bool all = spin_ge(x.s_theta_version, NX * ver);
                    for (int k = 1; k < NX && all; ++k) all = spin_ge(x.s_xarrived + k, phase + 1u);
                    if (!all) { dead = true; break; }
                    asm volatile("" ::: "memory");
                    b0 = 0.f; b1 = 0.f;
                    if (upd) {
                        for (int k = 0; k < NX; ++k) {
                            b0 += xpart[((phase & 1u) * NX + k) * 128 + lane * 2];
                            b1 += xpart[((phase & 1u) * NX + k) * 128 + lane * 2 + 1];
                        }
                    }
                }
            }
            if (upd && xw == 0) {
                float n0, n1;
                if constexpr (!OPT) {
                    n0 = th_old[c] - scale * b0;
                    n1 = th_old[c + 1] - scale * b1;
                } else {
                    float m0 = a.opt.m[c], m1 = a.opt.m[c + 1];
                    float s0 = a.opt.kind == kOptAdam ? a.opt.s[c] : 0.f, s1 = a.opt.kind == kOptAdam ? a.opt.s[c + 1] : 0.f;
                    n0 = opt_update(a.opt, th_old[c], b0 / (float)nb, alpha_s, m0, s0, oc1, oc2);
                    n1 = opt_update(a.opt, th_old[c + 1], b1 / (float)nb, alpha_s, m1, s1, oc1, oc2);
                    a.opt.m[c] = m0; a.opt.m[c + 1] = m1;
                    if (a.opt.kind == kOptAdam) { a.opt.s[c] = s0; a.opt.s[c + 1] = s1; }
                }
                const u32x4 nw = word_pair(n0, n1, tag);
#pragma unroll
                for (int r = 0; r < kThetaCopies; ++r)
                    __builtin_amdgcn_raw_buffer_store_b128(nw, thw, (unsigned)c * 8u, (unsigned)(r * pp * 8), kAgentScope);
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // `red` is reused by the next chunk of pairs
            if constexpr (NX > 1) {
                if (xw == 0 && lane == 0) __hip_atomic_store(x.s_xconsumed, phase + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                ++phase;
            }
        }
        if (dead) break;
        // 2. the whole new theta, from this workgroup's copy
        // (one address register per lane again; the buffer is that copy alone, so loads beyond its row of words are
        // answered with zeros by the range check without going to memory, and are not looked at)
        const __amdgpu_buffer_rsrc_t mine = words_rsrc(a.ll_theta + ((size_t)(s & 1) * kThetaCopies + (size_t)(g % kThetaCopies)) * pp, (unsigned)(pp * 8));
        const unsigned copy_off = (unsigned)lane * 16u;
        for (int c0 = 128 * xw; c0 < p && !dead; c0 += 128 * NX * U2) {
            u32x4 w[U2];
            for (;;) {
                asm volatile("" ::: "memory");
#pragma unroll
                for (int u = 0; u < U2; ++u)
                    w[u] = __builtin_amdgcn_raw_buffer_load_b128(mine, copy_off, (unsigned)(c0 + 128 * NX * u) * 8u, kAgentScope);
                asm volatile("" ::: "memory");
                unsigned miss = 0u;
#pragma unroll
                for (int u = 0; u < U2; ++u)
                    if (c0 + 2 * (lane + 64 * NX * u) < p) miss |= (w[u].y ^ tag) | (w[u].w ^ tag);
                if (__builtin_amdgcn_ballot_w64(miss != 0u) == 0ull) break;
                if (guard.expired()) { dead = true; break; }
            }
            if (dead) break;
#pragma unroll
            for (int u = 0; u < U2; ++u) {
                const int c = c0 + 2 * (lane + 64 * NX * u);
                if (c < p) {
                    th_new[c] = as_float(w[u].x);
                    th_new[c + 1] = as_float(w[u].z);
                }
            }
        }
        if (dead) break;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        if (lane == 0) __hip_atomic_fetch_add(x.s_theta_version, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    if (dead) {
        if (lane == 0) {
            __hip_atomic_store(a.sync + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(x.s_abort, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        return;
    }
    if (g == 0 && xw == 0) {
        if constexpr (NX > 1) {
            if (!spin_ge(x.s_theta_version, NX * (unsigned)(last - first))) return;
            asm volatile("" ::: "memory");
        }
        const lds_f32* fin = x.th + ((unsigned)(last - first) & 1u) * x.th_stride;
        for (int c = lane; c < p; c += 64) a.theta[c] = fin[c];
    }
}

}  // namespace
}  // namespace bmgd
