// Fused mini-batch gradient + update for rows of 1025 .. 4096 floats (least squares, logistic), persistent over
// all steps of up to four passes, on G workgroups (G a multiple of 8, one per compute unit).
//
// One step of eq. (2.1) moves n rows of 4 p bytes once through the device and then has to wait for the new theta;
// the kernel's job is to keep the memory system busy through that wait.  Three decisions follow from measurements
// on the device:
//
//   * A workgroup takes its rows together.  Eight "row" wavefronts split every row by columns (wavefront w owns
//     columns [w C, (w + 1) C), C = 256 or 512; a lane holds one or two float4 of a row), so a compute unit advances
//     row by row (a row every 0.7 us at full rate) instead of each wavefront owning whole rows (a row every 6 us
//     per wavefront, and a step that ends when the slowest of 2048 wavefronts has had its turn).  A lane's slice of
//     theta and of the gradient sum lives in registers; nothing of a step's arithmetic goes through shared memory
//     except the eight partial dot products of a row, which the wavefronts exchange in groups of kGroupRows rows.
//   * Rows are requested far ahead and never waited for by anything but their own use.  Each row wavefront holds a
//     ring of kGroups groups of rows in registers, requested across step boundaries: while an exchange resolves, the
//     rows of the next step keep arriving.  Loads return to a wavefront in the order it issued them, so a wavefront
//     that has rows in flight must not poll for the exchange (its poll would come back behind its newest rows):
//     row wavefronts issue no load but their rows (and, right behind them, the responses and the next row indices), and
//   * a ninth wavefront does the exchange (glm_exchange.h).  It has no rows in flight, so its polls return at the latency
//     of the fabric.  Two trips over the fabric per step.  (Measured: under the row traffic a trip costs about 2 us
//     whether the words come from the same die or another, and a wavefront that asks for a phase's words in two
//     batches pays twice, so a die-local first stage - one more trip - loses; loads that would be served from a
//     die's L2 without leaving it, other than atomics, do not exist in this mode of the hardware.)
//
// Waits: row wavefronts only ever wait on shared-memory flags (which the exchange wavefront always releases, also
// when it gives up); the exchange wavefront's polls are bounded by the wall clock (PollGuard).
#include "glm_exchange.h"

#include <algorithm>

namespace bmgd {

namespace {

constexpr int kSplitBlock = kRoleBlock;
constexpr int kGroupRows = 4;                        // rows whose partial dot products are exchanged together
constexpr int kGroups = 3;                           // groups of rows a row wavefront holds (used, or in flight)

// Wait until every lane's word (one address per lane) equals want, or the word at `abort_addr` is non-zero.
__device__ __forceinline__ void lds_wait_all_eq(unsigned addr, unsigned want, unsigned abort_addr)
{
    unsigned t;
    asm volatile("1:\n\t"
                 "ds_read_b32 %0, %1\n\t"
                 "s_waitcnt lgkmcnt(0)\n\t"
                 "v_cmp_ne_u32_e32 vcc, %0, %2\n\t"
                 "s_cbranch_vccz 2f\n\t"
                 "ds_read_b32 %0, %3\n\t"
                 "s_waitcnt lgkmcnt(0)\n\t"
                 "v_cmp_ne_u32_e32 vcc, 0, %0\n\t"
                 "s_cbranch_vccnz 2f\n\t"
                 "s_branch 1b\n"
                 "2:"
                 : "=&v"(t) : "v"(addr), "v"(want), "v"(abort_addr) : "vcc", "memory");
}

template <int CH, bool OPT>
__global__ void __launch_bounds__(kSplitBlock) glm_split_kernel(GlmArgs a)
{
    extern __shared__ __align__(16) float smem[];
    __shared__ int s_abort;                          // set by the exchange wavefront when a wait ran out
    __shared__ unsigned s_theta_version;             // versions of theta delivered to shared memory so far
    __shared__ unsigned s_published;                 // row wavefronts that have stored their sums, counted over all steps

    constexpr int WCOLS = 256 * CH;                  // columns a row wavefront owns
    constexpr int P_PAD = kRowWaves * WCOLS;
    constexpr int GR = kGroupRows;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int G = gridDim.x;
    const int g = blockIdx.x;
    const int p = a.p;
    const int pp = (p + 15) & ~15;
    lds_f32* th = (lds_f32*)smem;                    // [2][P_PAD]: theta, by version parity
    // (pointers into shared memory carry its address space, so that accesses through them are shared-memory
    // instructions and are counted apart from the row loads)
    volatile lds_f32* pd = (volatile lds_f32*)(smem + 2 * P_PAD);   // [2][kRowWaves][GR]: partial dot products of a group, by group parity
    volatile lds_u32* pd_seq = (volatile lds_u32*)(smem + 2 * P_PAD + 2 * kRowWaves * GR);   // [2][kRowWaves]: their sequence numbers
    lds_f32* red = (lds_f32*)(smem + 2 * P_PAD + 2 * kRowWaves * GR + 2 * kRowWaves);   // [64][2] scratch of the exchange wavefront
    lds_f32* sums = red + 2 * 64;                    // [P_PAD]: the workgroup's gradient sums of a step, on their way out
    const int first = a.s_begin, last = a.s_end;

    // both copies of theta: columns beyond p stay zero for good (rows are read at column 0 there)
    for (int c = tid; c < 2 * P_PAD; c += kSplitBlock) th[c] = c < p ? a.theta[c] : 0.f;
    if (tid < 2 * kRowWaves) pd_seq[tid] = 0u;
    if (tid == 0) { s_abort = 0; s_theta_version = 0u; s_published = 0u; }
    __syncthreads();                                 // the only barrier: from here on the wavefronts meet through flags

    const StepGeometry geo(a);
    auto batch_rows = [&](int s) { return geo.batch_rows(s); };
    auto batch_base = [&](int s) { return geo.batch_base(s); };

    const int rw = role_of(wave);
    if (rw == -2) return;                            // they only keep the exchange wavefront's SIMD free of row loads
    if (rw >= 0) {
        // ------------------------------------------------------------------------------------ row wavefronts
        // Workgroup g takes rows g, g + G, g + 2 G, ... of a mini-batch, in groups of GR; a step has at least one
        // group (a group without rows contributes nothing), so every step ends with a publication.
        auto groups_of = [&](int s) {
            const int nb = batch_rows(s);
            const int mine = g < nb ? (nb - g + G - 1) / G : 0;
            return max(1, (mine + GR - 1) / GR);
        };
        const int col0 = rw * WCOLS + 4 * lane;    // first column of this lane's chunk 0; chunk ch starts 256 ch further

        // A slot of the ring: one group of rows.  Besides the rows it carries, in lanes r < GR, the response of row r
        // and the index of the row that takes its place at the slot's next request.  Both are loaded right behind
        // the slot's rows, so they have arrived when the rows have (loads return in order) and waiting for them waits
        // for nothing else.  (Loads through the scalar path would be counted together with the shared-memory
        // accesses, out of order: every access to shared memory would then wait for them, microseconds under load.)
        struct Slot {
            float4 x[GR][CH];                        // this lane's part of the group's rows
            float y;                                 // lane r < GR: response of row r
            int idx_next;                            // lane r < GR: row that follows row r in this slot
            unsigned ok;                             // bit r: row r exists (uniform)
            unsigned ok_next;
        };
        Slot S0, S1, S2;
        static_assert(kGroups == 3, "the ring is written out for three groups");
        const int lr = lane & (GR - 1);              // the row of a group this lane looks after (lanes >= GR repeat them)

        int sq = first, kq = 0, nq = groups_of(first);   // the group whose row indices are loaded next
        auto load_idx = [&](Slot& S) {
            const bool live = sq < last;
            const int sc = live ? sq : first;
            const int nb = batch_rows(sc);
            const size_t base = batch_base(sc);
            const int j = (kq * GR + lr) * G + g;
            S.idx_next = a.perm[base + (size_t)(live && j < nb ? j : 0)];
            S.ok_next = 0u;
#pragma unroll
            for (int r = 0; r < GR; ++r) S.ok_next |= live && (kq * GR + r) * G + g < nb ? (1u << r) : 0u;
            if (live) {
                if (kq + 1 < nq) ++kq;
                else { ++sq; kq = 0; nq = groups_of(min(sq, last - 1)); }
            }
        };
        auto request = [&](Slot& S) {
            const int idxv = S.idx_next;
#pragma unroll
            for (int r = 0; r < GR; ++r) {
                const int idx = __builtin_amdgcn_readlane(idxv, r);
                const float* row = a.X + (size_t)idx * (size_t)p;
#pragma unroll
                for (int ch = 0; ch < CH; ++ch) {
                    const int c = col0 + 256 * ch;
                    S.x[r][ch] = *reinterpret_cast<const float4*>(row + (c < p ? c : 0));   // beyond p: theta is 0 there
                }
            }
            S.y = a.y[idxv];
            S.ok = S.ok_next;
            load_idx(S);
        };
        load_idx(S0); load_idx(S1); load_idx(S2);
        request(S0); request(S1); request(S2);

        float4 thr[CH], acc[CH];
#pragma unroll
        for (int ch = 0; ch < CH; ++ch) acc[ch] = make_float4(0.f, 0.f, 0.f, 0.f);
        int su = first, ku = 0, nu = groups_of(first);   // the group that is used next
        unsigned kg = 0u;                            // groups used so far

        const unsigned abort_addr = (unsigned)(uintptr_t)(lds_u32*)&s_abort;
        const unsigned version_addr = (unsigned)(uintptr_t)(lds_u32*)&s_theta_version;
        // Use the rows in S (group ku of step su), refill S, end the step if that was its last group.  Straight-line
        // code with one conditional (the publication): the loop around it has its only exit at the bottom, so a
        // wavefront may run up to two groups past the last step; those groups use rows requested beyond the end
        // (valid addresses), publish nothing and wait for nothing that will not come.
        auto process = [&](Slot& S) {
            const bool live = su < last;
            if (ku == 0) {
                // theta of this step: version su - first, delivered by the exchange wavefront
                const unsigned want = (unsigned)(min(su, last) - first);
                lds_wait_ge(version_addr, want, abort_addr);
                const lds_f32* src = th + (want & 1u) * P_PAD + col0;
#pragma unroll
                for (int ch = 0; ch < CH; ++ch)
                    thr[ch] = make_float4(src[256 * ch], src[256 * ch + 1], src[256 * ch + 2], src[256 * ch + 3]);
            }
            // this wavefront's part of the group's dot products
            float d[GR];
#pragma unroll
            for (int r = 0; r < GR; ++r) {
                float t = 0.f;
#pragma unroll
                for (int ch = 0; ch < CH; ++ch) {
                    t = fmaf(S.x[r][ch].x, thr[ch].x, t);
                    t = fmaf(S.x[r][ch].y, thr[ch].y, t);
                    t = fmaf(S.x[r][ch].z, thr[ch].z, t);
                    t = fmaf(S.x[r][ch].w, thr[ch].w, t);
                }
                d[r] = group_sum(t, 64);
            }
            // exchange them: one writer per wavefront, values first, then the sequence number; a reader that sees the
            // number of this group reads values stored before it (shared memory serves requests in order)
            const unsigned par = kg & 1u;
            if (lane == 0) {
#pragma unroll
                for (int r = 0; r < GR; ++r) pd[(par * kRowWaves + rw) * GR + r] = d[r];
                pd_seq[par * kRowWaves + rw] = kg + 1u;
            }
            lds_wait_all_eq((unsigned)(uintptr_t)(pd_seq + par * kRowWaves + (lane & (kRowWaves - 1))), kg + 1u, abort_addr);
            float v = lane < kRowWaves * GR ? pd[par * kRowWaves * GR + lane] : 0.f;
            v = slot_sum(v, GR);                     // lane r < GR: the whole dot product of row r
            const float res = lane < GR && ((S.ok >> lane) & 1u) != 0u ? residual(a.model, v, S.y) : 0.f;
#pragma unroll
            for (int r = 0; r < GR; ++r) {
                const float rr = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, res), r));
#pragma unroll
                for (int ch = 0; ch < CH; ++ch) {
                    acc[ch].x = fmaf(rr, S.x[r][ch].x, acc[ch].x);
                    acc[ch].y = fmaf(rr, S.x[r][ch].y, acc[ch].y);
                    acc[ch].z = fmaf(rr, S.x[r][ch].z, acc[ch].z);
                    acc[ch].w = fmaf(rr, S.x[r][ch].w, acc[ch].w);
                }
            }
            kg += 1u;
            const bool step_ends = live && ku + 1 >= nu;
            if (step_ends) {
                // This lane's columns of the workgroup's sums go to shared memory; the exchange wavefront sends them
                // out (a store issued here would stand in this SIMD's queue behind the rows requested for the next
                // step, for microseconds).
#pragma unroll
                for (int ch = 0; ch < CH; ++ch) {
                    lds_f32* dst = sums + col0 + 256 * ch;
                    dst[0] = acc[ch].x; dst[1] = acc[ch].y; dst[2] = acc[ch].z; dst[3] = acc[ch].w;
                    acc[ch] = make_float4(0.f, 0.f, 0.f, 0.f);
                }
                if (lane == 0) __hip_atomic_fetch_add(&s_published, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
            request(S);
            ku = step_ends ? 0 : (live ? ku + 1 : 0);
            su += step_ends ? 1 : 0;
            nu = step_ends ? groups_of(min(su, last - 1)) : nu;
        };
#pragma clang loop unroll(disable)
        do {
            process(S0);
            process(S1);
            process(S2);
        } while (su < last && __hip_atomic_load(&s_abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) == 0);
        return;                                      // rows requested beyond the last step land in registers that die here
    }

    // ------------------------------------------------------------------------------------ exchange wavefront
    const ExchangeLds x{th, P_PAD, red, sums, 1, P_PAD, (unsigned)kRowWaves,
                        (lds_u32*)&s_published, (lds_u32*)&s_theta_version, (lds_i32*)&s_abort, nullptr, nullptr};
    exchange_wavefront<OPT, 1, 32, 32>(a, x, lane, 0);
}

using KernelFn = void (*)(GlmArgs);

KernelFn split_kernel(int ch, bool opt)
{
    if (ch == 1) return opt ? glm_split_kernel<1, true> : glm_split_kernel<1, false>;
    return opt ? glm_split_kernel<2, true> : glm_split_kernel<2, false>;
}

}  // namespace

size_t glm_split_lds_bytes(int ch)
{
    return (size_t)(3 * kRowWaves * 256 * ch + 2 * kRowWaves * kGroupRows + 2 * kRowWaves + 2 * 64 + 16) * sizeof(float);
}

int glm_split_block() { return kSplitBlock; }

hipError_t glm_split_prepare(int ch, bool opt, int* max_groups)
{
    KernelFn fn = split_kernel(ch, opt);
    const size_t lds = glm_split_lds_bytes(ch);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    int per_cu = 0;
    e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(fn), kSplitBlock, lds);
    if (e != hipSuccess) return e;
    int dev = 0;
    hipDeviceProp_t prop;
    if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
    if ((e = hipGetDeviceProperties(&prop, dev)) != hipSuccess) return e;
    *max_groups = per_cu * prop.multiProcessorCount;
    return hipSuccess;
}

hipError_t glm_split_launch(int ch, bool opt, int G, const GlmArgs& args, hipStream_t stream)
{
    if (G < 8 || G % 8 != 0 || args.s_begin >= args.s_end || args.p % 4 != 0 || args.p > kRowWaves * 256 * ch)
        return hipErrorInvalidValue;
    hipLaunchKernelGGL(split_kernel(ch, opt), dim3(G), dim3(kSplitBlock), glm_split_lds_bytes(ch), stream, args);
    return hipGetLastError();
}

}  // namespace bmgd
