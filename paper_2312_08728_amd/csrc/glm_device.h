// Device-side helpers shared by the GLM kernels: lane reductions (DPP / permlane swaps), the link function, flagged
// words (the exchange between workgroups) and the bounded wait.  Included by the kernel sources only.
#pragma once

#include <hip/hip_runtime.h>

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

// The same two sums without branches on L (every stage is executed and its result kept or dropped): for code whose
// control flow must stay a straight line.
__device__ __forceinline__ float group_sum_flat(float v, int L)
{
    float t;
    t = dpp_mov<0xB1>(v); v += L >= 2 ? t : 0.f;
    t = dpp_mov<0x4E>(v); v += L >= 4 ? t : 0.f;
    t = dpp_mov<0x141>(v); v += L >= 8 ? t : 0.f;
    t = dpp_mov<0x140>(v); v += L >= 16 ? t : 0.f;
    t = swap16_sum(v); v = L >= 32 ? t : v;
    t = swap32_sum(v); v = L >= 64 ? t : v;
    return v;
}

__device__ __forceinline__ float slot_sum_flat(float v, int L)
{
    float t;
    t = dpp_mov<0x121>(v); v += L <= 1 ? t : 0.f;
    t = dpp_mov<0x122>(v); v += L <= 2 ? t : 0.f;
    t = dpp_mov<0x124>(v); v += L <= 4 ? t : 0.f;
    t = dpp_mov<0x128>(v); v += L <= 8 ? t : 0.f;
    t = swap16_sum(v); v = L <= 16 ? t : v;
    t = swap32_sum(v); v = L <= 32 ? t : v;
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
    // Called after a failed poll; reports true when the wait must be given up.  Reading the clock is also the
    // back-off (polls travel over the fabric; a storm of them slows the very stores they wait for).  The abort flag
    // is looked at on every 32nd miss only: it lives in global memory, and a load from it costs a whole trip over
    // the fabric, as much as the poll that just failed.
    __device__ __forceinline__ bool expired()
    {
        const long long now = wall_clock64();
        if (t0 == 0) t0 = now;
        ++misses;
        if (now - t0 > timeout) {
            __hip_atomic_store(flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return true;
        }
        if ((misses & 31u) != 0u) return false;
        return __hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u;
    }
    __device__ __forceinline__ void arm() { t0 = 0; misses = 0; }
};

}  // namespace
}  // namespace bmgd
