// Device helpers shared by the contraction kernels (contract.hip, contract_wave.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

// Unguarded load of the 4 words at p with the widest access the operand's alignment allows.
template <int VEC>
__device__ __forceinline__ uint4 load4(const uint32_t *p)
{
    if (VEC == 4) return *reinterpret_cast<const uint4 *>(p);
    if (VEC == 2) {
        const uint2 lo = *reinterpret_cast<const uint2 *>(p), hi = *reinterpret_cast<const uint2 *>(p + 2);
        return make_uint4(lo.x, lo.y, hi.x, hi.y);
    }
    return make_uint4(p[0], p[1], p[2], p[3]);
}

// p points at word k0 of a plane of kend words; words at or beyond kend read as zero.  k0 and kend are
// multiples of VEC (the launch code picks VEC so), so a group of VEC words lies wholly inside or wholly
// outside the plane.  Branch-free: an outside group is fetched from the plane's last group and discarded.
template <int VEC>
__device__ __forceinline__ uint4 load4_tail(const uint32_t *p, int k0, int kend)
{
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 4; e += VEC) {
        const bool ok = k0 + e < kend;
        const uint32_t *q = p + (ok ? e : kend - VEC - k0);
        if (VEC == 4) {
            const uint4 t = *reinterpret_cast<const uint4 *>(q);
            w[0] = ok ? t.x : 0u; w[1] = ok ? t.y : 0u; w[2] = ok ? t.z : 0u; w[3] = ok ? t.w : 0u;
        } else if (VEC == 2) {
            const uint2 t = *reinterpret_cast<const uint2 *>(q);
            w[e] = ok ? t.x : 0u; w[e + 1] = ok ? t.y : 0u;
        } else {
            const uint32_t t = *q;
            w[e] = ok ? t : 0u;
        }
    }
    return make_uint4(w[0], w[1], w[2], w[3]);
}

// acc[n] += popcount(a & w[n]) for a group of N outputs that share the activation word `a`:
// exactly one v_and_b32 and one accumulating v_bcnt_u32_b32 per output, the ANDs running two
// instructions ahead of the BCNTs that consume them.  Written as asm because the optimiser
// otherwise re-associates the accumulation chains into trees of partial sums (extra adds and
// registers), and as one block per group because every separate asm statement costs a wait state.
template <int N>
__device__ __forceinline__ void and_popc_group(int (&acc)[N], uint32_t a, const uint32_t (&w)[N]);

template <>
__device__ __forceinline__ void and_popc_group<2>(int (&acc)[2], uint32_t a, const uint32_t (&w)[2])
{
    uint32_t t0, t1;
    asm("v_and_b32 %2, %4, %5\n\t"
        "v_and_b32 %3, %4, %6\n\t"
        "v_bcnt_u32_b32 %0, %2, %0\n\t"
        "v_bcnt_u32_b32 %1, %3, %1"
        : "+v"(acc[0]), "+v"(acc[1]), "=&v"(t0), "=&v"(t1)
        : "v"(a), "v"(w[0]), "v"(w[1]));
}

template <>
__device__ __forceinline__ void and_popc_group<4>(int (&acc)[4], uint32_t a, const uint32_t (&w)[4])
{
    uint32_t t0, t1;
    asm("v_and_b32 %4, %6, %7\n\t"
        "v_and_b32 %5, %6, %8\n\t"
        "v_bcnt_u32_b32 %0, %4, %0\n\t"
        "v_and_b32 %4, %6, %9\n\t"
        "v_bcnt_u32_b32 %1, %5, %1\n\t"
        "v_and_b32 %5, %6, %10\n\t"
        "v_bcnt_u32_b32 %2, %4, %2\n\t"
        "v_bcnt_u32_b32 %3, %5, %3"
        : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]), "=&v"(t0), "=&v"(t1)
        : "v"(a), "v"(w[0]), "v"(w[1]), "v"(w[2]), "v"(w[3]));
}

template <>
__device__ __forceinline__ void and_popc_group<6>(int (&acc)[6], uint32_t a, const uint32_t (&w)[6])
{
    uint32_t t0, t1;
    asm("v_and_b32 %6, %8, %9\n\t"
        "v_and_b32 %7, %8, %10\n\t"
        "v_bcnt_u32_b32 %0, %6, %0\n\t"
        "v_and_b32 %6, %8, %11\n\t"
        "v_bcnt_u32_b32 %1, %7, %1\n\t"
        "v_and_b32 %7, %8, %12\n\t"
        "v_bcnt_u32_b32 %2, %6, %2\n\t"
        "v_and_b32 %6, %8, %13\n\t"
        "v_bcnt_u32_b32 %3, %7, %3\n\t"
        "v_and_b32 %7, %8, %14\n\t"
        "v_bcnt_u32_b32 %4, %6, %4\n\t"
        "v_bcnt_u32_b32 %5, %7, %5"
        : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]), "+v"(acc[4]), "+v"(acc[5]), "=&v"(t0), "=&v"(t1)
        : "v"(a), "v"(w[0]), "v"(w[1]), "v"(w[2]), "v"(w[3]), "v"(w[4]), "v"(w[5]));
}

template <>
__device__ __forceinline__ void and_popc_group<8>(int (&acc)[8], uint32_t a, const uint32_t (&w)[8])
{
    uint32_t t0, t1;
    asm("v_and_b32 %8, %10, %11\n\t"
        "v_and_b32 %9, %10, %12\n\t"
        "v_bcnt_u32_b32 %0, %8, %0\n\t"
        "v_and_b32 %8, %10, %13\n\t"
        "v_bcnt_u32_b32 %1, %9, %1\n\t"
        "v_and_b32 %9, %10, %14\n\t"
        "v_bcnt_u32_b32 %2, %8, %2\n\t"
        "v_and_b32 %8, %10, %15\n\t"
        "v_bcnt_u32_b32 %3, %9, %3\n\t"
        "v_and_b32 %9, %10, %16\n\t"
        "v_bcnt_u32_b32 %4, %8, %4\n\t"
        "v_and_b32 %8, %10, %17\n\t"
        "v_bcnt_u32_b32 %5, %9, %5\n\t"
        "v_and_b32 %9, %10, %18\n\t"
        "v_bcnt_u32_b32 %6, %8, %6\n\t"
        "v_bcnt_u32_b32 %7, %9, %7"
        : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]), "+v"(acc[4]), "+v"(acc[5]), "+v"(acc[6]),
          "+v"(acc[7]), "=&v"(t0), "=&v"(t1)
        : "v"(a), "v"(w[0]), "v"(w[1]), "v"(w[2]), "v"(w[3]), "v"(w[4]), "v"(w[5]), "v"(w[6]), "v"(w[7]));
}

__device__ __forceinline__ void popc_acc(int &acc, uint32_t a)
{
    asm("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc) : "v"(a));
}

// n / d for 0 <= n, n * d < 2^32, with magic = ceil(2^32 / d) computed on the host (0 stands for d = 1).
// Branch-free on purpose (the mask adds n back when d = 1): the magic is uniform, and the compiler
// otherwise turns the two cases into a branch, which a wave that is alone on its SIMD pays for in full.
__device__ __forceinline__ int fast_div(int n, uint32_t magic)
{
    const uint32_t one = (uint32_t)-(int)(magic == 0u);
    return (int)(__umulhi((uint32_t)n, magic) + ((uint32_t)n & one));
}

// n / d where the host could not promise n * d < 2^32: magic 1 (no divisor has it) asks for the hardware's
// division sequence instead, about ten times as many instructions.
__device__ __forceinline__ int checked_div(int n, int d, uint32_t magic)
{
    return __builtin_expect(magic == 1u, 0) ? n / d : fast_div(n, magic);
}

}  // namespace
