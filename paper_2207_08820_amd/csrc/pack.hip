// Bitplane packing for gfx950 (Section V of arXiv 2207.08820: operands are split into
// separate bitplanes), with the forward quantizer of Section IV fused in front for float input.
//
// The output words of all rows form one flat sequence (row-major over [row][word]); a wave
// takes 32 consecutive words = 1024 elements per step.  Each lane loads 4 consecutive elements
// (one dword of bytes, or one float4) so that a wave reads whole contiguous segments, reduces them
// to their bit patterns, and parks the 4 pattern bytes in LDS.  Reading the bytes back with a
// stride of one byte per lane puts 64 consecutive elements into the 64 lanes, and one wave64
// ballot per plane then yields two finished 32-bit words at once.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "dlrt.h"
#include "launch.h"

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

template <int N, int I = 0, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<N, I + 1>(f);
    }
}

struct Quant {
    float lo, hi;
    int mask;     // (1 << bits) - 1
    int bipolar;  // bit = value > 0
};

// Put the two halves of a wave-uniform 64-bit ballot into lanes LANE and LANE + 1 of `old`, leaving
// the other lanes (two VALU ops).  On gfx950 a VALU instruction that reads an SGPR as data needs two
// wait states after the VALU instruction that wrote it (here the v_cmp of the ballot); the compiler
// inserts them for its own code but cannot see into asm, so the block carries its own s_nop.
template <int LANE>
__device__ __forceinline__ uint32_t put_lane_pair(unsigned long long m, uint32_t old)
{
    const uint32_t lo = (uint32_t)m, hi = (uint32_t)(m >> 32);
    asm("s_nop 1\n\t"
        "v_writelane_b32 %0, %1, %3\n\t"
        "v_writelane_b32 %0, %2, %4"
        : "+v"(old)
        : "s"(lo), "s"(hi), "n"(LANE), "n"(LANE + 1));
    return old;
}

template <int SRC>
__device__ __forceinline__ uint32_t patterns_of_4(const dlrt::PackArgs &p, const Quant &q, int64_t r, int64_t k,
                                                  bool aligned)
{
    // Returns the bit patterns of elements k..k+3 of row r, one per byte; elements at or beyond K are 0.
    int v[4] = {0, 0, 0, 0};
    if (SRC == DLRT_SRC_F32) {
        const float *s = static_cast<const float *>(p.src) + r * p.ld + k;
        float x[4] = {0.f, 0.f, 0.f, 0.f};
        if (aligned && k + 4 <= p.K) {
            const float4 t = *reinterpret_cast<const float4 *>(s);
            x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (k + e < p.K) x[e] = s[e];
        }
        const float sc = p.scale[p.scale_per_row ? r : 0];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            // Section IV: round(clip(t / s, lo, hi)); IEEE division, ties to even
            const float t = fminf(fmaxf(x[e] / sc, q.lo), q.hi);
            v[e] = (k + e < p.K) ? (int)rintf(t) : 0;
        }
    } else {
        const uint8_t *s = static_cast<const uint8_t *>(p.src) + r * p.ld + k;
        uint32_t w = 0;
        if (aligned && k + 4 <= p.K) {
            w = *reinterpret_cast<const uint32_t *>(s);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (k + e < p.K) w |= (uint32_t)s[e] << (8 * e);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t b = (w >> (8 * e)) & 0xffu;
            v[e] = SRC == DLRT_SRC_I8 ? (int)(int8_t)b : (int)b;
        }
    }
    uint32_t out = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const uint32_t pat = q.bipolar ? (v[e] > 0 ? 1u : 0u) : ((uint32_t)v[e] & (uint32_t)q.mask);
        out |= pat << (8 * e);
    }
    return out;
}

template <int SRC, int BITS>
__global__ __launch_bounds__(kThreads) void pack_kernel(const dlrt::PackArgs p, const Quant q, int64_t Kw,
                                                        int64_t total_words, int aligned)
{
    __shared__ uint32_t park[kWaves][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint8_t *bytes = reinterpret_cast<const uint8_t *>(park[wave]);
    const int64_t steps = (total_words + 31) / 32;

    // every wave of a block runs the same number of iterations so that the barriers match
    for (int64_t it = blockIdx.x; it * kWaves < steps; it += gridDim.x) {
        const int64_t base = (it * kWaves + wave) * 32;  // first flat word of this wave's step
        uint32_t outw[BITS];
#pragma unroll
        for (int b = 0; b < BITS; ++b) outw[b] = 0;

        static_for<4>([&](auto sub_c) {
            constexpr int sub = decltype(sub_c)::value;
            const int64_t wi = base + sub * 8 + (lane >> 3);
            uint32_t pat = 0;
            if (wi < total_words) {
                const int64_t r = wi / Kw, kwd = wi - r * Kw;
                pat = patterns_of_4<SRC>(p, q, r, kwd * 32 + 4 * (lane & 7), aligned != 0);
            }
            __syncthreads();
            park[wave][lane] = pat;
            __syncthreads();
            static_for<4>([&](auto t_c) {
                constexpr int t = decltype(t_c)::value;
                const uint32_t v = bytes[64 * t + lane];
#pragma unroll
                for (int b = 0; b < BITS; ++b) {
                    const unsigned long long m = __ballot((v >> b) & 1u);
                    // words sub*8 + 2t and sub*8 + 2t + 1 of this step belong to those lanes
                    outw[b] = put_lane_pair<sub * 8 + 2 * t>(m, outw[b]);
                }
            });
        });

        const int64_t wi = base + lane;
        if (lane < 32 && wi < total_words) {
            const int64_t r = wi / Kw, kwd = wi - r * Kw;
            const int64_t outer = r / p.taps, tap = r - outer * p.taps;
            uint32_t *d = p.dst + outer * p.outer_stride + tap * p.tap_stride + kwd;
#pragma unroll
            for (int b = 0; b < BITS; ++b) d[b * p.plane_stride] = outw[b];
        }
    }
}

template <int SRC>
dlrt_status launch_bits(const dlrt::PackArgs &p, const Quant &q, int64_t Kw, int64_t total, int aligned,
                        unsigned blocks, hipStream_t stream)
{
    switch (p.bits) {
    case 1: hipLaunchKernelGGL((pack_kernel<SRC, 1>), dim3(blocks), dim3(kThreads), 0, stream, p, q, Kw, total, aligned); break;
    case 2: hipLaunchKernelGGL((pack_kernel<SRC, 2>), dim3(blocks), dim3(kThreads), 0, stream, p, q, Kw, total, aligned); break;
    case 3: hipLaunchKernelGGL((pack_kernel<SRC, 3>), dim3(blocks), dim3(kThreads), 0, stream, p, q, Kw, total, aligned); break;
    case 4: hipLaunchKernelGGL((pack_kernel<SRC, 4>), dim3(blocks), dim3(kThreads), 0, stream, p, q, Kw, total, aligned); break;
    default: return DLRT_ERR_BITS;
    }
    return hipGetLastError() == hipSuccess ? DLRT_OK : DLRT_ERR_LAUNCH;
}

}  // namespace

namespace dlrt {

dlrt_status launch_pack(const PackArgs &p, hipStream_t stream)
{
    const int64_t Kw = (p.K + 31) / 32;
    const int64_t total = p.rows * Kw;
    Quant q{};
    q.mask = (1 << p.bits) - 1;
    q.bipolar = p.enc == DLRT_BIPOLAR;
    if (p.enc == DLRT_UNSIGNED) { q.lo = 0.f; q.hi = (float)((1 << p.bits) - 1); }
    else if (p.enc == DLRT_TWOS) { q.lo = -(float)(1 << (p.bits - 1)); q.hi = (float)((1 << (p.bits - 1)) - 1); }
    else { q.lo = -1.f; q.hi = 1.f; }

    const uintptr_t addr = reinterpret_cast<uintptr_t>(p.src);
    int aligned;
    if (p.src_type == DLRT_SRC_F32) aligned = addr % 16 == 0 && p.ld % 4 == 0;
    else aligned = addr % 4 == 0 && p.ld % 4 == 0;

    const int64_t steps = (total + 31) / 32;
    int64_t blocks = (steps + kWaves - 1) / kWaves;
    if (blocks > 256 * 16) blocks = 256 * 16;  // grid-stride beyond 16 blocks per compute unit
    if (blocks < 1) blocks = 1;

    switch (p.src_type) {
    case DLRT_SRC_U8: return launch_bits<DLRT_SRC_U8>(p, q, Kw, total, aligned, (unsigned)blocks, stream);
    case DLRT_SRC_I8: return launch_bits<DLRT_SRC_I8>(p, q, Kw, total, aligned, (unsigned)blocks, stream);
    case DLRT_SRC_F32: return launch_bits<DLRT_SRC_F32>(p, q, Kw, total, aligned, (unsigned)blocks, stream);
    default: return DLRT_ERR_SHAPE;
    }
}

}  // namespace dlrt
