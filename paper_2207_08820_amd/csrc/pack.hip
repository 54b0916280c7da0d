// Bitplane packing for gfx950 (Section V of arXiv 2207.08820: operands are split into
// separate bitplanes), with the forward quantizer of Section IV fused in front for float input.
//
// One lane builds one output word per plane: it loads the 32 elements of that word (two 16-byte
// loads for byte sources; neighbouring lanes take neighbouring words, so a wave reads 2 KB of
// contiguous input), isolates bit p of every byte with a shift and a mask, and lets
// v_dot4_u32_u8 gather the four bits of a dword: a dot product of the 0/1 bytes with the byte
// vector {1,2,4,8} (or {16,32,64,128} for the odd dword of a pair) IS the 4-bit gather, and its
// accumulator operand chains two dwords into a finished byte of the output word.  That is about
// 0.75 VALU instructions per element and plane, against 4 for a wave64 ballot (compare + mask +
// moving the two ballot words into the lanes that store them), which measured 0.19 of the HBM
// roofline on 4096 x 4096 bytes; no LDS, no barriers.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dlrt.h"
#include "launch.h"

namespace {

constexpr int kThreads = 256;

struct Quant {
    float lo, hi;
    int bipolar;  // bit = value > 0
};

__device__ __forceinline__ uint32_t dot4(uint32_t a, uint32_t b, uint32_t c)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_udot4(a, b, c, false);
#else
    (void)a; (void)b;
    return c;  // host pass of the single-source compile: never executed
#endif
}

// x[d] holds elements 4d .. 4d+3 of the word as bytes whose low BITS bits are the pattern.
template <int BITS>
__device__ __forceinline__ void gather32(const uint32_t (&x)[8], uint32_t (&out)[BITS])
{
#pragma unroll
    for (int p = 0; p < BITS; ++p) {
        uint32_t word = 0;
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            const uint32_t even = (x[2 * h] >> p) & 0x01010101u, odd = (x[2 * h + 1] >> p) & 0x01010101u;
            const uint32_t byte = dot4(odd, 0x80402010u, dot4(even, 0x08040201u, 0u));
            word |= byte << (8 * h);
        }
        out[p] = word;
    }
}

// bytes -> 0/1 per byte for "value > 0" (bipolar bit); SIGNED: bytes are int8, else uint8
template <bool SIGNED>
__device__ __forceinline__ uint32_t positive_bytes(uint32_t x)
{
    const uint32_t nonzero = (((x & 0x7f7f7f7fu) + 0x7f7f7f7fu) | x) & 0x80808080u;  // bit 7 set iff byte != 0
    return (SIGNED ? (nonzero & ~x) : nonzero) >> 7;
}

template <int SRC, int BITS>
__global__ __launch_bounds__(kThreads) void pack_kernel(const dlrt::PackArgs p, const Quant q, int64_t Kw,
                                                        int64_t total_words, int aligned)
{
    const int64_t wi = (int64_t)blockIdx.x * kThreads + threadIdx.x;  // flat output word, row-major
    if (wi >= total_words) return;
    const int64_t r = wi / Kw, kwd = wi - r * Kw;
    const int64_t k0 = kwd * 32;
    const int valid = (int)(p.K - k0 < 32 ? p.K - k0 : 32);  // elements of this word inside the row

    uint32_t x[8];
    if (SRC == DLRT_SRC_F32) {
        const float *s = static_cast<const float *>(p.src) + r * p.ld + k0;
        // one scale for the tensor, one per row, or one per group of `taps` rows (an output channel's taps)
        const float sc = p.scale[p.scale_per_row == 0 ? 0 : p.scale_per_row == 1 ? r : r / p.taps];
#pragma unroll
        for (int d = 0; d < 8; ++d) {
            float v[4] = {0.f, 0.f, 0.f, 0.f};
            if (aligned && 4 * d + 4 <= valid) {
                const float4 t = *reinterpret_cast<const float4 *>(s + 4 * d);
                v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (4 * d + e < valid) v[e] = s[4 * d + e];
            }
            uint32_t w = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                // Section IV: round(clip(t / s, lo, hi)); IEEE division, ties to even.  Bipolar has no zero
                // level, so its quantizer is the sign of t / s with zero counted as +1.
                const float ts = v[e] / sc;
                const int qi = (int)rintf(fminf(fmaxf(ts, q.lo), q.hi));
                const uint32_t pat = q.bipolar ? (ts >= 0.0f ? 1u : 0u) : ((uint32_t)qi & 0xffu);
                w |= (4 * d + e < valid ? pat : 0u) << (8 * e);
            }
            x[d] = w;
        }
    } else {
        const uint8_t *s = static_cast<const uint8_t *>(p.src) + r * p.ld + k0;
        if (aligned && valid == 32) {
            const uint4 lo = *reinterpret_cast<const uint4 *>(s), hi = *reinterpret_cast<const uint4 *>(s + 16);
            x[0] = lo.x; x[1] = lo.y; x[2] = lo.z; x[3] = lo.w;
            x[4] = hi.x; x[5] = hi.y; x[6] = hi.z; x[7] = hi.w;
        } else {
#pragma unroll
            for (int d = 0; d < 8; ++d) {
                uint32_t w = 0;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (4 * d + e < valid) w |= (uint32_t)s[4 * d + e] << (8 * e);
                x[d] = w;
            }
        }
        if (q.bipolar) {
#pragma unroll
            for (int d = 0; d < 8; ++d) x[d] = positive_bytes<SRC == DLRT_SRC_I8>(x[d]);
        }
    }

    uint32_t out[BITS];
    gather32<BITS>(x, out);
    const int64_t outer = r / p.taps, tap = r - outer * p.taps;
    uint32_t *d = p.dst + outer * p.outer_stride + tap * p.tap_stride + kwd;
#pragma unroll
    for (int b = 0; b < BITS; ++b) d[b * p.plane_stride] = out[b];
}

template <int SRC>
dlrt_status launch_bits(const dlrt::PackArgs &p, const Quant &q, int64_t Kw, int64_t total, int aligned,
                        unsigned blocks, hipStream_t stream)
{
    switch (p.bits) {
    case 1: return dlrt::enqueue(pack_kernel<SRC, 1>, dim3(blocks), dim3(kThreads), 0, stream, p, q, Kw, total, aligned);
    case 2: return dlrt::enqueue(pack_kernel<SRC, 2>, dim3(blocks), dim3(kThreads), 0, stream, p, q, Kw, total, aligned);
    case 3: return dlrt::enqueue(pack_kernel<SRC, 3>, dim3(blocks), dim3(kThreads), 0, stream, p, q, Kw, total, aligned);
    case 4: return dlrt::enqueue(pack_kernel<SRC, 4>, dim3(blocks), dim3(kThreads), 0, stream, p, q, Kw, total, aligned);
    }
    return DLRT_ERR_BITS;
}

}  // namespace

namespace dlrt {

dlrt_status launch_pack(const PackArgs &p, hipStream_t stream)
{
    const int64_t Kw = (p.K + 31) / 32;
    const int64_t total = p.rows * Kw;
    Quant q{};
    q.bipolar = p.enc == DLRT_BIPOLAR;
    if (p.enc == DLRT_UNSIGNED) { q.lo = 0.f; q.hi = (float)((1 << p.bits) - 1); }
    else if (p.enc == DLRT_TWOS) { q.lo = -(float)(1 << (p.bits - 1)); q.hi = (float)((1 << (p.bits - 1)) - 1); }
    else { q.lo = -1.f; q.hi = 1.f; }

    // 16-byte loads need every word's first element 16-byte aligned: base and row stride multiples
    // of 16 bytes (a word's 32 elements are 32 or 128 bytes, so words within a row stay aligned)
    const uintptr_t addr = reinterpret_cast<uintptr_t>(p.src);
    const int64_t esize = p.src_type == DLRT_SRC_F32 ? 4 : 1;
    const int aligned = addr % 16 == 0 && (p.ld * esize) % 16 == 0;

    const int64_t blocks = (total + kThreads - 1) / kThreads;
    if (blocks > 0x7fffffffLL) return DLRT_ERR_SHAPE;

    switch (p.src_type) {
    case DLRT_SRC_U8: return launch_bits<DLRT_SRC_U8>(p, q, Kw, total, aligned, (unsigned)blocks, stream);
    case DLRT_SRC_I8: return launch_bits<DLRT_SRC_I8>(p, q, Kw, total, aligned, (unsigned)blocks, stream);
    case DLRT_SRC_F32: return launch_bits<DLRT_SRC_F32>(p, q, Kw, total, aligned, (unsigned)blocks, stream);
    default: return DLRT_ERR_SHAPE;
    }
}

}  // namespace dlrt
